// Shared device helpers of libw4a4 (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/w4a4.h"

namespace w4a4 {

constexpr int kWave = 64;

// ---- wavefront reductions (64 lanes) -------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
    return v;
}

// ---- reduce-scatter of 32 values over the 32 lanes of a half wave ---------------------
// On entry every lane of a 32-lane half holds v[0..31]; on return v[0] of lane c (c = lane & 31)
// is op over the 32 lanes of v[c].  Five halving steps; in the step for index bit b a lane
// keeps the entries whose bit b equals its own lane bit b and hands the others to a partner
// whose lane bit b differs and whose higher bits agree.  Bit 4 swaps 16-lane rows between two
// registers in place; bits 3..0 pair the lanes through the cross-lane operand modes
// (row mirror, half-row mirror, two quad permutes), so no step goes through the LDS.
template <int CTRL, typename T>
__device__ __forceinline__ T dpp_fetch(T x) {
    static_assert(sizeof(T) == 4, "one register");
    const int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(T, r);
}
template <int O, int CTRL, typename T, typename Op>
__device__ __forceinline__ void reduce_scatter_step(T (&v)[32], int lane, Op op) {
    const bool up = (lane & O) != 0;
#pragma unroll
    for (int k = 0; k < O; ++k) {
        const T keep = up ? v[k + O] : v[k];
        const T send = up ? v[k] : v[k + O];
        v[k] = op(keep, dpp_fetch<CTRL>(send));
    }
}
template <typename T, typename Op>
__device__ __forceinline__ void reduce_scatter32(T (&v)[32], int lane, Op op) {
    static_assert(sizeof(T) == 4, "one register per value");
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        // rows 1 and 3 of v[k] change places with rows 0 and 2 of v[k+16]: afterwards both
        // registers hold, in every lane, the two partial results of the entry that lane keeps
        const auto sw = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, v[k]),
                                                         __builtin_bit_cast(unsigned, v[k + 16]), false, false);
        v[k] = op(__builtin_bit_cast(T, (unsigned)sw[0]), __builtin_bit_cast(T, (unsigned)sw[1]));
    }
    reduce_scatter_step<8, 0x140>(v, lane, op);                   // row mirror: lane i <-> 15 - i
    reduce_scatter_step<4, 0x141>(v, lane, op);                   // half-row mirror: i <-> 7 - i
    reduce_scatter_step<2, 0x4E>(v, lane, op);                    // quad permute [2,3,0,1]
    reduce_scatter_step<1, 0xB1>(v, lane, op);                    // quad permute [1,0,3,2]
}

// ---- the Sec. 3.1 mappings, b = 4 ----------------------------------------------------
// A vector's range is summarised as (lo, inv, S): code = rne(clamp((x - lo) * inv)).
// The reciprocal is one correctly rounded fp32 divide per vector; the per-element
// multiply and the round-to-nearest-even are separate fp32 operations (the library is
// compiled without FMA contraction), so codes are reproducible bit for bit.
struct Range {
    float lo;    // 0 for the symmetric mapping, min(x) for the asymmetric one
    float inv;   // 7/absmax or 15/(max-min); 0 for a constant vector
    float S;     // absmax/7 or (max-min)/15; 1 for a constant vector
};

__device__ __forceinline__ Range range_sym(float amax) {
    Range r;
    r.lo = 0.0f;
    if (amax == 0.0f) { r.inv = 0.0f; r.S = 1.0f; }
    else { r.inv = 7.0f / amax; r.S = amax / 7.0f; }
    return r;
}
__device__ __forceinline__ Range range_asym(float lo, float hi) {
    Range r;
    r.lo = lo;
    if (hi == lo) { r.inv = 0.0f; r.S = 1.0f; }
    else { float d = hi - lo; r.inv = 15.0f / d; r.S = d / 15.0f; }
    return r;
}
template <int MODE>
__device__ __forceinline__ int code_of(float x, const Range &r) {
    if (MODE == W4A4_SYM) {
        float t = x * r.inv;
        t = fminf(fmaxf(t, -8.0f), 7.0f);
        return (int)rintf(t);
    } else {
        float d = x - r.lo;
        float t = d * r.inv;
        t = fminf(fmaxf(t, 0.0f), 15.0f);
        return (int)rintf(t);
    }
}

// erf-form GELU (Sec. 4.2 names GELU; BERT's is the erf form): gelu(x) = x * Phi(x) with
// Phi the standard normal CDF.  Evaluated as  max(x,0) - t * Phi(-t),  t = min(|x|, 6), with
// Phi(-t) = 2^q(t) and q a degree-7 polynomial fitted to log2 Phi(-t) on [0,6].  The form
// keeps RELATIVE accuracy in the negative tail (where gelu is tiny) and costs eight FMAs and
// one v_exp_f32, about a third of a libm-grade erff.  Against the float64 erf form: relative
// error < 5e-6 wherever |gelu| exceeds the smallest fp16 subnormal, absolute error < 7e-7.
struct GeluParts { float relu, t, p; };                          // gelu(x) = relu - t * p
__device__ __forceinline__ GeluParts gelu_parts(float x) {
    GeluParts g;
    g.t = fminf(fabsf(x), 6.0f);
    float q = -1.889626219e-06f;
    q = __fmaf_rn(q, g.t, 6.268139987e-05f);
    q = __fmaf_rn(q, g.t, -9.388679173e-04f);
    q = __fmaf_rn(q, g.t, 8.539461531e-03f);
    q = __fmaf_rn(q, g.t, -5.402068794e-02f);
    q = __fmaf_rn(q, g.t, -4.584097862e-01f);
    q = __fmaf_rn(q, g.t, -1.151269197e+00f);
    q = __fmaf_rn(q, g.t, -9.999943376e-01f);
    g.p = __builtin_amdgcn_exp2f(q);
    // max(x, 0) as a signed integer maximum on the bit pattern (one instruction, no NaN canonicalisation)
    g.relu = __int_as_float(max(__float_as_int(x), 0));
    return g;
}
__device__ __forceinline__ float gelu_erf(float x) {
    const GeluParts g = gelu_parts(x);
    return __fmaf_rn(-g.t, g.p, g.relu);
}
// GELU for the fp16 stores.  An fp16 result carries 11 significant bits, so the stores use a cheaper form of the
// same evaluation: q of degree 5 (fitted to log2 Phi(-t) on [0,6] with the error weighted by what an fp16 result
// can show), relative error < 9e-5 wherever |gelu| is a normal fp16 number, i.e. at most one fp16 step from the
// float64 erf form and equal to its rounding for about 95 % of the values.  The leading coefficient is negative
// and q falls monotonically beyond the fitted range (q(6) = -30, q(12) = -124), so t needs no clamp: for large
// |x| the correction t * 2^q underflows to zero by itself and the result is max(x,0).  The last FMA and the
// conversion are one instruction per half (v_fma_mix*_f16: fp32 sources, |x| and the negation as operand
// modifiers, the exact fused result rounded ONCE to fp16).  Every fp16 GELU output of the library goes through
// here, so all kernels agree bit for bit.  Eight instructions per value; gelu_erf() above (degree 7) remains the
// form for fp32 results that are quantized afterwards, where its extra accuracy decides codes.
__device__ __forceinline__ float gelu_tail_f16(float x) {        // Phi(-|x|) to fp16 accuracy
    const float t = fabsf(x);
    float q = -3.204851180e-04f;
    q = __fmaf_rn(q, t, 5.827001986e-03f);
    q = __fmaf_rn(q, t, -4.823611915e-02f);
    q = __fmaf_rn(q, t, -4.641228736e-01f);
    q = __fmaf_rn(q, t, -1.149174450e+00f);
    q = __fmaf_rn(q, t, -1.000121072e+00f);
    return __builtin_amdgcn_exp2f(q);
}
__device__ __forceinline__ uint32_t gelu_erf_half2(float x0, float x1) {
    const float p0 = gelu_tail_f16(x0), p1 = gelu_tail_f16(x1);
    const float r0 = __int_as_float(max(__float_as_int(x0), 0)), r1 = __int_as_float(max(__float_as_int(x1), 0));
    uint32_t d;
    asm("v_fma_mixlo_f16 %0, -|%1|, %2, %3" : "=v"(d) : "v"(x0), "v"(p0), "v"(r0));
    asm("v_fma_mixhi_f16 %0, -|%1|, %2, %3" : "+v"(d) : "v"(x1), "v"(p1), "v"(r1));
    return d;
}
__device__ __forceinline__ unsigned short gelu_erf_half(float x) {
    const float p = gelu_tail_f16(x);
    const float r = __int_as_float(max(__float_as_int(x), 0));
    uint32_t d;
    asm("v_fma_mixlo_f16 %0, -|%1|, %2, %3" : "=v"(d) : "v"(x), "v"(p), "v"(r));
    return (unsigned short)(d & 0xFFFFu);
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() {
    return hipGetLastError() == hipSuccess ? W4A4_OK : W4A4_ERR_HIP;
}

// Kernel-boundary timestamps for the caller's roofline figure (w4a4_time_next_gemm): when the
// thread is armed, the GEMM launch goes through hipExtLaunchKernelGGL, which stamps the two events
// with the start and the end of the kernel itself, and disarms.
struct KernelTimer { hipEvent_t start = nullptr, stop = nullptr; };
KernelTimer &kernel_timer();                                     // thread-local, lives in api.hip
template <typename... KArgs, typename... Args>
inline void launch_gemm(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    KernelTimer &t = kernel_timer();
    if (t.start || t.stop) {
        hipExtLaunchKernelGGL(kern, grid, block, (unsigned)lds, st, t.start, t.stop, 0, args...);
        t = KernelTimer{};
    } else {
        hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
    }
}

// Per-device launch state of one kernel instantiation: the dynamic-LDS limit already granted and the CU
// count.  Function attributes and CU counts belong to a device and a process may use several, so both are
// kept per device (races between threads are benign: the calls are idempotent).
constexpr int kMaxDevices = 16;
// Per-kernel, per-device launch state.  The LDS limit of a kernel only ever grows: raising it happens under
// the mutex, reading it does not need one.
struct KernelState {
    std::atomic<size_t> lds[kMaxDevices] = {};
    std::atomic<int> cus[kMaxDevices] = {};
    std::atomic<int> occ[kMaxDevices] = {};                        // workgroups of this kernel a CU holds at once (0 = not asked yet)
    std::mutex grow;
};
// Lets `kern` use `lds` bytes of dynamic LDS on the current device.  Returns that device's CU count, or -1.
inline int prepare_kernel(const void *kern, size_t lds, KernelState &ks) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    if (lds > ks.lds[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(ks.grow);
        if (lds > ks.lds[dev].load(std::memory_order_relaxed)) {
            if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return -1;
            ks.lds[dev].store(lds, std::memory_order_release);
        }
    }
    int cus = ks.cus[dev].load(std::memory_order_relaxed);
    if (!cus) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return -1;
        ks.cus[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

// Workgroups of `kern` (block size `threads`, `lds` bytes of dynamic LDS) that the runtime says one CU holds at
// once on the current device; asked once per kernel and device.  Kernels whose workgroups wait for each other
// size their grid from this figure, never from the attributes they were compiled with.  Returns -1 on error.
inline int resident_per_cu(const void *kern, int threads, size_t lds, KernelState &ks) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    int occ = ks.occ[dev].load(std::memory_order_relaxed);
    if (!occ) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, threads, lds) != hipSuccess || occ < 0) return -1;
        if (occ == 0) return 0;                                    // does not fit at all: nothing to remember
        ks.occ[dev].store(occ, std::memory_order_relaxed);
    }
    return occ;
}

// How the token-wise quantizer of the FP6 operand layout (see w4a4_layout) splits a row of K codes: lanes per token
// (LPR: 8, 16, 32 or 64, a divisor of K / 32) and operands of 32 codes per lane (OPL = K / 32 / LPR).  The fewest lanes
// that keep OPL <= 2 (a lane then holds at most eight 16-byte chunks, what the quantizer runs fastest with), else
// <= 3, 4, 6.  False for a K the layout is not offered for.
inline bool fp6_plan(int K, int *lpr, int *opl) {
    if (K <= 0 || K % 64 || K > 10240) return false;           // (the quantizer stages eight rows in 64 KB of LDS)
    const int n_op = K / 32;
    for (int most : {2, 3, 4, 6})
        for (int l = 8; l <= 64; l <<= 1)
            if (n_op % l == 0 && n_op / l <= most) {
                *lpr = l;
                *opl = n_op / l;
                return true;
            }
    return false;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace w4a4
