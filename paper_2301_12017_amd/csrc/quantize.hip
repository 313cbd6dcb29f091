// Row-wise INT4 quantization kernels: token-wise activations (step a1), offline weights
// (step a0) and the requantize of fp32 rows used behind the GEMM.
//
// One wavefront owns one row.  The row is read once with 16-byte loads, kept in
// registers, reduced with wave shuffles (absmax, or min and max), mapped to codes with
// the Sec. 3.1 formulas and written as one dword (eight codes) per lane per step, so
// both the read and the write are fully coalesced.  HBM traffic is the algorithmic
// minimum: 2 bytes in and half a byte out per element.
#include "common.hpp"

namespace w4a4 {

constexpr int kRowsPerBlock = 4;      // four waves, one row each
constexpr int kMaxGroups = 512;       // code-sum slots per row held in LDS

template <typename T> struct Load8;
template <> struct Load8<__half> {
    // eight consecutive fp16 -> fp32
    static __device__ __forceinline__ void load(const __half *p, float (&v)[8]) {
        uint4 raw = *reinterpret_cast<const uint4 *>(p);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float2 f = __half22float2(h[i]);
            v[2 * i] = f.x;
            v[2 * i + 1] = f.y;
        }
    }
};
template <> struct Load8<float> {
    static __device__ __forceinline__ void load(const float *p, float (&v)[8]) {
        float4 a = *reinterpret_cast<const float4 *>(p);
        float4 b = *reinterpret_cast<const float4 *>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};

// X: [rows, ldx] elements, first K used.  q: [rows, K/2] bytes.  s,z: [rows].
// gsum: [rows, ng] code sums over runs of G elements (NULL = not wanted).
// ITERS = ceil(K / 512): every lane holds ITERS chunks of eight elements.
// LAYOUT: 0 = canonical nibbles; 1 = MFMA operand layout of activations; 2 = MFMA operand layout of
// weights (the nibbles of a byte swapped).  In both, the element that lands in the HIGH nibble is stored as a
// two's-complement value and the one in the LOW nibble as an unsigned one, so that `byte & 0xF0` and `byte & 0x0F`
// are int8 MFMA operands as they stand:
//   symmetric codes c in [-8,7]:  high nibble c, low nibble c + 8;
//   unsigned codes u in [0,15]:   high nibble u - 8, low nibble u.
// psum receives the code sums the GEMM needs to take the offsets out again:
//   symmetric, layout 1: psum[row] = sum of the odd-position codes; layout 2: of the even-position codes;
//   unsigned,  layout 1: psum[g * rows + row] = 128 * (sum of the even-position codes of K-group g), the C operand
//                        of that group's first MFMAs;
//   unsigned,  layout 2: psum[row + row / psum_per] = sum of the odd-position codes (rows are (channel, group)
//                        pairs, psum_per groups per channel: one spare word per channel follows its sums).
template <int MODE, typename T, int ITERS, int LAYOUT>
__global__ __launch_bounds__(kRowsPerBlock *kWave) void quantize_rows_kernel(
    const T *__restrict__ X, long ldx, int rows, int K, int G, uint8_t *__restrict__ q,
    float *__restrict__ s, float *__restrict__ z, int32_t *__restrict__ gsum, int ng,
    int32_t *__restrict__ psum, int psum_per) {
    __shared__ int32_t gs[kRowsPerBlock][kMaxGroups];
    __shared__ int32_t es[LAYOUT == 1 && MODE == W4A4_ASYM ? kRowsPerBlock : 1][LAYOUT == 1 && MODE == W4A4_ASYM ? kMaxGroups : 1];
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const long row = (long)blockIdx.x * kRowsPerBlock + wave;
    if (row >= rows) return;                       // whole wave leaves; no block barrier below
    const int nchunks = K / 8;
    const T *xr = X + row * ldx;

    float v[ITERS][8];
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        if (c < nchunks) {
            Load8<T>::load(xr + (long)c * 8, v[it]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (MODE == W4A4_SYM) hi = fmaxf(hi, fabsf(v[it][e]));
                else { hi = fmaxf(hi, v[it][e]); lo = fminf(lo, v[it][e]); }
            }
        }
    }
    Range r;
    if (MODE == W4A4_SYM) {
        r = range_sym(wave_max(hi));
    } else {
        r = range_asym(wave_min(lo), wave_max(hi));
    }
    if (lane == 0) {
        s[row] = r.S;
        if (MODE == W4A4_ASYM) z[row] = r.lo;
    }
    constexpr bool GROUP_PSUM = LAYOUT == 1 && MODE == W4A4_ASYM;    // even-position sums per K-group
    if (gsum || GROUP_PSUM) {
        for (int g = lane; g < ng; g += kWave) {
            gs[wave][g] = 0;
            if (GROUP_PSUM) es[wave][g] = 0;
        }
        // lanes of one wave run in lockstep and LDS operations of a wave complete in
        // order, so the zeroes land before the adds below.
        __builtin_amdgcn_wave_barrier();
    }
    const int cpg = G / 8;                         // chunks per code-sum group
    uint32_t *qr = reinterpret_cast<uint32_t *>(q + row * (long)(K / 2));
    int part = 0;                                  // this lane's share of psum
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        if (c < nchunks) {
            uint32_t packed = 0;
            int sum = 0, esum_c = 0;
            // offset that turns a code into the nibble stored for it: symmetric codes gain 8 in the low nibble,
            // unsigned ones lose 8 in the high nibble
            constexpr int kLowAdd = MODE == W4A4_SYM ? 8 : 0, kHighAdd = MODE == W4A4_SYM ? 0 : -8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int code = code_of<MODE>(v[it][e], r);
                sum += code;
                if (LAYOUT == 0) {
                    packed |= (uint32_t)(code & 0xF) << (4 * e);
                } else if (LAYOUT == 1) {                        // odd elements sit in the high nibbles
                    if (MODE == W4A4_SYM) { if (e & 1) part += code; }
                    else if (!(e & 1)) esum_c += code;
                    packed |= (uint32_t)((code + ((e & 1) ? kHighAdd : kLowAdd)) & 0xF) << (4 * e);
                } else {                                         // nibbles swapped: even elements sit in the high nibbles
                    if (MODE == W4A4_SYM) { if (!(e & 1)) part += code; }
                    else if (e & 1) part += code;
                    packed |= (uint32_t)((code + ((e & 1) ? kLowAdd : kHighAdd)) & 0xF) << (4 * (e ^ 1));
                }
            }
            qr[c] = packed;
            if (gsum) atomicAdd(&gs[wave][c / cpg], sum);
            if (GROUP_PSUM) atomicAdd(&es[wave][c / cpg], esum_c);
        }
    }
    if (LAYOUT != 0 && !GROUP_PSUM) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, kWave);
        if (lane == 0) psum[MODE == W4A4_ASYM ? row + row / psum_per : row] = part;
    }
    if (gsum || GROUP_PSUM) {
        __builtin_amdgcn_wave_barrier();
        for (int g = lane; g < ng; g += kWave) {
            if (gsum) gsum[row * (long)ng + g] = gs[wave][g];
            if (GROUP_PSUM) psum[(long)g * rows + row] = 128 * es[wave][g];
        }
    }
}

// Row quantizer for fp16 activations (step a1, the run-time one), trimmed for the vector ALU: the
// range is taken on packed fp16 (v_pk_max_f16 on |x|, exact), the row stays in registers as raw
// fp16 (16 bytes per lane per chunk) and is converted once for the codes, rounding is an fp32 add
// of 1.5*2^23 (round-to-nearest-even, then the code sits in the low mantissa bits), symmetric
// codes are produced in offset binary so that nibble sums are byte sums (v_sad_u8) and one XOR per
// dword gives the wanted layout.  Loads go through a buffer descriptor of the row (chunks past K
// read as zero).  A wave owns rows w, w + W, ... of W waves and requests its next row before it
// touches the current one.  Code sums per K-group are segmented wave reductions (cpg = chunks per
// group must be a power of two <= 64, or the group is the whole row).
template <int MODE, int ITERS, int LAYOUT>
__global__ __launch_bounds__(kRowsPerBlock *kWave) void quantize_stream_kernel(
    const __half *__restrict__ X, long ldx, int rows, int K, uint8_t *__restrict__ q,
    float *__restrict__ s, float *__restrict__ z, int32_t *__restrict__ gsum, int ng, int cpg,
    int32_t *__restrict__ psum) {
    const int lane = threadIdx.x % kWave;
    const int nwaves = gridDim.x * kRowsPerBlock;
    const int nchunks = K / 8;
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    auto load_row = [&](long row, u4 (&raw)[ITERS]) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<__half *>(X + row * ldx), (short)0, K * 2, 0x00020000);
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
            raw[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, (lane + it * kWave) * 16, 0, 0);
    };
    auto unpack8 = [&](const u4 &r, float (&v)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __half2 h = *reinterpret_cast<const __half2 *>(&reinterpret_cast<const uint32_t *>(&r)[i]);
            const float2 f = __half22float2(h);
            v[2 * i] = f.x;
            v[2 * i + 1] = f.y;
        }
    };
    long row = (long)blockIdx.x * kRowsPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    u4 cur[ITERS], nxt[ITERS];
    if (row < rows) load_row(row, cur);
    while (row < rows) {
        const long next = row + nwaves;
        if (next < rows) load_row(next, nxt);
        // ---- range of the row, on packed fp16 (the maximum of fp16 values is exact in fp16)
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 hi2, lo2;
        {
            const uint32_t first = cur[0][0];
            const uint32_t init = MODE == W4A4_SYM ? 0u : (first & 0xFFFFu) * 0x10001u;   // SYM: 0; ASYM: element 0 twice
            hi2 = *reinterpret_cast<const h2 *>(&init);
            lo2 = hi2;
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            // chunks past K read as zero: harmless for |x| maxima; for min/max they are replaced by the row's
            // first element
            const bool in = lane + it * kWave < nchunks;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t d = cur[it][i];
                if (MODE == W4A4_SYM) {
                    d &= 0x7FFF7FFFu;
                    hi2 = __builtin_elementwise_max(hi2, *reinterpret_cast<const h2 *>(&d));
                } else {
                    const uint32_t sub = *reinterpret_cast<const uint32_t *>(&hi2);
                    if (!in) d = sub;
                    hi2 = __builtin_elementwise_max(hi2, *reinterpret_cast<const h2 *>(&d));
                    lo2 = __builtin_elementwise_min(lo2, *reinterpret_cast<const h2 *>(&d));
                }
            }
        }
        float hi = fmaxf((float)hi2[0], (float)hi2[1]);
        Range r;
        if (MODE == W4A4_SYM) {
            r = range_sym(wave_max(hi));
        } else {
            // lanes past K started from THEIR chunk's first element (zeros): take lane 0's as the neutral value
            const float lo = fminf((float)lo2[0], (float)lo2[1]);
            const bool any = lane < nchunks;
            const float hi0 = __shfl(hi, 0, kWave), lo0 = __shfl(lo, 0, kWave);
            r = range_asym(wave_min(any ? lo : lo0), wave_max(any ? hi : hi0));
        }
        if (lane == 0) {
            s[row] = r.S;
            if (MODE == W4A4_ASYM) z[row] = r.lo;
        }
        // ---- codes.  rne(t) for |t| < 2^22 is the low mantissa of t + 1.5*2^23 (the fp32 add rounds to
        // nearest even); the clamp of the definition cannot bind (|t| <= 7(1+2^-23), resp. t in [0, 15(1+2^-23)]).
        // Symmetric codes are produced in offset binary (code + 8: the +8 rides in the constant) so that nibble
        // sums are plain byte sums; one XOR per dword then gives the layout wanted.
        constexpr float kMagic = MODE == W4A4_SYM ? 12582920.0f : 12582912.0f;
        // symmetric codes leave offset binary where two's complement is wanted; unsigned codes of the operand
        // layout lose 8 in the high nibbles (u - 8 in two's complement is u with its top bit flipped)
        constexpr uint32_t kFlip = LAYOUT != 0 ? 0x80808080u : MODE == W4A4_ASYM ? 0u : 0x88888888u;
        constexpr bool GROUP_PSUM = LAYOUT != 0 && MODE == W4A4_ASYM;   // 128 * even-position sums per K-group
        uint32_t *qr = reinterpret_cast<uint32_t *>(q + row * (long)(K / 2));
        int part = 0, total = 0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int c = lane + it * kWave;
            float v[8];
            unpack8(cur[it], v);
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t;
                if (MODE == W4A4_SYM) t = v[e] * r.inv;
                else { float d = v[e] - r.lo; t = d * r.inv; }
                const float u = t + kMagic;
                packed |= (__float_as_uint(u) & 0xFu) << (4 * e);
            }
            const bool in = c < nchunks;
            const uint32_t even = packed & 0x0F0F0F0Fu, odd = (packed >> 4) & 0x0F0F0F0Fu;
            int sum = 0, esum_c = 0;
            if (gsum) sum = (int)__builtin_amdgcn_sad_u8(even, 0u, __builtin_amdgcn_sad_u8(odd, 0u, 0u)) - (MODE == W4A4_SYM ? 64 : 0);
            if (GROUP_PSUM) esum_c = (int)__builtin_amdgcn_sad_u8(even, 0u, 0u);
            if (LAYOUT != 0 && MODE == W4A4_SYM && in) part += (int)__builtin_amdgcn_sad_u8(odd, 0u, 0u) - 32;
            if (in) {
                qr[c] = packed ^ kFlip;
                total += sum;
                if (GROUP_PSUM) part += esum_c;
            } else {
                sum = 0;
                esum_c = 0;
            }
            if ((gsum || GROUP_PSUM) && ng > 1) {               // groups of cpg lanes, all inside this `it`
                for (int o = 1; o < cpg; o <<= 1) {
                    if (gsum) sum += __shfl_xor(sum, o, kWave);
                    if (GROUP_PSUM) esum_c += __shfl_xor(esum_c, o, kWave);
                }
                if ((lane & (cpg - 1)) == 0 && in) {
                    if (gsum) gsum[row * (long)ng + c / cpg] = sum;
                    if (GROUP_PSUM) psum[(long)(c / cpg) * rows + row] = 128 * esum_c;
                }
            }
        }
        if (gsum && ng == 1) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) total += __shfl_xor(total, o, kWave);
            if (lane == 0) gsum[row] = total;
        }
        if (LAYOUT != 0 && (!GROUP_PSUM || ng == 1)) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, kWave);
            if (lane == 0) psum[row] = GROUP_PSUM ? 128 * part : part;
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) cur[it] = nxt[it];
        row = next;
    }
}

// c[n] = sum over k of the dequantized weight, group by group in fp32:
// c = c + (S*RW + G*zero), each operation separately rounded.
__global__ void weight_rowsum_kernel(const float *__restrict__ scale, const float *__restrict__ zero,
                                     const int32_t *__restrict__ gsum, int N, int ng, int G,
                                     float *__restrict__ c) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float acc = 0.0f;
    for (int g = 0; g < ng; ++g) {
        float S = scale[(long)n * ng + g];
        float Z = zero ? zero[(long)n * ng + g] : 0.0f;
        float t = S * (float)gsum[(long)n * ng + g];
        float u = (float)G * Z;
        float w = t + u;
        acc = acc + w;
    }
    c[n] = acc;
}

template <int MODE, typename T, int LAYOUT = 0>
static int launch_rows(const T *X, long ldx, int rows, int K, int G, uint8_t *q, float *s, float *z,
                       int32_t *gsum, int ng, hipStream_t st, int32_t *psum = nullptr, int psum_per = 1) {
    if (rows == 0) return W4A4_OK;
    const int iters = (K / 8 + kWave - 1) / kWave;
    dim3 grid((rows + kRowsPerBlock - 1) / kRowsPerBlock), block(kRowsPerBlock * kWave);
#define W4A4_QL(I)                                                                                  \
    hipLaunchKernelGGL((quantize_rows_kernel<MODE, T, I, LAYOUT>), grid, block, 0, st, X, ldx, rows, K, G, q, \
                       s, z, gsum, ng, psum, psum_per)
    if (iters <= 1) W4A4_QL(1);
    else if (iters <= 2) W4A4_QL(2);
    else if (iters <= 4) W4A4_QL(4);
    else if (iters <= 8) W4A4_QL(8);
    else if (iters <= 16) W4A4_QL(16);
    else if (iters <= 32) W4A4_QL(32);
    else return W4A4_ERR_UNSUPPORTED_SHAPE;
#undef W4A4_QL
    return launch_status();
}

// ---- the run-time quantizer, several tokens per wave ------------------------------------------------------------
// quantize_stream_kernel spends most of its instructions on what a row costs once (two wave-wide reductions
// through the LDS crossbar, the division, addressing), and at K = 1024 a lane holds only sixteen elements: a
// 12288 x 1024 matrix took 6 us of vector-ALU issue per SIMD against 5 us of memory time.  Here a row is owned by
// LPR = 16, 32 or 64 lanes (the smallest that keeps <= 8 chunks of eight elements per lane), so a wave quantizes
// 64 / LPR tokens with one instruction stream; reductions inside 16 lanes use the cross-lane operand modes (quad
// permutes, half-row and row mirror) instead of the LDS; and a code costs four instructions: conversion fused
// with the first arithmetic step, the second step, the rounding add, and one shift-add that appends it to the
// packed word.  The last works because bits(t + 1.5*2^23 + b) = 0x4B400000 + (code + b) (b = 8 for the symmetric
// mapping, offset binary; 0 for the asymmetric one): shifted left by 4e and summed over e (mod 2^32) that is the
// packed word plus the constant 0x3F400000, taken off once per word.
// LAYOUT 0 (canonical) or 1 (MFMA operand layout of activations).  Symmetric mapping (Sec. 3.1): no K-group sums;
// with LAYOUT 1, psum[row] = sum of the odd-position codes.  Asymmetric mapping: gsum[row * ng + g] = sum of the
// codes of K-group g (when asked for) and, with LAYOUT 1, psum[g * rows + row] = 128 * (sum of its even-position
// codes), for groups of 128 elements (the sixteen chunks of a group are the sixteen lanes of a DPP row in one
// register slot) or one group per row.
// Same arithmetic, same codes as the kernels above.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int LPR>
__device__ __forceinline__ float sub_max(float v) {                 // maximum over the LPR lanes that own a row
    v = fmaxf(v, __int_as_float(dpp_move<0xB1>(__float_as_int(v))));     // quad_perm [1,0,3,2]
    v = fmaxf(v, __int_as_float(dpp_move<0x4E>(__float_as_int(v))));     // quad_perm [2,3,0,1]
    v = fmaxf(v, __int_as_float(dpp_move<0x141>(__float_as_int(v))));    // half-row mirror
    if (LPR >= 16) v = fmaxf(v, __int_as_float(dpp_move<0x140>(__float_as_int(v))));   // row mirror
    if (LPR >= 32) v = fmaxf(v, __shfl_xor(v, 16, kWave));
    if (LPR >= 64) v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}
__device__ __forceinline__ int row16_sum(int v) {                   // sum over the sixteen lanes of a DPP row
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return v;
}
template <int LPR>
__device__ __forceinline__ int sub_sum(int v) {
    v = row16_sum(v);
    if (LPR >= 32) v += __shfl_xor(v, 16, kWave);
    if (LPR >= 64) v += __shfl_xor(v, 32, kWave);
    return v;
}

// EXACT: K / 8 == LPR * CPL, no chunk of a lane lies past K.  ng: K-groups of the asymmetric psum (1 or K / 128).
template <int MODE, int LPR, int CPL, int LAYOUT, bool EXACT>
__global__ __launch_bounds__(kRowsPerBlock *kWave) void quantize_tok_rows_kernel(
    const __half *__restrict__ X, long ldx, int rows, int K, uint8_t *__restrict__ q, float *__restrict__ s,
    float *__restrict__ z, int32_t *__restrict__ gsum, int32_t *__restrict__ psum, int ng) {
    constexpr int RPW = kWave / LPR;                            // tokens per wave
    constexpr bool ASYM = MODE == W4A4_ASYM;
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x % kWave, l = lane % LPR;
    const long row = ((long)blockIdx.x * kRowsPerBlock + threadIdx.x / kWave) * RPW + lane / LPR;
    const int nchunks = K / 8;
    const bool live = row < rows;
    const u4 *src = reinterpret_cast<const u4 *>(X + (live ? row : (long)rows - 1) * ldx);
    u4 raw[CPL];
    // chunks past K: zeros under the symmetric mapping (code 0, no effect on absmax); the row's first chunk under
    // the asymmetric one (no effect on minimum and maximum; their codes are neither stored nor summed)
    u4 fill = {0u, 0u, 0u, 0u};
    if (ASYM && !EXACT) fill = src[0];
#pragma unroll
    for (int it = 0; it < CPL; ++it) {
        const int c = l + it * LPR;
        raw[it] = (EXACT || c < nchunks) ? src[c] : fill;
    }
    Range r;
    if constexpr (!ASYM) {
        // ---- absmax: |x| of finite fp16 values orders like its 15-bit pattern, so the maximum is taken on packed
        // unsigned 16-bit integers (exact, and no NaN canonicalisation as a floating-point maximum would add)
        typedef unsigned short us2 __attribute__((ext_vector_type(2)));
        us2 hi2 = {0, 0};
#pragma unroll
        for (int it = 0; it < CPL; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t d = raw[it][i] & 0x7FFF7FFFu;
                hi2 = __builtin_elementwise_max(hi2, *reinterpret_cast<const us2 *>(&d));
            }
        const unsigned short hmax = hi2[0] > hi2[1] ? hi2[0] : hi2[1];
        r = range_sym(sub_max<LPR>(__half2float(__ushort_as_half(hmax))));
        if (l == 0 && live) s[row] = r.S;
    } else {
        // ---- minimum and maximum on packed fp16 (exact: the extremes of fp16 values are fp16 values)
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        auto halves = [](uint32_t w) { return __builtin_bit_cast(h2, w); };
        h2 hi2 = halves(raw[0][0]), lo2 = hi2;
#pragma unroll
        for (int it = 0; it < CPL; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (it == 0 && i == 0) continue;
                const h2 d = halves(raw[it][i]);
                hi2 = __builtin_elementwise_max(hi2, d);
                lo2 = __builtin_elementwise_min(lo2, d);
            }
        const float hi = sub_max<LPR>(fmaxf((float)hi2[0], (float)hi2[1]));
        const float lo = -sub_max<LPR>(-fminf((float)lo2[0], (float)lo2[1]));
        r = range_asym(lo, hi);
        if (l == 0 && live) {
            s[row] = r.S;
            z[row] = r.lo;
        }
    }
    // ---- codes
    constexpr float kMagic = ASYM ? 12582912.0f : 12582920.0f;  // 1.5 * 2^23 (+ 8: offset binary)
    constexpr uint32_t kBits = 0x3F400000u;                     // sum over e of (0x4B400000 << 4e) mod 2^32
    // symmetric codes leave offset binary where two's complement is wanted; unsigned codes of the operand layout
    // lose 8 in the high nibbles (u - 8 in two's complement is u with its top bit flipped)
    constexpr uint32_t kFlip = LAYOUT != 0 ? 0x80808080u : ASYM ? 0u : 0x88888888u;
    const float neg_lo = -r.lo;
    uint32_t *qr = reinterpret_cast<uint32_t *>(q + row * (long)(K / 2));
    int part = 0, total = 0;
#pragma unroll
    for (int it = 0; it < CPL; ++it) {
        const int c = l + it * LPR;
        const bool in = EXACT || c < nchunks;
        uint32_t acc = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // the mixed-precision fused multiply-add reads the fp16 half directly and rounds once: with a zero
            // addend it is the conversion and the fp32 multiply, t = (float)x * inv; with the factor 1 it is the
            // conversion and the fp32 subtraction, d = (float)x - lo
            const uint32_t w = raw[it][e >> 1];
            float t;
            if constexpr (!ASYM) {
                if (e & 1) asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(t) : "v"(w), "v"(r.inv));
                else asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(t) : "v"(w), "v"(r.inv));
            } else {
                float d;
                if (e & 1) asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(neg_lo));
                else asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(neg_lo));
                t = d * r.inv;
            }
            const float u = t + kMagic;
            acc = (__float_as_uint(u) << (4 * e)) + acc;
        }
        const uint32_t packed = acc - kBits;                    // nibble e = code (+ 8 under the symmetric mapping)
        if (live && in) qr[c] = packed ^ kFlip;
        if (LAYOUT != 0 && !ASYM) part += (int)__builtin_amdgcn_sad_u8((packed >> 4) & 0x0F0F0F0Fu, 0u, 0u) - 32;
        if constexpr (ASYM) {
            // both sums of a chunk ride in one register: all eight codes above bit 16, the even positions below
            // (a K-group of 128 holds at most 64 * 15 there)
            const uint32_t ev = __builtin_amdgcn_sad_u8(packed & 0x0F0F0F0Fu, 0u, 0u);
            const uint32_t all = __builtin_amdgcn_sad_u8((packed >> 4) & 0x0F0F0F0Fu, 0u, ev);
            const int both = in ? (int)((all << 16) | ev) : 0;
            if (ng == 1) {
                part += both & 0xFFFF;
                total += both >> 16;
            } else if (LAYOUT != 0 || gsum) {                   // chunks 16 j .. 16 j + 15 are K-group j
                const int gs = row16_sum(both);
                if ((l & 15) == 0 && live && in) {
                    if (LAYOUT != 0) psum[(long)(c >> 4) * rows + row] = 128 * (gs & 0xFFFF);
                    if (gsum) gsum[row * (long)ng + (c >> 4)] = gs >> 16;
                }
            }
        }
    }
    if (ASYM && ng == 1 && gsum) {
        total = sub_sum<LPR>(total);
        if (l == 0 && live) gsum[row] = total;
    }
    if (LAYOUT != 0 && (!ASYM || ng == 1)) {
        part = sub_sum<LPR>(part);
        if (l == 0 && live) psum[row] = ASYM ? 128 * part : part;
    }
}

template <int MODE, int LAYOUT>
static int launch_tok_rows(const __half *X, long ldx, int rows, int K, uint8_t *q, float *s, float *z,
                           int32_t *gsum, hipStream_t st, int32_t *psum, int ng) {
    if (rows == 0) return W4A4_OK;
    const int nchunks = K / 8;
    if (nchunks > 8 * kWave) return -100;
    const int lpr = nchunks <= 8 * 16 ? 16 : nchunks <= 8 * 32 ? 32 : 64;
    const int cpl = (nchunks + lpr - 1) / lpr;
    const long per_block = (long)kRowsPerBlock * (kWave / lpr);
    dim3 grid((unsigned)((rows + per_block - 1) / per_block)), block(kRowsPerBlock * kWave);
#define W4A4_QF(L, C)                                                                                       \
    do {                                                                                                    \
        if (nchunks == L * C)                                                                               \
            hipLaunchKernelGGL((quantize_tok_rows_kernel<MODE, L, C, LAYOUT, true>), grid, block, 0, st, X, ldx, rows, K, q, s, z, gsum, psum, ng); \
        else                                                                                                \
            hipLaunchKernelGGL((quantize_tok_rows_kernel<MODE, L, C, LAYOUT, false>), grid, block, 0, st, X, ldx, rows, K, q, s, z, gsum, psum, ng); \
    } while (0)
#define W4A4_QFL(L)                                                                                         \
    do {                                                                                                    \
        if (cpl <= 2) W4A4_QF(L, 2);                                                                        \
        else if (cpl <= 4) W4A4_QF(L, 4);                                                                   \
        else if (cpl <= 6) W4A4_QF(L, 6);                                                                   \
        else W4A4_QF(L, 8);                                                                                 \
    } while (0)
    if (lpr == 16) W4A4_QFL(16);
    else if (lpr == 32) W4A4_QFL(32);
    else W4A4_QFL(64);
#undef W4A4_QFL
#undef W4A4_QF
    return launch_status();
}

// ---- the FP6 operand layout (symmetric codes as FP6 E2M3 numbers; see w4a4_layout) -------------------------------
// A row of K codes is K / 32 MFMA operands of 32 codes (24 bytes); operands 2b and 2b + 1 form the row's 48-byte
// block b, [16 bytes at 16h | 8 bytes at 32 + 8h] for operand 2b + h.  Rows are stored in panels (64 tokens, or 128
// output channels in the order that gives a lane of the GEMM adjacent channels), block b of all rows of a panel
// contiguously, so that the GEMM's tile loads are whole kilobytes of consecutive addresses; matrices are padded
// with zero rows to whole panels.  Operand o of a row holds codes 32o .. 32o+31 in its 6-bit fields 0 .. 31 (little
// endian), for activations and weights alike.  In the token-wise quantizer a token is owned by LPR lanes and lane l
// converts operands l, l + LPR, ...: it loads the 64 bytes of an operand's fp16 values itself (four 16-byte loads; a
// wave's loads cover every cache line they touch completely), and the hardware conversion, which interleaves its two
// sixteen-value sources, takes the even-position values as one source and the odd-position ones as the other - the two
// halves of the dwords as loaded.
typedef float v16f_q __attribute__((ext_vector_type(16)));
typedef unsigned int v6u_q __attribute__((ext_vector_type(6)));

// Token-wise symmetric quantizer into the FP6 layout: same range and same codes as the kernels above (t = x * 7/absmax
// in fp32, round to nearest even; |t| <= 7(1+2^-23), so the clamp of the definition cannot bind); the rounded value,
// an integer of magnitude <= 7, is exactly representable in FP6 E2M3, so the hardware conversion of 32 fp32 values
// to 32 packed FP6 fields is exact.  Two vector instructions per code plus one conversion per 32.
template <int LPR, int OPL>
__global__ __launch_bounds__(8 * kWave) void quantize_fp6_rows_kernel(
    const __half *__restrict__ X, long ldx, int rows, uint8_t *__restrict__ q, float *__restrict__ s) {
    constexpr int RPW = kWave / LPR, NJ = 4 * OPL;
    constexpr int KB = LPR * OPL / 2;                           // 48-byte blocks (64 codes) per row
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u2 __attribute__((ext_vector_type(2)));
    const int lane = threadIdx.x % kWave, l = lane % LPR;
    // a workgroup owns a multiple of eight consecutive rows: 384 contiguous bytes of every block, whole cache lines
    // that no other workgroup (on another XCD, behind another L2) writes to
    const long row = ((long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave) * RPW + lane / LPR;
    const bool live = row < rows;                               // rows up to the end of the last 64-row panel are written as zeros
    const bool padded = row < (((long)rows + 63) & ~63L);
    const u4 *src = reinterpret_cast<const u4 *>(X + (live ? row : (long)rows - 1) * ldx);
    u4 raw[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) raw[j] = src[4 * ((j >> 2) * LPR + l) + (j & 3)];
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    us2 hi2 = {0, 0};
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t d = raw[j][i] & 0x7FFF7FFFu;
            hi2 = __builtin_elementwise_max(hi2, *reinterpret_cast<const us2 *>(&d));
        }
    const unsigned short hmax = hi2[0] > hi2[1] ? hi2[0] : hi2[1];
    const Range r = range_sym(sub_max<LPR>(__half2float(__ushort_as_half(hmax))));
    if (l == 0 && live) s[row] = r.S;
    // The operands go to LDS first, laid out as this workgroup's part of the panel ([block][row of the workgroup][48
    // bytes]), and from there to memory in runs of whole cache lines: written straight from the lanes, every store
    // instruction would touch 32 blocks 3 KB apart with 32 bytes each, which costs a 12288 x 4096 matrix 6 of 32 us.
    extern __shared__ __attribute__((aligned(16))) uint8_t stage6[];
    const int rows_wg = (blockDim.x / kWave) * RPW;             // 8, 16 or 32: a multiple of 8, so 384-byte multiples per block
    const int r_wg = (threadIdx.x / kWave) * RPW + lane / LPR;
    uint8_t *srow = stage6 + r_wg * 48;
#pragma unroll
    for (int o = 0; o < OPL; ++o) {
        v16f_q a, b;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t w = raw[4 * o + jj][e >> 1];
                float t;
                if (e & 1) asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(t) : "v"(w), "v"(r.inv));
                else asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(t) : "v"(w), "v"(r.inv));
                const float c = __builtin_rintf(t);
                if (e & 1) b[4 * jj + (e >> 1)] = c;            // field 2i of the conversion's result is a[i], field 2i+1 is b[i]
                else a[4 * jj + (e >> 1)] = c;
            }
        v6u_q w6 = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(a, b, 1.0f);
        if (!live) w6 = v6u_q{0u, 0u, 0u, 0u, 0u, 0u};
        const int idx = o * LPR + l;
        uint8_t *blk = srow + (idx >> 1) * (rows_wg * 48);
        *reinterpret_cast<u4 *>(blk + (idx & 1) * 16) = u4{w6[0], w6[1], w6[2], w6[3]};
        // the 8-byte part: at 32 + 8h, the two halves exchanged in rows 16 .. 31 of every 32 (LDS banks of the GEMM's reads)
        *reinterpret_cast<u2 *>(blk + 32 + (((idx & 1) ^ (int)((row >> 4) & 1)) * 8)) = u2{w6[4], w6[5]};
    }
    __syncthreads();
    // rows of the workgroup: row0 .. row0 + rows_wg - 1 (inside one panel: rows_wg divides 64); block b of them lies at
    // panel + b * 3072 + (row0 % 64) * 48, rows_wg * 48 bytes long
    const long row0 = (long)blockIdx.x * rows_wg;
    if (row0 < (((long)rows + 63) & ~63L)) {
        uint8_t *dst = q + (row0 >> 6) * ((long)KB * 3072) + (row0 & 63) * 48;
        const int per_block = rows_wg * 3;                      // 16-byte pieces per block
        for (int pc = threadIdx.x; pc < KB * per_block; pc += blockDim.x) {
            const int bq = pc / per_block, within = pc - bq * per_block;
            *reinterpret_cast<u4 *>(dst + (long)bq * 3072 + within * 16) = *reinterpret_cast<const u4 *>(stage6 + pc * 16);
        }
    }
}

static int launch_fp6_rows(const __half *X, long ldx, int rows, int K, uint8_t *q, float *s, hipStream_t st) {
    if (rows == 0) return W4A4_OK;
    int lpr = 0, opl = 0;
    if (!fp6_plan(K, &lpr, &opl)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int rpw = kWave / lpr, waves = rpw >= 2 ? 4 : 8;      // 8 .. 32 rows per workgroup
    const long per_block = (long)waves * rpw;
    const long padded = ((long)rows + 63) & ~63L;
    dim3 grid((unsigned)(padded / per_block)), block(waves * kWave);
    const size_t lds = (size_t)per_block * (K / 64) * 48;       // the workgroup's rows, staged (60 KB at most: fp6_plan)
    if (lds > 64 * 1024) return W4A4_ERR_UNSUPPORTED_SHAPE;
#define W4A4_Q6(L, O) \
    case O: hipLaunchKernelGGL((quantize_fp6_rows_kernel<L, O>), grid, block, lds, st, X, ldx, rows, q, s); break
#define W4A4_Q6L(L)                                                                                        \
    switch (opl) { W4A4_Q6(L, 1); W4A4_Q6(L, 2); W4A4_Q6(L, 3); W4A4_Q6(L, 4); W4A4_Q6(L, 5); W4A4_Q6(L, 6); default: return W4A4_ERR_UNSUPPORTED_SHAPE; }
    if (lpr == 8) { W4A4_Q6L(8) }
    else if (lpr == 16) { W4A4_Q6L(16) }
    else if (lpr == 32) { W4A4_Q6L(32) }
    else { W4A4_Q6L(64) }
#undef W4A4_Q6L
#undef W4A4_Q6
    return launch_status();
}

// FP6 E2M3 field of a code in [-7, 7]: sign, then the magnitude as (exponent, three mantissa bits)
__device__ __forceinline__ uint32_t fp6_field(int c) {
    const int m = c < 0 ? -c : c;
    const uint32_t mag = m == 0 ? 0u : m == 1 ? 8u : m < 4 ? 8u + 4u * (uint32_t)m : 16u + 2u * (uint32_t)m;   // 1 | 2, 3 | 4 .. 7
    return (c < 0 ? 32u : 0u) | mag;
}

// Offline weight quantizer into the FP6 layout (symmetric, one scale per output channel): one wave per channel of
// the padded matrix (channels past N are written as zeros), the range over the whole row, then every lane assembles
// whole operands of 32 consecutive codes.  Same range and codes as quantize_rows_kernel;
// gsum[n] = sum of the codes of the row.  Channel n lives in panel n / 128, storage row (n % 4) * 32 + (n % 128) / 4.
__global__ __launch_bounds__(kRowsPerBlock *kWave) void quantize_weight_fp6_kernel(
    const __half *__restrict__ W, int N, int K, uint8_t *__restrict__ q, float *__restrict__ s,
    int32_t *__restrict__ gsum) {
    const int lane = threadIdx.x % kWave;
    const long n = (long)blockIdx.x * kRowsPerBlock + threadIdx.x / kWave;
    if (n >= (((long)N + 127) & ~127L)) return;
    const bool live = n < N;
    const __half *w = W + (live ? n : 0) * K;
    float amax = 0.0f;
    for (int k = lane; k < K; k += kWave) amax = fmaxf(amax, fabsf(__half2float(w[k])));
    const Range r = range_sym(wave_max(amax));
    if (lane == 0 && live) s[n] = r.S;
    const int p = (int)(n & 3) * 32 + (int)((n & 127) >> 2);
    uint8_t *qrow = q + (n >> 7) * ((long)(K / 64) * 6144) + p * 48;
    int total = 0;
    for (int idx = lane; idx < K / 32; idx += kWave) {
        uint32_t words[6] = {0, 0, 0, 0, 0, 0};
        for (int e = 0; e < 32; ++e) {
            const int c = live ? code_of<W4A4_SYM>(__half2float(w[32 * idx + e]), r) : 0;
            total += c;
            const int bit = 6 * e;
            const uint32_t f = fp6_field(c);
            words[bit >> 5] |= f << (bit & 31);
            if ((bit & 31) > 26) words[(bit >> 5) + 1] |= f >> (32 - (bit & 31));
        }
        uint8_t *blk = qrow + (long)(idx >> 1) * 6144;
        uint32_t *lo = reinterpret_cast<uint32_t *>(blk + (idx & 1) * 16);
        lo[0] = words[0]; lo[1] = words[1]; lo[2] = words[2]; lo[3] = words[3];
        uint32_t *tl = reinterpret_cast<uint32_t *>(blk + 32 + (((idx & 1) ^ ((p >> 4) & 1)) * 8));   // halves exchanged in storage rows 16 .. 31 of every 32
        tl[0] = words[4]; tl[1] = words[5];
    }
    if (gsum && live) {
        for (int o = 32; o > 0; o >>= 1) total += __shfl_xor(total, o, kWave);
        if (lane == 0) gsum[n] = total;
    }
}

// Streaming launch for fp16 activations; returns -100 when the shape needs the general kernel
// (K-groups whose chunk count is not a power of two <= 64).
template <int MODE, int LAYOUT>
static int launch_stream(const __half *X, long ldx, int rows, int K, int G, uint8_t *q, float *s, float *z,
                         int32_t *gsum, int ng, hipStream_t st, int32_t *psum) {
    if (rows == 0) return W4A4_OK;
    const int cpg = G / 8;
    // several tokens per wave: symmetric layers that want no K-group sums, asymmetric ones whose sums are per
    // row or per group of 128
    if (MODE == W4A4_SYM ? !gsum : (ng == 1 || cpg == 16)) {
        const int rc = launch_tok_rows<MODE, LAYOUT>(X, ldx, rows, K, q, s, z, gsum, st, psum, ng);
        if (rc != -100) return rc;
    }
    if ((gsum || (LAYOUT != 0 && MODE == W4A4_ASYM)) && ng > 1 && (cpg > 64 || (cpg & (cpg - 1)))) return -100;
    const int iters = (K / 8 + kWave - 1) / kWave;
    // One row per wave measured fastest on MI355X (a 12288 x 1024 activation matrix: 8.1 us against 9.6 us
    // with two rows per wave and the second row's loads in flight under the first row's arithmetic): the
    // dispatcher keeps the CUs fed, and more, shorter waves hide the reduction latency better.  The row loop
    // of the kernel only matters beyond 2^22 rows.
    const long rpw = (rows + (1L << 22) - 1) >> 22;
    const long waves = (rows + rpw - 1) / rpw;
    dim3 grid((unsigned)((waves + kRowsPerBlock - 1) / kRowsPerBlock)), block(kRowsPerBlock * kWave);
#define W4A4_QS(I)                                                                                       \
    hipLaunchKernelGGL((quantize_stream_kernel<MODE, I, LAYOUT>), grid, block, 0, st, X, ldx, rows, K, q, s, z, \
                       gsum, ng, cpg, psum)
    if (iters <= 1) W4A4_QS(1);
    else if (iters <= 2) W4A4_QS(2);
    else if (iters <= 4) W4A4_QS(4);
    else if (iters <= 8) W4A4_QS(8);
    else return -100;
#undef W4A4_QS
    return launch_status();
}

// Shared argument checks for a row quantizer.  elem_bytes: 2 (fp16) or 4 (fp32).
static int check_rows(const void *X, int rows, int K, long ldx, int mode, int group, const void *q,
                      const void *s, const void *z, int elem_bytes, int *ng_out) {
    if (rows < 0 || K <= 0 || ldx < K) return W4A4_ERR_INVALID_ARG;
    if (mode != W4A4_SYM && mode != W4A4_ASYM) return W4A4_ERR_INVALID_ARG;
    if (group < 0) return W4A4_ERR_INVALID_ARG;
    if (rows > 0 && (!X || !q || !s || (mode == W4A4_ASYM && !z))) return W4A4_ERR_INVALID_ARG;
    if (K % 32 || (ldx * elem_bytes) % 16 || !aligned16(X) || !aligned16(q)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (K > 16384) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int G = group == 0 ? K : group;
    if (G % 32 || K % G) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (K / G > kMaxGroups) return W4A4_ERR_UNSUPPORTED_SHAPE;
    *ng_out = K / G;
    return W4A4_OK;
}

// Requantize of fp32 rows (used behind the GEMM); same mapping as quantize_act.
// layout 1: codes in the MFMA operand layout of activations, gsum[rows] = odd-position sums.
int quantize_rows_f32(const float *Y, int rows, int K, long ld, int mode, int group, uint8_t *q,
                      float *s, float *z, int32_t *gsum, hipStream_t st, int layout) {
    int ng = 0;
    int rc = check_rows(Y, rows, K, ld, mode, group, q, s, z, 4, &ng);
    if (rc) return rc;
    const int G = group == 0 ? K : group;
    if (layout == W4A4_LAYOUT_MFMA)
        return launch_rows<W4A4_SYM, float, 1>(Y, ld, rows, K, K, q, s, z, nullptr, 1, st, gsum);
    return mode == W4A4_SYM ? launch_rows<W4A4_SYM, float>(Y, ld, rows, K, G, q, s, z, gsum, ng, st)
                            : launch_rows<W4A4_ASYM, float>(Y, ld, rows, K, G, q, s, z, gsum, ng, st);
}

// Layout check shared by the two quantizer entry points.  The operand layout exists for symmetric codes with one
// weight scale per channel and for unsigned codes with weight groups that are multiples of 128 (or one group).
static int check_layout(int layout, int mode, int group, int K, const void *psum, int rows) {
    if (layout == W4A4_LAYOUT_FP6) {                            // symmetric codes, one scale per row, a K the layout exists for
        int lpr = 0, opl = 0;
        if (mode != W4A4_SYM) return W4A4_ERR_INVALID_ARG;
        if ((group != 0 && group != K) || !fp6_plan(K, &lpr, &opl)) return W4A4_ERR_UNSUPPORTED_SHAPE;
        return W4A4_OK;
    }
    if (layout != W4A4_LAYOUT_CANONICAL && layout != W4A4_LAYOUT_MFMA) return W4A4_ERR_INVALID_ARG;
    if (layout == W4A4_LAYOUT_MFMA) {
        if (mode == W4A4_SYM) {
            if (group != 0 && group != K) return W4A4_ERR_UNSUPPORTED_SHAPE;
        } else {
            const int G = group == 0 ? K : group;
            if (G % 128 || K % 128) return W4A4_ERR_UNSUPPORTED_SHAPE;
        }
        if (rows > 0 && !psum) return W4A4_ERR_INVALID_ARG;
    }
    return W4A4_OK;
}

// Last word of a channel's row of the operand-layout sums of unsigned weights: the fp32 bits of
// 8 * sum_g sw[n,g] * (float)WO[n,g], WO = the odd-position code sums in the words before it (ascending g, every
// operation rounded): what the offsets of the layout add to sum_g sw[n,g] * P_g for every token.
__global__ void weight_odd_term_kernel(const float *__restrict__ scale, int32_t *__restrict__ esum, int N, int ng) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float acc = 0.0f;
    for (int g = 0; g < ng; ++g) {
        const float t = scale[(long)n * ng + g] * 8.0f;
        const float u = t * (float)esum[(long)n * (ng + 1) + g];
        acc = acc + u;
    }
    esum[(long)n * (ng + 1) + ng] = __float_as_int(acc);
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_quantize_act(const void *X_f16, int M, int K, int ldx, int mode, int group,
                                 uint8_t *q, float *scale, float *zero, int32_t *gsum, int layout,
                                 int32_t *osum, void *stream) {
    int ng = 0;
    int rc = check_rows(X_f16, M, K, ldx, mode, group, q, scale, zero, 2, &ng);
    if (rc) return rc;
    rc = check_layout(layout, mode, group, K, osum, M);
    if (rc) return rc;
    const int G = group == 0 ? K : group;
    const __half *X = static_cast<const __half *>(X_f16);
    hipStream_t st = as_stream(stream);
    if (layout == W4A4_LAYOUT_FP6) {
        if (gsum) return W4A4_ERR_UNSUPPORTED_SHAPE;            // no K-group code sums in this layout
        return launch_fp6_rows(X, ldx, M, K, q, scale, st);
    }
    const bool olay = layout == W4A4_LAYOUT_MFMA;
    rc = olay ? (mode == W4A4_SYM ? launch_stream<W4A4_SYM, 1>(X, ldx, M, K, G, q, scale, zero, gsum, ng, st, osum)
                                  : launch_stream<W4A4_ASYM, 1>(X, ldx, M, K, G, q, scale, zero, gsum, ng, st, osum))
         : mode == W4A4_SYM ? launch_stream<W4A4_SYM, 0>(X, ldx, M, K, G, q, scale, zero, gsum, ng, st, nullptr)
                            : launch_stream<W4A4_ASYM, 0>(X, ldx, M, K, G, q, scale, zero, gsum, ng, st, nullptr);
    if (rc != -100) return rc;                                  // else: a shape only the general kernel takes
    if (olay)
        return mode == W4A4_SYM
                   ? launch_rows<W4A4_SYM, __half, 1>(X, ldx, M, K, G, q, scale, zero, gsum, ng, as_stream(stream), osum)
                   : launch_rows<W4A4_ASYM, __half, 1>(X, ldx, M, K, G, q, scale, zero, gsum, ng, as_stream(stream), osum);
    return mode == W4A4_SYM
               ? launch_rows<W4A4_SYM, __half>(X, ldx, M, K, G, q, scale, zero, gsum, ng, as_stream(stream))
               : launch_rows<W4A4_ASYM, __half>(X, ldx, M, K, G, q, scale, zero, gsum, ng, as_stream(stream));
}

extern "C" int w4a4_quantize_weight(const void *W_f16, int N, int K, int mode, int group, uint8_t *q,
                                    float *scale, float *zero, int32_t *gsum, float *rowsum_deq,
                                    int layout, int32_t *esum, void *stream) {
    // A weight matrix [N,K] with groups of G along K is the row matrix [N*ng, G]:
    // every (channel, group) pair is one independent vector (App. A).
    if (N < 0 || K <= 0 || group < 0) return W4A4_ERR_INVALID_ARG;
    const int G = group == 0 ? K : group;
    if (K % 32 || G % 32 || K % G) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int ng = K / G;
    if (rowsum_deq && N > 0 && !gsum) return W4A4_ERR_INVALID_ARG;   // c[n] is built from the code sums
    long rows = (long)N * ng;
    if (rows > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    int one = 0;
    int rc = check_rows(W_f16, (int)rows, G, G, mode, 0, q, scale, zero, 2, &one);
    if (rc) return rc;
    rc = check_layout(layout, mode, group, K, esum, N);
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const __half *W = static_cast<const __half *>(W_f16);
    if (layout == W4A4_LAYOUT_FP6) {
        if (N > 0) {
            hipLaunchKernelGGL(quantize_weight_fp6_kernel, dim3((((N + 127) & ~127) + kRowsPerBlock - 1) / kRowsPerBlock),
                               dim3(kRowsPerBlock * kWave), 0, st, W, N, K, q, scale, gsum);
            rc = launch_status();
        }
    } else if (layout == W4A4_LAYOUT_MFMA && mode == W4A4_SYM)
        rc = launch_rows<W4A4_SYM, __half, 2>(W, G, (int)rows, G, G, q, scale, zero, gsum, 1, st, esum);
    else if (layout == W4A4_LAYOUT_MFMA)
        rc = launch_rows<W4A4_ASYM, __half, 2>(W, G, (int)rows, G, G, q, scale, zero, gsum, 1, st, esum, ng);
    else
        rc = mode == W4A4_SYM
                 ? launch_rows<W4A4_SYM, __half>(W, G, (int)rows, G, G, q, scale, zero, gsum, 1, st)
                 : launch_rows<W4A4_ASYM, __half>(W, G, (int)rows, G, G, q, scale, zero, gsum, 1, st);
    if (rc) return rc;
    if (rowsum_deq && N > 0) {
        hipLaunchKernelGGL(weight_rowsum_kernel, dim3((N + 255) / 256), dim3(256), 0, st, scale,
                           mode == W4A4_ASYM ? zero : nullptr, gsum, N, ng, G, rowsum_deq);
        rc = launch_status();
    }
    if (rc == W4A4_OK && layout == W4A4_LAYOUT_MFMA && mode == W4A4_ASYM && N > 0) {
        hipLaunchKernelGGL(weight_odd_term_kernel, dim3((N + 255) / 256), dim3(256), 0, st, scale, esum, N, ng);
        rc = launch_status();
    }
    return rc;
}
