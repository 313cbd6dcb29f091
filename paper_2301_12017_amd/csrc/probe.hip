// Measurement probes of libw4a4: what the matrix pipe and the memory system of the device deliver on their own,
// so that a kernel's rate can be read against a measured ceiling beside the nominal one.  Neither computes
// anything of the method.
#include "gemm_common.hpp"

namespace w4a4 {

// Register-only loop of independent v_mfma_i32_32x32x32_i8 (eight accumulators per wave, no memory traffic in the
// loop).  The operand registers are the caller's: all-zero operands give the pipe's rate at the clock the chip
// keeps when the multipliers see no switching activity, INT4 codes widened as the GEMM kernels widen them give the
// rate at the clock it keeps on real data (the chip lowers its clock with the switching activity of the operands).
__global__ __launch_bounds__(256) void mfma_probe_kernel(const uint32_t *__restrict__ operands, int iters, uint32_t *sink) {
    const int lane = threadIdx.x & 63;
    v4i a[2], b[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            a[s][r] = (int)operands[lane * 16 + s * 8 + r];
            b[s][r] = (int)operands[lane * 16 + s * 8 + 4 + r];
        }
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 0x7fffffff) sink[0] = (uint32_t)s;                   // keeps the loop alive; practically never taken
}

// The same loop on the FP6 form of the matrix instruction (v_mfma_f32_32x32x64_f8f6f4, both operands E2M3): per
// lane two A and two B operands of 32 six-bit fields each (24 bytes, the first six of eight words).
typedef int v8i_p __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256) void mfma_fp6_probe_kernel(const uint32_t *__restrict__ operands, int iters, uint32_t *sink) {
    const int lane = threadIdx.x & 63;
    v8i_p a[2], b[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            a[s][r] = r < 6 ? (int)operands[lane * 32 + s * 16 + r] : 0;
            b[s][r] = r < 6 ? (int)operands[lane * 32 + s * 16 + 8 + r] : 0;
        }
    v16f acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 1], b[(i >> 1) & 1], acc[i], 2, 2, 0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[0] = 1u;                            // keeps the loop alive; practically never taken
}

// Streaming kernel: every lane reads 16 bytes per step, consecutive lanes consecutive addresses, grid-stride;
// with a destination it writes what it read (a copy), without one it folds the data into one word per lane and
// stores nothing: the rate a read-mostly, HBM-bound kernel such as the token-wise quantizer can hope for.
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4 *__restrict__ src, u32x4 *dst, size_t n16, uint32_t *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4 x = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        if (dst) __builtin_nontemporal_store(v, dst + i);
        else x ^= v;
    }
    if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u) sink[0] = x[0];   // keeps the loads alive
}

}  // namespace w4a4

using namespace w4a4;

static int probe_cus() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return -1;
    return cus;
}

extern "C" long w4a4_probe_mfma(const uint32_t *operands, int iters, uint32_t *sink, void *stream) {
    if (!operands || !sink || iters <= 0) return W4A4_ERR_INVALID_ARG;
    const int cus = probe_cus();
    if (cus < 0) return W4A4_ERR_HIP;
    const unsigned grid = (unsigned)cus * 2;                      // two waves on every SIMD, as the GEMM kernels run
    launch_gemm(mfma_probe_kernel, dim3(grid), dim3(256), 0, as_stream(stream), operands, iters, sink);
    if (launch_status() != W4A4_OK) return W4A4_ERR_HIP;
    return (long)grid * 4 * 8 * (long)iters;                      // wave-level MFMA instructions issued
}

extern "C" long w4a4_probe_mfma_fp6(const uint32_t *operands, int iters, uint32_t *sink, void *stream) {
    if (!operands || !sink || iters <= 0) return W4A4_ERR_INVALID_ARG;
    const int cus = probe_cus();
    if (cus < 0) return W4A4_ERR_HIP;
    const unsigned grid = (unsigned)cus * 2;                      // two waves on every SIMD
    launch_gemm(mfma_fp6_probe_kernel, dim3(grid), dim3(256), 0, as_stream(stream), operands, iters, sink);
    if (launch_status() != W4A4_OK) return W4A4_ERR_HIP;
    return (long)grid * 4 * 8 * (long)iters;                      // wave-level MFMA instructions issued
}

extern "C" int w4a4_probe_stream(const void *src, void *dst, size_t bytes, uint32_t *sink, void *stream) {
    if (!src || !sink || bytes < 16 || bytes % 16 || !aligned16(src) || (dst && !aligned16(dst))) return W4A4_ERR_INVALID_ARG;
    const int cus = probe_cus();
    if (cus < 0) return W4A4_ERR_HIP;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    const size_t cap = (size_t)cus * 16;                          // 16 workgroups of four waves per CU: every wave slot taken
    if (blocks > cap) blocks = cap;
    launch_gemm(stream_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream),
                static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), n16, sink);
    return launch_status();
}
