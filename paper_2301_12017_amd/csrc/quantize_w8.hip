// Row-wise symmetric INT8 quantization of fp16 rows: the quantizer of the INT8 sibling of the path
// (Sec. 3.1 with b = 8: S = absmax / 127, code = rne(x * (127 / absmax)); token-wise for activations,
// per output channel for weights, App. A).  One code per byte.  Same structure as the INT4 row
// quantizer: one wavefront per row, 16-byte loads, the row in registers as raw fp16, the range on
// packed fp16, rounding by an fp32 add of 1.5 * 2^23 (the clamp of the mapping cannot bind:
// |t| <= 127 (1 + 2^-23)); eight codes leave as eight bytes per lane and step.  HBM-bound: 2 bytes in,
// 1 byte out per element.
#include "common.hpp"

namespace w4a4 {

constexpr int kQ8RowsPerBlock = 4;

template <int ITERS>
__global__ __launch_bounds__(kQ8RowsPerBlock *kWave) void quantize_rows8_kernel(
    const __half *__restrict__ X, long ldx, int rows, int K, int8_t *__restrict__ q, float *__restrict__ s) {
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const int lane = threadIdx.x % kWave;
    const long row = (long)blockIdx.x * kQ8RowsPerBlock + threadIdx.x / kWave;
    if (row >= rows) return;                                    // whole wave leaves; no block barrier below
    const int nchunks = K / 8;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__half *>(X + row * ldx), (short)0, K * 2, 0x00020000);
    u4 raw[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) raw[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, (lane + it * kWave) * 16, 0, 0);
    uint32_t zero = 0;
    h2 mx = *reinterpret_cast<const h2 *>(&zero);
#pragma unroll
    for (int it = 0; it < ITERS; ++it)                          // chunks past K read as zero: harmless for |x| maxima
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t d = raw[it][i] & 0x7FFF7FFFu;
            mx = __builtin_elementwise_max(mx, *reinterpret_cast<const h2 *>(&d));
        }
    const float amax = wave_max(fmaxf((float)mx[0], (float)mx[1]));
    float inv, S;
    if (amax == 0.0f) { inv = 0.0f; S = 1.0f; }
    else { inv = 127.0f / amax; S = amax / 127.0f; }
    if (lane == 0) s[row] = S;
    uint2 *qr = reinterpret_cast<uint2 *>(q + row * (long)K);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        uint32_t u[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t d = raw[it][i];
            const float2 f = __half22float2(*reinterpret_cast<const __half2 *>(&d));
            const float t0 = f.x * inv, t1 = f.y * inv;
            u[2 * i] = __float_as_uint(t0 + 12582912.0f);           // the code is the low byte of the sum
            u[2 * i + 1] = __float_as_uint(t1 + 12582912.0f);
        }
        const uint32_t lo = __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u) | __builtin_amdgcn_perm(u[3], u[2], 0x04000c0cu);
        const uint32_t hi = __builtin_amdgcn_perm(u[5], u[4], 0x0c0c0400u) | __builtin_amdgcn_perm(u[7], u[6], 0x04000c0cu);
        if (c < nchunks) qr[c] = make_uint2(lo, hi);
    }
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w8a8_quantize_rows(const void *X_f16, int M, int K, int ldx, int8_t *q, float *scale, void *stream) {
    if (M < 0 || K <= 0 || ldx < K) return W4A4_ERR_INVALID_ARG;
    if (M > 0 && (!X_f16 || !q || !scale)) return W4A4_ERR_INVALID_ARG;
    if (K % 32 || K > 16384 || (ldx * 2) % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return W4A4_OK;
    if (!aligned16(X_f16) || !aligned16(q)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int iters = (K / 8 + kWave - 1) / kWave;
    dim3 grid((unsigned)((M + kQ8RowsPerBlock - 1) / kQ8RowsPerBlock)), block(kQ8RowsPerBlock * kWave);
    hipStream_t st = as_stream(stream);
    const __half *X = static_cast<const __half *>(X_f16);
#define W8_Q(I) hipLaunchKernelGGL((quantize_rows8_kernel<I>), grid, block, 0, st, X, (long)ldx, M, K, q, scale)
    if (iters <= 1) W8_Q(1);
    else if (iters <= 2) W8_Q(2);
    else if (iters <= 4) W8_Q(4);
    else if (iters <= 8) W8_Q(8);
    else if (iters <= 16) W8_Q(16);
    else W8_Q(32);
#undef W8_Q
    return launch_status();
}
