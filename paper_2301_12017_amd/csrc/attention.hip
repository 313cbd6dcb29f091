// FP16 attention between the QKV projection and the attention output (Sec. 4.2 keeps the attention
// in FP16 and takes its kernel from elsewhere; this is a plain stand-in so that a whole encoder
// layer can be timed): softmax(q.k / sqrt(64)) V per sequence and head, no mask, fp32 arithmetic.
// One workgroup per (sequence, head, block of 4 or 16 queries): the keys and values of the head go to
// LDS once, then each of the four waves takes one query at a time: a lane scores keys lane,
// lane + 64, ..., the wave reduces maximum and sum, and lane d accumulates output feature d.
#include "common.hpp"

namespace w4a4 {
namespace {

constexpr int kHead = 64;             // features per head
constexpr int kAttnWaves = 4;
constexpr int kKeyPitch = kHead / 2 + 1;   // key rows in 32-bit words, padded: lanes read different rows

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__global__ __launch_bounds__(kAttnWaves *kWave) void attention_f16_kernel(const __half *qkv, __half *ctx, int seq,
                                                                            int heads, int qblock) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint32_t *k_lds = reinterpret_cast<uint32_t *>(smem);                       // [seq][kKeyPitch] half2
    const int k_words = (seq * kKeyPitch + 3) & ~3;                              // keeps the value rows 16-byte aligned
    __half *v_lds = reinterpret_cast<__half *>(k_lds + k_words);                 // [seq][64]
    float *p_lds = reinterpret_cast<float *>(v_lds + (size_t)seq * kHead);       // [waves][seq]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qblocks = (seq + qblock - 1) / qblock;
    const int qb = blockIdx.x % qblocks, head = (blockIdx.x / qblocks) % heads, b = blockIdx.x / (qblocks * heads);
    const int h = heads * kHead;
    const long ld = 3L * h;
    const __half *base = qkv + (long)b * seq * ld + head * kHead;

    // keys and values of this head: 8 halves per thread and step
    for (int i = tid; i < seq * (kHead / 8); i += kAttnWaves * kWave) {
        const int row = i / (kHead / 8), c = i % (kHead / 8);
        const uint4 kk = *reinterpret_cast<const uint4 *>(base + row * ld + h + c * 8);
        const uint4 vv = *reinterpret_cast<const uint4 *>(base + row * ld + 2 * h + c * 8);
        uint32_t *kd = k_lds + row * kKeyPitch + c * 4;
        kd[0] = kk.x; kd[1] = kk.y; kd[2] = kk.z; kd[3] = kk.w;
        *reinterpret_cast<uint4 *>(v_lds + row * kHead + c * 8) = vv;
    }
    __syncthreads();

    float *p = p_lds + wave * seq;
    for (int qi = wave; qi < qblock; qi += kAttnWaves) {
        const int i = qb * qblock + qi;
        if (i >= seq) break;                                    // uniform per wave; no barrier below
        // the query, the same 64 values in every lane
        uint32_t q2[kHead / 2];
        const uint4 *qp = reinterpret_cast<const uint4 *>(base + i * ld);
#pragma unroll
        for (int c = 0; c < kHead / 8; ++c) {
            const uint4 t = qp[c];
            q2[4 * c] = t.x; q2[4 * c + 1] = t.y; q2[4 * c + 2] = t.z; q2[4 * c + 3] = t.w;
        }
        // scores of keys lane, lane + 64, ...
        float m = -INFINITY;
        for (int k = lane; k < seq; k += kWave) {
            const uint32_t *kr = k_lds + k * kKeyPitch;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < kHead / 2; ++w) {
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                const uint32_t kw = kr[w];
                s = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, q2[w]), __builtin_bit_cast(h2, kw), s, false);   // fp32 sum of exact products
            }
            s *= 0.125f;                                        // 1 / sqrt(64)
            p[k] = s;
            m = fmaxf(m, s);
        }
        m = wave_max(m);
        float sum = 0.0f;
        for (int k = lane; k < seq; k += kWave) {
            const float e = expf(p[k] - m);
            p[k] = e;
            sum += e;
        }
        sum = wave_sum_f(sum);
        __builtin_amdgcn_wave_barrier();                        // the wave's LDS writes are in order; keep the compiler from moving the reads up
        // output feature `lane`
        float acc = 0.0f;
#pragma unroll 8
        for (int k = 0; k < seq; ++k) acc = fmaf(p[k], __half2float(v_lds[k * kHead + lane]), acc);
        ctx[((long)b * seq + i) * h + head * kHead + lane] = __float2half(acc / sum);
        __builtin_amdgcn_wave_barrier();                        // p is reused by the wave's next query
    }
}

}  // namespace
}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_attention_f16(const void *QKV_f16, int batch, int seq, int heads, void *ctx_f16, void *stream) {
    if (batch < 0 || seq < 0 || heads <= 0) return W4A4_ERR_INVALID_ARG;
    if (batch == 0 || seq == 0) return W4A4_OK;
    if (!QKV_f16 || !ctx_f16) return W4A4_ERR_INVALID_ARG;
    if (seq > 512 || heads > 1024) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(QKV_f16) || !aligned16(ctx_f16)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    // sixteen queries share one copy of the head's keys and values; with few sequences and heads four do, so that
    // the launch still covers the chip
    const int qblock = (long)batch * heads * ((seq + 15) / 16) >= 512 ? 16 : 4;
    const long blocks = (long)batch * heads * ((seq + qblock - 1) / qblock);
    if (blocks > 0x7fffffffL || (long)batch * seq * 3 * heads * kHead >= 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const size_t lds = (size_t)((seq * kKeyPitch + 3) & ~3) * 4 + (size_t)seq * kHead * 2 + (size_t)kAttnWaves * seq * 4;
    static KernelState ks;
    if (prepare_kernel(reinterpret_cast<const void *>(attention_f16_kernel), lds, ks) < 0) return W4A4_ERR_HIP;
    hipLaunchKernelGGL(attention_f16_kernel, dim3((unsigned)blocks), dim3(kAttnWaves * kWave), lds, as_stream(stream),
                       static_cast<const __half *>(QKV_f16), static_cast<__half *>(ctx_f16), seq, heads, qblock);
    return hipGetLastError() == hipSuccess ? W4A4_OK : W4A4_ERR_HIP;
}
