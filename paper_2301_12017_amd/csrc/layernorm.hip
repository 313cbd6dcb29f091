// LayerNorm (+ residual) of fp16 token rows fused with the token-wise INT4 quantize (Sec. 4.2:
// the quantize of an activation is fused with the bias-add, GELU or LayerNorm that produces
// it, so the activation reaches the next GEMM already packed).
//
//     v    = x + r                         (r optional)
//     mean = sum(v) / K,   var = sum((v - mean)^2) / K        (biased, two passes over registers)
//     y    = (v - mean) * rstd * gamma + beta,   rstd = 1 / sqrt(var + eps)
//
// in fp32, every operation separately rounded.  y is then quantized per token exactly like an
// activation row (step a1: range over the row, t = y * (7/absmax) or (y - min) * (15/(max-min)),
// round to nearest even) from its fp32 value, and optionally stored as fp16 for the residual
// stream.  HBM-bound: 2 (+2) bytes in and 0.5 (+2) bytes out per element.
//
// One wavefront owns one token: 16-byte loads, the row stays in registers (K <= 4096: eight
// chunks of eight elements per lane), sums and ranges are reduced with wave shuffles, codes
// leave as one dword per lane and step (FP6 operand layout: the four lanes of a quad hold one
// operand of 32 codes, of which three store eight bytes each).
#include "common.hpp"

namespace w4a4 {

constexpr int kLnRowsPerBlock = 4;

struct LnArgs {
    const __half *X, *R; long ldx;       // [M, ldx] each; R may be NULL
    const __half *gamma, *beta;          // [K]
    float eps;
    __half *Y;                           // [M, K] or NULL
    uint8_t *q; float *s, *z;            // [M, K/2], [M], [M]
    int32_t *gsum; int ng, cpg;          // [M, ng] code sums of runs of cpg chunks (NULL = not wanted)
    int32_t *psum;                       // [M] odd-position code sums (MFMA operand layout)
    int M, K;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ void halves8(const uint4 &raw, float (&v)[8]) {
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h[i]);
        v[2 * i] = f.x;
        v[2 * i + 1] = f.y;
    }
}

// One lane's eight codes of chunk c of a row (fields 8 (c % 4) .. + 7 of operand c / 4) as 48 bits {lo, hi16}, and the
// next lane's: the four lanes of a quad hold one operand of 24 bytes, of which lanes 0, 1 and 2 store bytes 0 .. 7,
// 8 .. 15 (the operand's sixteen-byte part) and 16 .. 23 (its eight-byte part).  See w4a4_layout for the addresses.
__device__ __forceinline__ void fp6_store_chunk(uint8_t *q, int K, long row, int c, uint32_t lo, uint32_t hi,
                                                uint32_t nlo, uint32_t nhi) {
    const int j = c & 3, o = c >> 2, b = o >> 1, e = o & 1;
    if (j == 3) return;
    // bytes 8j .. 8j+7 of the quad's 24: own bytes 2j .. 5, then the next lane's 0 .. 2j+1
    uint32_t w0, w1;
    if (j == 0) { w0 = lo; w1 = (hi & 0xFFFFu) | (nlo << 16); }
    else if (j == 1) { w0 = (lo >> 16) | (hi << 16); w1 = nlo; }
    else { w0 = (hi & 0xFFFFu) | (nlo << 16); w1 = (nlo >> 16) | (nhi << 16); }
    const long r = row & 63;
    uint8_t *blk = q + ((row >> 6) * (long)(K / 64) + b) * 3072 + r * 48;
    uint8_t *dst = j < 2 ? blk + 16 * e + 8 * j : blk + 32 + 8 * (e ^ (int)((r >> 4) & 1));
    *reinterpret_cast<uint2 *>(dst) = make_uint2(w0, w1);
}

// LAYOUT: 0 canonical nibbles, 1 the MFMA operand layout of activations, 2 the FP6 operand layout (both: symmetric codes only)
template <int MODE, int ITERS, int LAYOUT>
__global__ __launch_bounds__(kLnRowsPerBlock *kWave) void layernorm_quantize_kernel(LnArgs a) {
    const int lane = threadIdx.x % kWave;
    const long row = (long)blockIdx.x * kLnRowsPerBlock + threadIdx.x / kWave;
    const int K = a.K, nchunks = K / 8;
    if (row >= a.M) {                                           // whole wave leaves; no block barrier below
        if constexpr (LAYOUT == 2) {                            // the layout stores whole 64-token panels: zero rows behind M
            if (row < (((long)a.M + 63) & ~63L)) {
#pragma unroll
                for (int it = 0; it < ITERS; ++it)
                    if (lane + it * kWave < nchunks) fp6_store_chunk(a.q, K, row, lane + it * kWave, 0u, 0u, 0u, 0u);
            }
        }
        return;
    }
    const __half *xr = a.X + row * a.ldx;
    const __half *rr = a.R ? a.R + row * a.ldx : nullptr;

    // ---- v = x + r, in registers ------------------------------------------------------------------
    float v[ITERS][8];
    float sum = 0.0f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        if (c < nchunks) {
            halves8(*reinterpret_cast<const uint4 *>(xr + c * 8), v[it]);
            if (rr) {
                float t[8];
                halves8(*reinterpret_cast<const uint4 *>(rr + c * 8), t);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[it][e] = v[it][e] + t[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += v[it][e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[it][e] = 0.0f;
        }
    }
    const float inv_k = 1.0f / (float)K;
    const float mean = wave_sum(sum) * inv_k;
    float sq = 0.0f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        if (lane + it * kWave < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[it][e] = v[it][e] - mean;
                const float d2 = v[it][e] * v[it][e];
                sq += d2;
            }
        }
    }
    const float var = wave_sum(sq) * inv_k;
    const float rstd = 1.0f / sqrtf(var + a.eps);

    // ---- y = (v - mean) * rstd * gamma + beta; fp16 copy; range of the row ---------------------------
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        if (c < nchunks) {
            float g[8], b[8];
            halves8(*reinterpret_cast<const uint4 *>(a.gamma + c * 8), g);
            halves8(*reinterpret_cast<const uint4 *>(a.beta + c * 8), b);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float y = v[it][e] * rstd;
                y = y * g[e];
                y = y + b[e];
                v[it][e] = y;
                if (MODE == W4A4_SYM) hi = fmaxf(hi, fabsf(y));
                else { hi = fmaxf(hi, y); lo = fminf(lo, y); }
            }
            if (a.Y) {
                __half2 h[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = __floats2half2_rn(v[it][2 * i], v[it][2 * i + 1]);
                typedef unsigned int u4 __attribute__((ext_vector_type(4)));
                // written once, read by a later kernel: keep it out of the way of the rows still being read
                __builtin_nontemporal_store(*reinterpret_cast<const u4 *>(h), reinterpret_cast<u4 *>(a.Y + row * (long)K + c * 8));
            }
        }
    }
    const Range r = MODE == W4A4_SYM ? range_sym(wave_max(hi)) : range_asym(wave_min(lo), wave_max(hi));
    if (lane == 0) {
        a.s[row] = r.S;
        if (MODE == W4A4_ASYM) a.z[row] = r.lo;
    }

    // ---- codes: rne(t) is the low mantissa of t + 1.5*2^23 (the clamp of the mapping cannot bind);
    //      symmetric codes in offset binary (+8 rides in the constant) so that nibble sums are byte sums,
    //      one XOR per dword then gives the layout wanted -------------------------------------------------
    if constexpr (LAYOUT == 2) {
        // t = rne(y * 7/absmax) is an integer of magnitude <= 7; the FP8 E4M3 encoding of t / 64, which the pack
        // conversion produces two at a time (the division is its scale operand), is `sign 0 0 e e m m m` with the
        // exponent and mantissa bits of t's FP6 E2M3 encoding: a field is that byte without its two zero bits
        typedef short v2s __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int c = lane + it * kWave;
            uint32_t f24[2];
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                float t[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = __builtin_rintf(v[it][4 * p + e] * r.inv);
                v2s pk = {0, 0};
                pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, t[0], t[1], 64.0f, false);
                pk = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(pk, t[2], t[3], 64.0f, true);
                const uint32_t b4 = __builtin_bit_cast(uint32_t, pk);
                const uint32_t f4 = (b4 & 0x1F1F1F1Fu) | ((b4 >> 2) & 0x20202020u);   // four 6-bit fields, one per byte
                const uint32_t p2 = (f4 & 0x003F003Fu) | ((f4 >> 2) & 0x0FC00FC0u);   // two 12-bit pairs, one per half
                f24[p] = (p2 & 0x00000FFFu) | ((p2 >> 4) & 0x00FFF000u);              // 24 bits
            }
            const uint32_t lo = f24[0] | (f24[1] << 24), hi = f24[1] >> 8;            // 48 bits
            const uint32_t nlo = dpp_fetch<0xF9>(lo), nhi = dpp_fetch<0xF9>(hi);      // quad permute [1,2,3,3]: the next lane's
            if (c < nchunks) fp6_store_chunk(a.q, K, row, c, lo, hi, nlo, nhi);
        }
        return;
    }
    constexpr float kMagic = MODE == W4A4_SYM ? 12582920.0f : 12582912.0f;
    constexpr uint32_t kFlip = MODE == W4A4_ASYM ? 0u : LAYOUT == 0 ? 0x88888888u : 0x80808080u;
    uint32_t *qr = reinterpret_cast<uint32_t *>(a.q + row * (long)(K / 2));
    int part = 0, total = 0;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int c = lane + it * kWave;
        const bool in = c < nchunks;
        uint32_t packed = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t;
            if (MODE == W4A4_SYM) t = v[it][e] * r.inv;
            else { const float d = v[it][e] - r.lo; t = d * r.inv; }
            const float u = t + kMagic;
            packed |= (__float_as_uint(u) & 0xFu) << (4 * e);
        }
        const uint32_t even = packed & 0x0F0F0F0Fu, odd = (packed >> 4) & 0x0F0F0F0Fu;
        int s8 = 0;
        if (a.gsum && in)
            s8 = (int)__builtin_amdgcn_sad_u8(even, 0u, __builtin_amdgcn_sad_u8(odd, 0u, 0u)) - (MODE == W4A4_SYM ? 64 : 0);
        if (LAYOUT != 0 && in) part += (int)__builtin_amdgcn_sad_u8(odd, 0u, 0u) - 32;
        if (in) qr[c] = packed ^ kFlip;                         // (a plain store: the next GEMM reads the codes from cache)
        total += s8;
        if (a.gsum && a.ng > 1) {                               // groups of cpg lanes, all inside this `it`
            for (int o = 1; o < a.cpg; o <<= 1) s8 += __shfl_xor(s8, o, kWave);
            if ((lane & (a.cpg - 1)) == 0 && in) a.gsum[row * (long)a.ng + c / a.cpg] = s8;
        }
    }
    if (a.gsum && a.ng == 1) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) total += __shfl_xor(total, o, kWave);
        if (lane == 0) a.gsum[row] = total;
    }
    if (LAYOUT != 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, kWave);
        if (lane == 0) a.psum[row] = part;
    }
}

template <int MODE, int LAYOUT>
static int launch_ln(const LnArgs &a, hipStream_t st) {
    const int iters = (a.K / 8 + kWave - 1) / kWave;
    const long rows = LAYOUT == 2 ? (((long)a.M + 63) & ~63L) : a.M;     // (FP6: the zero rows that fill the last panel too)
    dim3 grid((unsigned)((rows + kLnRowsPerBlock - 1) / kLnRowsPerBlock)), block(kLnRowsPerBlock * kWave);
#define W4A4_LN(I) hipLaunchKernelGGL((layernorm_quantize_kernel<MODE, I, LAYOUT>), grid, block, 0, st, a)
    if (iters <= 1) W4A4_LN(1);
    else if (iters <= 2) W4A4_LN(2);
    else if (iters <= 4) W4A4_LN(4);
    else if (iters <= 8) W4A4_LN(8);
    else return W4A4_ERR_UNSUPPORTED_SHAPE;
#undef W4A4_LN
    return launch_status();
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_layernorm_quantize(const void *X_f16, const void *R_f16, int M, int K, int ldx,
                                       const void *gamma_f16, const void *beta_f16, float eps, void *Y_f16,
                                       int mode, int group, uint8_t *q, float *scale, float *zero, int32_t *gsum,
                                       int layout, int32_t *osum, void *stream) {
    if (M < 0 || K <= 0 || ldx < K || group < 0 || !(eps >= 0.0f)) return W4A4_ERR_INVALID_ARG;
    if (mode != W4A4_SYM && mode != W4A4_ASYM) return W4A4_ERR_INVALID_ARG;
    if (layout != W4A4_LAYOUT_CANONICAL && layout != W4A4_LAYOUT_MFMA && layout != W4A4_LAYOUT_FP6) return W4A4_ERR_INVALID_ARG;
    if (layout != W4A4_LAYOUT_CANONICAL && mode != W4A4_SYM) return W4A4_ERR_INVALID_ARG;
    if (layout == W4A4_LAYOUT_FP6 && gsum) return W4A4_ERR_INVALID_ARG;        // no code sums travel with that layout
    if (M > 0 && (!X_f16 || !gamma_f16 || !beta_f16 || !q || !scale || (mode == W4A4_ASYM && !zero) ||
                  (layout == W4A4_LAYOUT_MFMA && !osum)))
        return W4A4_ERR_INVALID_ARG;
    if (K % 32 || K > 4096 || (ldx * 2) % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int G = group == 0 ? K : group;
    if (G % 32 || K % G) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (layout != W4A4_LAYOUT_CANONICAL && G != K) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (layout == W4A4_LAYOUT_FP6) {                            // a row length the layout is offered for
        int lpr = 0, opl = 0;
        if (!fp6_plan(K, &lpr, &opl)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    const int ng = K / G, cpg = G / 8;
    if (gsum && ng > 1 && (cpg > 64 || (cpg & (cpg - 1)))) return W4A4_ERR_UNSUPPORTED_SHAPE;   // segmented wave sums
    if (M == 0) return W4A4_OK;
    if (!aligned16(X_f16) || (R_f16 && !aligned16(R_f16)) || !aligned16(gamma_f16) || !aligned16(beta_f16) ||
        (Y_f16 && !aligned16(Y_f16)) || !aligned16(q))
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    LnArgs a;
    a.X = static_cast<const __half *>(X_f16); a.R = static_cast<const __half *>(R_f16); a.ldx = ldx;
    a.gamma = static_cast<const __half *>(gamma_f16); a.beta = static_cast<const __half *>(beta_f16);
    a.eps = eps; a.Y = static_cast<__half *>(Y_f16);
    a.q = q; a.s = scale; a.z = zero; a.gsum = gsum; a.ng = ng; a.cpg = cpg; a.psum = osum;
    a.M = M; a.K = K;
    hipStream_t st = as_stream(stream);
    if (layout == W4A4_LAYOUT_MFMA) return launch_ln<W4A4_SYM, 1>(a, st);
    if (layout == W4A4_LAYOUT_FP6) return launch_ln<W4A4_SYM, 2>(a, st);
    return mode == W4A4_SYM ? launch_ln<W4A4_SYM, 0>(a, st) : launch_ln<W4A4_ASYM, 0>(a, st);
}
