// Stand-alone dequantize epilogue (step a3 applied to int32 accumulators that are
// already in memory).  It is the unfused counterpart of the epilogue that w4a4_linear
// runs inside the GEMM: the same formulas, in the same operation order.
//
// One wavefront owns one output row; a lane handles eight consecutive columns at a
// time (two 16-byte accumulator loads per K-group, one 16-byte fp16 store or one dword
// of packed codes).  For the requantize form the row is evaluated twice -- once for
// its range, once for the codes -- because the evaluation is deterministic and cheaper
// than parking a whole row in registers for arbitrary N.
#include "common.hpp"

namespace w4a4 {

struct EpiArgs {
    const int32_t *acc;    // [ng, M, N]
    int M, N, ng;
    const float *sa, *za;  // [M]
    const int32_t *RA;     // [M, ng]
    const float *sw, *zw;  // [N, ng]
    const float *c;        // [N]
    const __half *bias;    // [N] or null
    int act;
    // outputs
    __half *out16;         // [M, N]
    uint8_t *outq;         // [M, N/2]
    float *outs, *outz;    // [M]
    int32_t *outg;         // [M, rng]
    int rG, rng;           // requant group length and count
};

// y[e] for columns n0..n0+7 of row m.  Operation order is part of the contract:
//   SYM, ng == 1:  y = ((float)P * sa) * sw
//   otherwise:     t1 = sum_g sw[n,g]*(float)P_g ; y = sa*t1
//   ASYM adds:     t2 = sum_g zw[n,g]*(float)RA[m,g] ; y = y + sa*t2 ; y = y + za*c[n]
// then + bias, then GELU (GELU32; the fp16 store applies its own, rounded once to fp16).
template <int MODE, bool GELU32 = true>
__device__ __forceinline__ void dequant8(const EpiArgs &a, long m, int n0, float (&y)[8]) {
    const float sa = a.sa[m];
    if (MODE == W4A4_SYM && a.ng == 1) {
        const int4 *p = reinterpret_cast<const int4 *>(a.acc + m * a.N + n0);
        int4 p0 = p[0], p1 = p[1];
        int pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = (float)pv[e] * sa;
            y[e] = t * a.sw[n0 + e];
        }
    } else {
        float t1[8], t2[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { t1[e] = 0.0f; t2[e] = 0.0f; }
        for (int g = 0; g < a.ng; ++g) {
            const int4 *p = reinterpret_cast<const int4 *>(a.acc + ((long)g * a.M + m) * a.N + n0);
            int4 p0 = p[0], p1 = p[1];
            int pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            float ra = MODE == W4A4_ASYM ? (float)a.RA[m * a.ng + g] : 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float u = a.sw[(long)(n0 + e) * a.ng + g] * (float)pv[e];
                t1[e] = t1[e] + u;
                if (MODE == W4A4_ASYM) {
                    float w = a.zw[(long)(n0 + e) * a.ng + g] * ra;
                    t2[e] = t2[e] + w;
                }
            }
        }
        const float za = MODE == W4A4_ASYM ? a.za[m] : 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = sa * t1[e];
            if (MODE == W4A4_ASYM) {
                float p = sa * t2[e];
                float q = za * a.c[n0 + e];
                v = v + p;
                v = v + q;
            }
            y[e] = v;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (a.bias) y[e] = y[e] + __half2float(a.bias[n0 + e]);
        if (GELU32 && a.act == W4A4_ACT_GELU) y[e] = gelu_erf(y[e]);
    }
}

// REQ: -1 fp16 store, else the w4a4_mode of the requantized output.
template <int MODE, int REQ>
__global__ __launch_bounds__(256) void dequant_rows_kernel(EpiArgs a) {
    __shared__ int32_t gs[4][512];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const long m = (long)blockIdx.x * 4 + wave;
    if (m >= a.M) return;
    const int nchunks = a.N / 8;
    float y[8];
    if (REQ < 0) {
        for (int c = lane; c < nchunks; c += kWave) {
            dequant8<MODE, false>(a, m, c * 8, y);
            uint4 w;
            if (a.act == W4A4_ACT_GELU) {
                w = uint4{gelu_erf_half2(y[0], y[1]), gelu_erf_half2(y[2], y[3]), gelu_erf_half2(y[4], y[5]), gelu_erf_half2(y[6], y[7])};
            } else {
                __half2 h[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = __floats2half2_rn(y[2 * i], y[2 * i + 1]);
                w = *reinterpret_cast<uint4 *>(h);
            }
            *reinterpret_cast<uint4 *>(a.out16 + m * a.N + c * 8) = w;
        }
        return;
    }
    float lo = INFINITY, hi = -INFINITY;
    for (int c = lane; c < nchunks; c += kWave) {
        dequant8<MODE>(a, m, c * 8, y);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (REQ == W4A4_SYM) hi = fmaxf(hi, fabsf(y[e]));
            else { hi = fmaxf(hi, y[e]); lo = fminf(lo, y[e]); }
        }
    }
    Range r = REQ == W4A4_SYM ? range_sym(wave_max(hi)) : range_asym(wave_min(lo), wave_max(hi));
    if (lane == 0) {
        a.outs[m] = r.S;
        if (REQ == W4A4_ASYM) a.outz[m] = r.lo;
    }
    if (a.outg) {
        for (int g = lane; g < a.rng; g += kWave) gs[wave][g] = 0;
        __builtin_amdgcn_wave_barrier();
    }
    uint32_t *qr = reinterpret_cast<uint32_t *>(a.outq + m * (long)(a.N / 2));
    const int cpg = a.rG / 8;
    for (int c = lane; c < nchunks; c += kWave) {
        dequant8<MODE>(a, m, c * 8, y);
        uint32_t packed = 0;
        int sum = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int code = code_of<(REQ < 0 ? 0 : REQ)>(y[e], r);
            sum += code;
            packed |= (uint32_t)(code & 0xF) << (4 * e);
        }
        qr[c] = packed;
        if (a.outg) atomicAdd(&gs[wave][c / cpg], sum);
    }
    if (a.outg) {
        __builtin_amdgcn_wave_barrier();
        for (int g = lane; g < a.rng; g += kWave) a.outg[m * a.rng + g] = gs[wave][g];
    }
}

}  // namespace w4a4

using namespace w4a4;

// Checks shared with the fused path live in gemm.hip; declared here.
namespace w4a4 {
int check_layer(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, const void *out,
                const float *out_scale, const float *out_zero, int *ng, int *rng);
}

extern "C" int w4a4_dequant_epilogue(const int32_t *acc, const w4a4_act *A, const w4a4_weight *W,
                                     const w4a4_epilogue *ep, void *out, float *out_scale,
                                     float *out_zero, int32_t *out_gsum, void *stream) {
    int ng = 0, rng = 0;
    int rc = check_layer(A, W, ep, out, out_scale, out_zero, &ng, &rng);
    if (rc) return rc;
    if (ep->requant && ep->requant_layout != W4A4_LAYOUT_CANONICAL) return W4A4_ERR_UNSUPPORTED_SHAPE;   // canonical codes only
    if (A->M == 0) return W4A4_OK;
    if (!acc) return W4A4_ERR_INVALID_ARG;
    if (!aligned16(acc)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    EpiArgs a;
    a.acc = acc; a.M = A->M; a.N = W->N; a.ng = ng;
    a.sa = A->scale; a.za = A->zero; a.RA = A->gsum;
    a.sw = W->scale; a.zw = W->zero; a.c = W->rowsum_deq;
    a.bias = static_cast<const __half *>(ep->bias_f16); a.act = ep->act;
    a.out16 = static_cast<__half *>(out); a.outq = static_cast<uint8_t *>(out);
    a.outs = out_scale; a.outz = out_zero; a.outg = ep->requant ? out_gsum : nullptr;
    a.rG = ep->requant_group == 0 ? W->N : ep->requant_group; a.rng = rng;
    dim3 grid((a.M + 3) / 4), block(256);
    hipStream_t st = as_stream(stream);
    const int req = ep->requant ? ep->requant_mode : -1;
#define W4A4_EL(MODE, REQ) hipLaunchKernelGGL((dequant_rows_kernel<MODE, REQ>), grid, block, 0, st, a)
    if (A->mode == W4A4_SYM) {
        if (req < 0) W4A4_EL(W4A4_SYM, -1);
        else if (req == W4A4_SYM) W4A4_EL(W4A4_SYM, W4A4_SYM);
        else W4A4_EL(W4A4_SYM, W4A4_ASYM);
    } else {
        if (req < 0) W4A4_EL(W4A4_ASYM, -1);
        else if (req == W4A4_SYM) W4A4_EL(W4A4_ASYM, W4A4_SYM);
        else W4A4_EL(W4A4_ASYM, W4A4_ASYM);
    }
#undef W4A4_EL
    return launch_status();
}
