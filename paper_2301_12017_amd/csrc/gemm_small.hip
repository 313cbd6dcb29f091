// Linear layer for small token counts with the activation quantize inside the GEMM kernel:
//   out = epilogue( Q(X) * Wq^T ),  Q = the symmetric per-token INT4 mapping of Sec. 3.1.
//
// At batch 1 x sequence 128 (M = 128) a linear layer is a few microseconds of work and the
// launch of a kernel costs about as much (Sec. 4.2: at small batch x sequence the launch overhead
// and the memory-bound quantize kernels are what hurts).  So this path spends arithmetic to save
// a launch: every workgroup quantizes the rows of its 32 tokens itself, into LDS, and multiplies
// from there; codes and scales never reach memory.  The result is bit for bit what
// w4a4_quantize_act followed by w4a4_linear gives (same fp32 operations in the same order, exact
// integer sums).
//
//   * tile: 32 tokens x 32 (or 64) channels per workgroup of NW = 4, 8 or 16 waves;
//   * pass 1: the 32 x K fp16 rows are read ONCE, fully coalesced (2 NW consecutive lanes per token),
//     and stay in registers (at most 16 chunks of 16 bytes per lane) while the range of each token
//     is reduced over its lanes; then every lane quantizes its own registers: t = x * (7/absmax),
//     rne(t) by adding 1.5 * 2^23 (the clamp of the mapping cannot bind for symmetric codes); the
//     code then sits in the low byte of the sum and v_perm_b32 gathers four of them into an int8
//     MFMA operand register, in the order the weight widening produces (even codes, odd codes of
//     a packed dword).  The int8 tile goes to LDS (row pitch K + 16 bytes: conflict-free 16-byte
//     reads of 32 consecutive rows);
//   * the packed weight codes of the tile's channels are requested together with the activation
//     rows, coalesced as well, and parked in LDS beside the activation codes;
//   * pass 2: the waves split K in blocks of 64 codes (interleaved) and read both operands from
//     LDS in MFMA order; weights are widened to 16 * code, activations stay 1 * code: the
//     accumulators hold 16 * P;
//   * the int32 partial sums of the waves are added in LDS and the accumulator registers of the
//     tile are dealt round robin to the waves for the epilogue.
#include "gemm_common.hpp"

namespace w4a4 {

struct SmallArgs {
    const __half *X; long ldx;       // [M, K] fp16, row stride in elements (fp16-activation form)
    const uint8_t *Aq; long lda;     // [M, K/2] canonical packed codes, row stride in bytes (packed form)
    const float *sa;                 // [M] token scales (packed form)
    int32_t *acc_out;                // packed form only: store the int32 sums P [M, N] instead of fp16 outputs
    const uint8_t *Wq; long ldw;     // canonical packed codes [N, K/2]; INT8 sibling: int8 codes [N, K]
    const float *sw;                 // [N]
    const __half *bias; int act;
    __half *out;                     // [M, N]
    int M, N, K, tiles_n;
};

// 16-byte chunks held by one lane: of its token row (K <= 4096: 512 chunks over 2 NW * 32 / TM lanes), and of
// the weight tile on its way to LDS (the launcher checks the latter)
constexpr int small_xchunks(int tm) { return tm == 16 ? 8 : 16; }
constexpr int small_wchunks(int nw) { return nw == 16 ? 4 : 6; }

// eight fp16 values -> their codes, as two operand registers: bytes (c0,c2,c4,c6) and (c1,c3,c5,c7)
// (NATURAL: bytes (c0,c1,c2,c3) and (c4,c5,c6,c7) instead: the order of one-byte weight codes)
template <bool NATURAL = false>
__device__ __forceinline__ void codes8(const u32x4 &x, float inv, uint32_t &even, uint32_t &odd) {
    uint32_t u[8];
    const float nzero = -0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // t = fp32(x) * inv in one instruction: v_fma_mix_f32 reads the fp16 half directly and rounds the
        // product once to fp32 (the addend -0 changes nothing), exactly what convert-then-multiply gives
        float t0, t1;
        asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(t0) : "v"(x[i]), "v"(inv), "v"(nzero));
        asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(t1) : "v"(x[i]), "v"(inv), "v"(nzero));
        u[2 * i] = __float_as_uint(t0 + 12582912.0f);
        u[2 * i + 1] = __float_as_uint(t1 + 12582912.0f);
    }
    if (NATURAL) {
        even = __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u) | __builtin_amdgcn_perm(u[3], u[2], 0x04000c0cu);
        odd = __builtin_amdgcn_perm(u[5], u[4], 0x0c0c0400u) | __builtin_amdgcn_perm(u[7], u[6], 0x04000c0cu);
    } else {
        even = __builtin_amdgcn_perm(u[2], u[0], 0x0c0c0400u) | __builtin_amdgcn_perm(u[6], u[4], 0x04000c0cu);
        odd = __builtin_amdgcn_perm(u[3], u[1], 0x0c0c0400u) | __builtin_amdgcn_perm(u[7], u[5], 0x04000c0cu);
    }
}

// NW waves, FN column fragments of 32 channels, TM = 32 or 16 tokens per workgroup (with 16 the upper
// half of the MFMA rows repeats the lower one and is not stored), WLDS: the weight tile is staged in LDS.
// PACKED: the activations arrive already quantized (packed codes + token scales, the output of
// w4a4_quantize_act or of a producer kernel): pass 1 only parks their tile in LDS, and both operands are
// widened to 16 * code on their way into the MFMA (the sums hold 256 * P).
// W8: the INT8 sibling.  Tokens are quantized with 127 levels per side (or arrive as one int8 code per
// byte when PACKED), the weights are one int8 code per byte, and both go into the MFMA as they are (the
// sums hold P).
template <int NW, int FN, int TM, bool WLDS, bool PACKED, bool W8 = false>
__global__ __launch_bounds__(NW * 64) void linear_f16act_kernel(SmallArgs a) {
    constexpr int NT = NW * 64, LPR = NT / TM;                  // LPR consecutive lanes share a token in pass 1
    constexpr int RV = TM / 2;                                  // accumulator registers per fragment that hold real rows
    constexpr int R = RV * FN;                                  // ... of the tile
    constexpr int RPW = (R + NW - 1) / NW;                      // ... finished by one wave
    constexpr int WCH = WLDS ? small_wchunks(NW) : 1;
    constexpr int XCH = PACKED ? 1 : small_xchunks(TM);
    constexpr int ACH = PACKED ? (W8 ? 8 : 4) : 1;              // 16-byte chunks of the packed activation tile per lane
    constexpr bool NIBBLES = PACKED && !W8;                     // activation codes arrive two per byte
    static_assert(LPR <= 64 && (LPR & (LPR - 1)) == 0, "a token's lanes sit in one wave");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int wpitch = (W8 ? a.K : a.K / 2) + 16, pitch = NIBBLES ? a.K / 2 + 16 : a.K + 16;
    uint8_t *codes = smem;                                      // [TM][pitch] int8 activation codes (packed codes if PACKED)
    uint8_t *wt = codes + TM * pitch;                           // [32 FN][wpitch] packed weight codes (WLDS)
    int *s_sum = reinterpret_cast<int *>(wt + (WLDS ? 32 * FN * wpitch : 0));   // [R][64]
    float *s_S = reinterpret_cast<float *>(s_sum + R * 64);     // [TM]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m0 = (blockIdx.x / a.tiles_n) * TM, n0 = (blockIdx.x % a.tiles_n) * (32 * FN);
    const __amdgpu_buffer_rsrc_t x_rsrc = PACKED ? make_rsrc(a.Aq, (uint32_t)((long)(a.M - 1) * a.lda + (W8 ? a.K : a.K / 2)))
                                                 : make_rsrc(a.X, (uint32_t)(((long)(a.M - 1) * a.ldx + a.K) * 2));
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(a.Wq, (uint32_t)((long)a.N * a.ldw));
    const int r = lane & 31, h = lane >> 5;                     // pass 2: token / channel r, K half h
    const int nb = a.K / 64;

    // ---- requests, in the order they are needed: activation rows, weights, channel constants ----------------
    const int row = tid / LPR, c0 = tid % LPR;
    const int nchunks = a.K / 8;                                // 16-byte chunks of an activation row
    const int wcpr = W8 ? a.K / 16 : a.K / 32;                  // 16-byte chunks of a row of weight codes
    u32x4 x[XCH];
    u32x4 ast[ACH];
    int arow_i[ACH];
    uint32_t adst_i[ACH];
    if constexpr (!PACKED) {
        const uint32_t base = (uint32_t)min(m0 + row, a.M - 1) * (uint32_t)a.ldx * 2u;
#pragma unroll
        for (int i = 0; i < XCH; ++i)               // (chunks past the row are requested but never used)
            if (i * LPR < nchunks) x[i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, base + (uint32_t)(c0 + i * LPR) * 16, 0, 0);
    } else {
        // the packed tile, coalesced like the weight tile below (rows past M fall outside the descriptor: zeros)
        const int stepq = NT / wcpr, stepr = NT % wcpr;
        int rw = tid / wcpr, cl = tid % wcpr;
        uint32_t src = (uint32_t)(m0 + rw) * (uint32_t)a.lda + (uint32_t)cl * 16, dst = (uint32_t)(rw * pitch + cl * 16);
        const uint32_t src_q = (uint32_t)stepq * (uint32_t)a.lda + (uint32_t)stepr * 16, dst_q = (uint32_t)(stepq * pitch + stepr * 16);
        const uint32_t src_c = (uint32_t)a.lda - (uint32_t)wcpr * 16, dst_c = (uint32_t)(pitch - wcpr * 16);
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            arow_i[i] = rw; adst_i[i] = dst;
            if (i * NT < TM * wcpr) ast[i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, src, 0, 0);
            rw += stepq; cl += stepr; src += src_q; dst += dst_q;
            if (cl >= wcpr) { cl -= wcpr; ++rw; src += src_c; dst += dst_c; }
        }
    }
    // weights: the whole tile, coalesced (consecutive lanes walk a channel's row), on its way to LDS; when
    // it does not fit there, pass 2 fetches its operands itself (lane (c, h): 16 bytes of channel c)
    u32x4 wst[WCH];
    // chunk tid + i NT of the tile sits in row wrow_i, column wcol_i: one division, then carries
    int wrow_i[WCH];                                            // its row, or 32 FN and more past the tile
    uint32_t wdst_i[WCH];                                       // its byte offset in the LDS tile
    if constexpr (WLDS) {
        const int stepq = NT / wcpr, stepr = NT % wcpr;
        int rw = tid / wcpr, cl = tid % wcpr;
        uint32_t src = (uint32_t)(n0 + rw) * (uint32_t)a.ldw + (uint32_t)cl * 16, dst = (uint32_t)(rw * wpitch + cl * 16);
        const uint32_t src_q = (uint32_t)stepq * (uint32_t)a.ldw + (uint32_t)stepr * 16, dst_q = (uint32_t)(stepq * wpitch + stepr * 16);
        const uint32_t src_c = (uint32_t)a.ldw - (uint32_t)wcpr * 16, dst_c = (uint32_t)(wpitch - wcpr * 16);   // carry into the next row
#pragma unroll
        for (int i = 0; i < WCH; ++i) {
            wrow_i[i] = rw; wdst_i[i] = dst;
            if (i * NT < 32 * FN * wcpr) wst[i] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, src, 0, 0);
            rw += stepq; cl += stepr; src += src_q; dst += dst_q;
            if (cl >= wcpr) { cl -= wcpr; ++rw; src += src_c; dst += dst_c; }
        }
    }
    // channel constants of the accumulator registers this wave finishes (register qq of the tile belongs to
    // wave qq % NW), as raw bits: nothing here waits for a load
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(a.sw, (uint32_t)a.N * 4u);
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(a.bias, a.bias ? (uint32_t)a.N * 2u : 0u);   // no bias: reads zero
    uint32_t sw_raw[RPW];
    unsigned short b_raw[RPW];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const int qq = wave + k * NW, n = n0 + 32 * (qq / RV) + r;
        sw_raw[k] = __builtin_amdgcn_raw_buffer_load_b32(sw_rsrc, (uint32_t)n * 4u, 0, 0);
        b_raw[k] = __builtin_amdgcn_raw_buffer_load_b16(b_rsrc, (uint32_t)n * 2u, 0, 0);
    }
    for (int e = tid; e < R * 64; e += NT) s_sum[e] = 0;

    // ---- pass 1: ranges, codes into LDS ----------------------------------------------------------------------
    if constexpr (PACKED) {
        if (tid < TM) s_S[tid] = a.sa[min(m0 + tid, a.M - 1)];
#pragma unroll
        for (int i = 0; i < ACH; ++i)
            if (i * NT < TM * wcpr && arow_i[i] < TM) *reinterpret_cast<u32x4 *>(codes + adst_i[i]) = ast[i];
    } else {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        uint32_t zero = 0;
        h2 mx = *reinterpret_cast<const h2 *>(&zero);
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            if (i * LPR < nchunks && c0 + i * LPR < nchunks) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t d = x[i][k] & 0x7FFF7FFFu;
                    mx = __builtin_elementwise_max(mx, *reinterpret_cast<const h2 *>(&d));
                }
            }
        }
        float amax = fmaxf((float)mx[0], (float)mx[1]);
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, kWave));
        Range rg = range_sym(amax);
        if (W8) {                                                // Sec. 3.1 with b = 8: 127 levels per side
            if (amax == 0.0f) { rg.inv = 0.0f; rg.S = 1.0f; }
            else { rg.inv = 127.0f / amax; rg.S = amax / 127.0f; }
        }
        if (c0 == 0) s_S[row] = rg.S;
        uint8_t *dst = codes + row * pitch;
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int c = c0 + i * LPR;
            if (i * LPR < nchunks && c < nchunks) {
                uint32_t ev, od;
                codes8<W8>(x[i], rg.inv, ev, od);
                *reinterpret_cast<uint2 *>(dst + c * 8) = make_uint2(ev, od);
            }
        }
    }
    if constexpr (WLDS) {
#pragma unroll
        for (int i = 0; i < WCH; ++i) {
            if (i * NT < 32 * FN * wcpr && wrow_i[i] < 32 * FN) *reinterpret_cast<u32x4 *>(wt + wdst_i[i]) = wst[i];
        }
    }
    __syncthreads();

    // ---- pass 2: this wave's share of K (a rolled loop: the accumulators stay in place) ----------------------
    v16i acc[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[j][q] = 0;
    const uint8_t *arow = codes + (r % TM) * pitch + h * (NIBBLES ? 16 : 32);
    const uint8_t *wrow = wt + r * wpitch + h * (W8 ? 32 : 16);
#pragma unroll 1
    for (int b = wave; b < nb; b += NW) {
        v4i alo, ahi;
        if constexpr (NIBBLES) {
            const u32x4 ap = *reinterpret_cast<const u32x4 *>(arow + b * 32);
            alo = widen2<true>(ap[0], ap[1]);
            ahi = widen2<true>(ap[2], ap[3]);
        } else {
            alo = *reinterpret_cast<const v4i *>(arow + b * 64);
            ahi = *reinterpret_cast<const v4i *>(arow + b * 64 + 16);
        }
        if constexpr (W8) {
            // one-byte codes: lane (r, h) takes 32 bytes of channel r, two MFMA operands as they are
            v4i w0[FN], w1[FN];
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                if constexpr (WLDS) {
                    w0[j] = *reinterpret_cast<const v4i *>(wrow + 32 * j * wpitch + b * 64);
                    w1[j] = *reinterpret_cast<const v4i *>(wrow + 32 * j * wpitch + b * 64 + 16);
                } else {
                    const uint32_t off = (uint32_t)(n0 + 32 * j + r) * (uint32_t)a.ldw + (uint32_t)(b * 64 + h * 32);
                    const u32x4 t0 = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, off, 0, 0);
                    const u32x4 t1 = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, off + 16, 0, 0);
                    w0[j] = v4i{(int)t0[0], (int)t0[1], (int)t0[2], (int)t0[3]};
                    w1[j] = v4i{(int)t1[0], (int)t1[1], (int)t1[2], (int)t1[3]};
                }
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo, w0[j], acc[j], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi, w1[j], acc[j], 0, 0, 0);
        } else {
        u32x4 wv[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            if constexpr (WLDS) wv[j] = *reinterpret_cast<const u32x4 *>(wrow + 32 * j * wpitch + b * 32);
            else wv[j] = __builtin_amdgcn_raw_buffer_load_b128(
                     w_rsrc, (uint32_t)(n0 + 32 * j + r) * (uint32_t)a.ldw + (uint32_t)(b * 32 + h * 16), 0, 0);
        }
#pragma unroll
        for (int j = 0; j < FN; ++j)
            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo, widen2<true>(wv[j][0], wv[j][1]), acc[j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < FN; ++j)
            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi, widen2<true>(wv[j][2], wv[j][3]), acc[j], 0, 0, 0);
        }
    }

    // ---- add the partial sums of the waves in LDS (exact, so the order is free).  Accumulator register q of
    //      lane (c, h) is row 8 (q / 4) + 4 h + q % 4: with TM = 16 only registers 0 .. 7 hold real rows ----------
    if (wave < nb) {
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < RV; ++q) atomicAdd(&s_sum[(j * RV + q) * 64 + lane], acc[j][q]);
    }
    __syncthreads();
    const bool ints = PACKED && a.acc_out != nullptr;
    const __amdgpu_buffer_rsrc_t o_rsrc = ints ? make_rsrc(a.acc_out, (uint32_t)((long)a.M * a.N * 4))
                                               : make_rsrc(a.out, (uint32_t)((long)a.M * a.N * 2));
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const int qq = wave + k * NW;
        if (qq >= R) break;
        const int j = qq / RV, q = qq % RV;
        const int n = n0 + 32 * j + r;
        const bool n_ok = n < a.N;
        const int trow = frag_row(0, q, lane);
        if (ints) {                                              // parity export: P itself
            const uint32_t ioff = n_ok ? ((uint32_t)(m0 + trow) * (uint32_t)a.N + (uint32_t)n) * 4u : kPoison;
            __builtin_amdgcn_raw_buffer_store_b32((uint32_t)(W8 ? s_sum[qq * 64 + lane] : s_sum[qq * 64 + lane] >> 8), o_rsrc, ioff, 0, 0);
            continue;
        }
        // the sums hold 16 * P (256 * P if PACKED, P itself for the INT8 sibling); a power of two, so the rescaled
        // weight scale is exact
        const float swn = __uint_as_float(sw_raw[k]) * (W8 ? 1.0f : PACKED ? 0.00390625f : 0.0625f);
        float y = ((float)s_sum[qq * 64 + lane] * s_S[trow]) * swn;
        if (a.bias) y = y + __half2float(__ushort_as_half(b_raw[k]));
        const uint32_t off = n_ok ? ((uint32_t)(m0 + trow) * (uint32_t)a.N + (uint32_t)n) * 2u : kPoison;   // rows >= M fall off the end
        if (a.act == W4A4_ACT_GELU) __builtin_amdgcn_raw_buffer_store_b16(gelu_erf_half(y), o_rsrc, off, 0, 0);
        else __builtin_amdgcn_raw_buffer_store_b16(__half_as_ushort(__float2half_rn(y)), o_rsrc, off, 0, 0);
    }
}

template <int NW, int FN, int TM, bool WLDS, bool PACKED, bool W8 = false>
static int launch_small(SmallArgs &a, hipStream_t st) {
    a.tiles_n = (a.N + 32 * FN - 1) / (32 * FN);
    const long tiles = (long)((a.M + TM - 1) / TM) * a.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const size_t lds = TM * (size_t)((PACKED && !W8 ? a.K / 2 : a.K) + 16) + (WLDS ? 32 * FN * (size_t)((W8 ? a.K : a.K / 2) + 16) : 0) +
                       (size_t)(TM / 2) * FN * 64 * 4 + TM * 4;
    auto kern = linear_f16act_kernel<NW, FN, TM, WLDS, PACKED, W8>;
    static KernelState ks;
    if (prepare_kernel(reinterpret_cast<const void *>(kern), lds, ks) < 0) return W4A4_ERR_HIP;
    launch_gemm(kern, dim3((unsigned)tiles), dim3(NW * 64), lds, st, a);
    return launch_status();
}

// Shape policy.  Waves: enough that none walks more than four blocks of K nor holds more than 16 chunks of
// a row.  Tile: every column tile re-quantizes (or re-reads) its token rows, so fewer, wider tiles do less
// redundant work, but a tile is one CU's job: 32 x 32 while that gives at most one workgroup per CU, 32 x 64
// beyond, and 16-token tiles when 32-token tiles would leave more than half of the CUs idle.  The weight
// tile is staged in LDS (coalesced loads) whenever it fits beside the activation codes.
template <bool PACKED, bool W8 = false>
static int small_dispatch(SmallArgs &a, hipStream_t st) {
    const int M = a.M, N = a.N, K = a.K;
    const long t32 = (long)((M + 31) / 32) * ((N + 31) / 32);
    const bool wide = t32 > 256, low = t32 <= 128;
    const size_t code_b = (size_t)(low ? 16 : 32) * ((PACKED && !W8 ? K / 2 : K) + 16), wt_b = (size_t)(wide ? 64 : 32) * ((W8 ? K : K / 2) + 16);
    const int nw = K > 1536 ? 16 : K > 384 ? 8 : 4;
    const long wchunks = ((long)(wide ? 64 : 32) * (K / (W8 ? 16 : 32)) + nw * 64 - 1) / (nw * 64);   // per lane
    const bool wlds = code_b + wt_b <= 144 * 1024 && wchunks <= small_wchunks(nw);   // beside the sums, within a CU's 160 KB
#define W4A4_SMALL(NW)                                                                                  \
    do {                                                                                                \
        if (wide) return wlds ? launch_small<NW, 2, 32, true, PACKED, W8>(a, st) : launch_small<NW, 2, 32, false, PACKED, W8>(a, st); \
        if (low) return wlds ? launch_small<NW, 1, 16, true, PACKED, W8>(a, st) : launch_small<NW, 1, 16, false, PACKED, W8>(a, st);  \
        return wlds ? launch_small<NW, 1, 32, true, PACKED, W8>(a, st) : launch_small<NW, 1, 32, false, PACKED, W8>(a, st);     \
    } while (0)
    if (K > 1536) W4A4_SMALL(16);
    if (K > 384) W4A4_SMALL(8);
    W4A4_SMALL(4);
#undef W4A4_SMALL
}

// The same kernel on activations that are already quantized (canonical packed codes + token scales): the
// small-problem schedule of w4a4_linear / w4a4_gemm_i32.  Requires symmetric per-channel operands,
// K % 64 == 0, K <= 4096, lda % 16 == 0, 32-bit offsets.
int launch_small_packed(int out_kind, GemmArgs &g, hipStream_t st) {
    if (out_kind != OUT_F16 && out_kind != OUT_I32) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (g.K % 64 || g.K > 4096 || g.lda % 16 || (long)g.M * g.lda >= 0x7fffffffL || (long)g.N * g.ldw >= 0x7fffffffL ||
        ((long)g.M + 32) * g.N * 4 >= 0x7fffffffL)
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    SmallArgs a{};
    a.Aq = g.Aq; a.lda = g.lda; a.sa = g.sa;
    a.Wq = g.Wq; a.ldw = g.ldw; a.sw = g.sw;
    a.bias = g.bias; a.act = g.act;
    if (out_kind == OUT_I32) a.acc_out = static_cast<int32_t *>(g.out);
    else a.out = static_cast<__half *>(g.out);
    a.M = g.M; a.N = g.N; a.K = g.K;
    return small_dispatch<true>(a, st);
}

// The INT8 sibling's small-problem path on int8 codes that are already in memory (w8a8_linear / w8a8_gemm_i32
// for at most 512 tiles of 32 x 32).  g.lda / g.ldw are row strides in bytes = codes.
bool small8_ok(const GemmArgs &g) {
    return g.K % 64 == 0 && g.K <= 4096 && g.lda % 16 == 0 && (long)((g.M + 31) / 32) * ((g.N + 31) / 32) <= 512 &&
           (long)g.M * g.lda < 0x7fffffffL && (long)g.N * g.ldw < 0x7fffffffL && ((long)g.M + 32) * g.N * 4 < 0x7fffffffL;
}
int launch_small_packed8(int out_kind, GemmArgs &g, hipStream_t st) {
    if ((out_kind != OUT_F16 && out_kind != OUT_I32) || !small8_ok(g)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    SmallArgs a{};
    a.Aq = g.Aq; a.lda = g.lda; a.sa = g.sa;
    a.Wq = g.Wq; a.ldw = g.ldw; a.sw = g.sw;
    a.bias = g.bias; a.act = g.act;
    if (out_kind == OUT_I32) a.acc_out = static_cast<int32_t *>(g.out);
    else a.out = static_cast<__half *>(g.out);
    a.M = g.M; a.N = g.N; a.K = g.K;
    return small_dispatch<true, true>(a, st);
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_linear_f16act(const void *X_f16, int M, int K, int ldx, const w4a4_weight *W,
                                  const w4a4_epilogue *ep, void *out, void *stream) {
    if (!W || !ep || M < 0 || K <= 0 || ldx < K || W->N <= 0 || W->K != K) return W4A4_ERR_INVALID_ARG;
    if (ep->act != W4A4_ACT_NONE && ep->act != W4A4_ACT_GELU) return W4A4_ERR_INVALID_ARG;
    if (W->mode != W4A4_SYM && W->mode != W4A4_ASYM) return W4A4_ERR_INVALID_ARG;
    if (W->mode != W4A4_SYM || W->layout != W4A4_LAYOUT_CANONICAL || (W->group != 0 && W->group != K) || ep->requant)
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (K % 64 || K > 4096 || W->N % 8 || (ldx * 2) % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;   // 16 waves x 4 blocks
    if (M == 0) return W4A4_OK;
    if (!X_f16 || !W->q || !W->scale || !out) return W4A4_ERR_INVALID_ARG;
    if (!aligned16(X_f16) || !aligned16(W->q) || !aligned16(out)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if ((long)M * ldx * 2 >= 0x7fffffffL || (long)W->N * (K / 2) >= 0x7fffffffL || ((long)M + 32) * W->N * 2 >= 0x7fffffffL)
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    SmallArgs a{};
    a.X = static_cast<const __half *>(X_f16); a.ldx = ldx;
    a.Wq = W->q; a.ldw = K / 2; a.sw = W->scale;
    a.bias = static_cast<const __half *>(ep->bias_f16); a.act = ep->act;
    a.out = static_cast<__half *>(out);
    a.M = M; a.N = W->N; a.K = K; a.tiles_n = 0;
    return small_dispatch<false>(a, as_stream(stream));
}

extern "C" int w8a8_linear_f16act(const void *X_f16, int M, int K, int ldx, const int8_t *Wq, const float *sw, int N,
                                  const w4a4_epilogue *ep, void *out, void *stream) {
    if (!ep || M < 0 || K <= 0 || ldx < K || N <= 0) return W4A4_ERR_INVALID_ARG;
    if (ep->act != W4A4_ACT_NONE && ep->act != W4A4_ACT_GELU) return W4A4_ERR_INVALID_ARG;
    if (ep->requant) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (K % 64 || K > 4096 || N % 8 || (ldx * 2) % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return W4A4_OK;
    if (!X_f16 || !Wq || !sw || !out) return W4A4_ERR_INVALID_ARG;
    if (!aligned16(X_f16) || !aligned16(Wq) || !aligned16(out) || (ep->bias_f16 && !aligned16(ep->bias_f16)))
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    if ((long)M * ldx * 2 >= 0x7fffffffL || (long)N * K >= 0x7fffffffL || ((long)M + 32) * N * 2 >= 0x7fffffffL)
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    SmallArgs a{};
    a.X = static_cast<const __half *>(X_f16); a.ldx = ldx;
    a.Wq = reinterpret_cast<const uint8_t *>(Wq); a.ldw = K; a.sw = sw;
    a.bias = static_cast<const __half *>(ep->bias_f16); a.act = ep->act;
    a.out = static_cast<__half *>(out);
    a.M = M; a.N = N; a.K = K; a.tiles_n = 0;
    return small_dispatch<false, true>(a, as_stream(stream));
}
