// Generic INT4 x INT4 -> INT32 GEMM kernel with the fused epilogue: any M, any N % 8 == 0,
// any K % 32 == 0, symmetric or asymmetric codes, weights with or without K-groups.
// It is the fallback of the pipelined kernel (gemm_pipe.hip) and the kernel for grouped /
// asymmetric layers and small problems.
//
//   * Both operands stay packed (two codes per byte) through the 16-byte global loads and
//     in LDS; they are widened to int8 in registers right before v_mfma_i32_32x32x32_i8.
//   * A workgroup owns a BM x BN tile; K is walked in steps of 128 codes (64 bytes per row)
//     through two LDS stages, the global loads of step t+1 in flight during step t.  LDS
//     rows are padded to 80 bytes so 16-byte reads of consecutive rows hit distinct banks.
//   * The activation tile supplies the MFMA rows, the weight tile the MFMA columns.  Weight
//     rows are placed in LDS so that MFMA column c of fragment f is output channel c*FN + f
//     of the wave's span: a lane ends up with FN consecutive channels of one token.
//   * With K-groups (always for the asymmetric mapping) the int32 partial sums are folded
//     into fp32 accumulators at every group boundary: t1 += sw[n,g] * (float)P_g.
#include "gemm_common.hpp"

namespace w4a4 {

// FM x FN MFMA fragments (32x32 each) per wave, WM x WN waves per workgroup.
// MODE: w4a4_mode of the operands.  GROUPED: weights carry K-groups (fp32 accumulation
// across groups) -- always true for ASYM.  OUT: what is stored.
template <int FM, int FN, int WM, int WN, int MODE, bool GROUPED, int OUT>
__global__ __launch_bounds__(WM *WN * 64) void gemm_kernel(GemmArgs g) {
    constexpr bool SGN = MODE == W4A4_SYM;
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
    constexpr int A_STAGE = BM * kRowB, B_STAGE = BN * kRowB;
    constexpr int A_CH = BM * 4, B_CH = BN * 4;                 // 16-byte chunks per K step
    constexpr int A_PT = (A_CH + NT - 1) / NT, B_PT = (B_CH + NT - 1) / NT;
    static_assert(GROUPED || MODE == W4A4_SYM, "the asymmetric mapping uses the grouped path");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint8_t *As = smem;
    uint8_t *Bs = smem + 2 * A_STAGE;
    float *sa_lds = reinterpret_cast<float *>(smem + 2 * A_STAGE + 2 * B_STAGE);   // token scales
    float *za_lds = sa_lds + BM;                                                   // token zero points
    // K-group parameters of the tile, staged once: sw_lds[g][n], zw_lds[g][n], ra_lds[g][m]
    float *sw_lds = za_lds + BM;
    float *zw_lds = sw_lds + (GROUPED ? g.ng * BN : 0);
    float *ra_lds = zw_lds + (MODE == W4A4_ASYM ? g.ng * BN : 0);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- tile of this workgroup: XCD x gets a contiguous range of tiles -------------
    const int tile = xcd_tile(blockIdx.x, g.tiles_m * g.tiles_n);
    const int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    const int Kb = g.K / 2;                                     // packed bytes per row

    // ---- per-thread global->LDS plan ------------------------------------------------
    const uint8_t *a_src[A_PT], *b_src[B_PT];
    int a_dst[A_PT], b_dst[B_PT];
    bool a_ok[A_PT], b_ok[B_PT];
    int a_kb[A_PT], b_kb[B_PT];
#pragma unroll
    for (int i = 0; i < A_PT; ++i) {
        const int ch = tid + i * NT, row = ch >> 2, kc = ch & 3;
        a_ok[i] = ch < A_CH && (m0 + row) < g.M;
        a_kb[i] = kc * 16;
        a_src[i] = g.Aq + (long)(m0 + row) * g.lda + kc * 16;
        a_dst[i] = ch < A_CH ? row * kRowB + kc * 16 : -1;
    }
#pragma unroll
    for (int i = 0; i < B_PT; ++i) {
        const int ch = tid + i * NT, p = ch >> 2, kc = ch & 3;
        // LDS row p of the weight tile holds output channel nl (see header comment)
        const int w = p / (FN * 32), rem = p % (FN * 32), f = rem / 32, c = rem % 32;
        const int nl = w * (FN * 32) + c * FN + f;
        b_ok[i] = ch < B_CH && (n0 + nl) < g.N;
        b_kb[i] = kc * 16;
        b_src[i] = g.Wq + (long)(n0 + nl) * g.ldw + kc * 16;
        b_dst[i] = ch < B_CH ? p * kRowB + kc * 16 : -1;
    }
    uint4 ra[A_PT], rb[B_PT];
    auto gload = [&](int kt) {
        const int kb = kt * (kBK / 2);
#pragma unroll
        for (int i = 0; i < A_PT; ++i) {
            ra[i] = make_uint4(0, 0, 0, 0);
            if (a_ok[i] && kb + a_kb[i] < Kb) ra[i] = *reinterpret_cast<const uint4 *>(a_src[i] + kb);
        }
#pragma unroll
        for (int i = 0; i < B_PT; ++i) {
            rb[i] = make_uint4(0, 0, 0, 0);
            if (b_ok[i] && kb + b_kb[i] < Kb) rb[i] = *reinterpret_cast<const uint4 *>(b_src[i] + kb);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PT; ++i)
            if (a_dst[i] >= 0) *reinterpret_cast<uint4 *>(As + buf * A_STAGE + a_dst[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_PT; ++i)
            if (b_dst[i] >= 0) *reinterpret_cast<uint4 *>(Bs + buf * B_STAGE + b_dst[i]) = rb[i];
    };

    // ---- accumulators -----------------------------------------------------------------
    v16i acc[FM][FN];
    float facc[GROUPED ? FM : 1][GROUPED ? FN : 1][16];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
            if constexpr (GROUPED) {
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[i][j][r] = 0.0f;
            }
        }

    const int a_rd = (wm * FM * 32 + (lane & 31)) * kRowB + (lane >> 5) * 16;
    const int b_rd = (wn * FN * 32 + (lane & 31)) * kRowB + (lane >> 5) * 16;
    auto compute = [&](int buf) {
        const uint8_t *ab = As + buf * A_STAGE + a_rd;
        const uint8_t *bb = Bs + buf * B_STAGE + b_rd;
#pragma unroll
        for (int ks = 0; ks < kBK / 64; ++ks) {
            v4i a0[FM], a1[FM], b0[FN], b1[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                widen<SGN>(*reinterpret_cast<const uint4 *>(ab + i * 32 * kRowB + ks * 32), a0[i], a1[i]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                widen<SGN>(*reinterpret_cast<const uint4 *>(bb + j * 32 * kRowB + ks * 32), b0[j], b1[j]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
        }
    };

    // output coordinates of this lane
    const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;     // FN consecutive channels from here
    const bool n_ok = n_lane < g.N;
    const int n_local = wn * FN * 32 + (lane & 31) * FN;
    auto m_of = [&](int i, int r) { return m0 + wm * FM * 32 + frag_row(i, r, lane); };

    // Rescale at a group boundary:  t1 += sw[n,g] * (float)P_g   (one mul, one add).
    auto fold_group = [&](int grp) {
        float swg[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) swg[j] = sw_lds[grp * BN + n_local + j];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int P = SGN ? (acc[i][j][r] >> 8) : acc[i][j][r];
                    if (OUT == OUT_I32) {
                        const int m = m_of(i, r);
                        if (n_ok && m < g.M)
                            static_cast<int32_t *>(g.out)[((long)grp * g.M + m) * g.N + n_lane + j] = P;
                    } else {
                        float u = swg[j] * (float)P;
                        facc[GROUPED ? i : 0][GROUPED ? j : 0][r] = facc[GROUPED ? i : 0][GROUPED ? j : 0][r] + u;
                    }
                    acc[i][j][r] = 0;
                }
    };

    // ---- main loop ----------------------------------------------------------------------
    const int KT = (g.K + kBK - 1) / kBK;
    const EpiLane<FN> epi = epilogue_prefetch<FN, MODE, GROUPED, OUT>(g, n_lane);
    stage_token_params<BM, NT, MODE>(g, m0, sa_lds, za_lds, tid);     // visible after the first barrier
    if constexpr (GROUPED) {
        for (int e = tid; e < BN * g.ng; e += NT) {                   // global [N][ng] -> LDS [ng][BN]
            const int nl = e / g.ng, grp = e % g.ng, n = n0 + nl;
            sw_lds[grp * BN + nl] = n < g.N ? g.sw[(long)n * g.ng + grp] : 0.0f;
            if (MODE == W4A4_ASYM) zw_lds[grp * BN + nl] = n < g.N ? g.zw[(long)n * g.ng + grp] : 0.0f;
        }
        if (MODE == W4A4_ASYM) {
            for (int e = tid; e < BM * g.ng; e += NT) {
                const int ml = e / g.ng, grp = e % g.ng, m = m0 + ml;
                ra_lds[grp * BM + ml] = m < g.M ? (float)g.RA[(long)m * g.ng + grp] : 0.0f;
            }
        }
    }
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) gload(kt + 1);
        compute(buf);
        if (GROUPED && (kt + 1) % g.steps_per_group == 0) fold_group(kt / g.steps_per_group);
        if (kt + 1 < KT) lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------
    tile_epilogue<FM, FN, MODE, GROUPED, OUT>(g, acc, facc, epi, m0, wm * FM * 32, lane, sa_lds, za_lds, zw_lds, ra_lds,
                                              n_local, BM, BN);
}

template <int FM, int FN, int WM, int WN, int MODE, bool GROUPED, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    size_t lds = 2 * (size_t)(BM + BN) * kRowB + 2 * BM * sizeof(float);
    if (GROUPED) lds += (size_t)g.ng * (BN * (MODE == W4A4_ASYM ? 2 : 1) + (MODE == W4A4_ASYM ? BM : 0)) * sizeof(float);
    if (lds > 160 * 1024) return W4A4_ERR_UNSUPPORTED_SHAPE;      // K-group tables do not fit next to this tile
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_kernel<FM, FN, WM, WN, MODE, GROUPED, OUT>;
    static KernelState ks;
    if (prepare_kernel(reinterpret_cast<const void *>(kern), lds, ks) < 0) return W4A4_ERR_HIP;
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    launch_gemm(kern, dim3((unsigned)tiles), dim3(WM * WN * 64), lds, st, g);
    return launch_status();
}

// variant: 0 = 64x128, 1 = 64x64, 2 = 32x32
template <int MODE, bool GROUPED, int OUT>
static int launch_variant(int variant, GemmArgs &g, hipStream_t st) {
    switch (variant) {
        case 0: return launch_one<1, 2, 2, 2, MODE, GROUPED, OUT>(g, st);
        case 1: return launch_one<1, 1, 2, 2, MODE, GROUPED, OUT>(g, st);
        case 2: return launch_one<1, 1, 1, 1, MODE, GROUPED, OUT>(g, st);
        default: return W4A4_ERR_INVALID_ARG;
    }
}

int launch_generic(int variant, int mode, bool grouped, int out_kind, GemmArgs &g, hipStream_t st) {
#define W4A4_GO(MODE, GR)                                                        \
    switch (out_kind) {                                                          \
        case OUT_F16: return launch_variant<MODE, GR, OUT_F16>(variant, g, st);  \
        case OUT_F32: return launch_variant<MODE, GR, OUT_F32>(variant, g, st);  \
        default: return launch_variant<MODE, GR, OUT_I32>(variant, g, st);       \
    }
    if (mode == W4A4_SYM) {
        if (grouped) { W4A4_GO(W4A4_SYM, true) } else { W4A4_GO(W4A4_SYM, false) }
    } else {
        W4A4_GO(W4A4_ASYM, true)
    }
#undef W4A4_GO
}

}  // namespace w4a4
