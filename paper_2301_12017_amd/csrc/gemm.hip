// INT4 x INT4 -> INT32 GEMM with the fused dequantize epilogue (steps a2 + a3).
//
// Design for gfx950 (no INT4 matrix instruction exists, the int8 MFMA is the target):
//   * Both operands stay PACKED (two codes per byte) in HBM, through the 16-byte
//     global loads and in LDS; they are widened to int8 only in registers, right
//     before v_mfma_i32_32x32x32_i8.  LDS traffic and footprint are half of an int8
//     GEMM's.
//   * Widening a packed dword d (codes k0..k7) uses the nibble's position instead of a
//     sign extension:  (d << 4) & 0xF0F0F0F0  holds 16*k0,16*k2,16*k4,16*k6 as int8 and
//     d & 0xF0F0F0F0  holds 16*k1,16*k3,16*k5,16*k7.  Both operands are widened the
//     same way, so the MFMA accumulates 256 * sum(qa*qw) exactly (|acc| <= 2^26 at
//     K = 4096) and an arithmetic shift by 8 recovers the integer dot product.  The
//     k order inside one MFMA is permuted identically for both operands, which leaves
//     the sum unchanged.  Unsigned codes use the 0x0F0F0F0F masks and no scaling.
//   * A workgroup owns a BM x BN output tile, K is walked in steps of 128 codes
//     (64 bytes per row) through two LDS stages: the global loads of step t+1 are in
//     flight while step t is multiplied.  LDS rows are padded to 80 bytes so the
//     16-byte operand reads of 16 consecutive rows fall in distinct banks.
//   * The activation tile supplies the MFMA rows and the weight tile the MFMA columns.
//     Weight rows are placed in LDS so that MFMA column c of fragment f is output
//     channel c*FN + f of the wave's span: a lane then holds FN consecutive output
//     channels of one token and stores them with one vector store, 32 lanes covering
//     a contiguous run of the output row.
//   * Weights with K-groups (and the asymmetric mapping) rescale the int32 partial
//     sums into fp32 accumulators at every group boundary; the zero-point terms of
//     the asymmetric mapping are added in the epilogue.
//   * Workgroup ids are remapped so that each of the 8 XCDs (one L2 each) works on a
//     contiguous range of tiles that share activation row panels.
#include "common.hpp"

namespace w4a4 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 128;           // codes per K step
constexpr int kRowB = 80;          // LDS row pitch in bytes: 64 of codes + 16 of padding
constexpr int kXcd = 8;

enum { OUT_F16 = 0, OUT_F32 = 1, OUT_I32 = 2 };

struct GemmArgs {
    const uint8_t *Aq; long lda;
    const uint8_t *Wq; long ldw;
    int M, N, K;
    int ng, steps_per_group;       // K-groups of the weights, K steps per group
    const float *sa, *za; const int32_t *RA;
    const float *sw, *zw, *c;
    const __half *bias; int act;
    void *out;                     // fp16 [M,N] | fp32 [M,N] | int32 [ng,M,N]
    int tiles_m, tiles_n;
};

template <bool SIGNED_>
__device__ __forceinline__ void widen(const uint4 &p, v4i &lo, v4i &hi) {
    if (SIGNED_) {
        constexpr uint32_t m = 0xF0F0F0F0u;
        lo = v4i{(int)((p.x << 4) & m), (int)(p.x & m), (int)((p.y << 4) & m), (int)(p.y & m)};
        hi = v4i{(int)((p.z << 4) & m), (int)(p.z & m), (int)((p.w << 4) & m), (int)(p.w & m)};
    } else {
        constexpr uint32_t m = 0x0F0F0F0Fu;
        lo = v4i{(int)(p.x & m), (int)((p.x >> 4) & m), (int)(p.y & m), (int)((p.y >> 4) & m)};
        hi = v4i{(int)(p.z & m), (int)((p.z >> 4) & m), (int)(p.w & m), (int)((p.w >> 4) & m)};
    }
}

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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- tile of this workgroup: XCD x gets a contiguous range of tiles -------------
    const int total = g.tiles_m * g.tiles_n;
    int tile;
    {
        const int bid = blockIdx.x, x = bid % kXcd, i = bid / kXcd;
        const int per = total / kXcd, rem = total % kXcd;
        tile = x * per + (x < rem ? x : rem) + i;
    }
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
    auto m_of = [&](int i, int r) { return m0 + wm * FM * 32 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); };

    // Rescale at a group boundary:  t1 += sw[n,g] * (float)P_g   (one mul, one add).
    auto fold_group = [&](int grp) {
        float swg[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) swg[j] = n_ok ? g.sw[(long)(n_lane + j) * g.ng + grp] : 0.0f;
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
    if (!n_ok) return;
    if (GROUPED && OUT == OUT_I32) return;                       // planes were stored group by group
    float swv[FN], bv[FN], cv[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        swv[j] = (!GROUPED && OUT != OUT_I32) ? g.sw[n_lane + j] : 0.0f;
        bv[j] = (OUT != OUT_I32 && g.bias) ? __half2float(g.bias[n_lane + j]) : 0.0f;
        cv[j] = (MODE == W4A4_ASYM && OUT != OUT_I32) ? g.c[n_lane + j] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m_of(i, r);
            if (m >= g.M) continue;
            if (OUT == OUT_I32) {
                int32_t *o = static_cast<int32_t *>(g.out) + (long)m * g.N + n_lane;
#pragma unroll
                for (int j = 0; j < FN; ++j) o[j] = SGN ? (acc[i][j][r] >> 8) : acc[i][j][r];
                continue;
            }
            const float sam = g.sa[m];
            float y[FN];
            if (!GROUPED) {
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    float t = (float)(acc[i][j][r] >> 8) * sam;
                    y[j] = t * swv[j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < FN; ++j) y[j] = sam * facc[GROUPED ? i : 0][GROUPED ? j : 0][r];
                if (MODE == W4A4_ASYM) {
                    // t2 = sum_g zw[n,g] * (float)RA[m,g];  y += sa*t2;  y += za*c[n]
                    float t2[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) t2[j] = 0.0f;
                    for (int grp = 0; grp < g.ng; ++grp) {
                        const float ra_f = (float)g.RA[(long)m * g.ng + grp];
#pragma unroll
                        for (int j = 0; j < FN; ++j) {
                            float w = g.zw[(long)(n_lane + j) * g.ng + grp] * ra_f;
                            t2[j] = t2[j] + w;
                        }
                    }
                    const float zam = g.za[m];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        float p = sam * t2[j];
                        float q = zam * cv[j];
                        y[j] = y[j] + p;
                        y[j] = y[j] + q;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                if (g.bias) y[j] = y[j] + bv[j];
                if (g.act == W4A4_ACT_GELU) y[j] = gelu_erf(y[j]);
            }
            if (OUT == OUT_F32) {
                float *o = static_cast<float *>(g.out) + (long)m * g.N + n_lane;
#pragma unroll
                for (int j = 0; j < FN; ++j) o[j] = y[j];
            } else {
                __half *o = static_cast<__half *>(g.out) + (long)m * g.N + n_lane;
                if (FN == 1) {
                    o[0] = __float2half_rn(y[0]);
                } else {
                    __half2 h[FN / 2 > 0 ? FN / 2 : 1];
#pragma unroll
                    for (int j = 0; j < FN / 2; ++j) h[j] = __floats2half2_rn(y[2 * j], y[2 * j + 1]);
                    if (FN == 2) *reinterpret_cast<uint32_t *>(o) = *reinterpret_cast<uint32_t *>(h);
                    else if (FN == 4) *reinterpret_cast<uint2 *>(o) = *reinterpret_cast<uint2 *>(h);
                    else *reinterpret_cast<uint4 *>(o) = *reinterpret_cast<uint4 *>(h);
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Schedules (Sec. 4.2: the GEMM schedule is chosen per shape ahead of time).
struct Schedule {
    const char *name;
    int BM, BN, threads;
    bool grouped_ok;     // also built for the grouped / asymmetric path
};
// index = schedule number - 1
static const Schedule kSchedules[] = {
    {"256x256_8w", 256, 256, 512, false},
    {"256x256_4w", 256, 256, 256, false},
    {"128x256_4w", 128, 256, 256, true},
    {"192x256_4w", 192, 256, 256, false},
    {"64x128_4w", 64, 128, 256, true},
    {"64x64_4w", 64, 64, 256, true},
    {"32x32_1w", 32, 32, 64, true},
};
constexpr int kNumSchedules = sizeof(kSchedules) / sizeof(kSchedules[0]);

template <int FM, int FN, int WM, int WN, int MODE, bool GROUPED, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = 2 * (size_t)(BM + BN) * kRowB;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_kernel<FM, FN, WM, WN, MODE, GROUPED, OUT>;
    static bool attr_set = false;          // benign race: the attribute call is idempotent
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return W4A4_ERR_HIP;
        attr_set = true;
    }
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(WM * WN * 64), lds, st, g);
    return launch_status();
}

template <int MODE, bool GROUPED, int OUT>
static int launch_schedule(int schedule, GemmArgs &g, hipStream_t st) {
    switch (schedule) {
        case 3: return launch_one<2, 4, 2, 2, MODE, GROUPED, OUT>(g, st);
        case 5: return launch_one<1, 2, 2, 2, MODE, GROUPED, OUT>(g, st);
        case 6: return launch_one<1, 1, 2, 2, MODE, GROUPED, OUT>(g, st);
        case 7: return launch_one<1, 1, 1, 1, MODE, GROUPED, OUT>(g, st);
        default: break;
    }
    if constexpr (!GROUPED) {
        switch (schedule) {
            case 1: return launch_one<2, 4, 4, 2, MODE, false, OUT>(g, st);
            case 2: return launch_one<4, 4, 2, 2, MODE, false, OUT>(g, st);
            case 4: return launch_one<3, 4, 2, 2, MODE, false, OUT>(g, st);
            default: break;
        }
    }
    return W4A4_ERR_INVALID_ARG;
}

// Built-in shape table: large problems take the big tiles, small ones the tiles that
// still give every CU something to do.
static int pick_schedule(int M, int N, bool grouped) {
    const long big = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (big >= 128) return grouped ? 3 : 1;
    const long mid = (long)((M + 63) / 64) * ((N + 127) / 128);
    if (mid >= 256) return 5;
    const long small = (long)((M + 63) / 64) * ((N + 63) / 64);
    if (small >= 256) return 6;
    return 7;
}

static int run_gemm(GemmArgs &g, int mode, bool grouped, int out_kind, int schedule, hipStream_t st) {
    if (schedule == 0) schedule = pick_schedule(g.M, g.N, grouped);
    if (schedule < 1 || schedule > kNumSchedules) return W4A4_ERR_INVALID_ARG;
    if (grouped && !kSchedules[schedule - 1].grouped_ok) return W4A4_ERR_INVALID_ARG;
#define W4A4_GO(MODE, GR)                                                         \
    switch (out_kind) {                                                           \
        case OUT_F16: return launch_schedule<MODE, GR, OUT_F16>(schedule, g, st); \
        case OUT_F32: return launch_schedule<MODE, GR, OUT_F32>(schedule, g, st); \
        default: return launch_schedule<MODE, GR, OUT_I32>(schedule, g, st);      \
    }
    if (mode == W4A4_SYM) {
        if (grouped) { W4A4_GO(W4A4_SYM, true) } else { W4A4_GO(W4A4_SYM, false) }
    } else {
        W4A4_GO(W4A4_ASYM, true)
    }
#undef W4A4_GO
}

// ---------------------------------------------------------------------------------------------
// Argument validation shared by w4a4_linear, w4a4_gemm_i32 and w4a4_dequant_epilogue.
static int check_operands(const w4a4_act *A, const w4a4_weight *W, int *ng_out) {
    if (!A || !W) return W4A4_ERR_INVALID_ARG;
    if (A->M < 0 || A->K <= 0 || W->N <= 0 || W->K != A->K) return W4A4_ERR_INVALID_ARG;
    if (A->mode != W->mode || (A->mode != W4A4_SYM && A->mode != W4A4_ASYM)) return W4A4_ERR_INVALID_ARG;
    if (W->group < 0 || A->group < 0) return W4A4_ERR_INVALID_ARG;
    const int K = A->K;
    if (K % 32 || W->N % 8) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int G = W->group == 0 ? K : W->group;
    if (K % G || (W->group != 0 && G % kBK)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int ng = K / G;
    if (A->lda < K / 2) return W4A4_ERR_INVALID_ARG;
    if (A->lda % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (A->M > 0) {
        if (!A->q || !A->scale || !W->q || !W->scale) return W4A4_ERR_INVALID_ARG;
        if (A->mode == W4A4_ASYM) {
            if (!A->zero || !A->gsum || !W->zero || !W->rowsum_deq) return W4A4_ERR_INVALID_ARG;
            const int GA = A->group == 0 ? K : A->group;
            if (GA != G) return W4A4_ERR_INVALID_ARG;          // code sums must match the weight groups
        }
        if (!aligned16(A->q) || !aligned16(W->q)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    *ng_out = ng;
    return W4A4_OK;
}

int check_layer(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, const void *out,
                const float *out_scale, const float *out_zero, int *ng, int *rng) {
    int rc = check_operands(A, W, ng);
    if (rc) return rc;
    if (!ep) return W4A4_ERR_INVALID_ARG;
    if (ep->act != W4A4_ACT_NONE && ep->act != W4A4_ACT_GELU) return W4A4_ERR_INVALID_ARG;
    *rng = 1;
    if (ep->requant) {
        if (ep->requant_mode != W4A4_SYM && ep->requant_mode != W4A4_ASYM) return W4A4_ERR_INVALID_ARG;
        if (ep->requant_group < 0) return W4A4_ERR_INVALID_ARG;
        const int N = W->N;
        if (N % 32 || N > 8192) return W4A4_ERR_UNSUPPORTED_SHAPE;
        const int rG = ep->requant_group == 0 ? N : ep->requant_group;
        if (rG % 32 || N % rG || N / rG > 512) return W4A4_ERR_UNSUPPORTED_SHAPE;
        *rng = N / rG;
        if (A->M > 0 && (!out_scale || (ep->requant_mode == W4A4_ASYM && !out_zero))) return W4A4_ERR_INVALID_ARG;
    }
    if (A->M > 0) {
        if (!out) return W4A4_ERR_INVALID_ARG;
        if (!aligned16(out) || (ep->bias_f16 && !aligned16(ep->bias_f16))) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    return W4A4_OK;
}

int quantize_rows_f32(const float *Y, int rows, int K, long ld, int mode, int group, uint8_t *q,
                      float *s, float *z, int32_t *gsum, hipStream_t st);

static void fill_args(GemmArgs &g, const w4a4_act *A, const w4a4_weight *W, int ng) {
    g.Aq = A->q; g.lda = A->lda; g.Wq = W->q; g.ldw = W->K / 2;
    g.M = A->M; g.N = W->N; g.K = A->K;
    g.ng = ng; g.steps_per_group = (A->K / ng + kBK - 1) / kBK;
    g.sa = A->scale; g.za = A->zero; g.RA = A->gsum;
    g.sw = W->scale; g.zw = W->zero; g.c = W->rowsum_deq;
    g.bias = nullptr; g.act = W4A4_ACT_NONE; g.out = nullptr;
    g.tiles_m = g.tiles_n = 0;
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_schedule_count(void) { return kNumSchedules; }

extern "C" const char *w4a4_schedule_name(int schedule) {
    return (schedule >= 1 && schedule <= kNumSchedules) ? kSchedules[schedule - 1].name : "";
}

extern "C" size_t w4a4_workspace_bytes(int M, int N, int K, const w4a4_epilogue *ep) {
    (void)K;
    if (!ep || !ep->requant || M <= 0 || N <= 0) return 0;
    return (size_t)M * (size_t)N * sizeof(float);          // fp32 rows awaiting their per-token range
}

extern "C" int w4a4_gemm_i32(const w4a4_act *A, const w4a4_weight *W, int32_t *acc, int schedule, void *stream) {
    int ng = 0;
    int rc = check_operands(A, W, &ng);
    if (rc) return rc;
    if (A->M == 0) return W4A4_OK;
    if (!acc) return W4A4_ERR_INVALID_ARG;
    if (!aligned16(acc)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    GemmArgs g;
    fill_args(g, A, W, ng);
    g.out = acc;
    const bool grouped = A->mode == W4A4_ASYM || ng > 1;
    return run_gemm(g, A->mode, grouped, OUT_I32, schedule, as_stream(stream));
}

extern "C" int w4a4_linear(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, void *out,
                           float *out_scale, float *out_zero, int32_t *out_gsum, void *workspace,
                           size_t workspace_bytes, void *stream) {
    int ng = 0, rng = 0;
    int rc = check_layer(A, W, ep, out, out_scale, out_zero, &ng, &rng);
    if (rc) return rc;
    if (A->M == 0) return W4A4_OK;
    const size_t need = w4a4_workspace_bytes(A->M, W->N, A->K, ep);
    if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) return W4A4_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    GemmArgs g;
    fill_args(g, A, W, ng);
    g.bias = static_cast<const __half *>(ep->bias_f16);
    g.act = ep->act;
    const bool grouped = A->mode == W4A4_ASYM || ng > 1;
    if (!ep->requant) {
        g.out = out;
        return run_gemm(g, A->mode, grouped, OUT_F16, ep->schedule, st);
    }
    // Requantize: the per-token range needs the whole output row, which no single tile
    // sees.  The GEMM leaves the fp32 rows in the workspace and the row quantizer turns
    // them into packed codes.
    g.out = workspace;
    rc = run_gemm(g, A->mode, grouped, OUT_F32, ep->schedule, st);
    if (rc) return rc;
    return quantize_rows_f32(static_cast<const float *>(workspace), A->M, W->N, W->N, ep->requant_mode,
                             ep->requant_group, static_cast<uint8_t *>(out), out_scale, out_zero, out_gsum, st);
}
