// Dispatch and C entry points of the GEMM side of libw4a4: schedule table, argument
// validation, w4a4_linear / w4a4_gemm_i32 / w4a4_workspace_bytes.
#include "gemm_common.hpp"

namespace w4a4 {

// Schedules (Sec. 4.2: the GEMM schedule is chosen per shape ahead of time).  A schedule
// names a kernel family and a tile variant of it.  Every schedule is picked by the built-in
// shape tables below for some shape; forcing one (w4a4_epilogue.schedule) is for measurements
// and parity tests.
enum Family {
    F_PIPE,      // pipelined kernel on canonical codes (symmetric, per-channel, K % 128 == 0): many tokens whose
                 // operands were left in the canonical layout
    F_GENERIC,   // any mode / grouping / K % 32: small and odd shapes
    F_OLAY,      // persistent kernel on operands in the MFMA operand layout
    F_GROUP,     // persistent kernel for K-grouped / asymmetric layers
    F_SMALL,     // small-problem kernel: the waves of a workgroup split K (symmetric per-channel, K % 64 == 0)
    F_FP6        // persistent kernel on operands in the FP6 operand layout (FP6 matrix pipe, exact integer results)
};
struct Schedule {
    const char *name;
    int family;
    int variant;
    bool grouped_ok;     // usable for K-grouped / asymmetric layers
};
// index = schedule number - 1
static const Schedule kSchedules[] = {
    {"pipe_128x256", F_PIPE, 0, false},
    {"pipe_192x128", F_PIPE, 1, false},
    {"generic_64x128", F_GENERIC, 0, true},
    {"generic_64x64", F_GENERIC, 1, true},
    {"generic_32x32", F_GENERIC, 2, true},
    {"olay_128x256", F_OLAY, 0, false},
    {"olay_192x128", F_OLAY, 1, false},
    {"olay_128x128", F_OLAY, 2, false},
    {"group_128x128", F_GROUP, 0, true},
    {"small_splitk", F_SMALL, 0, false},
    {"fp6_128x256", F_FP6, 0, false},
    {"fp6_192x128", F_FP6, 1, false},
    {"fp6_128x128", F_FP6, 2, false},
    {"fp6_192x256", F_FP6, 3, false},
};
constexpr int kNumSchedules = sizeof(kSchedules) / sizeof(kSchedules[0]);
enum { S_PIPE_128x256 = 1, S_PIPE_192x128, S_GEN_64x128, S_GEN_64x64, S_GEN_32x32, S_OLAY_128x256, S_OLAY_192x128,
       S_OLAY_128x128, S_GROUP, S_SMALL, S_FP6_128x256, S_FP6_192x128, S_FP6_128x128, S_FP6_192x256 };

static bool pipe_ok(const GemmArgs &g, bool grouped, int kstep = kBK) {
    // 32-bit buffer offsets and whole K steps
    return !grouped && g.K % kstep == 0 && (long)g.M * g.lda < 0x7fffffffL && (long)g.N * g.ldw < 0x7fffffffL;
}

// The small-problem kernel: symmetric per-channel layers in the canonical layout, fp16 or int32 output.
static bool small_ok(const GemmArgs &g, bool grouped, int out_kind) {
    return !grouped && (out_kind == OUT_F16 || out_kind == OUT_I32) && g.K % 64 == 0 && g.K <= 4096 && g.lda % 16 == 0 &&
           (long)g.M * g.lda < 0x7fffffffL && (long)g.N * g.ldw < 0x7fffffffL && ((long)g.M + 32) * g.N * 4 < 0x7fffffffL;
}

// LDS of the group kernel: three stages of a 128 x 128 tile (plus, in the operand layout, a column of token sums
// each), token parameters, and the group tables zw[ng][128] and RA[ng][128]; two workgroups share a CU's 160 KB.
static bool group_tables_fit(int ng, bool olay) {
    return (size_t)ng * 256 * 4 + 3 * (256 * 64 + (olay ? 512 : 0)) + 2048 <= 80 * 1024;
}
static bool group_ok(const GemmArgs &g, bool grouped) {
    return grouped && g.K % kBK == 0 && g.K >= 2 * kBK && (long)g.M * g.lda < 0x7fffffffL &&
           (long)g.N * g.ldw < 0x7fffffffL && (long)g.N * (g.ng + 1) * 4 < 0x7fffffffL && (long)g.M * g.ng * 4 < 0x7fffffffL &&
           group_tables_fit(g.ng, g.osum != nullptr);
}

// Built-in shape table of the canonical layout: large problems take the pipelined tiles (192 x 128 when the
// output is narrow, so that a 12288-token problem splits into a whole number of rounds of two
// workgroups per CU; 128 x 256 otherwise), small ones the generic tiles that still give every
// CU something to do.
static int pick_schedule(const GemmArgs &g, bool grouped, int out_kind) {
    // a few hundred 32 x 32 tiles at most: latency decides, the waves of a workgroup split K
    if ((long)((g.M + 31) / 32) * ((g.N + 31) / 32) <= 512 && small_ok(g, grouped, out_kind)) return S_SMALL;
    const long big = (long)((g.M + 127) / 128) * ((g.N + 255) / 256);
    if (big >= 256) {
        if (group_ok(g, grouped)) return S_GROUP;
        if (!pipe_ok(g, grouped)) return S_GEN_64x128;   // grouped layers: the 64 x 128 tile leaves LDS for the group tables
        return g.N <= 1024 ? S_PIPE_192x128 : S_PIPE_128x256;
    }
    const long mid = (long)((g.M + 63) / 64) * ((g.N + 127) / 128);
    if (mid >= 256) return S_GEN_64x128;
    // 64 x 64 tiles beat 32 x 32 ones wherever there are a few dozen of them (measured at 384 .. 1536 tokens)
    const long small = (long)((g.M + 63) / 64) * ((g.N + 63) / 64);
    if (small >= 64) return S_GEN_64x64;
    return S_GEN_32x32;
}

// The FP6 kernel: both operands in the FP6 layout, whole pairs of 64-code half steps, at least eight of them.
static bool fp6_ok(const GemmArgs &g, bool grouped) {
    int lpr = 0, opl = 0;
    return !grouped && g.K % kBK == 0 && g.K >= 4 * kBK && fp6_plan(g.K, &lpr, &opl) && g.lda % 48 == 0 &&
           ((long)g.M + 64) * g.lda < 0x7fffffffL && ((long)g.N + 128) * (g.K / 4 * 3) < 0x7fffffffL;
}

// CU count of the current device (the tile choice of the persistent kernel depends on it); 256 if it cannot be read.
static int device_cus() {
    static std::atomic<int> cached[kMaxDevices] = {};
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    cus = cached[dev].load(std::memory_order_relaxed);
    if (!cus) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        cached[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

// Tile choice of the persistent kernel.  What counts is the CU that ends up with the most tiles: n tiles
// of area a, worked on by min(n, workgroups per CU) co-resident workgroups.  Fitted to kernel times over
// M = 512 .. 16384 on the BERT-base and BERT-large shapes: one workgroup alone gets about half of what two
// get out of a CU's matrix pipe, three get 0.85 of it (LDS and cache contention); per unit of area the
// 192 x 128 tile is 8 % dearer than the 128 x 256 one (more operand registers unpacked per MFMA) and the
// 128 x 128 tile 6 % cheaper in the mid range, where it also leaves fewer CUs idle.  Below about 1500
// tokens a tile's K loop is latency-bound and the small tile gains nothing.
static int pick_olay(const GemmArgs &g) {
    const long cus = device_cus();
    auto cost = [&](int bm, int bn, int occ, double eff) {
        const long tiles = (long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn);
        const long n = (tiles + cus - 1) / cus;
        const long together = n < occ ? n : occ;
        const double rate = together == 1 ? 0.5 : together == 2 ? 1.0 : 0.85;
        return (double)n * bm * bn / (rate * eff);
    };
    int best = S_OLAY_128x256;
    double c = cost(128, 256, 2, 1.0);
    const double c192 = cost(192, 128, 2, 0.92);
    if (c192 < c) { best = S_OLAY_192x128; c = c192; }
    if (g.M >= 1536 && cost(128, 128, 3, 1.06) < c) best = S_OLAY_128x128;
    return best;
}

// Tile choice of the FP6 kernel, from kernel times on the BERT-large shapes at 12288 tokens (TOP/s of 192 x 256 with
// one wave per SIMD / 128 x 256 / 192 x 128): K = 4096 3350 / 3040 / 3110; K = 1024 with N = 3072 2450 / 2490 / 1950, with
// N = 4096 + GELU 2030 / 2260 / 2080, with N = 1024 1890 / 1960 / 1790.  Long K favours the big tile (least operand traffic per
// product, one workgroup per CU); otherwise two 128 x 256 workgroups per CU, whose epilogues and stores overlap better;
// few tiles fall back to the mid-range rule of the int8 kernel.
static int pick_fp6(const GemmArgs &g) {
    const long cus = device_cus();
    const long big = (long)((g.M + 191) / 192) * ((g.N + 255) / 256);
    if (g.K >= 2048 && g.K / 64 >= 9 && big * 4 >= 3 * cus) return S_FP6_192x256;
    const long mid = (long)((g.M + 127) / 128) * ((g.N + 255) / 256);
    if (mid >= cus) return S_FP6_128x256;
    const int o = pick_olay(g);
    return o == S_OLAY_128x256 ? S_FP6_128x256 : o == S_OLAY_192x128 ? S_FP6_192x128 : S_FP6_128x128;
}

// Resolves schedule 0 to the table's choice and checks everything a launcher of that family requires, so that
// a caller can still refuse the call with its outputs untouched.  Nothing is launched here.
static int resolve_schedule(const GemmArgs &g, bool grouped, int out_kind, int *schedule) {
    // the epilogue addresses the output with 32-bit byte offsets below 2^31
    if (((long)g.M + 512) * g.N * 4 >= 0x80000000L) return W4A4_ERR_UNSUPPORTED_SHAPE;   // (tile overhang included)
    const bool olay = g.layout == W4A4_LAYOUT_MFMA;             // operands in the MFMA operand layout
    const bool fp6 = g.layout == W4A4_LAYOUT_FP6;
    int sch = *schedule;
    // operand layout: symmetric per-channel layers run on the persistent kernel, unsigned (grouped) ones on the group kernel
    if (sch == 0) sch = fp6 ? pick_fp6(g) : olay ? (grouped ? S_GROUP : pick_olay(g)) : pick_schedule(g, grouped, out_kind);
    if (sch < 1 || sch > kNumSchedules) return W4A4_ERR_INVALID_ARG;
    const Schedule &s = kSchedules[sch - 1];
    if (grouped && !s.grouped_ok) return W4A4_ERR_INVALID_ARG;
    // a kernel family understands one layout, except the group kernel, which reads grouped layers in either
    if (fp6 != (s.family == F_FP6)) return W4A4_ERR_INVALID_ARG;
    if (!fp6 && (olay ? !(s.family == (grouped ? F_GROUP : F_OLAY)) : s.family == F_OLAY)) return W4A4_ERR_INVALID_ARG;
    const bool q4 = out_kind == OUT_Q4 || out_kind == OUT_Q4M || out_kind == OUT_Q6;
    if ((out_kind == OUT_Q6) != (q4 && fp6)) return W4A4_ERR_UNSUPPORTED_SHAPE;   // FP6 codes come from the FP6 kernel, and only they
    switch (s.family) {
        case F_FP6:
            if (!fp6_ok(g, grouped)) return W4A4_ERR_UNSUPPORTED_SHAPE;
            if (q4) {
                int lpr = 0, opl = 0;
                if (s.variant != 0) return W4A4_ERR_INVALID_ARG;
                // the output is the next layer's activation operand: whole 256-column tiles, a row length the layout is
                // offered for, 32-bit byte offsets
                if (g.N % 256 || !fp6_plan(g.N, &lpr, &opl) || (((long)g.M + 191) * g.N / 4 * 3) >= 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
                const int lim = fp6_requant_max_tiles_n();
                if (lim < 0) return W4A4_ERR_HIP;
                if (g.N / 256 > lim) return W4A4_ERR_UNSUPPORTED_SHAPE;
            }
            break;
        case F_OLAY:
            if (!pipe_ok(g, grouped) || g.K < 2 * kBK || (long)g.M * g.ldo * 4 >= 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
            if (q4) {
                if (s.variant != 0) return W4A4_ERR_INVALID_ARG;
                const int lim = olay_requant_max_tiles_n(out_kind == OUT_Q4M);
                if (lim < 0) return W4A4_ERR_HIP;
                if ((g.N + 255) / 256 > lim) return W4A4_ERR_UNSUPPORTED_SHAPE;
            }
            break;
        case F_SMALL:
            if (!small_ok(g, grouped, out_kind)) return W4A4_ERR_UNSUPPORTED_SHAPE;
            break;
        case F_GROUP:
            if (!group_ok(g, grouped) || q4) return W4A4_ERR_UNSUPPORTED_SHAPE;
            break;
        case F_PIPE:
            if (!pipe_ok(g, grouped) || out_kind == OUT_Q4M) return W4A4_ERR_UNSUPPORTED_SHAPE;
            if (out_kind == OUT_Q4) {
                if (s.variant != 0) return W4A4_ERR_INVALID_ARG;
                const int lim = pipe_requant_max_tiles();
                if (lim < 0) return W4A4_ERR_HIP;
                if ((long)((g.M + 127) / 128) * ((g.N + 255) / 256) > lim) return W4A4_ERR_UNSUPPORTED_SHAPE;
            }
            break;
        default:
            if (q4) return W4A4_ERR_UNSUPPORTED_SHAPE;
            break;
    }
    *schedule = sch;
    return W4A4_OK;
}

static int run_gemm(GemmArgs &g, int mode, bool grouped, int out_kind, int schedule, hipStream_t st) {
    const int rc = resolve_schedule(g, grouped, out_kind, &schedule);
    if (rc) return rc;
    const Schedule &s = kSchedules[schedule - 1];
    switch (s.family) {
        case F_OLAY: return launch_olay(s.variant, out_kind, g, st);
        case F_FP6: return launch_fp6(s.variant, out_kind, g, st);
        case F_SMALL: return launch_small_packed(out_kind, g, st);
        case F_GROUP: return launch_group(mode, out_kind, g, st);
        case F_PIPE: return launch_pipe(s.variant, out_kind, g, st);
        default: return launch_generic(s.variant, mode, grouped, out_kind, g, st);
    }
}

// ---------------------------------------------------------------------------------------------
// Argument validation shared by w4a4_linear, w4a4_gemm_i32 and w4a4_dequant_epilogue.
static int check_operands(const w4a4_act *A, const w4a4_weight *W, int *ng_out) {
    if (!A || !W) return W4A4_ERR_INVALID_ARG;
    if (A->M < 0 || A->K <= 0 || W->N <= 0 || W->K != A->K) return W4A4_ERR_INVALID_ARG;
    if (A->mode != W->mode || (A->mode != W4A4_SYM && A->mode != W4A4_ASYM)) return W4A4_ERR_INVALID_ARG;
    if (W->group < 0 || A->group < 0) return W4A4_ERR_INVALID_ARG;
    if (A->layout != W->layout) return W4A4_ERR_INVALID_ARG;
    if (A->layout != W4A4_LAYOUT_CANONICAL && A->layout != W4A4_LAYOUT_MFMA && A->layout != W4A4_LAYOUT_FP6) return W4A4_ERR_INVALID_ARG;
    if (A->layout == W4A4_LAYOUT_FP6) {
        int lpr = 0, opl = 0;
        if (A->mode != W4A4_SYM) return W4A4_ERR_INVALID_ARG;
        if ((W->group != 0 && W->group != W->K) || (A->group != 0 && A->group != A->K)) return W4A4_ERR_UNSUPPORTED_SHAPE;
        if (A->K % kBK || A->K < 4 * kBK || !fp6_plan(A->K, &lpr, &opl)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    if (A->layout == W4A4_LAYOUT_MFMA) {
        if (A->ldo < 1) return W4A4_ERR_INVALID_ARG;
        if (A->M > 0 && (!A->osum || !W->esum)) return W4A4_ERR_INVALID_ARG;
        if (A->K % kBK || A->K < 2 * kBK) return W4A4_ERR_UNSUPPORTED_SHAPE;
        if (A->mode == W4A4_SYM) {
            if (W->group != 0 && W->group != W->K) return W4A4_ERR_UNSUPPORTED_SHAPE;
        } else {                                                // unsigned codes: whole K steps per weight group
            const int G = W->group == 0 ? W->K : W->group;
            if (G % kBK || W->K % G || !group_tables_fit(W->K / G, true)) return W4A4_ERR_UNSUPPORTED_SHAPE;
        }
    }
    const int K = A->K;
    if (K % 32 || W->N % 8) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int G = W->group == 0 ? K : W->group;
    if (K % G || (W->group != 0 && G % kBK)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const int ng = K / G;
    if (A->lda < (A->layout == W4A4_LAYOUT_FP6 ? K / 4 * 3 : K / 2)) return W4A4_ERR_INVALID_ARG;
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
        if (ep->requant_layout != W4A4_LAYOUT_CANONICAL && ep->requant_layout != W4A4_LAYOUT_MFMA &&
            ep->requant_layout != W4A4_LAYOUT_FP6) return W4A4_ERR_INVALID_ARG;
        if (ep->requant_layout != W4A4_LAYOUT_CANONICAL && ep->requant_mode != W4A4_SYM) return W4A4_ERR_INVALID_ARG;
        // FP6 codes are written by the FP6 kernel's own epilogue, for one range per token
        if (ep->requant_layout == W4A4_LAYOUT_FP6 &&
            (A->layout != W4A4_LAYOUT_FP6 || (ep->requant_group != 0 && ep->requant_group != W->N))) return W4A4_ERR_UNSUPPORTED_SHAPE;
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
                      float *s, float *z, int32_t *gsum, hipStream_t st, int layout = 0);

static void fill_args(GemmArgs &g, const w4a4_act *A, const w4a4_weight *W, int ng) {
    g.Aq = A->q; g.lda = A->lda; g.Wq = W->q; g.ldw = A->layout == W4A4_LAYOUT_FP6 ? W->K / 4 * 3 : W->K / 2;
    g.layout = A->layout;
    g.M = A->M; g.N = W->N; g.K = A->K;
    g.ng = ng; g.steps_per_group = (A->K / ng + kBK - 1) / kBK;
    g.sa = A->scale; g.za = A->zero; g.RA = A->gsum;
    g.sw = W->scale; g.zw = W->zero; g.c = W->rowsum_deq;
    g.bias = nullptr; g.act = W4A4_ACT_NONE; g.out = nullptr;
    g.tiles_m = g.tiles_n = 0;
    g.rowmax = nullptr; g.arrived = nullptr; g.fault = nullptr; g.fault_sticky = nullptr; g.out_scale = nullptr;
    g.spin_limit = 0; g.wait_for = 0;
    const bool olay = A->layout == W4A4_LAYOUT_MFMA;
    g.osum = olay ? A->osum : nullptr; g.ldo = olay ? A->ldo : 0; g.esum = olay ? W->esum : nullptr;
    g.out_osum = nullptr; g.osum_slices = 1; g.slice_tiles = 0;
    g.stagger = 0;
}

}  // namespace w4a4

using namespace w4a4;

extern "C" int w4a4_schedule_count(void) { return kNumSchedules; }

extern "C" int w4a4_preferred_layout(int M, int N, int K, int mode, int group) {
    (void)N;
    // the operand layout exists for symmetric per-channel layers whose K the persistent kernel accepts, and for
    // unsigned codes with weight groups of whole K steps whose tables fit the group kernel's LDS;
    // small token counts (latency-bound, a handful of 128-row tiles) stay on the canonical kernels
    if (K % kBK || K < 2 * kBK || K <= 0) return W4A4_LAYOUT_CANONICAL;
    if (mode == W4A4_SYM) {
        if (group != 0 && group != K) return W4A4_LAYOUT_CANONICAL;
    } else {
        const int G = group == 0 ? K : group;
        if (G <= 0 || G % kBK || K % G || !group_tables_fit(K / G, true)) return W4A4_LAYOUT_CANONICAL;
    }
    return M >= 1536 ? W4A4_LAYOUT_MFMA : W4A4_LAYOUT_CANONICAL;   // (measured crossover between 1024 and 1536 tokens)
}

extern "C" const char *w4a4_schedule_name(int schedule) {
    return (schedule >= 1 && schedule <= kNumSchedules) ? kSchedules[schedule - 1].name : "";
}

// Fused requantize (one kernel: the column tiles of a row panel exchange per-token maxima and pack
// the codes from registers).  Two kernels can do it:
//   1 = the pipelined kernel on canonical operands, canonical symmetric codes out, no code sums; its whole
//       grid must be resident, which limits it to a few hundred tiles;
//   2 = the persistent kernel on operands in the MFMA operand layout; symmetric codes out in either
//       layout (the operand layout with odd-position sums per column slice of requant_group, which
//       must be whole 256-column tiles); the column tiles of a panel must fit one XCD's resident share.
//   3 = the FP6 kernel on operands in the FP6 layout, codes out in the FP6 layout (no sums); N in whole 256-column
//       tiles that fit one XCD's resident share.
// 0 = not fusable: the GEMM stores fp32 rows and the row quantizer packs them.
// The residency limits come from the runtime's occupancy figure for the kernel on the current device.
static int fused_requant_kind(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, bool want_gsum) {
    if (!ep->requant || ep->requant_mode != W4A4_SYM) return 0;
    if (A->layout == W4A4_LAYOUT_FP6) {
        // FP6 codes out: the FP6 kernel's own requantizing epilogue; other layouts: fp32 rows and the row quantizer
        if (ep->requant_layout != W4A4_LAYOUT_FP6 || want_gsum) return 0;
        if (ep->schedule != 0 && ep->schedule != S_FP6_128x256) return 0;
        if ((ep->requant_group != 0 && ep->requant_group != W->N) || W->N % 256) return 0;
        return W->N / 256 <= fp6_requant_max_tiles_n() ? 3 : 0;
    }
    if (A->mode != W4A4_SYM || (W->group != 0 && W->group != W->K)) return 0;
    if (A->K % kBK || (long)A->M * A->lda >= 0x7fffffffL || (long)W->N * (W->K / 2) >= 0x7fffffffL) return 0;
    if (((long)A->M + 512) * W->N * 4 >= 0x80000000L) return 0;
    const int tn = (W->N + 255) / 256;
    if (A->layout == W4A4_LAYOUT_MFMA) {
        if (ep->schedule != 0 && ep->schedule != S_OLAY_128x256) return 0;
        if (A->K < 2 * kBK || (long)A->M * A->ldo * 4 >= 0x7fffffffL) return 0;
        const bool mfma_out = ep->requant_layout == W4A4_LAYOUT_MFMA;
        if (tn > olay_requant_max_tiles_n(mfma_out)) return 0;
        if (mfma_out) {
            const int rg = ep->requant_group == 0 ? W->N : ep->requant_group;
            return (rg % 256 == 0 || rg == W->N) && W->N % rg == 0 && (rg == W->N || W->N % 256 == 0) ? 2 : 0;
        }
        return want_gsum ? 0 : 2;
    }
    if (ep->requant_layout != W4A4_LAYOUT_CANONICAL || want_gsum) return 0;
    if (ep->schedule != 0 && ep->schedule != S_PIPE_128x256) return 0;
    return (long)((A->M + 127) / 128) * tn <= pipe_requant_max_tiles() ? 1 : 0;
}
static size_t fused_workspace_bytes(int M) {
    return ((size_t)M + (size_t)(M + 127) / 128 + 4) * sizeof(uint32_t);
}

extern "C" size_t w4a4_workspace_bytes(int M, int N, int K, const w4a4_epilogue *ep) {
    (void)K;
    if (!ep || !ep->requant || M <= 0 || N <= 0) return 0;
    return (size_t)M * (size_t)N * sizeof(float);          // fp32 rows awaiting their per-token range
}

extern "C" size_t w4a4_linear_workspace_bytes(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep,
                                              int want_gsum) {
    if (!A || !W || !ep || !ep->requant || A->M <= 0 || W->N <= 0) return 0;
    if (fused_requant_kind(A, W, ep, want_gsum != 0)) return fused_workspace_bytes(A->M);
    return (size_t)A->M * (size_t)W->N * sizeof(float);
}

// Clears two word ranges (a fill kernel rather than a memset, so that the call can be captured in a graph).
__global__ void zero_words_kernel(uint32_t *p, int n, uint32_t *p2, int n2) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
    else if (i - n < n2) p2[i - n] = 0;
}

// ---- the device-wide fault flag of the fused requantize ---------------------------------------------------
// A workgroup that gives up waiting for its siblings sets the last word of that call's workspace AND this
// flag, which callers that never see the workspace of an inner w4a4_linear (w4a4_ffn, w4a4_encoder_layer)
// read through w4a4_fused_fault_check.  One copy per device; host code uses the address the runtime reports
// for the current device, never the symbol's name.
static __device__ int fused_fault_flag;
static int *fault_flag_address() {
    static std::atomic<int *> addr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    int *p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(fused_fault_flag)) != hipSuccess || !p) return nullptr;
        addr[dev].store(p, std::memory_order_release);
    }
    return p;
}

extern "C" int w4a4_fused_fault_check(void *stream) {
    int *flag = fault_flag_address();
    if (!flag) return W4A4_ERR_HIP;
    hipStream_t st = as_stream(stream);
    int host = 0;
    if (hipMemcpyAsync(&host, flag, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return W4A4_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return W4A4_ERR_HIP;
    if (host) {
        hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t *>(flag), 1, nullptr, 0);
        if (hipStreamSynchronize(st) != hipSuccess) return W4A4_ERR_HIP;
    }
    return host ? 1 : 0;
}

// Test hook: the fused requantize kernels launched by this thread from now on poll at most `spin_limit` times
// and wait for `extra_arrivals` more column tiles than a row panel has.  (0, 0) restores the defaults.  With
// extra_arrivals > 0 no panel ever completes, so every workgroup gives up after spin_limit polls, raises the
// fault words and exits normally: the way to exercise the give-up path without a hang.
static thread_local int tl_spin_limit = 0, tl_extra_arrivals = 0;
extern "C" int w4a4_debug_fused_wait(int spin_limit, int extra_arrivals) {
    if (spin_limit < 0 || extra_arrivals < 0) return W4A4_ERR_INVALID_ARG;
    tl_spin_limit = spin_limit;
    tl_extra_arrivals = extra_arrivals;
    return W4A4_OK;
}
constexpr int kSpinLimit = 1 << 22;

extern "C" int w4a4_pick_schedule(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep) {
    int ng = 0;
    if (!A || !W || !ep) return W4A4_ERR_INVALID_ARG;
    if (A->K <= 0 || W->N <= 0 || W->K != A->K || A->mode != W->mode || A->layout != W->layout) return W4A4_ERR_INVALID_ARG;
    const int G = W->group == 0 ? A->K : W->group;
    if (G <= 0 || A->K % G) return W4A4_ERR_UNSUPPORTED_SHAPE;
    ng = A->K / G;
    GemmArgs g;
    fill_args(g, A, W, ng);
    const bool grouped = A->mode == W4A4_ASYM || ng > 1;
    int out_kind = OUT_F16, schedule = ep->schedule;
    if (ep->requant) {
        const int fused = fused_requant_kind(A, W, ep, false);
        out_kind = !fused ? OUT_F32 : fused == 3 ? OUT_Q6 : (fused == 2 && ep->requant_layout == W4A4_LAYOUT_MFMA) ? OUT_Q4M : OUT_Q4;
        if (fused) schedule = fused == 1 ? S_PIPE_128x256 : fused == 3 ? S_FP6_128x256 : S_OLAY_128x256;
    }
    const int rc = resolve_schedule(g, grouped, out_kind, &schedule);
    return rc ? rc : schedule;
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

// w4a4_linear behind its argument checks.  `exchange` is the area the fused requantize exchanges row maxima
// through (fused_workspace_bytes(M) bytes, cleared here by a fill kernel); `rows_f32` receives the fp32 rows
// of a requantize that cannot be fused.  Whichever the layer does not need may be NULL.
static int linear_impl(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, void *out, float *out_scale,
                       float *out_zero, int32_t *out_gsum, int ng, int fused, uint32_t *exchange, void *rows_f32,
                       hipStream_t st) {
    GemmArgs g;
    fill_args(g, A, W, ng);
    g.bias = static_cast<const __half *>(ep->bias_f16);
    g.act = ep->act;
    const bool grouped = A->mode == W4A4_ASYM || ng > 1;
    if (!ep->requant) {
        g.out = out;
        return run_gemm(g, A->mode, grouped, OUT_F16, ep->schedule, st);
    }
    if (ep->requant_layout == W4A4_LAYOUT_MFMA) {
        if (!out_gsum) return W4A4_ERR_INVALID_ARG;            // receives the odd-position code sums
        if (!fused && ep->requant_group != 0 && ep->requant_group != W->N) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    if (fused) {
        // One kernel: the column tiles of a row panel exchange their row maxima through the exchange area and
        // pack the codes from registers.
        const int words = (int)(fused_workspace_bytes(A->M) / sizeof(uint32_t));
        const bool sums = fused == 2 && ep->requant_layout == W4A4_LAYOUT_MFMA;
        const int rg = ep->requant_group == 0 ? W->N : ep->requant_group;
        const int slices = sums ? W->N / rg : 1;
        const long n2 = sums ? (long)A->M * slices : 0;
        if (n2 + words > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
        g.rowmax = exchange;
        g.arrived = reinterpret_cast<int *>(exchange + A->M);
        g.fault = reinterpret_cast<int *>(exchange + words - 1);
        g.fault_sticky = fault_flag_address();
        if (!g.fault_sticky) return W4A4_ERR_HIP;
        g.spin_limit = tl_spin_limit > 0 ? tl_spin_limit : kSpinLimit;
        g.wait_for = tl_extra_arrivals > 0 ? (W->N + 255) / 256 + tl_extra_arrivals : 0;   // 0: the launcher fills in tiles_n
        g.out_scale = out_scale;
        g.out = out;
        g.out_osum = out_gsum; g.osum_slices = slices; g.slice_tiles = sums && slices > 1 ? rg / 256 : 0x40000000;
        const int out_kind = fused == 3 ? OUT_Q6 : fused == 1 ? OUT_Q4 : (sums ? OUT_Q4M : OUT_Q4);
        int schedule = fused == 1 ? S_PIPE_128x256 : fused == 3 ? S_FP6_128x256 : S_OLAY_128x256;
        // everything that can refuse the launch is checked before the outputs are touched
        const int rc = resolve_schedule(g, false, out_kind, &schedule);
        if (rc) return rc;
        hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((words + n2 + 255) / 256)), dim3(256), 0, st, exchange, words,
                           reinterpret_cast<uint32_t *>(out_gsum), (int)n2);
        return run_gemm(g, A->mode, false, out_kind, schedule, st);
    }
    // Requantize: the per-token range needs the whole output row, which no single tile
    // sees.  The GEMM leaves the fp32 rows in the workspace and the row quantizer turns
    // them into packed codes.
    if (ep->requant_layout == W4A4_LAYOUT_FP6) return W4A4_ERR_UNSUPPORTED_SHAPE;   // FP6 codes exist only fused
    g.out = rows_f32;
    const int rc = run_gemm(g, A->mode, grouped, OUT_F32, ep->schedule, st);
    if (rc) return rc;
    return quantize_rows_f32(static_cast<const float *>(rows_f32), A->M, W->N, W->N, ep->requant_mode,
                             ep->requant_group, static_cast<uint8_t *>(out), out_scale, out_zero, out_gsum, st,
                             ep->requant_layout);
}

extern "C" int w4a4_linear(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, void *out,
                           float *out_scale, float *out_zero, int32_t *out_gsum, void *workspace,
                           size_t workspace_bytes, void *stream) {
    int ng = 0, rng = 0;
    int rc = check_layer(A, W, ep, out, out_scale, out_zero, &ng, &rng);
    if (rc) return rc;
    if (A->M == 0) return W4A4_OK;
    const int fused = fused_requant_kind(A, W, ep, out_gsum != nullptr);
    if (ep->requant && ep->requant_layout == W4A4_LAYOUT_FP6) {     // no code sums in that layout, and only the fused kernel writes it
        if (out_gsum) return W4A4_ERR_INVALID_ARG;
        if (!fused) return W4A4_ERR_UNSUPPORTED_SHAPE;
    }
    const size_t need = !ep->requant ? 0 : fused ? fused_workspace_bytes(A->M) : (size_t)A->M * (size_t)W->N * sizeof(float);
    if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) return W4A4_ERR_WORKSPACE;
    return linear_impl(A, W, ep, out, out_scale, out_zero, out_gsum, ng, fused, static_cast<uint32_t *>(workspace),
                       workspace, as_stream(stream));
}

// ---- w4a4_linear for callers that cannot allocate -----------------------------------------------------------
// The exchange area of the fused requantize lives in a file-scope device array instead of a caller workspace.
// Each GPU the library runs on holds its own copy of the array at its own address until the process ends; host
// code never passes the array's name to a kernel or a copy (on the host the name is only a handle): it asks the
// runtime once per device, with that device current, for the copy's address and uses that pointer.
constexpr int kStaticMaxTokens = 65536;
constexpr int kScratchWords = kStaticMaxTokens + kStaticMaxTokens / 128 + 4;      // 264 208 bytes per device
static __device__ __align__(256) uint32_t scratch[kScratchWords];

static uint32_t *scratch_address() {
    static std::atomic<uint32_t *> addr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    uint32_t *p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
        p = static_cast<uint32_t *>(sym);
        addr[dev].store(p, std::memory_order_release);
    }
    return p;
}

extern "C" int w4a4_linear_static(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep, void *out,
                                  float *out_scale, float *out_zero, int32_t *out_gsum, void *stream) {
    int ng = 0, rng = 0;
    int rc = check_layer(A, W, ep, out, out_scale, out_zero, &ng, &rng);
    if (rc) return rc;
    if (A->M == 0) return W4A4_OK;
    int fused = 0;
    uint32_t *exchange = nullptr;
    if (ep->requant) {
        if (ep->requant_layout == W4A4_LAYOUT_FP6 && out_gsum) return W4A4_ERR_INVALID_ARG;
        fused = fused_requant_kind(A, W, ep, out_gsum != nullptr);
        // a requantize that cannot be fused needs M*N*4 bytes of fp32 rows: beyond what a static array should hold
        if (!fused) return W4A4_ERR_WORKSPACE;
        if (A->M > kStaticMaxTokens) return W4A4_ERR_WORKSPACE;
        exchange = scratch_address();
        if (!exchange) return W4A4_ERR_HIP;
    }
    return linear_impl(A, W, ep, out, out_scale, out_zero, out_gsum, ng, fused, exchange, nullptr, as_stream(stream));
}
