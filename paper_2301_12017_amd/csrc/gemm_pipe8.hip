// Pipelined INT4 x INT4 -> INT32 GEMM, "widen once" variant (symmetric codes, per-channel
// weight scales, K a multiple of 64).
//
// On gfx950 the vector ALU, not the matrix pipe, is the scarce resource of this layer: every
// v_mfma_i32_32x32x32_i8 (32 clocks) leaves room for only about four other vector
// instructions on the SIMD.  Widening the packed codes per wave and per fragment (as the
// other kernels do) costs 6*(FM+FN)/(FM*FN) VALU per MFMA because every fragment is widened
// by each wave that reads it.  Here the codes are widened ONCE per workgroup, on the way
// from the global-load registers into LDS:
//   * HBM holds packed codes; a thread loads 16 bytes (32 codes), widens them with the
//     (d<<4)&0xF0F0F0F0 / d&0xF0F0F0F0 trick to 32 int8 values (each 16*code) and writes two
//     16-byte LDS words.  LDS therefore holds int8 tiles, 64 codes (64 bytes, pitch 80) per
//     row per K step, and the MFMA operands are read from LDS with no further arithmetic.
//   * 3*(BM+BN)*2/NT VALU per K step per thread instead of 12*(FM+FN): 2.25 instead of 4.5
//     VALU per MFMA for the 128 x 256 tile.
//   * LDS traffic doubles (int8 instead of nibbles) but stays near half of the 256 B/clk the
//     CU delivers.
// Two LDS stages of one K step (64 codes) each, one workgroup barrier per K step (LDS-only
// fence), global loads two K steps ahead in two register sets, two workgroups per CU so the
// prologue and epilogue of one tile overlap the main loop of another.
#include "gemm_common.hpp"

namespace w4a4 {

constexpr int kBK8 = 64;           // codes per K step of this kernel
constexpr int kPitch8 = 80;        // LDS row pitch: 64 int8 + 16 bytes of padding

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_pipe8_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
    constexpr int STAGE = (BM + BN) * kPitch8;
    constexpr int CH = (BM + BN) * 2;                           // 16-byte packed chunks per K step
    constexpr int LD = CH / NT;                                 // per thread
    constexpr int NF = FM + FN, NM = FM * FN;
    static_assert(CH % NT == 0, "tile rows must split evenly over the threads");
    static_assert(NF <= NM && 2 * LD <= NM, "not enough MFMA slots to hide the memory operations");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *sa_lds = reinterpret_cast<float *>(smem + 2 * STAGE);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tile = xcd_tile(blockIdx.x, g.tiles_m * g.tiles_n);
    const int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    const int KT = g.K / kBK8;

    // ---- global -> LDS plan ---------------------------------------------------------------
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.Aq, (uint32_t)((long)(g.M - 1) * g.lda + g.K / 2));
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.Wq, (uint32_t)((long)g.N * g.ldw));
    int voff[LD], ldst[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int ch = tid + i * NT, row = ch >> 1, half = ch & 1;
        if (row < BM) {
            voff[i] = (m0 + row) * (int)g.lda + half * 16;       // rows >= M fall outside the buffer: zeros
            ldst[i] = row * kPitch8 + half * 32;
        } else {
            // LDS row p of the weight tile holds output channel nl: MFMA column c of fragment f
            // is channel c*FN + f of the wave's span.
            const int p = row - BM;
            const int w = p / (FN * 32), rem = p % (FN * 32), f = rem / 32, c = rem % 32;
            const int nl = w * (FN * 32) + c * FN + f;
            voff[i] = (n0 + nl) * (int)g.ldw + half * 16;
            ldst[i] = (BM + p) * kPitch8 + half * 32;
        }
    }
    static_assert((BM * 2) % NT == 0, "activation chunks must fill whole load rounds");
    auto k_off = [&](int kt) { return (kt < KT ? kt : KT - 1) * (kBK8 / 2); };   // past the end: re-read (unused)
    auto load_one = [&](u32x4 &dst, int i, int so) {
        dst = __builtin_amdgcn_raw_buffer_load_b128(i < (BM * 2) / NT ? a_rsrc : b_rsrc, voff[i], so, 0);
    };
    // widen 32 packed codes to 32 int8 (16*code) and park them in LDS
    auto widen_store = [&](const u32x4 &p, int i, int buf) {
        const v4i lo = widen2<true>(p.x, p.y), hi = widen2<true>(p.z, p.w);
        uint8_t *d = smem + buf * STAGE + ldst[i];
        *reinterpret_cast<v4i *>(d) = lo;
        *reinterpret_cast<v4i *>(d + 16) = hi;
    };

    // ---- operand fragments: read straight from LDS -------------------------------------------
    const int rd = (lane & 31) * kPitch8 + (lane >> 5) * 16;
    int frag_off[NF];
#pragma unroll
    for (int f = 0; f < FM; ++f) frag_off[f] = (wm * FM * 32 + f * 32) * kPitch8 + rd;
#pragma unroll
    for (int f = 0; f < FN; ++f) frag_off[FM + f] = (BM + wn * FN * 32 + f * 32) * kPitch8 + rd;
    auto read_frag = [&](int f, int buf, int k32) {
        return *reinterpret_cast<const v4i *>(smem + buf * STAGE + frag_off[f] + k32 * 32);
    };

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    auto lds_barrier = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // ---- prologue ------------------------------------------------------------------------------
    const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;
    const EpiLane<FN> epi = epilogue_prefetch<FN, W4A4_SYM, false, OUT>(g, n_lane);
    stage_token_params<BM, NT, W4A4_SYM>(g, m0, sa_lds, nullptr, tid);
    u32x4 s0[LD], s1[LD];                                       // register sets of the steps in flight
    v4i F0[NF], F1[NF];
#pragma unroll
    for (int i = 0; i < LD; ++i) load_one(s0[i], i, k_off(0));
#pragma unroll
    for (int i = 0; i < LD; ++i) load_one(s1[i], i, k_off(1));
#pragma unroll
    for (int i = 0; i < LD; ++i) widen_store(s0[i], i, 0);
#pragma unroll
    for (int i = 0; i < LD; ++i) load_one(s0[i], i, k_off(2));
    lds_barrier();
#pragma unroll
    for (int f = 0; f < NF; ++f) F0[f] = read_frag(f, 0, 0);

    // ---- main loop ---------------------------------------------------------------------------------
    // One K step (64 codes) = two sub-steps of NM MFMAs.  Slot k issues MFMA k and, behind it,
    // at most one LDS fragment read and half of a chunk's widen-and-store; the scheduling
    // barriers pin that order.  `sa`/`sb` alternate as the register set that holds step kt+1
    // (consumed now) and then receives step kt+3.
#define W4A4_MFMA(F, k)                                                                               \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(F[(k) / FN], F[FM + (k) % FN],      \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);  \
    __builtin_amdgcn_sched_barrier(0);
    constexpr int kBarSlot = NM - NF;
    auto step = [&](int kt, u32x4 (&sa)[LD]) {
        const int cur = kt & 1;
        const int so = k_off(kt + 3);
        // sub-step A: multiply k32 0; fetch k32 1 of this stage; widen step kt+1 into the other
        //             stage; request step kt+3 into the freed registers.
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_MFMA(F0, k)
            if (k < NF) F1[k] = read_frag(k, cur, 1);
            if (k < 2 * LD && (k & 1) == 0) widen_store(sa[k / 2], k / 2, cur ^ 1);
            if (k < 2 * LD && (k & 1) == 1) load_one(sa[k / 2], k / 2, so);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step B: multiply k32 1; after the barrier the other stage is complete: fetch its k32 0
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_MFMA(F1, k)
            if (k == kBarSlot) lds_barrier();
            if (k >= kBarSlot) F0[k - kBarSlot] = read_frag(k - kBarSlot, cur ^ 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
        step(kt, s1);
        step(kt + 1, s0);
    }
    if (kt < KT) step(kt, s1);
#undef W4A4_MFMA

    // ---- epilogue ---------------------------------------------------------------------------------
    float none[1][1][16];
    tile_epilogue<FM, FN, W4A4_SYM, false, OUT>(g, acc, none, epi, m0, wm * FM * 32, lane, sa_lds, nullptr);
}

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = 2 * (size_t)(BM + BN) * kPitch8 + BM * sizeof(float);
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_pipe8_kernel<FM, FN, WM, WN, OCC, OUT>;
    static KernelState ks;
    if (prepare_kernel(reinterpret_cast<const void *>(kern), lds, ks) < 0) return W4A4_ERR_HIP;
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    launch_gemm(kern, dim3((unsigned)tiles), dim3(WM * WN * 64), lds, st, g);
    return launch_status();
}

template <int OUT>
static int launch_variant(int variant, GemmArgs &g, hipStream_t st) {
    switch (variant) {
        case 0: return launch_one<2, 4, 2, 2, 2, OUT>(g, st);   // 128 x 256, two workgroups per CU
        case 1: return launch_one<4, 4, 2, 2, 1, OUT>(g, st);   // 256 x 256, one workgroup per CU
        default: return W4A4_ERR_INVALID_ARG;
    }
}

// Requires: symmetric codes, per-channel weight scales, K % 64 == 0, M*lda and N*ldw < 2^31.
int launch_pipe8(int variant, int out_kind, GemmArgs &g, hipStream_t st) {
    switch (out_kind) {
        case OUT_F16: return launch_variant<OUT_F16>(variant, g, st);
        case OUT_F32: return launch_variant<OUT_F32>(variant, g, st);
        default: return launch_variant<OUT_I32>(variant, g, st);
    }
}

}  // namespace w4a4
