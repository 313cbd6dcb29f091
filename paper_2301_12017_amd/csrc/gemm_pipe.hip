// Software-pipelined INT4 x INT4 -> INT32 GEMM for the large, MFMA-bound shapes
// (symmetric codes, one weight scale per output channel, K a multiple of 128).
//
// Same data path as the generic kernel (packed codes in HBM and LDS, widened to int8 in
// registers, v_mfma_i32_32x32x32_i8, fused epilogue) but the inner loop is arranged so
// that the matrix pipe never waits for the vector ALU:
//   * A K step of 128 codes is four sub-steps of 32 codes.  While the MFMAs of one
//     sub-step run, the same wave widens the operands of the next sub-step into a second
//     register set and issues the LDS reads of the one after; scheduling barriers pin
//     that interleave (one MFMA, six VALU, at most one LDS / memory operation per slot).
//   * Global loads are buffer loads (out-of-range rows read as zero, so ragged M and N
//     need no branches): the tile of step t+2 is requested while step t is multiplied,
//     its registers are written to the other LDS stage at the start of step t+1.
//   * One workgroup barrier per K step, with an LDS-only fence, so outstanding global
//     loads are never waited for at the barrier.
//   * Two workgroups fit on a CU (128 accumulator registers per lane each) so that the
//     epilogue and the prologue of one tile overlap the main loop of another.
#include "gemm_common.hpp"

namespace w4a4 {

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_pipe_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64;
    constexpr int STAGE = (BM + BN) * kRowB;
    constexpr int A_PT = BM * 4 / NT, B_PT = BN * 4 / NT, LD = A_PT + B_PT;
    constexpr int NF = FM + FN, NM = FM * FN;
    static_assert((BM * 4) % NT == 0 && (BN * 4) % NT == 0, "tile rows must split evenly over the threads");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *sa_lds = reinterpret_cast<float *>(smem + 2 * STAGE);      // per-token scales of the tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tile = xcd_tile(blockIdx.x, g.tiles_m * g.tiles_n);
    const int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    const int KT = g.K / kBK;

    // ---- global -> LDS plan: LD chunks of 16 bytes per thread per K step ----------------
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.Aq, (uint32_t)((long)(g.M - 1) * g.lda + g.K / 2));
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.Wq, (uint32_t)((long)g.N * g.ldw));
    int voff[LD], ldst[LD];
#pragma unroll
    for (int i = 0; i < A_PT; ++i) {
        const int ch = tid + i * NT, row = ch >> 2, kc = ch & 3;
        voff[i] = (m0 + row) * (int)g.lda + kc * 16;             // rows >= M fall outside the buffer: zeros
        ldst[i] = row * kRowB + kc * 16;
    }
#pragma unroll
    for (int i = 0; i < B_PT; ++i) {
        const int ch = tid + i * NT, p = ch >> 2, kc = ch & 3;
        // LDS row p of the weight tile holds output channel nl: MFMA column c of fragment f
        // is channel c*FN + f of the wave's span.
        const int w = p / (FN * 32), rem = p % (FN * 32), f = rem / 32, c = rem % 32;
        const int nl = w * (FN * 32) + c * FN + f;
        voff[A_PT + i] = (n0 + nl) * (int)g.ldw + kc * 16;
        ldst[A_PT + i] = BM * kRowB + p * kRowB + kc * 16;
    }
    u32x4 stg[LD];
    auto load_one = [&](int i, int so) {
        stg[i] = __builtin_amdgcn_raw_buffer_load_b128(i < A_PT ? a_rsrc : b_rsrc, voff[i], so, 0);
    };
    auto store_one = [&](int i, int buf) {
        *reinterpret_cast<u32x4 *>(smem + buf * STAGE + ldst[i]) = stg[i];
    };
    // K offset of step kt; past the end the last step is re-read (in bounds, never used)
    auto k_off = [&](int kt) { return (kt < KT ? kt : KT - 1) * (kBK / 2); };

    // ---- operand fragments -----------------------------------------------------------------
    const int rd = (lane & 31) * kRowB + (lane >> 5) * 16;
    int frag_off[NF];
#pragma unroll
    for (int f = 0; f < FM; ++f) frag_off[f] = (wm * FM * 32 + f * 32) * kRowB + rd;
#pragma unroll
    for (int f = 0; f < FN; ++f) frag_off[FM + f] = BM * kRowB + (wn * FN * 32 + f * 32) * kRowB + rd;
    auto read_frag = [&](int f, int buf, int ks) {
        return *reinterpret_cast<const u32x4 *>(smem + buf * STAGE + frag_off[f] + ks * 32);
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
    u32x4 P0[NF], P1[NF];
    v4i U0[NF], U1[NF];
#pragma unroll
    for (int i = 0; i < LD; ++i) load_one(i, k_off(0));
#pragma unroll
    for (int i = 0; i < LD; ++i) store_one(i, 0);
#pragma unroll
    for (int i = 0; i < LD; ++i) load_one(i, k_off(1));
    lds_barrier();
#pragma unroll
    for (int f = 0; f < NF; ++f) P0[f] = read_frag(f, 0, 0);
#pragma unroll
    for (int f = 0; f < NF; ++f) U0[f] = widen2<true>(P0[f].x, P0[f].y);

    // ---- main loop ---------------------------------------------------------------------------------
    // One iteration = 128 codes of K = four sub-steps of NM MFMAs.  The instruction order below
    // is the intended issue order; the scheduling barriers keep the compiler from regrouping it.
    // Slot k of a sub-step issues MFMA k and, behind it, the widening of fragment k for the
    // NEXT sub-step plus at most one LDS write + global load and one LDS read.
#define W4A4_SLOT_BEGIN(Ucur, k)                                                                          \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ucur[(k) / FN], Ucur[FM + (k) % FN],   \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
    constexpr int kBarSlot = NM - NF;                          // LDS reads of the next stage start here
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const int so = k_off(kt + 2);
        // sub-step 0: multiply (ks 0, low); widen (ks 0, high) -> U1; fetch ks 1 -> P1;
        //             park step kt+1 (in registers since the last iteration) in the other LDS
        //             stage and request step kt+2.
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U0, k)
            if (k < NF) U1[k] = widen2<true>(P0[k].z, P0[k].w);
            if (k < NF) P1[k] = read_frag(k, cur, 1);
            if (k < LD) { store_one(k, cur ^ 1); load_one(k, so); }
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 1: multiply (ks 0, high); widen (ks 1, low) -> U0
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U1, k)
            if (k < NF) U0[k] = widen2<true>(P1[k].x, P1[k].y);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 2: multiply (ks 1, low); widen (ks 1, high) -> U1; once every wave has passed
        //             the barrier the other stage is complete: fetch its ks 0 -> P0.
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U0, k)
            if (k < NF) U1[k] = widen2<true>(P1[k].z, P1[k].w);
            if (k == kBarSlot) lds_barrier();
            if (k >= kBarSlot) P0[k - kBarSlot] = read_frag(k - kBarSlot, cur ^ 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 3: multiply (ks 1, high); widen (next step's ks 0, low) -> U0
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U1, k)
            if (k < NF) U0[k] = widen2<true>(P0[k].x, P0[k].y);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef W4A4_SLOT_BEGIN

    // ---- epilogue ---------------------------------------------------------------------------------
    if constexpr (OUT == OUT_Q4) {
        tile_epilogue_requant<FM, FN>(g, acc, epi, m0, wm * FM * 32, lane, tid, tile / g.tiles_n, sa_lds,
                                      reinterpret_cast<float *>(smem));
    } else {
        float none[1][1][16];
        tile_epilogue<FM, FN, W4A4_SYM, false, OUT>(g, acc, none, epi, m0, wm * FM * 32, lane, sa_lds, nullptr);
    }
}

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
struct PipeLaunch {
    static constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    static constexpr size_t lds = 2 * (size_t)(BM + BN) * kRowB + BM * sizeof(float);
    static KernelState &state() { static KernelState ks; return ks; }
    static auto kernel() { return gemm_pipe_kernel<FM, FN, WM, WN, OCC, OUT>; }
    // workgroups of this kernel that are resident at once on the current device (-1: HIP error)
    static int slots() {
        const int cus = prepare_kernel(reinterpret_cast<const void *>(kernel()), lds, state());
        if (cus < 0) return -1;
        const int occ = resident_per_cu(reinterpret_cast<const void *>(kernel()), WM * WN * 64, lds, state());
        return occ < 0 ? -1 : cus * occ;
    }
};

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    using L = PipeLaunch<FM, FN, WM, WN, OCC, OUT>;
    g.tiles_m = (g.M + L::BM - 1) / L::BM;
    g.tiles_n = (g.N + L::BN - 1) / L::BN;
    if (prepare_kernel(reinterpret_cast<const void *>(L::kernel()), L::lds, L::state()) < 0) return W4A4_ERR_HIP;
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (OUT == OUT_Q4) {
        // the column tiles of a row panel wait for each other: the whole grid has to be resident
        const int slots = L::slots();
        if (slots < 0) return W4A4_ERR_HIP;
        if (tiles > slots) return W4A4_ERR_UNSUPPORTED_SHAPE;
        if (g.wait_for == 0) g.wait_for = g.tiles_n;
    }
    launch_gemm(L::kernel(), dim3((unsigned)tiles), dim3(WM * WN * 64), L::lds, st, g);
    return launch_status();
}

// Tiles (128 x 256) that the fused requantize of the pipelined kernel may use on the current device: its whole
// grid has to be resident (-1 = HIP error).
int pipe_requant_max_tiles() { return PipeLaunch<2, 4, 2, 2, 2, OUT_Q4>::slots(); }

template <int OUT>
static int launch_variant(int variant, GemmArgs &g, hipStream_t st) {
    switch (variant) {
        case 0: return launch_one<2, 4, 2, 2, 2, OUT>(g, st);   // 128 x 256, two workgroups per CU
        case 1: return launch_one<3, 2, 2, 2, 2, OUT>(g, st);   // 192 x 128, two workgroups per CU
        default: return W4A4_ERR_INVALID_ARG;
    }
}

// Requires: symmetric codes, per-channel weight scales, K % 128 == 0, M*lda and N*ldw < 2^31.
int launch_pipe(int variant, int out_kind, GemmArgs &g, hipStream_t st) {
    if (out_kind == OUT_Q4)                                     // fused requantize: the 128 x 256 tile only
        return variant == 0 ? launch_one<2, 4, 2, 2, 2, OUT_Q4>(g, st) : W4A4_ERR_INVALID_ARG;
    switch (out_kind) {
        case OUT_F16: return launch_variant<OUT_F16>(variant, g, st);
        case OUT_F32: return launch_variant<OUT_F32>(variant, g, st);
        default: return launch_variant<OUT_I32>(variant, g, st);
    }
}

}  // namespace w4a4
