// Pipelined INT4 x INT4 -> INT32 GEMM with direct global->LDS loads (symmetric codes,
// per-channel weight scales, K a multiple of 128).
//
// Same arithmetic as gemm_pipe.hip (packed codes in HBM and LDS, widened to int8 in registers
// right before v_mfma_i32_32x32x32_i8, fused epilogue) but the tiles never pass through
// vector registers on their way to LDS:
//   * `buffer_load_dwordx4 ... lds` writes 16 bytes per lane straight into LDS (a wave fills
//     1 KB = 16 tile rows of 64 bytes per instruction).  That removes the LDS-write
//     instructions (which hold the SIMD's register ports while they read 128-bit data), the
//     staging registers and the load->store dependency from the main loop.
//   * LDS rows are unpadded (the DMA writes contiguously); bank conflicts are avoided by an XOR
//     swizzle instead: physical 16-byte slot pc of row r holds logical chunk pc ^ ((r>>2)&3).
//     The global address of each lane is chosen accordingly, the fragment reads undo it.
//   * Three LDS stages of one K step (128 codes) each: the tile of step t+2 is requested while
//     step t is multiplied; a wave waits (vmcnt) only for its own loads of step t+1 right
//     before the one workgroup barrier of the step.
//   * Two workgroups per CU (2 x 72 KB of LDS), four waves of 64 x 128 each.
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt immediate for "vmcnt <= n and lgkmcnt == 0", expcnt unconstrained (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 0xF) | (0x7 << 4) | (0x0 << 8) | (((n >> 4) & 0x3) << 14); }

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_dma_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NT = WM * WN * 64, NW = WM * WN;
    constexpr int ROWB = kBK / 2;                               // 64 bytes of codes per row per K step
    constexpr int STAGE = (BM + BN) * ROWB, NS = 3;
    constexpr int BLOCKS = (BM + BN) / 16;                      // 1 KB DMA blocks per stage
    constexpr int LD = BLOCKS / NW;                             // DMA instructions per wave per K step
    constexpr int A_LD = (BM / 16) / NW;                        // the first A_LD of them fetch activations
    constexpr int NF = FM + FN, NM = FM * FN;
    static_assert(BLOCKS % NW == 0 && (BM / 16) % NW == 0, "DMA blocks must split evenly over the waves");
    static_assert(NF <= NM && LD <= NM, "not enough MFMA slots to hide the memory operations");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    float *sa_lds = reinterpret_cast<float *>(smem + NS * STAGE);      // per-token scales of the tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tile = xcd_tile(blockIdx.x, g.tiles_m * g.tiles_n);
    const int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    const int KT = g.K / kBK;

    // ---- global -> LDS plan ---------------------------------------------------------------------
    // DMA instruction i of this wave fills block b = wave + i*NW of the stage: tile rows 16b..16b+15.
    // Lane l supplies physical slot (r = l>>2, pc = l&3) of the block = logical chunk pc ^ ((row>>2)&3).
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.Aq, (uint32_t)((long)(g.M - 1) * g.lda + g.K / 2));
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(g.Wq, (uint32_t)((long)g.N * g.ldw));
    int voff[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int row = (wave + i * NW) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        if (i < A_LD) {
            voff[i] = (m0 + row) * (int)g.lda + c * 16;          // rows >= M fall outside the buffer: zeros
        } else {
            // LDS row p of the weight tile holds output channel nl: MFMA column cc of fragment f
            // is channel cc*FN + f of the wave's span.
            const int p = row - BM;
            const int w = p / (FN * 32), rem = p % (FN * 32), f = rem / 32, cc = rem % 32;
            const int nl = w * (FN * 32) + cc * FN + f;
            voff[i] = (n0 + nl) * (int)g.ldw + c * 16;
        }
    }
    // K offset of step kt; past the end the last step is re-read (in bounds, never used)
    auto k_off = [&](int kt) { return (kt < KT ? kt : KT - 1) * ROWB; };
    auto dma_one = [&](int i, int stage, int so) {
        uint8_t *dst = smem + stage * STAGE + (wave + i * NW) * 1024;
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature; it rejects the LDS cast
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LD ? a_rsrc : b_rsrc, (lds_ptr_t)dst, 16, voff[i], so, 0, 0);
#else
        (void)dst; (void)so;
#endif
    };

    // ---- operand fragments -----------------------------------------------------------------------
    // lane (r = lane&31, h = lane>>5) reads logical chunk ks*2 + h of its row
    const int swz = ((lane & 31) >> 2) & 3;
    const int rd0 = (lane & 31) * ROWB + (((lane >> 5) ^ swz) << 4);   // ks = 0;  ks = 1 is rd0 ^ 32
    int frag_off[NF];
#pragma unroll
    for (int f = 0; f < FM; ++f) frag_off[f] = (wm * FM * 32 + f * 32) * ROWB + rd0;
#pragma unroll
    for (int f = 0; f < FN; ++f) frag_off[FM + f] = (BM + wn * FN * 32 + f * 32) * ROWB + rd0;
    auto read_frag = [&](int f, int stage, int ks) {
        return *reinterpret_cast<const u32x4 *>(smem + stage * STAGE + (frag_off[f] ^ (ks << 5)));
    };

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    // Workgroup barrier that publishes the DMA-written stage: the wave first waits until at most
    // LD of its own DMA loads are outstanding (they complete in order, so the older stage has
    // landed) and its LDS operations have drained.  A release fence is deliberately not used
    // here: it would wait for ALL outstanding DMA loads, including the stage requested last.
    auto dma_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(LD));
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
    for (int i = 0; i < LD; ++i) dma_one(i, 0, k_off(0));
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 1, k_off(1));
    dma_barrier();                                              // step 0 has landed (step 1 may be in flight)
#pragma unroll
    for (int f = 0; f < NF; ++f) P0[f] = read_frag(f, 0, 0);
#pragma unroll
    for (int f = 0; f < NF; ++f) U0[f] = widen2<true>(P0[f].x, P0[f].y);

    // ---- main loop ---------------------------------------------------------------------------------
    // One iteration = 128 codes of K = four sub-steps of NM MFMAs.  The instruction order below
    // is the intended issue order; the scheduling barriers keep the compiler from regrouping it.
    // Slot k of a sub-step issues MFMA k and, behind it, the widening of fragment k for the
    // NEXT sub-step plus at most one LDS read and one DMA request.
#define W4A4_SLOT_BEGIN(Ucur, k)                                                                          \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ucur[(k) / FN], Ucur[FM + (k) % FN],   \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
    constexpr int kBarSlot = NM - NF;                          // LDS reads of the next stage start here
    int cur = 0;                                               // stage of step kt
    for (int kt = 0; kt < KT; ++kt) {
        const int nxt = cur == NS - 1 ? 0 : cur + 1;           // stage of step kt+1
        const int nx2 = nxt == NS - 1 ? 0 : nxt + 1;           // stage of step kt+2 (= stage of step kt-1)
        const int so = k_off(kt + 2);
        // sub-step 0: multiply (ks 0, low); widen (ks 0, high) -> U1; fetch ks 1 -> P1; request
        //             step kt+2 into the stage every wave finished reading before the last barrier.
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U0, k)
            if (k < NF) U1[k] = widen2<true>(P0[k].z, P0[k].w);
            if (k < NF) P1[k] = read_frag(k, cur, 1);
            if (k < LD) dma_one(k, nx2, so);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 1: multiply (ks 0, high); widen (ks 1, low) -> U0
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U1, k)
            if (k < NF) U0[k] = widen2<true>(P1[k].x, P1[k].y);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 2: multiply (ks 1, low); widen (ks 1, high) -> U1; this wave's loads of step
        //             kt+1 have landed (vmcnt), and after the barrier everyone's have: fetch its ks 0.
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U0, k)
            if (k < NF) U1[k] = widen2<true>(P1[k].z, P1[k].w);
            if (k == kBarSlot) dma_barrier();
            if (k >= kBarSlot) P0[k - kBarSlot] = read_frag(k - kBarSlot, nxt, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // sub-step 3: multiply (ks 1, high); widen (next step's ks 0, low) -> U0
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            W4A4_SLOT_BEGIN(U1, k)
            if (k < NF) U0[k] = widen2<true>(P0[k].x, P0[k].y);
            __builtin_amdgcn_sched_barrier(0);
        }
        cur = nxt;
    }
#undef W4A4_SLOT_BEGIN
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                  // no DMA may outlive the workgroup's LDS

    // ---- epilogue ---------------------------------------------------------------------------------
    float none[1][1][16];
    tile_epilogue<FM, FN, W4A4_SYM, false, OUT>(g, acc, none, epi, m0, wm * FM * 32, lane, sa_lds, nullptr);
}

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = 3 * (size_t)(BM + BN) * (kBK / 2) + BM * sizeof(float);
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_dma_kernel<FM, FN, WM, WN, OCC, OUT>;
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

// Requires: symmetric codes, per-channel weight scales, K % 128 == 0, M*lda and N*ldw < 2^31.
int launch_dma(int variant, int out_kind, GemmArgs &g, hipStream_t st) {
    switch (out_kind) {
        case OUT_F16: return launch_variant<OUT_F16>(variant, g, st);
        case OUT_F32: return launch_variant<OUT_F32>(variant, g, st);
        default: return launch_variant<OUT_I32>(variant, g, st);
    }
}

}  // namespace w4a4
