// Persistent INT8 x INT8 -> INT32 GEMM with the fused symmetric epilogue: the INT8 sibling of the
// INT4 path (the pipeline the paper measures INT4 against, Sec. 4.1 / 4.3).  On gfx950 both run on the
// same int8 MFMA, so this kernel is gemm_olay.hip with the nibble handling taken out:
//   * same persistent skeleton: HBM -> LDS by `buffer_load_dwordx4 ... lds` with scalar addressing, three
//     LDS stages of 64-byte rows with the XOR swizzle, the K steps of successive tiles as one stream, one
//     barrier per K step, two workgroups of four waves per CU, priority alternation, non-temporal stores;
//   * a K step is 64 codes (64 bytes per row, where the INT4 kernel moves 128 codes in the same bytes):
//     a 16-byte LDS read IS an MFMA operand, so there is no widening VALU work at all, but twice the
//     LDS reads, DMA instructions and barriers per MFMA;
//   * no code-sum corrections: the accumulators hold P itself.
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int kW8Step = 64;                                       // codes (= bytes) per row per K step

// s_waitcnt immediate for "vmcnt <= n", lgkmcnt and expcnt unconstrained (gfx9 encoding)
constexpr int w8_vmcnt_only(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | (((n >> 4) & 0x3) << 14); }

template <int FN>
struct W8Chan {
    float sw[FN];
    float bias[FN];
};

// Epilogue of one wave: y = ((float)P * sa[m]) * sw[n] (+ bias[n]) (GELU), each operation separately
// rounded; int32 export for parity.
template <int FM, int FN, int OUT, bool BIAS, bool GELU>
__device__ __forceinline__ void w8_epilogue(const GemmArgs &g, v16i (&acc)[FM][FN], const W8Chan<FN> &cp,
                                            uint32_t col_off, int m0, int row_w, int lane, const float *sa_lds) {
    constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
    const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * g.N * ESZ));
    const uint32_t row_bytes = (uint32_t)g.N * ESZ;
    const uint32_t lane_off = (uint32_t)(m0 + row_w + 4 * (lane >> 5)) * row_bytes + col_off;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rl = row_w + i * 32 + 8 * q + 4 * (lane >> 5);          // 4 consecutive rows
            const float4 sa4 = *reinterpret_cast<const float4 *>(sa_lds + rl);
            const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = q * 4 + rr;
                const uint32_t off = lane_off + (uint32_t)(i * 32 + 8 * q + rr) * row_bytes;
                if constexpr (OUT == OUT_I32) {
                    uint32_t w[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) w[j] = (uint32_t)acc[i][j][r];
                    store_words<FN, kStreamed>(o_rsrc, off, w);
                } else {
                    float y[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        float t = (float)acc[i][j][r] * sav[rr];
                        y[j] = t * cp.sw[j];
                        if constexpr (BIAS) y[j] = y[j] + cp.bias[j];
                    }
                    if constexpr (GELU) store_gelu_halves<FN, kStreamed>(o_rsrc, off, y);
                    else store_halves<FN, kStreamed>(o_rsrc, off, y);
                }
            }
        }
}

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_w8_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    constexpr int ROWB = kW8Step;                               // 64 bytes = 64 codes per row per K step
    constexpr int STAGE = (BM + BN) * ROWB, NS = 3;
    constexpr int BLOCKS = (BM + BN) / 16;                      // 1 KB DMA blocks per stage
    constexpr int LD = BLOCKS / NW;                             // tile DMA instructions per wave per K step
    constexpr int A_LD = (BM / 16) / NW;                        // the first A_LD of them fetch activations
    constexpr int NF = FM + FN, NM = FM * FN;
    constexpr int PB = BM / 64;                                 // 64-row blocks of token scales
    static_assert(BLOCKS % NW == 0 && (BM / 16) % NW == 0, "DMA blocks must split evenly over the waves");
    static_assert(NF <= NM && LD <= NM, "not enough MFMA slots to hide the memory operations");
    static_assert(BM % 64 == 0, "token parameters are fetched 64 rows per DMA instruction");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    // token scales of the tile, double buffered by tile parity: [2][ sa[BM] ]
    uint8_t *par = smem + NS * STAGE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int total = g.tiles_m * g.tiles_n, stride = gridDim.x;
    const int KT = g.K / kW8Step;

    // ---- global -> LDS plan (fixed for the whole kernel) -------------------------------------------
    // DMA instruction i of this wave fills block b = wave + i*NW of a stage: tile rows 16b..16b+15.
    // Lane l supplies physical slot (r = l>>2, pc = l&3) of the block = logical chunk pc ^ ((row>>2)&3).
    int voff[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int row = (wave + i * NW) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        if (i < A_LD) {
            voff[i] = row * (int)g.lda + c * 16;
        } else {
            // LDS row p of the weight tile holds output channel nl: MFMA column cc of fragment f
            // is channel cc*FN + f of the wave's span, so a lane ends up with FN adjacent channels.
            const int p = row - BM;
            const int w = p / (FN * 32), rem = p % (FN * 32), f = rem / 32, cc = rem % 32;
            const int nl = w * (FN * 32) + cc * FN + f;
            voff[i] = nl * (int)g.ldw + c * 16;
        }
    }
    // Descriptors of a tile: base at the tile origin, size = its valid rows.
    auto a_desc = [&](int m0) {
        const int rows = min(BM, g.M - m0);
        return make_rsrc(g.Aq + (long)m0 * g.lda, (uint32_t)((long)(rows - 1) * g.lda + g.K));
    };
    auto b_desc = [&](int n0) {
        const int rows = min(BN, g.N - n0);
        return make_rsrc(g.Wq + (long)n0 * g.ldw, (uint32_t)((long)rows * g.ldw));
    };
    auto dma_one = [&](int i, int stage, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, int so) {
        uint8_t *dst = smem + stage * STAGE + (wave + i * NW) * 1024;
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature; it rejects the LDS cast
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LD ? ra : rb, (lds_ptr_t)dst, 16, voff[i], so, 0, 0);
#else
        (void)dst; (void)ra; (void)rb; (void)so;
#endif
    };
    // Token scales by 4-byte DMA: waves [0, PB) fetch 64 scales each.
    const __amdgpu_buffer_rsrc_t sa_rsrc = make_rsrc(g.sa, (uint32_t)g.M * 4u);
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(g.sw, (uint32_t)g.N * 4u);
    const __amdgpu_buffer_rsrc_t bias_rsrc = make_rsrc(g.bias, g.bias ? (uint32_t)g.N * 2u : 0u);   // no bias: zeros
    auto dma_params = [&](int m0, int parity) {
        if (wave < PB) {
            uint8_t *dst = par + parity * (BM * 4) + wave * 256;
            const int vo = (m0 + wave * 64 + lane) * 4;
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(sa_rsrc, (lds_ptr_t)dst, 4, vo, 0, 0, 0);
#else
            (void)dst; (void)vo;
#endif
        }
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
    auto read_frag = [&](int f, int stage, int ks) {              // 16 bytes = the int8 operand of one MFMA
        return *reinterpret_cast<const v4i *>(smem + stage * STAGE + (frag_off[f] ^ (ks << 5)));
    };

    v16i acc[FM][FN];                                           // written by the first K step of every tile

    // ---- first tile: its first two K steps and parameters --------------------------------------------
    // Tile of virtual block id vb (workgroup id + k * grid size; vb % 8 = the XCD it runs on): every XCD
    // owns a contiguous range of tiles, so that the tiles of a row panel run on one XCD and share its L2.
    auto tile_of = [&](int v, int &t) {
        t = xcd_tile(v < total ? v : 0, total);
        return v < total;
    };
    int vb = blockIdx.x;                                        // virtual block id of the current tile
    int tile;
    if (!tile_of(vb, tile)) return;                             // (uniform) nothing to do for this workgroup
    int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    __amdgpu_buffer_rsrc_t a_cur = a_desc(m0), b_cur = b_desc(n0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 0, a_cur, b_cur, 0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 1, a_cur, b_cur, ROWB);
    dma_params(m0, 0);
    __builtin_amdgcn_s_waitcnt(w8_vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    v4i P0[NF], P1[NF];

    int cur = 0;                                                // LDS stage of the current K step
    int parity = 0;
    for (;;) {
        // first fragments of the tile (its first two K steps are in LDS and published)
#pragma unroll
        for (int f = 0; f < NF; ++f) P0[f] = read_frag(f, cur, 0);
        // ---- tile start: channel constants, origin of the next tile ------------------------------------
        // channel constants of this lane's FN adjacent channels: raw loads now (channels past N read
        // as zero), converted when the epilogue starts
        const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;
        static_assert(FN == 4 || FN == 2, "channel constants are fetched two or four at a time");
        u32x4 sw_raw;
        u32x2 bias_raw;
        if constexpr (FN == 4) {
            sw_raw = __builtin_amdgcn_raw_buffer_load_b128(sw_rsrc, n_lane * 4, 0, 0);
            bias_raw = __builtin_amdgcn_raw_buffer_load_b64(bias_rsrc, n_lane * 2, 0, 0);
        } else {
            const u32x2 s2 = __builtin_amdgcn_raw_buffer_load_b64(sw_rsrc, n_lane * 4, 0, 0);
            sw_raw = u32x4{s2[0], s2[1], 0, 0};
            bias_raw = u32x2{__builtin_amdgcn_raw_buffer_load_b32(bias_rsrc, n_lane * 2, 0, 0), 0};
        }
        const int vb_next = vb + stride;
        int tile_next;
        const bool has_next = tile_of(vb_next, tile_next);
        if (!has_next) tile_next = tile;
        const int m0n = (tile_next / g.tiles_n) * BM, n0n = (tile_next % g.tiles_n) * BN;
        const __amdgpu_buffer_rsrc_t a_nxt = a_desc(m0n), b_nxt = b_desc(n0n);

        // ---- main loop: one iteration = 64 codes of K = two sub-steps of NM MFMAs ------------------------
        // The instruction order below is the intended issue order; the scheduling barriers keep the
        // compiler from regrouping it.  The operands need no widening: a 16-byte LDS read is an operand.
#define W8_SLOT(P, k)                                                                                     \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(P[(k) / FN], P[FM + (k) % FN],         \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        // the first MFMA into an accumulator of a tile takes a zero C operand (an inline constant)
#define W8_SLOT_ZERO(P, k)                                                                                \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(P[(k) / FN], P[FM + (k) % FN],         \
                                                                   v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);
        constexpr int kBarSlot = NM - NF;                      // LDS reads of the next stage start here
        auto k_step = [&](auto first_tag, auto last_tag, int kt) {
            constexpr bool FIRST = decltype(first_tag)::value; // first K step of the tile
            constexpr bool LAST = decltype(last_tag)::value;   // last K step of the tile
            const int nxt = cur == NS - 1 ? 0 : cur + 1;       // stage of stream step +1
            const int nx2 = nxt == NS - 1 ? 0 : nxt + 1;       // stage of stream step +2 (= step -1)
            // stream step +2 is K step kt+2 of this tile, or K step kt+2-KT of the next one (when there
            // is none: a harmless in-bounds re-read, so that the load counting stays uniform)
            const bool own = !LAST && kt + 2 < KT;
            const __amdgpu_buffer_rsrc_t ra = own ? a_cur : a_nxt, rb = own ? b_cur : b_nxt;
            const int so = (own ? kt + 2 : kt + 2 - KT) * ROWB;
            // sub-step 0: multiply codes 0..31 of the step; fetch codes 32..63 -> P1; request stream step +2
            //             into the stage every wave finished reading before the last barrier.
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                if constexpr (FIRST) { W8_SLOT_ZERO(P0, k) } else { W8_SLOT(P0, k) }
                if (k < NF) P1[k] = read_frag(k, cur, 1);
                if (k < LD) dma_one(k, nx2, ra, rb, so);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 1: multiply codes 32..63; this wave's loads of stream step +1 have landed (vmcnt), and
            //             after the barrier everyone's have: fetch its codes 0..31 -> P0.  At the end of a tile
            //             BOTH prefetched steps of the next tile are waited for; the next tile reads its first
            //             fragments itself.
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W8_SLOT(P1, k)
                if (k == kBarSlot) {
                    __builtin_amdgcn_s_waitcnt(w8_vmcnt_only(LAST ? 0 : LD));
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                }
                if (!LAST && k >= kBarSlot) P0[k - kBarSlot] = read_frag(k - kBarSlot, nxt, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
        };
        k_step(std::true_type{}, std::false_type{}, 0);
        // every wave has passed a barrier of this tile, so nobody reads the previous tile's parameters
        // any more: fetch the next tile's into that buffer (complete at this tile's last barrier)
        dma_params(m0n, parity ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        for (int kt = 1; kt < KT - 1; ++kt) k_step(std::false_type{}, std::false_type{}, kt);
        k_step(std::false_type{}, std::true_type{}, KT - 1);
#undef W8_SLOT
#undef W8_SLOT_ZERO

        // ---- epilogue of this tile ------------------------------------------------------------------
        {
            constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
            const uint32_t col_off = n_lane < g.N ? (uint32_t)n_lane * ESZ : kPoison;
            W8Chan<FN> cp;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                cp.sw[j] = __uint_as_float(sw_raw[j]);
                const uint32_t b2 = bias_raw[j >> 1];
                cp.bias[j] = __half2float(__ushort_as_half((unsigned short)((j & 1) ? b2 >> 16 : b2 & 0xFFFFu)));
            }
            const float *sa_lds = reinterpret_cast<const float *>(par + parity * (BM * 4));
            const int row_w = wm * FM * 32;
            const bool bias = g.bias != nullptr, gelu = g.act == W4A4_ACT_GELU;
            if (OUT == OUT_I32 || (!bias && !gelu)) w8_epilogue<FM, FN, OUT, false, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (bias && !gelu) w8_epilogue<FM, FN, OUT, true, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (!bias && gelu) w8_epilogue<FM, FN, OUT, false, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else w8_epilogue<FM, FN, OUT, true, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
        }
        if (!has_next) break;
        vb = vb_next; tile = tile_next; m0 = m0n; n0 = n0n; a_cur = a_nxt; b_cur = b_nxt; parity ^= 1;
    }
    __builtin_amdgcn_s_waitcnt(w8_vmcnt_only(0));                  // no DMA may outlive the workgroup's LDS
}


template <int FM, int FN, int WM, int WN, int OCC, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    constexpr size_t lds = 3 * (size_t)(BM + BN) * kW8Step + 2 * BM * 4;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_w8_kernel<FM, FN, WM, WN, OCC, OUT>;
    static KernelState ks;
    const int cus = prepare_kernel(reinterpret_cast<const void *>(kern), lds, ks);
    if (cus < 0) return W4A4_ERR_HIP;
    const int slots = cus * OCC;                                // workgroups that are resident at once on this device
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const unsigned grid = (unsigned)(tiles < slots ? tiles : slots);
    launch_gemm(kern, dim3(grid), dim3(WM * WN * 64), lds, st, g);
    return launch_status();
}

bool small8_ok(const GemmArgs &g);                              // gemm_small.hip: the split-K kernel for small problems
int launch_small_packed8(int out_kind, GemmArgs &g, hipStream_t st);

// Tile choice as for the INT4 kernel: the largest number of tiles any CU ends up with times the tile area.
// A few hundred 32 x 32 tiles at most go to the small-problem kernel instead (latency decides there).
static int launch_w8(int out_kind, GemmArgs &g, hipStream_t st) {
    if (small8_ok(g)) return launch_small_packed8(out_kind, g, st);
    const long cus = 256;
    auto cost = [&](int bm, int bn) {
        const long tiles = (long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn);
        return (double)((tiles + cus - 1) / cus) * bm * bn;
    };
    const bool wide = cost(128, 256) <= cost(192, 128);
    if (out_kind == OUT_I32)
        return wide ? launch_one<2, 4, 2, 2, 2, OUT_I32>(g, st) : launch_one<3, 2, 2, 2, 2, OUT_I32>(g, st);
    return wide ? launch_one<2, 4, 2, 2, 2, OUT_F16>(g, st) : launch_one<3, 2, 2, 2, 2, OUT_F16>(g, st);
}

}  // namespace w4a4

using namespace w4a4;

static int w8_check(const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw, int N, int K,
                    const void *out) {
    if (M < 0 || N <= 0 || K <= 0 || lda < K) return W4A4_ERR_INVALID_ARG;
    if (K % kW8Step || K < 2 * kW8Step || N % 8 || lda % 16) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return W4A4_OK;
    if (!Aq || !sa || !Wq || !sw || !out) return W4A4_ERR_INVALID_ARG;
    if (!aligned16(Aq) || !aligned16(Wq) || !aligned16(out)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    if ((long)M * lda >= 0x7fffffffL || (long)N * K >= 0x7fffffffL || ((long)M + 512) * N * 4 >= 0x80000000L)
        return W4A4_ERR_UNSUPPORTED_SHAPE;
    return W4A4_OK;
}

static void w8_fill(GemmArgs &g, const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw,
                    int N, int K) {
    g = GemmArgs{};
    g.Aq = reinterpret_cast<const uint8_t *>(Aq); g.lda = lda;
    g.Wq = reinterpret_cast<const uint8_t *>(Wq); g.ldw = K;
    g.M = M; g.N = N; g.K = K; g.ng = 1; g.steps_per_group = K / kW8Step;
    g.sa = sa; g.sw = sw; g.act = W4A4_ACT_NONE;
}

extern "C" int w8a8_linear(const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw,
                           int N, int K, const w4a4_epilogue *ep, void *out, void *stream) {
    if (!ep || (ep->act != W4A4_ACT_NONE && ep->act != W4A4_ACT_GELU)) return W4A4_ERR_INVALID_ARG;
    if (ep->requant) return W4A4_ERR_UNSUPPORTED_SHAPE;
    int rc = w8_check(Aq, lda, sa, M, Wq, sw, N, K, out);
    if (rc || M == 0) return rc;
    if (ep->bias_f16 && !aligned16(ep->bias_f16)) return W4A4_ERR_UNSUPPORTED_SHAPE;
    GemmArgs g;
    w8_fill(g, Aq, lda, sa, M, Wq, sw, N, K);
    g.bias = static_cast<const __half *>(ep->bias_f16);
    g.act = ep->act;
    g.out = out;
    return launch_w8(OUT_F16, g, as_stream(stream));
}

extern "C" int w8a8_gemm_i32(const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw,
                             int N, int K, int32_t *acc, void *stream) {
    int rc = w8_check(Aq, lda, sa, M, Wq, sw, N, K, acc);
    if (rc || M == 0) return rc;
    GemmArgs g;
    w8_fill(g, Aq, lda, sa, M, Wq, sw, N, K);
    g.out = acc;
    return launch_w8(OUT_I32, g, as_stream(stream));
}
