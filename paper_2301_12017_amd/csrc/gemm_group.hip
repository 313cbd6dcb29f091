// Persistent INT4 x INT4 -> INT32 GEMM for K-grouped and / or asymmetric layers (canonical
// codes, weight groups that are multiples of 128 along K, K >= 256).
//
// Sec. 4.3 notes that the asymmetric mapping costs extra "bias term" work; with weight K-groups
// (App. A) the work is larger still, because the int32 sums of every group have to be scaled by
// that group's weight scale before they may be added up:
//     t1[m,n] = sum_g sw[n,g] * (float)P_g[m,n],      P_g = sum_{k in g} qa[m,k] * qw[n,k]
//     y       = sa[m]*t1 + sa[m] * sum_g zw[n,g]*(float)RA[m,g] + za[m]*c[n] + bias[n]
// (every operation separately rounded, groups in ascending order).  That is three vector-ALU
// instructions per accumulator and group for t1 and two for the zero-point sum, far more than
// the MFMAs of a 128-code group leave room for, so this kernel is bound by the vector ALU and
// is built to keep everything else off it:
//   * tiles travel HBM -> LDS by `buffer_load_dwordx4 ... lds` with scalar addressing, unpadded
//     LDS rows with an XOR swizzle, three LDS stages, persistent workgroups whose K steps form
//     one stream across tiles (as in gemm_olay.hip);
//   * the first MFMA of a group takes a zero C operand, so accumulators are never cleared;
//   * token scales / zero points, and for asymmetric layers the group tables zw[g][n] and
//     RA[g][m] of the tile, go to LDS by 4-byte DMA at the start of the tile; a group's weight
//     scales are fetched into two registers when the group starts;
//   * 128 x 128 tiles, four waves of 64 x 64 (64 integer + 64 fp32 accumulators per lane), two
//     workgroups per CU so that one's group folds overlap the other's MFMAs.
// Symmetric grouped layers run here too (signed codes are widened to 16*code, so the sums carry
// a factor 256 that the group scale absorbs exactly).
//
// OLAY = true is the same kernel on unsigned codes kept in the MFMA operand layout (see w4a4_layout), built to
// take vector-ALU work out of it:
//   * one v_and per operand register instead of a shift and a mask (activations: low nibble u, high nibble
//     u - 8; weights: nibbles swapped).  A group's accumulator then holds 16*(P_g - 8*AE[m,g] - 8*WO[n,g]) with AE
//     the token's even-position code sum and WO the channel's odd-position code sum of the group.  The token term
//     costs nothing: 128*AE[m,g] arrives with the group's K step in LDS (one 4-byte DMA per row, the array is kept
//     group-major for that) and is the C operand of the group's first MFMAs, shared by the column fragments.  The
//     channel term is a constant per channel over all groups, 8 * sum_g sw[n,g]*WO[n,g], precomputed with the
//     weights; the fp32 accumulators start from it.
//   * the fold is a conversion and ONE fused multiply-add per accumulator and group,
//     t1 = fma(sw[n,g]/16, (float)acc, t1), and the zero-point sum, the token scale, the zero-point product and
//     the bias are fused multiply-adds as well:  y = fma(sa, fma-chain(zw[n,g], RA[m,g], t1), fma(za, c[n], b[n])).
//   The result is the same real number as the definition's, evaluated with fewer roundings and in another
//   order; fp32 rounding noise of the large cancelling terms of the unsigned mapping is of the same size in both
//   (a few units of 2^-24 * |sa * t1|), so fp16 outputs agree to that noise, not bit for bit.  The int32 planes
//   (OUT_I32) are exact: P_g = (acc + 128*WO[n,g]) / 16.
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt immediate for "vmcnt <= n", lgkmcnt and expcnt unconstrained (gfx9 encoding)
static constexpr int vmcnt_only(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | (((n >> 4) & 0x3) << 14); }

template <int MODE, int OUT, bool OLAY, bool SPG1>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void gemm_group_kernel(GemmArgs g) {
    static_assert(!OLAY || MODE == W4A4_ASYM, "the symmetric operand layout has its own kernel");
    constexpr bool SGN = MODE == W4A4_SYM;
    constexpr int FM = 2, FN = 2, WM = 2, WN = 2;
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    constexpr int ROWB = kBK / 2;                               // 64 bytes of codes per row per K step
    constexpr int CODES = (BM + BN) * ROWB;                     // code bytes of a stage
    constexpr int STAGE = CODES + (OLAY ? BM * 4 : 0), NS = 3; // OLAY: + the step's column of 128*AE, one word per row
    constexpr int LD = (BM + BN) / 16 / NW;                     // tile DMA instructions per wave per K step
    constexpr int LDT = LD + (OLAY ? 1 : 0);                    // ... the token-sum column included
    constexpr int A_LD = (BM / 16) / NW;                        // the first A_LD of them fetch activations
    constexpr int NF = FM + FN, NM = FM * FN;
    static_assert(NF <= NM && LD <= NM, "not enough MFMA slots to hide the memory operations");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    uint8_t *par = smem + NS * STAGE;                           // [2 parities][ sa[BM] | za[BM] ]
    float *zw_tab = reinterpret_cast<float *>(par + 2 * 2 * BM * 4);          // [ng][BN]   (ASYM)
    int *ra_tab = reinterpret_cast<int *>(zw_tab + (size_t)g.ng * BN);         // [ng][BM]   (ASYM)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int total = g.tiles_m * g.tiles_n, stride = gridDim.x;
    const int KT = g.K / kBK, spg = g.steps_per_group;

    // ---- global -> LDS plan (fixed for the whole kernel) -------------------------------------------
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
    auto a_desc = [&](int m0) {
        const int rows = min(BM, g.M - m0);
        return make_rsrc(g.Aq + (long)m0 * g.lda, (uint32_t)((long)(rows - 1) * g.lda + g.K / 2));
    };
    auto b_desc = [&](int n0) {
        const int rows = min(BN, g.N - n0);
        return make_rsrc(g.Wq + (long)n0 * g.ldw, (uint32_t)((long)rows * g.ldw));
    };
    auto dma4 = [&](__amdgpu_buffer_rsrc_t rs, void *dst, int vo, int so = 0) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature; it rejects the LDS cast
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)dst, 4, vo, so, 0, 0);
#else
        (void)rs; (void)dst; (void)vo; (void)so;
#endif
    };
    // OLAY: the token sums 128*AE, kept group-major [ng][M], so that the column of one group is contiguous
    const __amdgpu_buffer_rsrc_t ae_rsrc = make_rsrc(g.osum, OLAY ? (uint32_t)((long)g.ng * g.M * 4) : 0u);
    auto dma_one = [&](int i, int stage, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, int so) {
        uint8_t *dst = smem + stage * STAGE + (wave + i * NW) * 1024;
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LD ? ra : rb, (lds_ptr_t)dst, 16, voff[i], so, 0, 0);
#else
        (void)dst; (void)ra; (void)rb; (void)so;
#endif
    };
    // the token-sum column of K step `kt` of the tile whose first row is m0: every wave fetches the 64 rows of its
    // half of the tile (two waves fetch each half: same words to the same place, so that all waves issue the same
    // number of loads per K step and one wait count fits all)
    auto dma_col = [&](int stage, int m0, int kt) {
        if constexpr (OLAY)
            dma4(ae_rsrc, smem + stage * STAGE + CODES + wm * 256, (wm * 64 + lane) * 4, ((SPG1 ? kt : kt / spg) * g.M + m0) * 4);
    };
    const __amdgpu_buffer_rsrc_t sa_rsrc = make_rsrc(g.sa, (uint32_t)g.M * 4u);
    const __amdgpu_buffer_rsrc_t za_rsrc = make_rsrc(g.za, MODE == W4A4_ASYM ? (uint32_t)g.M * 4u : 0u);
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(g.sw, (uint32_t)((long)g.N * g.ng * 4));
    const __amdgpu_buffer_rsrc_t zw_rsrc = make_rsrc(g.zw, MODE == W4A4_ASYM ? (uint32_t)((long)g.N * g.ng * 4) : 0u);
    const __amdgpu_buffer_rsrc_t ra_rsrc = make_rsrc(g.RA, MODE == W4A4_ASYM ? (uint32_t)((long)g.M * g.ng * 4) : 0u);
    const __amdgpu_buffer_rsrc_t c_rsrc = make_rsrc(g.c, MODE == W4A4_ASYM ? (uint32_t)g.N * 4u : 0u);
    const __amdgpu_buffer_rsrc_t bias_rsrc = make_rsrc(g.bias, g.bias ? (uint32_t)g.N * 2u : 0u);   // no bias: zeros
    // OLAY: per channel ng odd-position code sums WO and one fp32 word, 8 * sum_g sw*WO
    const __amdgpu_buffer_rsrc_t wo_rsrc = make_rsrc(g.esum, OLAY ? (uint32_t)((long)g.N * (g.ng + 1) * 4) : 0u);
    // Token parameters and group tables of a tile, 64 values per DMA instruction, dealt round robin to
    // the waves: blocks [0,2) scales, [2,4) zero points, then per group two blocks of zw and two of RA.
    auto dma_params = [&](int m0, int n0, int parity) {
        const int nblk = MODE == W4A4_ASYM ? 4 + 4 * g.ng : 2;
        for (int b = wave; b < nblk; b += NW) {
            const int half = b & 1;
            if (b < 4) {
                const bool is_sa = b < 2;
                const int m = m0 + half * 64 + lane;
                dma4(is_sa ? sa_rsrc : za_rsrc, par + parity * (2 * BM * 4) + (is_sa ? 0 : BM * 4) + half * 256, m * 4);
            } else {
                const int t = (b - 4) >> 1, grp = t >> 1;
                if ((t & 1) == 0) {
                    const int n = n0 + half * 64 + lane;
                    dma4(zw_rsrc, zw_tab + grp * BN + half * 64, (n * g.ng + grp) * 4);
                } else {
                    const int m = m0 + half * 64 + lane;
                    dma4(ra_rsrc, ra_tab + grp * BM + half * 64, (m * g.ng + grp) * 4);
                }
            }
        }
    };

    // ---- operand fragments -----------------------------------------------------------------------
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
    // canonical codes: a shift and a mask per register pair; operand layout: one AND per register, the activation
    // registers (low, high) meeting the weight registers (high, low)
    auto widen_lo = [&](int f, const u32x4 &p) {
        if constexpr (!OLAY) return widen2<SGN>(p.x, p.y);
        else return f < FM ? v4i{(int)(p.x & 0x0F0F0F0Fu), (int)(p.x & 0xF0F0F0F0u), (int)(p.y & 0x0F0F0F0Fu), (int)(p.y & 0xF0F0F0F0u)}
                           : v4i{(int)(p.x & 0xF0F0F0F0u), (int)(p.x & 0x0F0F0F0Fu), (int)(p.y & 0xF0F0F0F0u), (int)(p.y & 0x0F0F0F0Fu)};
    };
    auto widen_hi = [&](int f, const u32x4 &p) {
        if constexpr (!OLAY) return widen2<SGN>(p.z, p.w);
        else return f < FM ? v4i{(int)(p.z & 0x0F0F0F0Fu), (int)(p.z & 0xF0F0F0F0u), (int)(p.w & 0x0F0F0F0Fu), (int)(p.w & 0xF0F0F0F0u)}
                           : v4i{(int)(p.z & 0xF0F0F0F0u), (int)(p.z & 0x0F0F0F0Fu), (int)(p.w & 0xF0F0F0F0u), (int)(p.w & 0x0F0F0F0Fu)};
    };

    v16i acc[FM][FN];                                           // written by the first K step of every group
    v16f facc[FM][FN];
    // OLAY: acc[i][0] <- 128*AE of this wave's rows of fragment row i, from the column that came with `stage`
    // (accumulator layout: register 4q+rr of lane (c, h) is row 8q + 4h + rr): the C operand of the group's first MFMAs
    // The reads are issued as opaque instructions and waited for by hand: an LDS read the compiler can see makes it
    // wait for EVERY outstanding tile DMA first (it cannot tell which LDS bytes a DMA writes), which would expose the
    // memory latency of the prefetch once per group.  The column was published by the K step's barrier like the code
    // tiles.  LDS reads return in order, so the compiler's own wait counts only ever become more conservative.
    v4i cpart[FM][4];
    auto load_cinit = [&](int stage) {
        if constexpr (OLAY) {
            const uint32_t addr = (uint32_t)(uintptr_t)(lds_ptr_t)(smem + stage * STAGE + CODES) +
                                  (uint32_t)(wm * FM * 32 + 4 * (lane >> 5)) * 4u;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(cpart[i][q]) : "v"(addr), "n"(i * 128 + q * 32));
        }
    };
    auto take_cinit = [&]() {                                   // wait for the reads, then name them accumulators
        if constexpr (OLAY) {
            __builtin_amdgcn_s_waitcnt(0xC07F);                 // lgkmcnt(0), the other counters unconstrained
#pragma unroll
            for (int i = 0; i < FM; ++i)
                acc[i][0] = v16i{cpart[i][0][0], cpart[i][0][1], cpart[i][0][2], cpart[i][0][3],
                                 cpart[i][1][0], cpart[i][1][1], cpart[i][1][2], cpart[i][1][3],
                                 cpart[i][2][0], cpart[i][2][1], cpart[i][2][2], cpart[i][2][3],
                                 cpart[i][3][0], cpart[i][3][1], cpart[i][3][2], cpart[i][3][3]};
        }
    };

    int vb = blockIdx.x;
    int tile = xcd_tile(vb, total);
    int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    __amdgpu_buffer_rsrc_t a_cur = a_desc(m0), b_cur = b_desc(n0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 0, a_cur, b_cur, 0);
    dma_col(0, m0, 0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 1, a_cur, b_cur, ROWB);
    dma_col(1, m0, 1);
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    u32x4 P0[NF], P1[NF];
    v4i U0[NF], U1[NF];

    int cur = 0;                                                // LDS stage of the current K step
    int parity = 0;
    for (;;) {
#pragma unroll
        for (int f = 0; f < NF; ++f) P0[f] = read_frag(f, cur, 0);
        load_cinit(cur);
        // ---- tile start --------------------------------------------------------------------------------
        dma_params(m0, n0, parity);
        const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;          // FN = 2 adjacent channels
        const int n_local = wn * FN * 32 + (lane & 31) * FN;
        const u32x2 c_raw = __builtin_amdgcn_raw_buffer_load_b64(c_rsrc, n_lane * 4, 0, 0);
        const uint32_t bias_raw = __builtin_amdgcn_raw_buffer_load_b32(bias_rsrc, n_lane * 2, 0, 0);
        uint32_t kw_raw[FN] = {0u, 0u};                         // OLAY: what the layout's offsets add to t1, per channel
        if constexpr (OLAY) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
                kw_raw[j] = __builtin_amdgcn_raw_buffer_load_b32(wo_rsrc, ((n_lane + j) * (g.ng + 1) + g.ng) * 4, 0, 0);
        }
        const int vb_next = vb + stride;
        const bool has_next = vb_next < total;
        const int tile_next = xcd_tile(has_next ? vb_next : vb, total);
        const int m0n = (tile_next / g.tiles_n) * BM, n0n = (tile_next % g.tiles_n) * BN;
        const __amdgpu_buffer_rsrc_t a_nxt = a_desc(m0n), b_nxt = b_desc(n0n);
#pragma unroll
        for (int f = 0; f < NF; ++f) U0[f] = widen_lo(f, P0[f]);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[i][j][r] = OLAY ? __uint_as_float(kw_raw[j]) : 0.0f;

        // ---- main loop ---------------------------------------------------------------------------------
#define W4A4_SLOT_BEGIN(Ucur, k)                                                                          \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ucur[(k) / FN], Ucur[FM + (k) % FN],   \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        // The first MFMA of a group starts from a constant C operand.  For unsigned canonical codes whose sums go to
        // the fp32 fold that constant is the bit pattern of 1.0f: the group's sum P (0 <= P < 2^23) then sits in
        // the mantissa field, the accumulator read as a float is 1 + P * 2^-23 exactly, and
        // fma(sw * 2^23, that, -sw * 2^23) is sw * P rounded once: the int-to-float conversion and the multiply of
        // the definition in one instruction, with the same bits.
        constexpr bool BIASED = !SGN && !OLAY && OUT != OUT_I32;
        constexpr int kC0 = BIASED ? 0x3F800000 : 0;
#define W4A4_SLOT_BEGIN_ZERO(Ucur, k)                                                                     \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                                       \
        Ucur[(k) / FN], Ucur[FM + (k) % FN],                                                              \
        v16i{kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0}, 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        // operand layout: the group's first MFMAs take acc[i][0] = 128*AE as their C operand, the column fragments in
        // descending order so that fragment 0 is overwritten last
#define W4A4_SLOT_BEGIN_TOKEN(Ucur, k)                                                                    \
    acc[(k) / FN][FN - 1 - (k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                              \
        Ucur[(k) / FN], Ucur[FM + FN - 1 - (k) % FN], acc[(k) / FN][0], 0, 0, 0);                          \
    __builtin_amdgcn_sched_barrier(0);
        constexpr int kBarSlot = NM - NF;
        float swg[FN];                                          // weight scales of the current group (this lane's channels)
        int wog[FN] = {0, 0};                                   // OLAY, int32 export: its odd-position code sums
        int grp = 0;                                            // index of the current weight group
        // One K step.  Whether it opens a weight group (FOG) and whether it ends the tile (LAST) are compile-time
        // flags: a K step is then one straight block of code, and the slot order written here is the issue order.
        // (With a run-time "first of group" branch the compiler sank the widening of the next step's first operands
        // out of the last MFMA slots to the common head of the two branches, where it ran with the matrix pipe idle.)
        auto k_step = [&](auto fog_tag, auto last_tag, int kt) {
            constexpr bool FOG = decltype(fog_tag)::value;     // first K step of a weight group
            constexpr bool LAST = decltype(last_tag)::value;   // last K step of the tile
            const int nxt = cur == NS - 1 ? 0 : cur + 1;       // stage of stream step +1
            const int nx2 = nxt == NS - 1 ? 0 : nxt + 1;       // stage of stream step +2 (= step -1)
            const bool own = !LAST && kt + 2 < KT;
            const __amdgpu_buffer_rsrc_t ra = own ? a_cur : a_nxt, rb = own ? b_cur : b_nxt;
            const int kt2 = own ? kt + 2 : kt + 2 - KT;
            const int so = kt2 * ROWB;
            if constexpr (FOG) {                                // this group's scales: used when it is folded
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    swg[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(sw_rsrc, (n_lane + j) * g.ng * 4, grp * 4, 0));
                    if constexpr (OLAY && OUT == OUT_I32)
                        wog[j] = (int)__builtin_amdgcn_raw_buffer_load_b32(wo_rsrc, (n_lane + j) * (g.ng + 1) * 4, grp * 4, 0);
                }
                take_cinit();
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 0: multiply (ks 0, low); widen (ks 0, high) -> U1; fetch ks 1 -> P1; request stream step +2
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                if constexpr (FOG && OLAY) { W4A4_SLOT_BEGIN_TOKEN(U0, k) }
                else if constexpr (FOG) { W4A4_SLOT_BEGIN_ZERO(U0, k) }
                else { W4A4_SLOT_BEGIN(U0, k) }
                if (k < NF) U1[k] = widen_hi(k, P0[k]);
                if (k < NF) P1[k] = read_frag(k, cur, 1);
                if (k < LD) dma_one(k, nx2, ra, rb, so);
                if (k == LD - 1) dma_col(nx2, own ? m0 : m0n, kt2);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 1: multiply (ks 0, high); widen (ks 1, low) -> U0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U1, k)
                if (k < NF) U0[k] = widen_lo(k, P1[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 2: multiply (ks 1, low); widen (ks 1, high) -> U1; barrier; fetch the next step's ks 0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U0, k)
                if (k < NF) U1[k] = widen_hi(k, P1[k]);
                if (k == kBarSlot) {
                    __builtin_amdgcn_s_waitcnt(vmcnt_only(LAST ? 0 : LDT));
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                }
                if (!LAST && k >= kBarSlot) P0[k - kBarSlot] = read_frag(k - kBarSlot, nxt, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 3: multiply (ks 1, high); widen (next step's ks 0, low) -> U0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U1, k)
                if (!LAST && k < NF) U0[k] = widen_lo(k, P0[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
        };
        // group boundary: t1 += sw[n,g] * (float)P_g.  Canonical codes: one multiply, one add, each rounded, as the
        // definition has it.  Operand layout: a conversion and one fused multiply-add on 16*(P_g - 8*WO).
        auto fold_group = [&](auto last_tag) {
            constexpr bool LAST = decltype(last_tag)::value;   // last group of the tile
            if constexpr (OUT == OUT_I32) {
                int32_t *plane = static_cast<int32_t *>(g.out) + (long)grp * g.M * g.N;
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int m = m0 + wm * FM * 32 + frag_row(i, r, lane), n = n_lane + j;
                            const int v = OLAY ? (acc[i][j][r] + 128 * wog[j]) >> 4 : SGN ? (acc[i][j][r] >> 8) : acc[i][j][r];
                            if (m < g.M && n < g.N) plane[(long)m * g.N + n] = v;
                        }
                if (!LAST) load_cinit(cur);
            } else {
                float sc[FN];
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    sc[j] = OLAY ? swg[j] * 0.0625f : SGN ? swg[j] * 0.00390625f : BIASED ? swg[j] * 8388608.0f : swg[j];
                // column fragment 0 first: its accumulators then take the next group's C operand from LDS while
                // the other fragment is folded
#pragma unroll
                for (int j = 0; j < FN; ++j) {
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            if constexpr (OLAY) {
                                facc[i][j][r] = __fmaf_rn(sc[j], (float)acc[i][j][r], facc[i][j][r]);
                            } else {
                                const float u = BIASED ? __fmaf_rn(sc[j], __int_as_float(acc[i][j][r]), -sc[j])
                                                       : sc[j] * (float)acc[i][j][r];
                                facc[i][j][r] = facc[i][j][r] + u;
                            }
                        }
                    if (j == 0 && !LAST) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_cinit(cur);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            ++grp;
        };
        {
            const std::true_type yes{};
            const std::false_type no{};
            int kt = 0;
            if constexpr (SPG1) {                               // every K step is a group
                for (; kt < KT - 1; ++kt) { k_step(yes, no, kt); fold_group(no); }
                k_step(yes, yes, kt);
            } else {
                for (int gi = 0; gi < g.ng - 1; ++gi) {
                    k_step(yes, no, kt++);
                    for (int st = 1; st < spg; ++st) k_step(no, no, kt++);
                    fold_group(no);
                }
                k_step(yes, no, kt++);
                for (int st = 1; st < spg - 1; ++st) k_step(no, no, kt++);
                k_step(no, yes, kt);
            }
            fold_group(yes);
        }
#undef W4A4_SLOT_BEGIN
#undef W4A4_SLOT_BEGIN_ZERO
#undef W4A4_SLOT_BEGIN_TOKEN

        // ---- epilogue of this tile ------------------------------------------------------------------
        if constexpr (OUT != OUT_I32) {
            constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
            const float *sa_lds = reinterpret_cast<const float *>(par + parity * (2 * BM * 4));
            const float *za_lds = sa_lds + BM;
            const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * g.N * ESZ));
            const uint32_t row_bytes = (uint32_t)g.N * ESZ;
            const uint32_t col_off = n_lane < g.N ? (uint32_t)n_lane * ESZ : kPoison;
            const int row_w = wm * FM * 32;
            const uint32_t lane_off = (uint32_t)(m0 + row_w + 4 * (lane >> 5)) * row_bytes + col_off;
            const bool has_bias = g.bias != nullptr, gelu = g.act == W4A4_ACT_GELU;
            const float cv[FN] = {__uint_as_float(c_raw[0]), __uint_as_float(c_raw[1])};
            const float bv[FN] = {__half2float(__ushort_as_half((unsigned short)(bias_raw & 0xFFFFu))),
                                  __half2float(__ushort_as_half((unsigned short)(bias_raw >> 16)))};
            if constexpr (OLAY) {
                // sum_g zw[n,g] * RA[m,g]: a rank-ng product of the tile's two group tables, continued into the fp32
                // accumulators by the fp32 MFMA, two groups per instruction (lanes 0-31 carry group gp, lanes 32-63
                // group gp + 1; a missing last group contributes zeros)
                for (int gp = 0; gp < g.ng; gp += 2) {
                    const int gi = gp + (lane >> 5);
                    const bool live = gi < g.ng;
                    const int gs = live ? gi : gp;
                    float ta[FM], tb[FN];
#pragma unroll
                    for (int i = 0; i < FM; ++i) {
                        const int v = ra_tab[gs * BM + row_w + i * 32 + (lane & 31)];
                        ta[i] = live ? (float)v : 0.0f;
                    }
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const float v = zw_tab[gs * BN + n_local + j];
                        tb[j] = live ? v : 0.0f;
                    }
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
                            facc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(ta[i], tb[j], facc[i][j], 0, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int rl = row_w + i * 32 + 8 * q + 4 * (lane >> 5);      // 4 consecutive rows
                    const float4 sa4 = *reinterpret_cast<const float4 *>(sa_lds + rl);
                    const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
                    float y[4][FN];
                    if constexpr (OLAY) {
                        // y = fma(sa, t1 + sum_g zw*RA, fma(za, c, bias)); the zero-point sum is already in facc
                        const float4 za4 = *reinterpret_cast<const float4 *>(za_lds + rl);
                        const float zav[4] = {za4.x, za4.y, za4.z, za4.w};
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                            for (int j = 0; j < FN; ++j)
                                y[rr][j] = __fmaf_rn(sav[rr], facc[i][j][q * 4 + rr],
                                                     __fmaf_rn(zav[rr], cv[j], has_bias ? bv[j] : 0.0f));
                    } else {
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                            for (int j = 0; j < FN; ++j) y[rr][j] = sav[rr] * facc[i][j][q * 4 + rr];
                        if constexpr (MODE == W4A4_ASYM) {
                            const float4 za4 = *reinterpret_cast<const float4 *>(za_lds + rl);
                            const float zav[4] = {za4.x, za4.y, za4.z, za4.w};
                            float t2[4][FN];
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                                for (int j = 0; j < FN; ++j) t2[rr][j] = 0.0f;
                            for (int gi = 0; gi < g.ng; ++gi) {
                                const int4 ra4 = *reinterpret_cast<const int4 *>(ra_tab + gi * BM + rl);
                                const float2 zw2 = *reinterpret_cast<const float2 *>(zw_tab + gi * BN + n_local);
                                const float raf[4] = {(float)ra4.x, (float)ra4.y, (float)ra4.z, (float)ra4.w};
                                const float zwv[FN] = {zw2.x, zw2.y};
#pragma unroll
                                for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                                    for (int j = 0; j < FN; ++j) {
                                        const float w = zwv[j] * raf[rr];
                                        t2[rr][j] = t2[rr][j] + w;
                                    }
                            }
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                                for (int j = 0; j < FN; ++j) {
                                    const float p = sav[rr] * t2[rr][j];
                                    const float z = zav[rr] * cv[j];
                                    y[rr][j] = y[rr][j] + p;
                                    y[rr][j] = y[rr][j] + z;
                                }
                        }
                        if (has_bias) {
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                                for (int j = 0; j < FN; ++j) y[rr][j] = y[rr][j] + bv[j];
                        }
                    }
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const uint32_t off = lane_off + (uint32_t)(i * 32 + 8 * q + rr) * row_bytes;
                        if constexpr (OUT == OUT_F32) {
                            uint32_t w[FN];
#pragma unroll
                            for (int j = 0; j < FN; ++j) w[j] = __float_as_uint(gelu ? gelu_erf(y[rr][j]) : y[rr][j]);
                            store_words<FN, kStreamed>(o_rsrc, off, w);
                        } else if (gelu) {
                            store_gelu_halves<FN, kStreamed>(o_rsrc, off, y[rr]);
                        } else {
                            store_halves<FN, kStreamed>(o_rsrc, off, y[rr]);
                        }
                    }
                }
        }
        if (!has_next) break;
        if constexpr (MODE == W4A4_ASYM) __syncthreads();       // the group tables are single: every wave is done reading them
        vb = vb_next; tile = tile_next; m0 = m0n; n0 = n0n; a_cur = a_nxt; b_cur = b_nxt; parity ^= 1;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));                  // no DMA may outlive the workgroup's LDS
}

template <int MODE, int OUT, bool OLAY, bool SPG1>
static int launch_spg(GemmArgs &g, hipStream_t st) {
    constexpr int BM = 128, BN = 128;
    const size_t tables = MODE == W4A4_ASYM ? (size_t)g.ng * (BM + BN) * 4 : 0;
    const size_t lds = 3 * ((size_t)(BM + BN) * (kBK / 2) + (OLAY ? BM * 4 : 0)) + 2 * 2 * BM * 4 + tables;
    if (lds > 80 * 1024) return W4A4_ERR_UNSUPPORTED_SHAPE;       // the group tables do not fit beside two workgroups' stages
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_group_kernel<MODE, OUT, OLAY, SPG1>;
    static KernelState ks;
    const int cus = prepare_kernel(reinterpret_cast<const void *>(kern), lds, ks);
    if (cus < 0) return W4A4_ERR_HIP;
    const int slots = cus * 2;                                  // workgroups that are resident at once
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    const unsigned grid = (unsigned)(tiles < slots ? tiles : slots);
    launch_gemm(kern, dim3(grid), dim3(256), lds, st, g);
    return launch_status();
}

template <int MODE, int OUT, bool OLAY>
static int launch_one(GemmArgs &g, hipStream_t st) {
    return g.steps_per_group == 1 ? launch_spg<MODE, OUT, OLAY, true>(g, st) : launch_spg<MODE, OUT, OLAY, false>(g, st);
}

// Requires: weight groups of g.steps_per_group * 128 codes (ng >= 1); K % 128 == 0, K >= 256;
// M*lda, N*ldw, N*(ng+1)*4 and M*ng*4 < 2^31.  Canonical codes, or (asymmetric layers) the operand layout with
// g.osum = 128 * even-position token sums [ng][M] and g.esum = odd-position channel sums [N][ng+1].
int launch_group(int mode, int out_kind, GemmArgs &g, hipStream_t st) {
    const bool olay = g.osum != nullptr;
    if (mode == W4A4_SYM) {
        if (olay) return W4A4_ERR_INVALID_ARG;
        switch (out_kind) {
            case OUT_F16: return launch_one<W4A4_SYM, OUT_F16, false>(g, st);
            case OUT_F32: return launch_one<W4A4_SYM, OUT_F32, false>(g, st);
            case OUT_I32: return launch_one<W4A4_SYM, OUT_I32, false>(g, st);
            default: return W4A4_ERR_INVALID_ARG;
        }
    }
    if (olay) {
        switch (out_kind) {
            case OUT_F16: return launch_one<W4A4_ASYM, OUT_F16, true>(g, st);
            case OUT_F32: return launch_one<W4A4_ASYM, OUT_F32, true>(g, st);
            case OUT_I32: return launch_one<W4A4_ASYM, OUT_I32, true>(g, st);
            default: return W4A4_ERR_INVALID_ARG;
        }
    }
    switch (out_kind) {
        case OUT_F16: return launch_one<W4A4_ASYM, OUT_F16, false>(g, st);
        case OUT_F32: return launch_one<W4A4_ASYM, OUT_F32, false>(g, st);
        case OUT_I32: return launch_one<W4A4_ASYM, OUT_I32, false>(g, st);
        default: return W4A4_ERR_INVALID_ARG;
    }
}

}  // namespace w4a4
