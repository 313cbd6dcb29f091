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
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt immediate for "vmcnt <= n", lgkmcnt and expcnt unconstrained (gfx9 encoding)
static constexpr int vmcnt_only(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | (((n >> 4) & 0x3) << 14); }

template <int MODE, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void gemm_group_kernel(GemmArgs g) {
    constexpr bool SGN = MODE == W4A4_SYM;
    constexpr int FM = 2, FN = 2, WM = 2, WN = 2;
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    constexpr int ROWB = kBK / 2;                               // 64 bytes of codes per row per K step
    constexpr int STAGE = (BM + BN) * ROWB, NS = 3;
    constexpr int LD = (BM + BN) / 16 / NW;                     // tile DMA instructions per wave per K step
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
    auto dma_one = [&](int i, int stage, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, int so) {
        uint8_t *dst = smem + stage * STAGE + (wave + i * NW) * 1024;
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature; it rejects the LDS cast
        __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LD ? ra : rb, (lds_ptr_t)dst, 16, voff[i], so, 0, 0);
#else
        (void)dst; (void)ra; (void)rb; (void)so;
#endif
    };
    auto dma4 = [&](__amdgpu_buffer_rsrc_t rs, void *dst, int vo) {
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)dst, 4, vo, 0, 0, 0);
#else
        (void)rs; (void)dst; (void)vo;
#endif
    };
    const __amdgpu_buffer_rsrc_t sa_rsrc = make_rsrc(g.sa, (uint32_t)g.M * 4u);
    const __amdgpu_buffer_rsrc_t za_rsrc = make_rsrc(g.za, MODE == W4A4_ASYM ? (uint32_t)g.M * 4u : 0u);
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(g.sw, (uint32_t)((long)g.N * g.ng * 4));
    const __amdgpu_buffer_rsrc_t zw_rsrc = make_rsrc(g.zw, MODE == W4A4_ASYM ? (uint32_t)((long)g.N * g.ng * 4) : 0u);
    const __amdgpu_buffer_rsrc_t ra_rsrc = make_rsrc(g.RA, MODE == W4A4_ASYM ? (uint32_t)((long)g.M * g.ng * 4) : 0u);
    const __amdgpu_buffer_rsrc_t c_rsrc = make_rsrc(g.c, MODE == W4A4_ASYM ? (uint32_t)g.N * 4u : 0u);
    const __amdgpu_buffer_rsrc_t bias_rsrc = make_rsrc(g.bias, g.bias ? (uint32_t)g.N * 2u : 0u);   // no bias: zeros
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

    v16i acc[FM][FN];                                           // written by the first K step of every group
    float facc[FM][FN][16];

    int vb = blockIdx.x;
    int tile = xcd_tile(vb, total);
    int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    __amdgpu_buffer_rsrc_t a_cur = a_desc(m0), b_cur = b_desc(n0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 0, a_cur, b_cur, 0);
#pragma unroll
    for (int i = 0; i < LD; ++i) dma_one(i, 1, a_cur, b_cur, ROWB);
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
        // ---- tile start --------------------------------------------------------------------------------
        dma_params(m0, n0, parity);
        const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;          // FN = 2 adjacent channels
        const int n_local = wn * FN * 32 + (lane & 31) * FN;
        const u32x2 c_raw = __builtin_amdgcn_raw_buffer_load_b64(c_rsrc, n_lane * 4, 0, 0);
        const uint32_t bias_raw = __builtin_amdgcn_raw_buffer_load_b32(bias_rsrc, n_lane * 2, 0, 0);
        const int vb_next = vb + stride;
        const bool has_next = vb_next < total;
        const int tile_next = xcd_tile(has_next ? vb_next : vb, total);
        const int m0n = (tile_next / g.tiles_n) * BM, n0n = (tile_next % g.tiles_n) * BN;
        const __amdgpu_buffer_rsrc_t a_nxt = a_desc(m0n), b_nxt = b_desc(n0n);
#pragma unroll
        for (int f = 0; f < NF; ++f) U0[f] = widen2<SGN>(P0[f].x, P0[f].y);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[i][j][r] = 0.0f;

        // ---- main loop ---------------------------------------------------------------------------------
#define W4A4_SLOT_BEGIN(Ucur, k)                                                                          \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ucur[(k) / FN], Ucur[FM + (k) % FN],   \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        // The first MFMA of a group starts from a constant C operand.  For unsigned codes whose sums go to
        // the fp32 fold that constant is the bit pattern of 1.0f: the group's sum P (0 <= P < 2^23) then sits in
        // the mantissa field, the accumulator read as a float is 1 + P * 2^-23 exactly, and
        // fma(sw * 2^23, that, -sw * 2^23) is sw * P rounded once: the int-to-float conversion and the multiply of
        // the definition in one instruction, with the same bits.
        constexpr bool BIASED = !SGN && OUT != OUT_I32;
        constexpr int kC0 = BIASED ? 0x3F800000 : 0;
#define W4A4_SLOT_BEGIN_ZERO(Ucur, k)                                                                     \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                                       \
        Ucur[(k) / FN], Ucur[FM + (k) % FN],                                                              \
        v16i{kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0, kC0}, 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        constexpr int kBarSlot = NM - NF;
        float swg[FN];                                          // weight scales of the current group (this lane's channels)
        int in_group = 0, grp = 0;                              // K steps done inside the current group; its index
        auto k_step = [&](auto last_tag, int kt) {
            constexpr bool LAST = decltype(last_tag)::value;   // last K step of the tile
            const int nxt = cur == NS - 1 ? 0 : cur + 1;       // stage of stream step +1
            const int nx2 = nxt == NS - 1 ? 0 : nxt + 1;       // stage of stream step +2 (= step -1)
            const bool own = !LAST && kt + 2 < KT;
            const __amdgpu_buffer_rsrc_t ra = own ? a_cur : a_nxt, rb = own ? b_cur : b_nxt;
            const int so = (own ? kt + 2 : kt + 2 - KT) * ROWB;
            const bool first_of_group = in_group == 0;
            if (first_of_group) {                               // (uniform) this group's scales: used when it is folded
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    swg[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(sw_rsrc, (n_lane + j) * g.ng * 4, grp * 4, 0));
            }
            // sub-step 0: multiply (ks 0, low); widen (ks 0, high) -> U1; fetch ks 1 -> P1; request stream step +2
            if (first_of_group) {
#pragma unroll
                for (int k = 0; k < NM; ++k) {
                    W4A4_SLOT_BEGIN_ZERO(U0, k)
                    if (k < NF) U1[k] = widen2<SGN>(P0[k].z, P0[k].w);
                    if (k < NF) P1[k] = read_frag(k, cur, 1);
                    if (k < LD) dma_one(k, nx2, ra, rb, so);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int k = 0; k < NM; ++k) {
                    W4A4_SLOT_BEGIN(U0, k)
                    if (k < NF) U1[k] = widen2<SGN>(P0[k].z, P0[k].w);
                    if (k < NF) P1[k] = read_frag(k, cur, 1);
                    if (k < LD) dma_one(k, nx2, ra, rb, so);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // sub-step 1: multiply (ks 0, high); widen (ks 1, low) -> U0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U1, k)
                if (k < NF) U0[k] = widen2<SGN>(P1[k].x, P1[k].y);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 2: multiply (ks 1, low); widen (ks 1, high) -> U1; barrier; fetch the next step's ks 0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U0, k)
                if (k < NF) U1[k] = widen2<SGN>(P1[k].z, P1[k].w);
                if (k == kBarSlot) {
                    __builtin_amdgcn_s_waitcnt(vmcnt_only(LAST ? 0 : LD));
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
                if (!LAST && k < NF) U0[k] = widen2<SGN>(P0[k].x, P0[k].y);
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
            // group boundary: t1 += sw[n,g] * (float)P_g  (one multiply, one add, each rounded, as the definition
            // has it; fusing them was measured to gain 8 % and costs bit-for-bit agreement with the definition)
            if (++in_group == spg) {
                if constexpr (OUT == OUT_I32) {
                    int32_t *plane = static_cast<int32_t *>(g.out) + (long)grp * g.M * g.N;
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int m = m0 + wm * FM * 32 + frag_row(i, r, lane), n = n_lane + j;
                                if (m < g.M && n < g.N) plane[(long)m * g.N + n] = SGN ? (acc[i][j][r] >> 8) : acc[i][j][r];
                            }
                } else {
                    float sc[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) sc[j] = SGN ? swg[j] * 0.00390625f : BIASED ? swg[j] * 8388608.0f : swg[j];
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const float u = BIASED ? __fmaf_rn(sc[j], __int_as_float(acc[i][j][r]), -sc[j])
                                                       : sc[j] * (float)acc[i][j][r];
                                facc[i][j][r] = facc[i][j][r] + u;
                            }
                }
                in_group = 0;
                ++grp;
            }
        };
        for (int kt = 0; kt < KT - 1; ++kt) k_step(std::false_type{}, kt);
        k_step(std::true_type{}, KT - 1);
#undef W4A4_SLOT_BEGIN
#undef W4A4_SLOT_BEGIN_ZERO

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
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int rl = row_w + i * 32 + 8 * q + 4 * (lane >> 5);      // 4 consecutive rows
                    const float4 sa4 = *reinterpret_cast<const float4 *>(sa_lds + rl);
                    const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
                    float y[4][FN];
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
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        if (has_bias) {
#pragma unroll
                            for (int j = 0; j < FN; ++j) y[rr][j] = y[rr][j] + bv[j];
                        }
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

template <int MODE, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    constexpr int BM = 128, BN = 128;
    const size_t tables = MODE == W4A4_ASYM ? (size_t)g.ng * (BM + BN) * 4 : 0;
    const size_t lds = 3 * (size_t)(BM + BN) * (kBK / 2) + 2 * 2 * BM * 4 + tables;
    if (lds > 80 * 1024) return W4A4_ERR_UNSUPPORTED_SHAPE;       // the group tables do not fit beside two workgroups' stages
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    auto kern = gemm_group_kernel<MODE, OUT>;
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

// Requires: canonical codes; weight groups of g.steps_per_group * 128 codes (ng >= 1); K % 128 == 0, K >= 256;
// M*lda, N*ldw, N*ng*4 and M*ng*4 < 2^31.
int launch_group(int mode, int out_kind, GemmArgs &g, hipStream_t st) {
    if (mode == W4A4_SYM) {
        switch (out_kind) {
            case OUT_F16: return launch_one<W4A4_SYM, OUT_F16>(g, st);
            case OUT_F32: return launch_one<W4A4_SYM, OUT_F32>(g, st);
            case OUT_I32: return launch_one<W4A4_SYM, OUT_I32>(g, st);
            default: return W4A4_ERR_INVALID_ARG;
        }
    }
    switch (out_kind) {
        case OUT_F16: return launch_one<W4A4_ASYM, OUT_F16>(g, st);
        case OUT_F32: return launch_one<W4A4_ASYM, OUT_F32>(g, st);
        case OUT_I32: return launch_one<W4A4_ASYM, OUT_I32>(g, st);
        default: return W4A4_ERR_INVALID_ARG;
    }
}

}  // namespace w4a4
