// Persistent INT4 x INT4 -> INT32 GEMM on operands kept in the MFMA operand layout
// (symmetric codes, per-channel weight scales, K a multiple of 128, K >= 256).
//
// What bounds this GEMM on gfx950 is the vector-ALU issue port of a SIMD: an int8
// 32x32x32 MFMA occupies it for about half of its 32 cycles, and every ordinary VALU
// instruction for four more.  So the design removes VALU work wherever it can:
//   * Operand layout (see w4a4_layout in w4a4.h): one v_and_b32 per MFMA operand register
//     instead of a shift and a mask (3 instead of 4.5 VALU per MFMA for a 64 x 128 wave
//     tile).  The contraction then yields 16*P + 128*(esum[n] + osum[m]).  The token term
//     costs nothing per accumulator: the first MFMA of a tile takes -128*osum[m] (sixteen
//     registers per 32 rows, shared by all column fragments) as its C operand; the channel
//     term is one integer add per accumulator in the epilogue.
//   * Tiles travel HBM -> LDS with `buffer_load_dwordx4 ... lds` (no staging registers, no
//     LDS-write instructions); all DMA addressing is scalar: the per-lane offsets are fixed
//     for the whole kernel, the tile origin lives in the buffer descriptor (SGPRs) and the
//     K offset in the instruction's scalar offset.  Rows past M / channels past N fall
//     outside the descriptor and read as zero.
//   * LDS rows are unpadded; bank conflicts are avoided by an XOR swizzle of the 16-byte
//     slots of a row (physical slot = logical chunk ^ ((row >> 2) & 3)).
//   * Workgroups are persistent and the K steps of successive tiles form ONE stream through
//     the three LDS stages: while the last two K steps of a tile are multiplied, the first
//     two of the next tile are already being fetched, so a tile has no load prologue.
//     Token scales / odd sums go to LDS by 4-byte DMA one tile ahead (the odd sums are needed
//     by the first MFMAs of the tile), channel constants to registers at the start of the tile.
//   * Two workgroups share a CU (2 x 74 KB of LDS), four waves of 64 x 128 each, so one
//     workgroup's epilogue stores overlap the other's main loop.
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt immediate for "vmcnt <= n", lgkmcnt and expcnt unconstrained (gfx9 encoding)
constexpr int vmcnt_only(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | (((n >> 4) & 0x3) << 14); }

// One v_and per register: activations give (even codes + 8, 16 * odd codes), weights give
// (16 * even codes, odd codes + 8); register r of one meets register r of the other.
__device__ __forceinline__ v4i widen_act(uint32_t x, uint32_t y) {
    return v4i{(int)(x & 0x0F0F0F0Fu), (int)(x & 0xF0F0F0F0u), (int)(y & 0x0F0F0F0Fu), (int)(y & 0xF0F0F0F0u)};
}
__device__ __forceinline__ v4i widen_wgt(uint32_t x, uint32_t y) {
    return v4i{(int)(x & 0xF0F0F0F0u), (int)(x & 0x0F0F0F0Fu), (int)(y & 0xF0F0F0F0u), (int)(y & 0x0F0F0F0Fu)};
}

template <int FN>
struct ChanParams {
    float sw[FN];      // weight scale / 16 (the accumulators hold 16 * P; a power of two, so exact)
    float bias[FN];
    int ne[FN];        // -128 * esum[n]
};

// Epilogue of one wave for the fp16 / fp32 / int32 outputs.  The accumulators already contain
// -128*osum[m] (C operand of the tile's first MFMAs), so v = acc - 128*esum[n] = 16*P exactly.
//   fp32 rows (they are quantized afterwards, where the operation order decides codes):
//     y = ((float)v * sa[m]) * (sw[n]/16) (+ bias[n]) (GELU), each operation separately rounded, which equals
//     ((float)P * sa) * sw of the definition bit for bit;
//   fp16 stores: three instructions per value instead of five,
//     y = fma(fma((float)acc, sw[n]/16, -128*esum[n]*sw[n]/16), sa[m], bias[n]),
//     the same real number evaluated with two roundings less and the channel term moved behind the conversion
//     (its product with the scale is formed once per tile).  The fp32 value differs from the definition's by a
//     few units in the last place, the fp16 result by at most one step and only on near-ties of the fp16 grid.
template <int FM, int FN, int OUT, bool BIAS, bool GELU>
__device__ __forceinline__ void olay_epilogue(const GemmArgs &g, v16i (&acc)[FM][FN], const ChanParams<FN> &cp,
                                              uint32_t col_off, int m0, int row_w, int lane,
                                              const float *sa_lds) {
    constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
    const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * g.N * ESZ));
    const uint32_t row_bytes = (uint32_t)g.N * ESZ;
    const uint32_t lane_off = (uint32_t)(m0 + row_w + 4 * (lane >> 5)) * row_bytes + col_off;
    float nsw[FN], bj[FN];                                      // channel term times the scale; bias (0 without one)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        nsw[j] = (float)cp.ne[j] * cp.sw[j];
        bj[j] = BIAS ? cp.bias[j] : 0.0f;
    }
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
                    for (int j = 0; j < FN; ++j) w[j] = (uint32_t)((acc[i][j][r] + cp.ne[j]) >> 4);
                    store_words<FN, kStreamed>(o_rsrc, off, w);
                } else if constexpr (OUT == OUT_F32) {
                    uint32_t w[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const float t = (float)(acc[i][j][r] + cp.ne[j]) * sav[rr];
                        float y = t * cp.sw[j];
                        if constexpr (BIAS) y = y + cp.bias[j];
                        w[j] = __float_as_uint(GELU ? gelu_erf(y) : y);
                    }
                    store_words<FN, kStreamed>(o_rsrc, off, w);
                } else {
                    float y[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        y[j] = __fmaf_rn(__fmaf_rn((float)acc[i][j][r], cp.sw[j], nsw[j]), sav[rr], bj[j]);
                    if constexpr (GELU) store_gelu_halves<FN, kStreamed>(o_rsrc, off, y);
                    else store_halves<FN, kStreamed>(o_rsrc, off, y);
                }
            }
        }
}

// Fused per-token requantize of one wave's part of the tile (symmetric output codes; Sec. 4.2:
// the next layer's quantize rides behind bias-add / GELU).  The range of a token needs the whole
// output row, which is spread over the tiles_n workgroups that hold the row panel's column
// tiles at this moment (all workgroups of the grid are resident), so:
//   1. every lane turns its accumulators into the fp32 outputs y (the operation order of the
//      fp32 store path), keeps them in the accumulator registers and notes max|y| of its four
//      channels for each of its 32 rows;
//   2. a butterfly over the 32 lanes that share the rows leaves lane c with the maximum of row
//      c, which it publishes with ONE atomic max on rowmax[m] (non-negative floats order like
//      integers);
//   3. the workgroup announces itself on arrived[panel] and waits until all tiles_n siblings
//      have (bounded; on expiry *fault is raised instead of hanging);
//   4. lane c fetches the final maximum of row c, derives scale = max/7 and 7/max and shares the
//      reciprocal through `scratch` (LDS, 64 floats per wave).  code = rne(y * (7/max)) as in
//      quantize_act: |y * (7/max)| <= 7(1+2^-23), so the clamp of the definition cannot bind and
//      the rounding is done by adding 1.5*2^23 + 8 (round-to-nearest-even of the fp32 add), which
//      leaves code+8 in the low four bits.  Eight codes per dword come from two neighbouring
//      lanes.  MFMA==true writes the operand layout of activations (even positions stay offset
//      binary, odd ones become two's complement) and accumulates the odd-position code sums of the
//      tile's column slice with one atomic add per row and wave; otherwise canonical nibbles.
template <int FM, int FN, bool MFMA>
__device__ __forceinline__ void olay_epilogue_requant(const GemmArgs &g, v16i (&acc)[FM][FN], const ChanParams<FN> &cp,
                                                       bool n_ok, int n_lane, int m0, int row_w, int lane, int tid,
                                                       int panel, int slice, bool first_cols, const float *sa_lds,
                                                       float *scratch) {
    static_assert(FN == 4 && FM == 2, "32 rows per half wave; two lanes assemble one dword of eight codes");
    const bool gelu = g.act == W4A4_ACT_GELU;
    const int h = lane >> 5, c = lane & 31;
    // 1. outputs in fp32, kept in place; vmax[i*16 + r] = bits of the max over this lane's channels
    //    (a non-negative, non-NaN float: such bit patterns order like unsigned integers)
    uint32_t vmax[32];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rl = row_w + i * 32 + 8 * q + 4 * h;
            const float4 sa4 = *reinterpret_cast<const float4 *>(sa_lds + rl);
            const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w};
            float y[4][FN];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    float t = (float)(acc[i][j][q * 4 + rr] + cp.ne[j]) * sav[rr];
                    t = t * cp.sw[j];
                    y[rr][j] = t + cp.bias[j];                    // 0 without a bias: changes at most the sign of a zero
                }
            }
            if (gelu) {                                           // uniform branch around 16 straight-line evaluations
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                    for (int j = 0; j < FN; ++j) y[rr][j] = gelu_erf(y[rr][j]);
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                float v = 0.0f;
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j][q * 4 + rr] = __float_as_int(y[rr][j]);
                    v = fmaxf(v, fabsf(y[rr][j]));
                }
                vmax[i * 16 + q * 4 + rr] = n_ok ? __float_as_uint(v) : 0u;   // channels past N do not count
            }
        }
    // 2. butterfly: after the step with offset o a lane keeps the rows whose index bit o equals
    //    its own lane bit o; after five steps lane c holds the maximum of row c.
    reduce_scatter32(vmax, lane, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
    const int m_c = m0 + row_w + frag_row(c >> 4, c & 15, lane);  // the row this lane is responsible for
    if (m_c < g.M) atomicMax(g.rowmax + m_c, vmax[0]);
    // 3. wait for the siblings of the row panel (bounded)
    panel_arrive_and_wait(g, panel, tid);
    // 4. ranges
    {
        const __amdgpu_buffer_rsrc_t mx_rsrc = make_rsrc(g.rowmax, (uint32_t)g.M * 4u);
        // an ordinary load that bypasses the non-coherent cache levels (sc0 | sc1); rows >= M read 0
        const float amax = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(mx_rsrc, m_c * 4, 0, 17));
        const Range rg = range_sym(amax);
        if (m_c < g.M && first_cols) g.out_scale[m_c] = rg.S;     // the wave that holds channel 0 of the row
        scratch[(tid & ~63) + lane] = rg.inv;
        __builtin_amdgcn_wave_barrier();
    }
    // packed rows are N/2 bytes; even lanes store a dword of eight codes, everything else is
    // sent to an offset the bounds check of the descriptor drops
    const __amdgpu_buffer_rsrc_t q_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * (g.N / 2)));
    const uint32_t row_b = (uint32_t)g.N / 2;
    const uint32_t lane_q = ((lane & 1) == 0 && n_ok)
                                ? (uint32_t)(m0 + row_w + 4 * h) * row_b + (uint32_t)(n_lane >> 1) : kPoison;
    constexpr float kMagic = 12582912.0f + 8.0f;                  // 1.5 * 2^23 + 8
    // even lanes fill the low half of a dword of eight codes, odd lanes the high half
    const uint32_t half_sel = (lane & 1) ? 0x04000c0cu : 0x0c0c0400u;
    int osum[32];                                                 // 16 * odd-position sums of (code + 8) per row (MFMA)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 iv4 = *reinterpret_cast<const float4 *>(scratch + (tid & ~63) + h * 32 + i * 16 + q * 4);
            const float ivv[4] = {iv4.x, iv4.y, iv4.z, iv4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = q * 4 + rr;
                uint32_t u[FN];
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const float t = __int_as_float(acc[i][j][r]) * ivv[rr];
                    u[j] = __float_as_uint(t + kMagic);           // low byte = rne(t) + 8, in 1 .. 15
                }
                // two codes per byte (bits above the byte are junk), then the two bytes into this
                // lane's half of the dword; the neighbour's half arrives through the quad permute
                const uint32_t p01 = (u[1] << 4) | u[0], p23 = (u[3] << 4) | u[2];
                const uint32_t half = __builtin_amdgcn_perm(p23, p01, half_sel);
                if (MFMA) osum[i * 16 + r] = n_ok ? (int)__builtin_amdgcn_sad_u8(half & 0xF0F0F0F0u, 0u, 0u) : 256;
                uint32_t packed = half | dpp_fetch<0xB1>(half);
                packed ^= MFMA ? 0x80808080u : 0x88888888u;       // offset binary -> two's complement where wanted
                __builtin_amdgcn_raw_buffer_store_b32(packed, q_rsrc, lane_q + (uint32_t)(i * 32 + 8 * q + rr) * row_b, 0, 0);
            }
        }
    if (MFMA) {
        // the same butterfly with sums: lane c ends with the sum over the wave's 128 channels of row c
        reduce_scatter32(osum, lane, [](int a, int b) { return a + b; });
        // in units of 1/16; every lane added 16 (two offsets of 8, or the neutral 16 of a lane past N)
        if (m_c < g.M) atomicAdd(g.out_osum + (long)m_c * g.osum_slices + slice, (osum[0] >> 4) - 32 * 16);
    }
}

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_olay_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    constexpr int ROWB = kBK / 2;                               // 64 bytes of codes per row per K step
    constexpr int STAGE = (BM + BN) * ROWB, NS = 3;
    constexpr int BLOCKS = (BM + BN) / 16;                      // 1 KB DMA blocks per stage
    constexpr int LD = BLOCKS / NW;                             // tile DMA instructions per wave per K step
    constexpr int A_LD = (BM / 16) / NW;                        // the first A_LD of them fetch activations
    constexpr int NF = FM + FN, NM = FM * FN;
    constexpr int PB = BM / 64;                                 // 64-row blocks of token scales (and as many of odd sums)
    static_assert(BLOCKS % NW == 0 && (BM / 16) % NW == 0, "DMA blocks must split evenly over the waves");
    static_assert(NF <= NM && LD <= NM, "not enough MFMA slots to hide the memory operations");
    static_assert(BM % 64 == 0, "token parameters are fetched 64 rows per DMA instruction");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    // token parameters of the tile, double buffered by tile parity: [2][ sa[BM] | osum[BM] ]
    uint8_t *par = smem + NS * STAGE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int total = g.tiles_m * g.tiles_n, stride = gridDim.x;
    const int KT = g.K / kBK;

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
    // Token parameters by 4-byte DMA: waves [0, PB) fetch 64 scales each, waves [PB, 2 PB) the odd sums.
    const __amdgpu_buffer_rsrc_t sa_rsrc = make_rsrc(g.sa, (uint32_t)g.M * 4u);
    const __amdgpu_buffer_rsrc_t os_rsrc = make_rsrc(g.osum, (uint32_t)(((long)(g.M - 1) * g.ldo + 1) * 4));
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(g.sw, (uint32_t)g.N * 4u);
    const __amdgpu_buffer_rsrc_t es_rsrc = make_rsrc(g.esum, (uint32_t)g.N * 4u);
    const __amdgpu_buffer_rsrc_t bias_rsrc = make_rsrc(g.bias, g.bias ? (uint32_t)g.N * 2u : 0u);   // no bias: zeros
    auto dma_params = [&](int m0, int parity) {
#pragma unroll
        for (int b0 = 0; b0 < 2 * PB; b0 += NW) {
            const int b = b0 + wave;                            // block b: scales of rows 64b.. (b < PB), else odd sums
            if (b < 2 * PB) {
                const bool is_sa = b < PB;
                const int blk = is_sa ? b : b - PB;
                uint8_t *dst = par + parity * (2 * BM * 4) + (is_sa ? 0 : BM * 4) + blk * 256;
                const int m = m0 + blk * 64 + lane;
                const int vo = is_sa ? m * 4 : m * (int)g.ldo * 4;
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(is_sa ? sa_rsrc : os_rsrc, (lds_ptr_t)dst, 4, vo, 0, 0, 0);
#else
                (void)dst; (void)vo;
#endif
            }
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
    auto read_frag = [&](int f, int stage, int ks) {
        return *reinterpret_cast<const u32x4 *>(smem + stage * STAGE + (frag_off[f] ^ (ks << 5)));
    };
    auto widen_lo = [&](int f, const u32x4 &p) { return f < FM ? widen_act(p.x, p.y) : widen_wgt(p.x, p.y); };
    auto widen_hi = [&](int f, const u32x4 &p) { return f < FM ? widen_act(p.z, p.w) : widen_wgt(p.z, p.w); };

    v16i acc[FM][FN];                                           // written by the first K step of every tile

    // ---- first tile: its first two K steps and parameters --------------------------------------------
    // Tile of virtual block id vb (workgroup id + k * grid size; vb % 8 = the XCD it runs on).  Every XCD
    // owns a contiguous range of tiles, so that the tiles of a row panel run on one XCD and share its
    // L2.  For the requantizing outputs the ranges are whole row panels: the column tiles of a panel
    // wait for each other, and a workgroup walks its XCD's tiles in increasing order, which together
    // rule out a cycle of waits.  Returns false when the XCD has no tile for this id.
    auto tile_of = [&](int v, int &t) {
        if constexpr (OUT == OUT_Q4 || OUT == OUT_Q4M) {
            const int x = v & (kXcd - 1), i = v >> 3;
            const int per = g.tiles_m / kXcd, rem = g.tiles_m % kXcd;
            const int cnt = per + (x < rem ? 1 : 0);
            t = (x * per + (x < rem ? x : rem)) * g.tiles_n + i;
            return i < cnt * g.tiles_n;
        } else {
            t = xcd_tile(v < total ? v : 0, total);
            return v < total;
        }
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
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    u32x4 P0[NF], P1[NF];
    v4i U0[NF], U1[NF];

    int cur = 0;                                                // LDS stage of the current K step
    int parity = 0;
    for (;;) {
        // first fragments of the tile (its first two K steps are in LDS and published)
#pragma unroll
        for (int f = 0; f < NF; ++f) P0[f] = read_frag(f, cur, 0);
        // ---- tile start: C operand of the first MFMAs, channel constants, origin of the next tile -----
        // acc[i][0] = -128 * osum of the rows of fragment row i (accumulator layout: register 4q+rr of
        // lane (c, h) is row 8q + 4h + rr).  The token parameters of this tile were fetched one tile ago.
        {
            const int *os_lds = reinterpret_cast<const int *>(par + parity * (2 * BM * 4) + BM * 4) + wm * FM * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int4 o = *reinterpret_cast<const int4 *>(os_lds + i * 32 + 8 * q);
                    acc[i][0][4 * q + 0] = __mul24(o.x, -128);
                    acc[i][0][4 * q + 1] = __mul24(o.y, -128);
                    acc[i][0][4 * q + 2] = __mul24(o.z, -128);
                    acc[i][0][4 * q + 3] = __mul24(o.w, -128);
                }
        }
        // channel constants of this lane's FN adjacent channels: raw loads now (channels past N read
        // as zero), converted when the epilogue starts
        const int n_lane = n0 + wn * FN * 32 + (lane & 31) * FN;
        static_assert(FN == 4 || FN == 2, "channel constants are fetched two or four at a time");
        u32x4 sw_raw, es_raw;
        u32x2 bias_raw;
        if constexpr (FN == 4) {
            sw_raw = __builtin_amdgcn_raw_buffer_load_b128(sw_rsrc, n_lane * 4, 0, 0);
            es_raw = __builtin_amdgcn_raw_buffer_load_b128(es_rsrc, n_lane * 4, 0, 0);
            bias_raw = __builtin_amdgcn_raw_buffer_load_b64(bias_rsrc, n_lane * 2, 0, 0);
        } else {
            const u32x2 s2 = __builtin_amdgcn_raw_buffer_load_b64(sw_rsrc, n_lane * 4, 0, 0);
            const u32x2 e2 = __builtin_amdgcn_raw_buffer_load_b64(es_rsrc, n_lane * 4, 0, 0);
            sw_raw = u32x4{s2[0], s2[1], 0, 0};
            es_raw = u32x4{e2[0], e2[1], 0, 0};
            bias_raw = u32x2{__builtin_amdgcn_raw_buffer_load_b32(bias_rsrc, n_lane * 2, 0, 0), 0};
        }
        const int vb_next = vb + stride;
        int tile_next;
        const bool has_next = tile_of(vb_next, tile_next);
        if (!has_next) tile_next = tile;
        const int m0n = (tile_next / g.tiles_n) * BM, n0n = (tile_next % g.tiles_n) * BN;
        const __amdgpu_buffer_rsrc_t a_nxt = a_desc(m0n), b_nxt = b_desc(n0n);
#pragma unroll
        for (int f = 0; f < NF; ++f) U0[f] = widen_lo(f, P0[f]);

        // ---- main loop: one iteration = 128 codes of K = four sub-steps of NM MFMAs -------------
        // The instruction order below is the intended issue order; the scheduling barriers keep
        // the compiler from regrouping it.  Slot k of a sub-step issues MFMA k and, behind it, the
        // widening of fragment k for the NEXT sub-step plus at most one LDS read and one DMA.
#define W4A4_SLOT_BEGIN(Ucur, k)                                                                          \
    acc[(k) / FN][(k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ucur[(k) / FN], Ucur[FM + (k) % FN],   \
                                                                   acc[(k) / FN][(k) % FN], 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);
        // the first MFMA into an accumulator of a tile takes acc[i][0] = -128 * osum as its C operand (column
        // fragments in descending order, so that fragment 0 is overwritten last): the accumulators are never
        // cleared and the token term of the layout correction is never added per element
#define W4A4_SLOT_BEGIN_FIRST(Ucur, k)                                                                    \
    acc[(k) / FN][FN - 1 - (k) % FN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                              \
        Ucur[(k) / FN], Ucur[FM + FN - 1 - (k) % FN], acc[(k) / FN][0], 0, 0, 0);                          \
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
            // sub-step 0: multiply (ks 0, low); widen (ks 0, high) -> U1; fetch ks 1 -> P1; request
            //             stream step +2 into the stage every wave finished reading before the last barrier.
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                if constexpr (FIRST) { W4A4_SLOT_BEGIN_FIRST(U0, k) } else { W4A4_SLOT_BEGIN(U0, k) }
                if (k < NF) U1[k] = widen_hi(k, P0[k]);
                if (k < NF) P1[k] = read_frag(k, cur, 1);
                if (k < LD) dma_one(k, nx2, ra, rb, so);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 1: multiply (ks 0, high); widen (ks 1, low) -> U0
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U1, k)
                if (k < NF) U0[k] = widen_lo(k, P1[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
            // sub-step 2: multiply (ks 1, low); widen (ks 1, high) -> U1; this wave's loads of stream
            //             step +1 have landed (vmcnt), and after the barrier everyone's have: fetch its ks 0.
            //             At the end of a tile BOTH prefetched steps of the next tile are waited for, so
            //             that the next tile's first barrier does not have to wait for this tile's stores;
            //             the next tile reads its first fragments itself.
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                W4A4_SLOT_BEGIN(U0, k)
                if (k < NF) U1[k] = widen_hi(k, P1[k]);
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
                if (!LAST && k < NF) U0[k] = widen_lo(k, P0[k]);
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
#undef W4A4_SLOT_BEGIN
#undef W4A4_SLOT_BEGIN_FIRST

        // ---- epilogue of this tile ------------------------------------------------------------------
        {
            constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
            const uint32_t col_off = n_lane < g.N ? (uint32_t)n_lane * ESZ : kPoison;
            ChanParams<FN> cp;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                cp.sw[j] = __uint_as_float(sw_raw[j]) * 0.0625f;
                cp.ne[j] = (int)es_raw[j] * -128;
                const uint32_t b2 = bias_raw[j >> 1];
                cp.bias[j] = __half2float(__ushort_as_half((unsigned short)((j & 1) ? b2 >> 16 : b2 & 0xFFFFu)));
            }
            const float *sa_lds = reinterpret_cast<const float *>(par + parity * (2 * BM * 4));
            const int row_w = wm * FM * 32;
            const bool bias = g.bias != nullptr, gelu = g.act == W4A4_ACT_GELU;
            if constexpr (OUT == OUT_Q4 || OUT == OUT_Q4M) {
                if constexpr (FM == 2 && FN == 4) {
                    const int tn = tile % g.tiles_n;
                    olay_epilogue_requant<FM, FN, OUT == OUT_Q4M>(g, acc, cp, n_lane < g.N, n_lane, m0, row_w, lane, tid,
                                                                  tile / g.tiles_n, tn / g.slice_tiles, tn == 0 && wn == 0,
                                                                  sa_lds, reinterpret_cast<float *>(par + 2 * 2 * BM * 4));
                }
            } else
            if (OUT == OUT_I32 || (!bias && !gelu)) olay_epilogue<FM, FN, OUT, false, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (bias && !gelu) olay_epilogue<FM, FN, OUT, true, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (!bias && gelu) olay_epilogue<FM, FN, OUT, false, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else olay_epilogue<FM, FN, OUT, true, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
        }
        if (!has_next) break;
        vb = vb_next; tile = tile_next; m0 = m0n; n0 = n0n; a_cur = a_nxt; b_cur = b_nxt; parity ^= 1;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_only(0));                  // no DMA may outlive the workgroup's LDS
}

// Launch geometry of one instantiation on the current device.  The requantizing outputs make the column tiles
// of a row panel wait for each other, so every workgroup of their grid must be resident: the grid is sized from
// what the runtime reports for this kernel (hipOccupancyMaxActiveBlocksPerMultiprocessor), capped by the
// occupancy the kernel was compiled for, and a panel's tiles_n tiles must fit into one XCD's share of it.
template <int FM, int FN, int WM, int WN, int OCC, int OUT>
struct OlayLaunch {
    static constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
    static constexpr size_t lds = 3 * (size_t)(BM + BN) * (kBK / 2) + 2 * 2 * BM * 4 + (OUT == OUT_Q4 || OUT == OUT_Q4M ? 1024 : 0);
    static KernelState &state() { static KernelState ks; return ks; }
    static auto kernel() { return gemm_olay_kernel<FM, FN, WM, WN, OCC, OUT>; }
    // resident workgroups on the current device (-1: HIP error)
    static int slots() {
        const int cus = prepare_kernel(reinterpret_cast<const void *>(kernel()), lds, state());
        if (cus < 0) return -1;
        if (OUT != OUT_Q4 && OUT != OUT_Q4M) return cus * OCC;    // no workgroup waits for another: any grid is safe
        const int occ = resident_per_cu(reinterpret_cast<const void *>(kernel()), WM * WN * 64, lds, state());
        if (occ < 0) return -1;
        return cus * (occ < OCC ? occ : OCC);
    }
};

template <int FM, int FN, int WM, int WN, int OCC, int OUT>
static int launch_one(GemmArgs &g, hipStream_t st) {
    using L = OlayLaunch<FM, FN, WM, WN, OCC, OUT>;
    g.tiles_m = (g.M + L::BM - 1) / L::BM;
    g.tiles_n = (g.N + L::BN - 1) / L::BN;
    const int slots = L::slots();
    if (slots < 0) return W4A4_ERR_HIP;
    const long tiles = (long)g.tiles_m * g.tiles_n;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    unsigned grid = (unsigned)(tiles < slots ? tiles : slots);
    if (OUT == OUT_Q4 || OUT == OUT_Q4M) {
        // every XCD walks whole row panels: ids up to 8 * (tiles of the fullest XCD); and the column tiles
        // of a panel must sit in different workgroups at the same time
        const long most = (long)((g.tiles_m + kXcd - 1) / kXcd) * g.tiles_n * kXcd;
        grid = (unsigned)(most < (slots & ~(kXcd - 1)) ? most : (slots & ~(kXcd - 1)));
        if (g.tiles_n > (int)(grid / kXcd)) return W4A4_ERR_UNSUPPORTED_SHAPE;
        if (g.wait_for == 0) g.wait_for = g.tiles_n;
    }
    if (grid == 0) return W4A4_ERR_UNSUPPORTED_SHAPE;
    launch_gemm(L::kernel(), dim3(grid), dim3(WM * WN * 64), L::lds, st, g);
    return launch_status();
}

// Column tiles of a row panel that the fused requantize of the persistent kernel can keep co-resident on the
// current device (0 = the kernel does not fit, -1 = HIP error): the limit on ceil(N / 256).
int olay_requant_max_tiles_n(bool mfma_out) {
    const int slots = mfma_out ? OlayLaunch<2, 4, 2, 2, 2, OUT_Q4M>::slots() : OlayLaunch<2, 4, 2, 2, 2, OUT_Q4>::slots();
    return slots < 0 ? -1 : (slots & ~(kXcd - 1)) / kXcd;
}

template <int OUT>
static int launch_variant(int variant, GemmArgs &g, hipStream_t st) {
    switch (variant) {
        case 0: return launch_one<2, 4, 2, 2, 2, OUT>(g, st);   // 128 x 256, two workgroups per CU
        case 1: return launch_one<3, 2, 2, 2, 2, OUT>(g, st);   // 192 x 128, two workgroups per CU
        case 2: return launch_one<2, 2, 2, 2, 3, OUT>(g, st);   // 128 x 128, three workgroups per CU: mid-sized problems
        default: return W4A4_ERR_INVALID_ARG;
    }
}

// Requires: MFMA operand layout on both sides (symmetric codes, per-channel weight scales),
// K % 128 == 0, K >= 256, M*lda and N*ldw < 2^31, M*ldo*4 < 2^31.
int launch_olay(int variant, int out_kind, GemmArgs &g, hipStream_t st) {
    switch (out_kind) {
        case OUT_F16: return launch_variant<OUT_F16>(variant, g, st);
        case OUT_F32: return launch_variant<OUT_F32>(variant, g, st);
        case OUT_I32: return launch_variant<OUT_I32>(variant, g, st);
        case OUT_Q4: return variant == 0 ? launch_one<2, 4, 2, 2, 2, OUT_Q4>(g, st) : W4A4_ERR_INVALID_ARG;
        case OUT_Q4M: return variant == 0 ? launch_one<2, 4, 2, 2, 2, OUT_Q4M>(g, st) : W4A4_ERR_INVALID_ARG;
        default: return W4A4_ERR_INVALID_ARG;
    }
}

}  // namespace w4a4
