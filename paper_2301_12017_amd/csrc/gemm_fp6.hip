// Persistent INT4 x INT4 GEMM on the FP6 matrix pipe (symmetric codes, per-channel weight scales).
//
// A symmetric 4-bit code c in [-7, 7] is exactly an FP6 E2M3 number (sign, two exponent bits, three mantissa
// bits: every integer up to 7 is representable), the products of two of them are exact in the FP32 accumulator of
// v_mfma_f32_32x32x64_f8f6f4, and so is their sum as long as it stays below 2^24 (K <= 342 000).  The FP32
// accumulator therefore holds the INT32 result of the method's integer GEMM bit for bit, and the FP6 form of the
// instruction runs at twice the rate of the int8 MFMA: what the INT4 tensor cores of the paper's hardware give a
// W4A4 layer (Sec. 4.2), gfx950 gives through its FP6 pipe.  Sign-magnitude operands also toggle fewer
// multiplier bits than two's complement ones, which counts on a chip whose clock follows its power draw.
//
// Operands arrive in the FP6 operand layout (see w4a4_layout in w4a4.h): per row and per 64 codes 48 bytes,
// [16: first part of the 24-byte operand of K-half 0 | 16: first part of K-half 1 | 8 + 8: their last parts], so
// that a lane fetches its MFMA operand with one 16-byte and one 8-byte LDS read, both aligned, and nothing is
// unpacked: the main loop has no vector-ALU work at all.  Output channels sit in their 128-channel panel in the
// order (n % 4) * 32 + n / 4, so that the lane that holds MFMA column cc of fragments 0 .. 3 holds channels
// 4cc .. 4cc+3.
//
// Structure (as the int8 kernel on the MFMA operand layout):
//   * tiles travel HBM -> LDS by `buffer_load_dwordx4 ... lds`; the layout stores block h of a 64-token (128-channel)
//     panel contiguously, so every DMA instruction moves one kilobyte of consecutive addresses (what the vector
//     memory path of a CU needs to keep up with the FP6 pipe: rows fetched 48 bytes at a time cost it three to four
//     times the cycles); all addressing is scalar; panels past the padded matrix fall outside the descriptor and
//     read as zero;
//   * LDS rows are 48 bytes: sixteen consecutive rows start in sixteen different groups of four banks, so the
//     operand reads have no bank conflicts without padding or swizzle;
//   * a ring of NS stages of 64 codes each: while half step h is multiplied, the operands of h+1 are read from LDS
//     and the tile data of h+2 .. h+NS-1 is in flight; one workgroup barrier per half step (after its first MFMA);
//   * persistent workgroups, the half steps of successive tiles form one stream through the ring, token scales go
//     to LDS by 4-byte DMA one tile ahead;
//   * two (three for the 128 x 128 tile) workgroups share a CU.
#include "gemm_common.hpp"

namespace w4a4 {

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));

// s_waitcnt immediate for "vmcnt <= n and lgkmcnt == 0", expcnt unconstrained (gfx9 encoding)
constexpr int vmcnt_and_lds(int n) { return (n & 0xF) | (0x7 << 4) | (0x0 << 8) | (((n >> 4) & 0x3) << 14); }

constexpr int kHalf = 64;          // codes per half step (one MFMA per accumulator)
constexpr int kRow6 = 48;          // bytes of a row per half step

template <int FN>
struct ChanParams6 {
    float sw[FN];
    float bias[FN];
};

// Epilogue of one wave.  The accumulators hold P exactly; every output follows the definition's operation order,
// each operation separately rounded: y = ((float)P * sa[m]) * sw[n] (+ bias[n]) (GELU), then the store's rounding.
template <int FM, int FN, int OUT, bool BIAS, bool GELU>
__device__ __forceinline__ void fp6_epilogue(const GemmArgs &g, v16f (&acc)[FM][FN], const ChanParams6<FN> &cp,
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
                    for (int j = 0; j < FN; ++j) w[j] = (uint32_t)(int)acc[i][j][r];
                    store_words<FN, kStreamed>(o_rsrc, off, w);
                } else {
                    float y[FN];
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const float t = acc[i][j][r] * sav[rr];
                        y[j] = t * cp.sw[j];
                        if constexpr (BIAS) y[j] = y[j] + cp.bias[j];
                    }
                    if constexpr (OUT == OUT_F32) {
                        uint32_t w[FN];
#pragma unroll
                        for (int j = 0; j < FN; ++j) w[j] = __float_as_uint(GELU ? gelu_erf(y[j]) : y[j]);
                        store_words<FN, kStreamed>(o_rsrc, off, w);
                    } else if constexpr (GELU) {
                        store_gelu_halves<FN, kStreamed>(o_rsrc, off, y);
                    } else {
                        store_halves<FN, kStreamed>(o_rsrc, off, y);
                    }
                }
            }
        }
}

// Fused per-token requantize of one wave's part of a 128 x 256 tile into the FP6 operand layout of activations
// (Sec. 4.2: the next layer's quantize rides behind bias-add / GELU; here the next layer's GEMM operand is written
// directly, 3/4 byte per output instead of the two bytes of an fp16 row).  The range of a token needs its whole
// output row, spread over the tiles_n workgroups that hold the row panel's column tiles at that moment, so the
// steps are those of the int8 kernel's requantizing epilogue: fp32 outputs in place (the definition's operation
// order), row maxima by a register butterfly and one atomic max per row, a bounded wait for the panel's siblings,
// then the codes.  A code t = rne(y * 7/max) is an integer of magnitude <= 7 (the clamp of the definition cannot
// bind) and exactly an FP6 E2M3 number, so the hardware conversion of 32 fp32 values to 32 packed fields serves here
// as in the token-wise quantizer: two conversions per 32 x 32 block of a lane's four channels, from whose results a
// row's 24 bits are cut.  A lane's four adjacent channels are those 24 bits; the lanes of a quad own twelve
// consecutive bytes of an operand, which three of them assemble as one dword each; the dwords of eight rows meet in
// LDS and leave as sixteen-byte stores.  No code sums travel with this layout.
template <int FM, int FN>
__device__ __forceinline__ void fp6_epilogue_requant(const GemmArgs &g, v16f (&acc)[FM][FN], const ChanParams6<FN> &cp,
                                                     int n_lane, int m0, int row_w, int lane, int tid, int panel,
                                                     bool first_cols, const float *sa_lds, float *scratch) {
    static_assert(FN == 4 && FM == 2, "32 rows per half wave; a lane holds four adjacent channels");
    const bool gelu = g.act == W4A4_ACT_GELU;
    const int h = lane >> 5, c = lane & 31;
    // 1. outputs in fp32, kept in place; vmax[i*16 + r] = bits of the max over this lane's channels (a non-negative,
    //    non-NaN float: such bit patterns order like unsigned integers).  N is a multiple of the tile width here.
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
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    float t = acc[i][j][q * 4 + rr] * sav[rr];
                    t = t * cp.sw[j];
                    y[rr][j] = t + cp.bias[j];                    // 0 without a bias: changes at most the sign of a zero
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
                    acc[i][j][q * 4 + rr] = y[rr][j];
                    v = fmaxf(v, fabsf(y[rr][j]));
                }
                vmax[i * 16 + q * 4 + rr] = __float_as_uint(v);
            }
        }
    // 2. butterfly: lane c ends with the maximum of row c of the wave's 64 (two halves of 32)
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
        scratch[(tid & ~63) * 4 + lane] = rg.inv;                 // 0 for rows >= M: their codes are written as zeros
        __builtin_amdgcn_wave_barrier();
    }
    // 5. codes.  The output is an activation matrix of N codes per row in the FP6 layout: panels of 64 tokens, block b
    //    (64 codes) of a panel's rows contiguous, a row's 48 bytes of a block = operand 2b+e as 16 bytes at 16e and 8
    //    bytes at 32 + 8e (at 40 - 8e in rows 16 .. 31 of every 32).  Lane c holds channels 4c .. 4c+3 of the wave's
    //    128-channel panel: bytes 3(c%8) .. +2 of operand c/8; quad lane j < 3 makes dword j of the quad's twelve bytes.
    //    The wave's 64 rows are one token panel and its 128 channels two blocks of it, so eight consecutive rows are 384
    //    consecutive bytes in each of the two blocks: the dwords of eight rows meet in LDS (768 bytes per wave, behind
    //    the wave's 64 ranges) and leave as 48 sixteen-byte stores.
    const int KBo = g.N / kHalf;
    const long out_bytes = (((long)g.M + 63) & ~63L) * KBo * kRow6;
    const __amdgpu_buffer_rsrc_t q_rsrc = make_rsrc(g.out, (uint32_t)out_bytes);
    const int op = (n_lane >> 5) & 3, ob = 12 * ((c >> 2) & 1) + 4 * (lane & 3);   // operand of the wave's four, byte of this lane's dword in it
    const int e = op & 1;
    uint8_t *stage8 = reinterpret_cast<uint8_t *>(scratch + (tid & ~63) * 4) + 256;
    uint32_t put[2];                                              // where this lane's dword goes in the staging area, by bit 4 of the row
#pragma unroll
    for (int sw = 0; sw < 2; ++sw)
        put[sw] = (uint32_t)(op >> 1) * 384u + (uint32_t)(4 * h) * kRow6 + (uint32_t)(ob < 16 ? 16 * e + ob : 32 + 8 * (e ^ sw) + (ob - 16));
    // lane L < 48 stores bytes 16L .. 16L+15 of the staging area: block L / 24 of the two, byte 16 (L % 24) of its eight rows
    const uint32_t blk0 = (uint32_t)(n_lane >> 7) * 2u;          // first of the wave's two blocks in the row
    const uint32_t get = lane >= 48 ? 0u : (uint32_t)lane * 16u;   // (the idle lanes re-read the first piece)
    const uint32_t lane_q = lane >= 48 ? kPoison
                            : (uint32_t)((m0 + row_w) >> 6) * ((uint32_t)KBo * (64 * kRow6)) +
                                  (blk0 + (uint32_t)(lane / 24)) * (64 * kRow6) + (uint32_t)(lane % 24) * 16u;
    // bytes of {next lane's 24 bits, own 24 bits} that make dword j: own[j..2], then next[0..j]
    const uint32_t sel = (lane & 3) == 0 ? 0x04020100u : (lane & 3) == 1 ? 0x05040201u : 0x06050402u;
    typedef unsigned int v6u __attribute__((ext_vector_type(6)));
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        // t = rne(y * 7/max), in place
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 iv4 = *reinterpret_cast<const float4 *>(scratch + (tid & ~63) * 4 + h * 32 + i * 16 + q * 4);
            const float ivv[4] = {iv4.x, iv4.y, iv4.z, iv4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j][q * 4 + rr] = __builtin_rintf(acc[i][j][q * 4 + rr] * ivv[rr]);
        }
        // 32 values -> 32 fields per conversion; it interleaves its two sources, so fields 2r and 2r+1 of `lo` are
        // channels 0 and 1 of row register r, of `hi` channels 2 and 3: twelve bits each per row
        const v6u lo = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(acc[i][0], acc[i][1], 1.0f);
        const v6u hi = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(acc[i][2], acc[i][3], 1.0f);
#pragma unroll
        for (int q = 0; q < 4; ++q) {                             // rows 8q .. 8q+7 of the 32: 4h + rr in this lane
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = 4 * q + rr;
                const int d = (12 * r) >> 5, o = (12 * r) & 31;
                uint32_t a12, b12;                                // b12 may keep bits above its twelve: they end up past bit 23
                if (o + 12 <= 32) {
                    a12 = __builtin_amdgcn_ubfe(lo[d], o, 12);
                    b12 = hi[d] >> o;
                } else {
                    a12 = __builtin_amdgcn_alignbit(lo[d + 1], lo[d], o) & 0xFFFu;
                    b12 = __builtin_amdgcn_alignbit(hi[d + 1], hi[d], o);
                }
                const uint32_t own = (b12 << 12) | a12;           // 24 bits (and junk above, which the byte select drops)
                const uint32_t nxt = dpp_fetch<0xF9>(own);        // quad permute [1,2,3,3]: the next lane's
                const uint32_t word = __builtin_amdgcn_perm(nxt, own, sel);
                if ((lane & 3) != 3) *reinterpret_cast<uint32_t *>(stage8 + put[q >> 1] + rr * kRow6) = word;
            }
            asm volatile("" ::: "memory");                        // the wave's LDS operations execute in program order
            const u32x4 out16 = *reinterpret_cast<const u32x4 *>(stage8 + get);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_raw_buffer_store_b128(out16, q_rsrc, lane_q + (uint32_t)(i * 32 + 8 * q) * kRow6, 0, 0);
        }
    }
}

template <int FM, int FN, int WM, int WN, int OCC, int NS, int OUT>
__global__ __attribute__((amdgpu_flat_work_group_size(WM *WN * 64, WM *WN * 64), amdgpu_waves_per_eu(OCC, OCC)))
void gemm_fp6_kernel(GemmArgs g) {
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    constexpr int REAL = (BM + BN) * 3 / 64;                    // 1 KB DMA blocks of a stage (64 slots of 16 bytes)
    constexpr int A_BLOCKS = BM * 3 / 64;                       // the first of them hold activations
    constexpr int BLOCKS = (REAL + NW - 1) / NW * NW;           // padded so that every wave issues as many
    constexpr int LD = BLOCKS / NW;                             // tile DMA instructions per wave per half step
    constexpr int STAGE = REAL * 1024;
    constexpr int NF = FM + FN, NM = FM * FN;
    constexpr int PB = BM / 64;                                 // 64-row blocks of token scales
    constexpr int RPS = 2;                                      // operand reads per MFMA slot, from slot 1 on: early, so that
                                                                // they have returned when the next half step starts
    static_assert((BM + BN) * 3 % 64 == 0 && BM * 3 % 64 == 0, "whole DMA blocks");
    static_assert(LD <= NM - 1 && (NF + RPS - 1) / RPS <= NM - 1, "not enough MFMA slots for the memory operations");
    static_assert(NS >= 3 && (NS - 2) * LD <= 63, "ring depth");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    uint8_t *dummy = smem + NS * STAGE;                         // where the padding blocks of every stage land (zeros)
    uint8_t *par = dummy + (BLOCKS > REAL ? 1024 : 0);          // token scales of the tile, double buffered: [2][BM]
                                                                // (OUT_Q6: followed by a kilobyte per wave: 64 row ranges, 768 bytes of codes on their way out)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int total = g.tiles_m * g.tiles_n, stride = gridDim.x;
    const int KT = g.K / kHalf;                                 // half steps per tile (even, >= NS + 2)

    // ---- global -> LDS plan (fixed for the whole kernel) -------------------------------------------
    // A stage is [BM token rows | BN channel rows] of 48 bytes, which is also how the operands lie in memory: block
    // h of a 64-token panel is 3 KB, of a 128-channel panel 6 KB, each contiguous.  DMA instruction i of this wave
    // moves kilobyte bi = wave + i*NW of the stage, every lane sixteen consecutive bytes: whole cache lines, in order.
    const int KB = g.K / kHalf;                                 // blocks per row = half steps per tile
    // a token panel is lda * 64 bytes long: KB blocks, or more when the activations are a column slice (whole blocks)
    // of a wider matrix, whose pointer then addresses the slice's first block in panel 0
    const int a_panel = (int)g.lda * 64;
    int dma_base[LD], dma_step[LD];                             // byte offset of the kilobyte in half step 0, and per half step
    int voff[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int bi = wave + i * NW;
        if (bi < A_BLOCKS) {
            dma_base[i] = (bi / 3) * a_panel + (bi % 3) * 1024;
            dma_step[i] = 3072;
        } else {
            const int bb = bi - A_BLOCKS;
            dma_base[i] = (bb / 6) * KB * 6144 + (bb % 6) * 1024;
            dma_step[i] = 6144;
        }
        voff[i] = bi < REAL ? lane * 16 : (int)kPoison;         // padding blocks: outside every descriptor, read as zero
    }
    // descriptors of a tile: from its first panel to the end of the (panel-padded) matrix - for a column slice, to the
    // end of the slice's blocks in the last panel
    const long a_bytes = ((((long)g.M + 63) >> 6) - 1) * a_panel + (long)KB * 3072, b_bytes = (((long)g.N + 127) & ~127L) * KB * 48;
    auto a_desc = [&](int m0) {
        const long off = (long)(m0 >> 6) * a_panel;
        return make_rsrc(g.Aq + off, (uint32_t)(a_bytes > off ? a_bytes - off : 0));
    };
    auto b_desc = [&](int n0) {
        const long off = (long)(n0 >> 7) * KB * 6144;
        return make_rsrc(g.Wq + off, (uint32_t)(b_bytes > off ? b_bytes - off : 0));
    };
    auto dma_one = [&](int i, int stage, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, int hstep) {
        const int bi = wave + i * NW;
        uint8_t *dst = bi < REAL ? smem + stage * STAGE + bi * 1024 : dummy;
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature; it rejects the LDS cast
        __builtin_amdgcn_raw_ptr_buffer_load_lds(bi < A_BLOCKS ? ra : rb, (lds_ptr_t)dst, 16, voff[i],
                                                 dma_base[i] + hstep * dma_step[i], 0, 0);
#else
        (void)dst; (void)ra; (void)rb; (void)hstep;
#endif
    };
    const __amdgpu_buffer_rsrc_t sa_rsrc = make_rsrc(g.sa, (uint32_t)g.M * 4u);
    const __amdgpu_buffer_rsrc_t sw_rsrc = make_rsrc(g.sw, (uint32_t)g.N * 4u);
    const __amdgpu_buffer_rsrc_t bias_rsrc = make_rsrc(g.bias, g.bias ? (uint32_t)g.N * 2u : 0u);   // no bias: zeros
    auto dma_params = [&](int m0, int parity) {
#pragma unroll
        for (int b0 = 0; b0 < PB; b0 += NW) {
            const int b = b0 + wave;                            // block b: scales of rows 64b ..
            if (b < PB) {
                uint8_t *dst = par + parity * (BM * 4) + b * 256;
                const int vo = (m0 + b * 64 + lane) * 4;
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(sa_rsrc, (lds_ptr_t)dst, 4, vo, 0, 0, 0);
#else
                (void)dst; (void)vo;
#endif
            }
        }
    };

    // ---- operand fragments -----------------------------------------------------------------------
    // lane (r = lane&31, h = lane>>5) reads the operand of K-half h of its row: 16 bytes at 16h, 8 bytes at 32 + 8h
    int frag16[NF];
#pragma unroll
    for (int f = 0; f < FM; ++f) frag16[f] = (wm * FM * 32 + f * 32 + (lane & 31)) * kRow6 + (lane >> 5) * 16;
#pragma unroll
    for (int f = 0; f < FN; ++f) {
        // fragment wn*FN + f of the tile's channels: panel (wn*FN + f) / 4, storage rows 32 * ((wn*FN + f) % 4) .. + 31,
        // which hold channels 4*cc + (wn*FN + f) % 4 of the panel: a lane ends up with FN adjacent channels
        const int gf = wn * FN + f;
        frag16[FM + f] = (BM + (gf >> 2) * 128 + (gf & 3) * 32 + (lane & 31)) * kRow6 + (lane >> 5) * 16;
    }
    // from the 16-byte part to the 8-byte part; rows 16 .. 31 of a 32-row group keep their two 8-byte parts in
    // the other order, so that the 32 lanes of one 8-byte read fall into 32 different pairs of banks
    const int tail = 32 + (((lane >> 5) ^ (lane >> 4)) & 1) * 8 - (lane >> 5) * 16;
    auto read_frag = [&](int f, int stage) {
        const uint8_t *p = smem + stage * STAGE + frag16[f];
        const v4i x = *reinterpret_cast<const v4i *>(p);
        const v2i y = *reinterpret_cast<const v2i *>(p + tail);
        return v8i{x[0], x[1], x[2], x[3], y[0], y[1], 0, 0};
    };
    // the fragments in the order the MFMAs of a half step first need them: A0, B0 .. B(FN-1), A1 .. A(FM-1)
    auto frag_in_order = [](int k) { return k == 0 ? 0 : k <= FN ? FM + k - 1 : k - FN; };

    v16f acc[FM][FN];                                           // written by the first half step of every tile

    // Tile of virtual block id v (workgroup id + k * grid size; v % 8 = the XCD it runs on): every XCD owns a
    // contiguous range of tiles, so that the tiles of a row panel run on one XCD and share its L2.
    // For the requantizing output the ranges are whole row panels: the column tiles of a panel wait for each other, and
    // a workgroup walks its XCD's tiles in increasing order, which together rule out a cycle of waits.
    auto tile_of = [&](int v, int &t) {
        if constexpr (OUT == OUT_Q6) {
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
    if constexpr (OUT == OUT_Q6) {
        // Every second row panel of an XCD starts a few microseconds late.  The requantizing epilogue is vector-ALU work
        // and a wait, the main loop matrix and memory work: two workgroups of a CU that are in different phases overlap
        // them, and the panel waits keep whatever phases the workgroups start with (the grid holds whole panels, so the
        // same workgroups meet at every wait).
        if (((int)(blockIdx.x >> 3) / g.tiles_n) & 1)
            for (int s = 0; s < g.stagger; ++s) __builtin_amdgcn_s_sleep(32);
    }
    int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
    __amdgpu_buffer_rsrc_t a_cur = a_desc(m0), b_cur = b_desc(n0);
    // ---- first tile: its first NS half steps and its token scales -----------------------------------
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int i = 0; i < LD; ++i) dma_one(i, s, a_cur, b_cur, s);
    dma_params(m0, 0);
    __builtin_amdgcn_s_waitcnt(vmcnt_and_lds(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    v8i Pa[NF], Pb[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) Pa[f] = read_frag(f, 0);

    int cur = 0;                                                // ring stage of the current half step
    int parity = 0;
    for (;;) {
        const int n_lane = n0 + ((wn * FN) >> 2) * 128 + (lane & 31) * 4 + ((wn * FN) & 3);
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

        // ---- main loop: one half step = 64 codes of K = NM MFMAs ---------------------------------------------
        // Slot k issues MFMA k; slot 0 then waits for this wave's tile DMAs of half step +1 and for its LDS
        // reads, and meets the other waves at the barrier: after it, half step +1 is published and the stage of
        // the current half step (whose operands every wave holds in registers) is free.  Slots 1 .. NM-1 read
        // the operands of half step +1 and request half step +NS into the freed stage.
        auto half_step = [&](auto first_tag, auto wait_tag, auto last_tag, v8i (&Pc)[NF], v8i (&Pn)[NF], int hs) {
            constexpr bool FIRST = decltype(first_tag)::value;  // first half step of the tile: the accumulators start at 0
            constexpr int WAIT = decltype(wait_tag)::value;     // 0: half step +1 is known to have landed; 1: wait for it
            constexpr bool LAST = decltype(last_tag)::value;    // last half step of the tile: wait for everything in flight
            const int nxt = cur == NS - 1 ? 0 : cur + 1;
            // stream step +NS is half step hs+NS of this tile, or hs+NS-KT of the next one (when there is none:
            // a harmless in-bounds re-read, so that the load counting stays uniform)
            const bool own = hs + NS < KT;
            const __amdgpu_buffer_rsrc_t ra = own ? a_cur : a_nxt, rb = own ? b_cur : b_nxt;
            const int so = own ? hs + NS : hs + NS - KT;
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                if constexpr (FIRST) {
                    const v16f zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    acc[k / FN][k % FN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(Pc[k / FN], Pc[FM + k % FN], zero, 2, 2, 0, 0, 0, 0);
                } else {
                    acc[k / FN][k % FN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(Pc[k / FN], Pc[FM + k % FN], acc[k / FN][k % FN], 2, 2, 0, 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (k == 0) {
                    if constexpr (LAST) __builtin_amdgcn_s_waitcnt(vmcnt_and_lds(0));
                    else if constexpr (WAIT) __builtin_amdgcn_s_waitcnt(vmcnt_and_lds((NS - 2) * LD));
                    else __builtin_amdgcn_s_waitcnt(vmcnt_and_lds(63));
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                } else {
#pragma unroll
                    for (int x = (k - 1) * RPS; x < k * RPS && x < NF; ++x) Pn[frag_in_order(x)] = read_frag(frag_in_order(x), nxt);
                    if (k - 1 < LD) dma_one(k - 1, cur, ra, rb, so);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
        };
        using yes = std::true_type;
        using no = std::false_type;
        using nowait = std::integral_constant<int, 0>;
        using wait = std::integral_constant<int, 1>;
        // The first NS-2 half steps of a tile find their successor landed (the last half step of the previous tile,
        // or the prologue, waited for everything); they must not wait on the counter, which the epilogue's stores
        // have filled since.
        half_step(yes{}, nowait{}, no{}, Pa, Pb, 0);
        // every wave has passed a barrier of this tile, so nobody reads the previous tile's scales any more: fetch
        // the next tile's into that buffer (complete at this tile's last barrier)
        dma_params(m0n, parity ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        int hs = 1;
        if constexpr (NS >= 4) { half_step(no{}, nowait{}, no{}, Pb, Pa, 1); hs = 2; }
        if constexpr (NS >= 5) { half_step(no{}, nowait{}, no{}, Pa, Pb, 2); hs = 3; }
        if constexpr (NS >= 6) { half_step(no{}, nowait{}, no{}, Pb, Pa, 3); hs = 4; }
        if constexpr (NS >= 7) { half_step(no{}, nowait{}, no{}, Pa, Pb, 4); hs = 5; }
        static_assert(NS <= 7, "unrolled prologue of a tile");
        if (hs & 1) {                                           // Pb holds the operands of half step hs
            for (; hs < KT - 1; hs += 2) {
                half_step(no{}, wait{}, no{}, Pb, Pa, hs);
                half_step(no{}, wait{}, no{}, Pa, Pb, hs + 1);
            }
            half_step(no{}, wait{}, yes{}, Pb, Pa, KT - 1);
        } else {
            for (; hs < KT - 2; hs += 2) {
                half_step(no{}, wait{}, no{}, Pa, Pb, hs);
                half_step(no{}, wait{}, no{}, Pb, Pa, hs + 1);
            }
            half_step(no{}, wait{}, no{}, Pa, Pb, KT - 2);
            half_step(no{}, wait{}, yes{}, Pb, Pa, KT - 1);
        }
        // Pa now holds the operands of the next tile's first half step

        // ---- epilogue of this tile ------------------------------------------------------------------
        {
            constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
            const uint32_t col_off = n_lane < g.N ? (uint32_t)n_lane * ESZ : kPoison;
            (void)col_off;
            ChanParams6<FN> cp;
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                cp.sw[j] = __uint_as_float(sw_raw[j]);
                const uint32_t b2 = bias_raw[j >> 1];
                cp.bias[j] = __half2float(__ushort_as_half((unsigned short)((j & 1) ? b2 >> 16 : b2 & 0xFFFFu)));
            }
            const float *sa_lds = reinterpret_cast<const float *>(par + parity * (BM * 4));
            const int row_w = wm * FM * 32;
            const bool bias = g.bias != nullptr, gelu = g.act == W4A4_ACT_GELU;
            if constexpr (OUT == OUT_Q6) {
                if constexpr (FM == 2 && FN == 4) {
                    const int tn = tile % g.tiles_n;
                    fp6_epilogue_requant<FM, FN>(g, acc, cp, n_lane, m0, row_w, lane, tid, tile / g.tiles_n, tn == 0 && wn == 0,
                                                 sa_lds, reinterpret_cast<float *>(par + 2 * BM * 4));
                }
            } else
            if (OUT == OUT_I32 || (!bias && !gelu)) fp6_epilogue<FM, FN, OUT, false, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (bias && !gelu) fp6_epilogue<FM, FN, OUT, true, false>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else if (!bias && gelu) fp6_epilogue<FM, FN, OUT, false, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
            else fp6_epilogue<FM, FN, OUT, true, true>(g, acc, cp, col_off, m0, row_w, lane, sa_lds);
        }
        if (!has_next) break;
        vb = vb_next; tile = tile_next; m0 = m0n; n0 = n0n; a_cur = a_nxt; b_cur = b_nxt; parity ^= 1;
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_and_lds(0));               // no DMA may outlive the workgroup's LDS
}

template <int FM, int FN, int WM, int WN, int OCC, int NS, int OUT>
struct Fp6Launch {
    static constexpr int BM = WM * FM * 32, BN = WN * FN * 32, NW = WM * WN;
    static constexpr int REAL = (BM + BN) * 3 / 64, BLOCKS = (REAL + NW - 1) / NW * NW;
    static constexpr size_t lds = (size_t)NS * REAL * 1024 + (BLOCKS > REAL ? 1024 : 0) + 2 * BM * 4 + (OUT == OUT_Q6 ? NW * 1024 : 0);
    static KernelState &state() { static KernelState ks; return ks; }
    static auto kernel() { return gemm_fp6_kernel<FM, FN, WM, WN, OCC, NS, OUT>; }
    // resident workgroups on the current device (-1: HIP error).  The requantizing output makes the column tiles of a
    // row panel wait for each other, so its grid is sized from what the runtime reports for this kernel, capped by the
    // occupancy it was compiled for.
    static int slots() {
        const int cus = prepare_kernel(reinterpret_cast<const void *>(kernel()), lds, state());
        if (cus < 0) return -1;
        if (OUT != OUT_Q6) return cus * OCC;
        const int occ = resident_per_cu(reinterpret_cast<const void *>(kernel()), NW * 64, lds, state());
        if (occ < 0) return -1;
        return cus * (occ < OCC ? occ : OCC);
    }
};

template <int FM, int FN, int WM, int WN, int OCC, int NS, int OUT>
static int launch_one6(GemmArgs &g, hipStream_t st) {
    using L = Fp6Launch<FM, FN, WM, WN, OCC, NS, OUT>;
    static_assert(L::lds * OCC <= 160 * 1024, "the workgroups of a CU share 160 KB of LDS");
    if (g.K / kHalf < NS + 2) return W4A4_ERR_UNSUPPORTED_SHAPE;
    g.tiles_m = (g.M + L::BM - 1) / L::BM;
    g.tiles_n = (g.N + L::BN - 1) / L::BN;
    const long slots = L::slots(), tiles = (long)g.tiles_m * g.tiles_n;
    if (slots < 0) return W4A4_ERR_HIP;
    if (tiles > 0x7fffffffL) return W4A4_ERR_UNSUPPORTED_SHAPE;
    unsigned grid = (unsigned)(tiles < slots ? tiles : slots);
    if (OUT == OUT_Q6) {
        // every XCD walks whole row panels: ids up to 8 * (tiles of the fullest XCD); and the column tiles of a panel
        // must sit in different workgroups at the same time
        const long most = (long)((g.tiles_m + kXcd - 1) / kXcd) * g.tiles_n * kXcd;
        grid = (unsigned)(most < (slots & ~(long)(kXcd - 1)) ? most : (slots & ~(long)(kXcd - 1)));
        if (g.N % L::BN || g.tiles_n > (int)(grid / kXcd)) return W4A4_ERR_UNSUPPORTED_SHAPE;
        if (g.wait_for == 0) g.wait_for = g.tiles_n;
        // Whole panels only, when the workgroups walk more than one round: the same tiles_n workgroups then meet at every
        // wait, and the half-tile offset between neighbouring panels (see the kernel) survives the rounds.
        const int per = (int)(grid / kXcd) / g.tiles_n;
        if (per >= 2 && most > (long)grid) {
            grid = (unsigned)(per * g.tiles_n * kXcd);
            g.stagger = 5;                                      // sleeps of 2048 cycles: measured best of 0 .. 17 at K = 1024 and 4096
        }
    }
    if (grid == 0) return W4A4_ERR_UNSUPPORTED_SHAPE;
    launch_gemm(L::kernel(), dim3(grid), dim3(WM * WN * 64), L::lds, st, g);
    return launch_status();
}

template <int OUT>
static int launch_variant6(int variant, GemmArgs &g, hipStream_t st) {
    switch (variant) {
        case 0: return launch_one6<2, 4, 2, 2, 2, 4, OUT>(g, st);   // 128 x 256, two workgroups per CU
        case 1: return launch_one6<3, 2, 2, 2, 2, 5, OUT>(g, st);   // 192 x 128, two workgroups per CU
        case 2: return launch_one6<2, 2, 2, 2, 3, 4, OUT>(g, st);   // 128 x 128, three workgroups per CU
        case 3: return launch_one6<3, 4, 2, 2, 1, 7, OUT>(g, st);   // 192 x 256, one workgroup per CU, one wave per SIMD
        default: return W4A4_ERR_INVALID_ARG;
    }
}

// Column tiles of a row panel that the fused requantize can keep co-resident on the current device (0 = the kernel
// does not fit, -1 = HIP error): the limit on N / 256.
int fp6_requant_max_tiles_n() {
    const int slots = Fp6Launch<2, 4, 2, 2, 2, 4, OUT_Q6>::slots();
    return slots < 0 ? -1 : (slots & ~(kXcd - 1)) / kXcd;
}

// Requires: FP6 operand layout on both sides (symmetric codes in [-7, 7], per-channel weight scales),
// K % 128 == 0, K >= 512, both padded operand matrices below 2^31 bytes; OUT_Q6: N % 256 == 0, the padded output
// matrix below 2^31 bytes, N / 256 within fp6_requant_max_tiles_n().
int launch_fp6(int variant, int out_kind, GemmArgs &g, hipStream_t st) {
    switch (out_kind) {
        case OUT_Q6: return variant == 0 ? launch_one6<2, 4, 2, 2, 2, 4, OUT_Q6>(g, st) : W4A4_ERR_INVALID_ARG;
        case OUT_F16: return launch_variant6<OUT_F16>(variant, g, st);
        case OUT_F32: return launch_variant6<OUT_F32>(variant, g, st);
        case OUT_I32: return launch_variant6<OUT_I32>(variant, g, st);
        default: return W4A4_ERR_INVALID_ARG;
    }
}

}  // namespace w4a4
