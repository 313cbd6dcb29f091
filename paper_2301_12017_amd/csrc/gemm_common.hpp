// Pieces shared by the GEMM kernels of libw4a4: argument block, the nibble widening and
// the fused epilogue (dequantize, zero-point terms, bias, GELU, store).
#pragma once
#include <type_traits>

#include "common.hpp"

namespace w4a4 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

// LDS reads the compiler cannot see.  A read it can see, issued while tile DMAs into LDS are in flight, makes it wait
// for every one of those DMAs first (it cannot tell which bytes a DMA writes): at the end of a tile that would
// expose the memory latency of the next tile's prefetch.  The caller guarantees that the bytes were published
// (their DMA waited for by its wave, then a workgroup barrier) and calls lds_unseen_wait on every value before
// its first use.  LDS reads return in order, so the compiler's own counts only become more conservative.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)p;                              // the low 32 bits of a generic LDS pointer are its LDS address
}
__device__ __forceinline__ v4f lds_unseen_b128(uint32_t addr) {
    v4f v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
__device__ __forceinline__ float lds_unseen_b32(uint32_t addr) {
    float v;
    asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
// waits for every LDS read of the wave; the values named here cannot be used before it
template <class T>
__device__ __forceinline__ void lds_unseen_wait(T &v) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v)); }
template <class T>
__device__ __forceinline__ void lds_unseen_also(T &v) { asm volatile("" : "+v"(v)); }   // ... behind an earlier wait

constexpr int kBK = 128;           // codes per K step
constexpr int kRowB = 80;          // LDS row pitch in bytes: 64 of codes + 16 of padding
constexpr int kXcd = 8;

enum { OUT_F16 = 0, OUT_F32 = 1, OUT_I32 = 2, OUT_Q4 = 3, OUT_Q4M = 4, OUT_Q6 = 5 };   // Q4: per-token requantized codes, canonical; Q4M: in the MFMA operand layout; Q6: in the FP6 operand layout

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
    // fused requantize (OUT_Q4): row maxima and arrival counters live in the caller's workspace
    uint32_t *rowmax;              // [M]       bit pattern of max |y| of the row, zeroed before the launch
    int *arrived;                  // [tiles_m] tiles of the row panel that have published their maxima
    int *fault;                    // [1]       set if a workgroup gave up waiting for its siblings
    int *fault_sticky;             // [1]       the device-wide flag behind w4a4_fused_fault_check, set together with *fault
    int spin_limit;                // polls of arrived[panel] before a workgroup gives up
    int wait_for;                  // arrivals a workgroup waits for: tiles_n (a test hook may ask for more)
    float *out_scale;              // [M]
    // MFMA operand layout: code sums that the contraction picks up (see w4a4_layout)
    const int32_t *osum; long ldo; // [M * ldo]  odd-position code sums of the tokens
    const int32_t *esum;           // [N]        even-position code sums of the channels
    int32_t *out_osum; int osum_slices, slice_tiles;   // requantized output: [M, osum_slices] sums, column
                                                       // tiles per slice
    int layout;                    // w4a4_layout of both operands
    int stagger;                   // fused requantize of the FP6 kernel: sleeps by which every second row panel starts late
};

// Widening of packed codes to int8 without sign extension.  For a packed dword d (codes
// k0..k7, low nibble first) of SIGNED codes, (d << 4) & 0xF0F0F0F0 holds 16*k0,16*k2,16*k4,
// 16*k6 and d & 0xF0F0F0F0 holds 16*k1,16*k3,16*k5,16*k7 as int8.  Both GEMM operands are
// widened the same way, so an int8 MFMA accumulates 256 * sum(qa*qw) exactly and the k
// permutation is common to both.  UNSIGNED codes use the 0x0F0F0F0F masks, unscaled.
// One 16-byte LDS read feeds two MFMA K-slices: (x,y) -> lo, (z,w) -> hi.
template <bool SIGNED_>
__device__ __forceinline__ v4i widen2(uint32_t x, uint32_t y) {
    if (SIGNED_) {
        constexpr uint32_t m = 0xF0F0F0F0u;
        return v4i{(int)((x << 4) & m), (int)(x & m), (int)((y << 4) & m), (int)(y & m)};
    } else {
        constexpr uint32_t m = 0x0F0F0F0Fu;
        return v4i{(int)(x & m), (int)((x >> 4) & m), (int)(y & m), (int)((y >> 4) & m)};
    }
}
template <bool SIGNED_>
__device__ __forceinline__ void widen(const uint4 &p, v4i &lo, v4i &hi) {
    lo = widen2<SIGNED_>(p.x, p.y);
    hi = widen2<SIGNED_>(p.z, p.w);
}

// XCD x (workgroup id % 8) gets a contiguous range of tiles, so the tiles that share an
// activation row panel run on one XCD and hit its L2.
__device__ __forceinline__ int xcd_tile(int bid, int total) {
    const int x = bid % kXcd, i = bid / kXcd;
    const int per = total / kXcd, rem = total % kXcd;
    return x * per + (x < rem ? x : rem) + i;
}

// Row of the output tile held in accumulator register r of fragment row i (32x32 MFMA
// layout: lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4).
__device__ __forceinline__ int frag_row(int i, int r, int lane) {
    return i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), (short)0, (int)bytes, 0x00020000);
}

// Store FN consecutive 32-bit or 16-bit values through a buffer descriptor: offsets past the
// end of the buffer (rows >= M, or the poisoned offset of a lane whose channels are >= N) are
// dropped by the hardware, so the epilogue needs no branches.
// AUX: cache-policy bits of the store (0 = default; kStreamed = non-temporal: the output is written once
// and not read by this kernel, so it should not displace the operand tiles in L2).
constexpr int kStreamed = 2;
template <int FN, int AUX = 0>
__device__ __forceinline__ void store_words(__amdgpu_buffer_rsrc_t rs, uint32_t off, const uint32_t (&w)[FN]) {
    if constexpr (FN == 1) __builtin_amdgcn_raw_buffer_store_b32(w[0], rs, off, 0, AUX);
    else if constexpr (FN == 2) __builtin_amdgcn_raw_buffer_store_b64(u32x2{w[0], w[1]}, rs, off, 0, AUX);
    else if constexpr (FN == 4) __builtin_amdgcn_raw_buffer_store_b128(u32x4{w[0], w[1], w[2], w[3]}, rs, off, 0, AUX);
    else {
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{w[0], w[1], w[2], w[3]}, rs, off, 0, AUX);
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{w[4], w[5], w[6], w[7]}, rs, off + 16, 0, AUX);
    }
}
template <int FN, int AUX = 0>
__device__ __forceinline__ void store_halves(__amdgpu_buffer_rsrc_t rs, uint32_t off, const float (&y)[FN]) {
    if constexpr (FN == 1) {
        __builtin_amdgcn_raw_buffer_store_b16(__half_as_ushort(__float2half_rn(y[0])), rs, off, 0, AUX);
    } else {
        uint32_t w[FN / 2];
#pragma unroll
        for (int j = 0; j < FN / 2; ++j) {
            __half2 h = __floats2half2_rn(y[2 * j], y[2 * j + 1]);
            w[j] = *reinterpret_cast<uint32_t *>(&h);
        }
        store_words<FN / 2, AUX>(rs, off, w);
    }
}

// GELU of FN pre-activations, stored as fp16 (see gelu_erf_half2)
template <int FN, int AUX = 0>
__device__ __forceinline__ void store_gelu_halves(__amdgpu_buffer_rsrc_t rs, uint32_t off, const float (&y)[FN]) {
    if constexpr (FN == 1) {
        __builtin_amdgcn_raw_buffer_store_b16(gelu_erf_half(y[0]), rs, off, 0, AUX);
    } else {
        uint32_t w[FN / 2];
#pragma unroll
        for (int j = 0; j < FN / 2; ++j) w[j] = gelu_erf_half2(y[2 * j], y[2 * j + 1]);
        store_words<FN / 2, AUX>(rs, off, w);
    }
}

constexpr uint32_t kPoison = 0x80000000u;     // an offset no output buffer reaches (M*N*4 < 2^31)

// Per-lane constants of the epilogue, fetched before the main loop so that their latency
// is hidden: the FN output channels of this lane start at n_lane.
template <int FN>
struct EpiLane {
    float sw[FN];      // per-channel weight scale (ungrouped layers), pre-divided by 256 for
                       // signed codes (the accumulators hold 256 * P; a power of two, so exact)
    float bias[FN];
    float c[FN];       // weight row sums (asymmetric layers)
    uint32_t col_off;  // byte offset of channel n_lane in an output row, or kPoison
    int nc;            // n_lane clamped into range, for loads
};

template <int FN, int MODE, bool GROUPED, int OUT>
__device__ __forceinline__ EpiLane<FN> epilogue_prefetch(const GemmArgs &g, int n_lane) {
    constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
    EpiLane<FN> e;
    const bool n_ok = n_lane < g.N;
    e.nc = n_ok ? n_lane : 0;
    e.col_off = n_ok ? (uint32_t)n_lane * ESZ : kPoison;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        e.sw[j] = (!GROUPED && OUT != OUT_I32) ? g.sw[e.nc + j] * (MODE == W4A4_SYM ? 0.00390625f : 1.0f) : 0.0f;
        e.bias[j] = (OUT != OUT_I32 && g.bias) ? __half2float(g.bias[e.nc + j]) : 0.0f;
        e.c[j] = (MODE == W4A4_ASYM && OUT != OUT_I32) ? g.c[e.nc + j] : 0.0f;
    }
    return e;
}

// Stage the per-token scales (and zero points) of the BM rows of a tile in LDS; rows past M
// read as zero.  Call before a workgroup barrier that precedes the epilogue.
template <int BM, int NT, int MODE>
__device__ __forceinline__ void stage_token_params(const GemmArgs &g, int m0, float *sa_lds, float *za_lds, int tid) {
    for (int r = tid; r < BM; r += NT) {
        const int m = m0 + r;
        sa_lds[r] = m < g.M ? g.sa[m] : 0.0f;
        if (MODE == W4A4_ASYM) za_lds[r] = m < g.M ? g.za[m] : 0.0f;
    }
}

// The fused epilogue of one wave.  The lane holds, for every (i, r), FN consecutive
// output channels n_lane..n_lane+FN-1 of token m0 + row_w + frag_row(i, r), row_w being the
// wave's first row inside the workgroup tile.  Operation order (every operation separately
// rounded):
//   SYM, per-channel:  y = ((float)P * sa[m]) * sw[n]     (evaluated on 256*P and sw/256)
//   grouped:           y = sa[m] * t1,  t1 = sum_g sw[n,g]*(float)P_g  (kept in facc)
//   ASYM adds:         t2 = sum_g zw[n,g]*(float)RA[m,g];  y = y + sa*t2;  y = y + za*c[n]
//   then + bias[n], then GELU; store fp16 / fp32 / (OUT_I32: the raw integer sums).
// Token parameters and (asymmetric layers) the group zero points / code sums come from LDS,
// channel parameters from registers, and stores go through a
// bounds-checked buffer descriptor (rows >= M and poisoned columns are dropped by the
// hardware), so the epilogue is straight-line code.
template <int FM, int FN, int MODE, bool GROUPED, int OUT>
__device__ __forceinline__ void tile_epilogue(const GemmArgs &g, v16i (&acc)[FM][FN],
                                              float (&facc)[GROUPED ? FM : 1][GROUPED ? FN : 1][16],
                                              const EpiLane<FN> &e, int m0, int row_w, int lane,
                                              const float *sa_lds, const float *za_lds,
                                              const float *zw_lds = nullptr, const float *ra_lds = nullptr,
                                              int n_local = 0, int BMt = 0, int BNt = 0) {
    constexpr bool SGN = MODE == W4A4_SYM;
    constexpr int ESZ = OUT == OUT_F16 ? 2 : 4;
    if (GROUPED && OUT == OUT_I32) return;                       // planes were stored group by group
    const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * g.N * ESZ));
    const uint32_t row_bytes = (uint32_t)g.N * ESZ;
    // offset of (row m0 + row_w + 4*(lane/32), channel n_lane); the per-(i,r) part is uniform
    const uint32_t lane_off = (uint32_t)(m0 + row_w + 4 * (lane >> 5)) * row_bytes + e.col_off;

    if constexpr (OUT == OUT_I32) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                uint32_t w[FN];
#pragma unroll
                for (int j = 0; j < FN; ++j) w[j] = (uint32_t)(SGN ? (acc[i][j][r] >> 8) : acc[i][j][r]);
                store_words<FN>(o_rsrc, lane_off + (uint32_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * row_bytes, w);
            }
    } else {
        const bool has_bias = g.bias != nullptr;
        auto body = [&](auto gelu_tag) {
            constexpr bool GELU = decltype(gelu_tag)::value;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int rl = row_w + i * 32 + 8 * q + 4 * (lane >> 5);      // 4 consecutive rows
                    const float4 sa4 = *reinterpret_cast<const float4 *>(sa_lds + rl);
                    float4 za4 = make_float4(0.f, 0.f, 0.f, 0.f);
                    if constexpr (MODE == W4A4_ASYM) za4 = *reinterpret_cast<const float4 *>(za_lds + rl);
                    const float sav[4] = {sa4.x, sa4.y, sa4.z, sa4.w}, zav[4] = {za4.x, za4.y, za4.z, za4.w};
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int r = q * 4 + rr;
                        const float sam = sav[rr];
                        float y[FN];
                        if constexpr (!GROUPED) {
#pragma unroll
                            for (int j = 0; j < FN; ++j) {
                                float t = (float)acc[i][j][r] * sam;
                                y[j] = t * e.sw[j];
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < FN; ++j) y[j] = sam * facc[GROUPED ? i : 0][GROUPED ? j : 0][r];
                            if constexpr (MODE == W4A4_ASYM) {
                                // zero points and code sums of the tile were staged in LDS as
                                // zw_lds[g][channel in tile] and ra_lds[g][row in tile] (as floats)
                                float t2[FN];
#pragma unroll
                                for (int j = 0; j < FN; ++j) t2[j] = 0.0f;
                                for (int grp = 0; grp < g.ng; ++grp) {
                                    const float ra_f = ra_lds[grp * BMt + rl + rr];
#pragma unroll
                                    for (int j = 0; j < FN; ++j) {
                                        float w = zw_lds[grp * BNt + n_local + j] * ra_f;
                                        t2[j] = t2[j] + w;
                                    }
                                }
#pragma unroll
                                for (int j = 0; j < FN; ++j) {
                                    float p = sam * t2[j];
                                    float z = zav[rr] * e.c[j];
                                    y[j] = y[j] + p;
                                    y[j] = y[j] + z;
                                }
                            }
                        }
                        if (has_bias) {
#pragma unroll
                            for (int j = 0; j < FN; ++j) y[j] = y[j] + e.bias[j];
                        }
                        const uint32_t off = lane_off + (uint32_t)(i * 32 + 8 * q + rr) * row_bytes;
                        if constexpr (OUT == OUT_F32) {
                            uint32_t w[FN];
#pragma unroll
                            for (int j = 0; j < FN; ++j) w[j] = __float_as_uint(GELU ? gelu_erf(y[j]) : y[j]);
                            store_words<FN>(o_rsrc, off, w);
                        } else if constexpr (GELU) {
                            store_gelu_halves<FN>(o_rsrc, off, y);
                        } else {
                            store_halves<FN>(o_rsrc, off, y);
                        }
                    }
                }
        };
        if (g.act == W4A4_ACT_GELU) body(std::true_type{});
        else body(std::false_type{});
    }
}


// Bounded wait of the fused requantize: thread 0 of a workgroup announces the workgroup on arrived[panel] and
// polls until g.wait_for column tiles of the row panel have done the same.  Only relaxed device-scope atomics
// are used (they are performed at the coherence point and bypass the L1): a release / acquire FENCE at device
// scope would write back and invalidate the whole L2 on every poll.  Ordering comes from waiting for this
// wave's atomics to be acknowledged (vmcnt) before the workgroup barrier that precedes the counter increment.
// The wait never hangs: after g.spin_limit polls the workgroup raises both fault words and carries on (its
// codes are then invalid; the host learns of it from w4a4_fused_fault_check or the workspace word).
__device__ __forceinline__ void panel_arrive_and_wait(const GemmArgs &g, int panel, int tid) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) {
        __hip_atomic_fetch_add(g.arrived + panel, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while (__hip_atomic_load(g.arrived + panel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < g.wait_for) {
            __builtin_amdgcn_s_sleep(1);
            if (++spins > g.spin_limit) {
                *g.fault = 1;
                *g.fault_sticky = 1;
                break;
            }
        }
    }
    __syncthreads();
}


// Fused per-token requantize of one wave's part of the tile (symmetric output codes, Sec. 4.2:
// the next layer's quantize rides behind bias-add / GELU).  The range of a token needs the
// whole output row, which is spread over the tiles_n workgroups of the row panel, so:
//   1. every lane turns its accumulators into the fp32 outputs y (same operation order as the
//      fp32 store path), keeps them in the accumulator registers and notes max|y| of its four
//      channels for each of its 32 rows;
//   2. a butterfly over the 32 lanes that share the rows (exchange with a partner per index bit while
//      halving the set of rows a lane is responsible for) leaves lane c with the maximum of
//      row c, which it publishes with ONE atomic max on rowmax[m] (non-negative floats order
//      like integers);
//   3. the workgroup announces itself on arrived[panel] and waits until all tiles_n siblings
//      have done so (they are co-resident: consecutive workgroup ids of one XCD; the wait is
//      bounded and raises *fault instead of hanging);
//   4. lane c fetches the final maximum of row c, derives scale = max/7 and 7/max and shares
//      the reciprocal with the other lanes of the row through `scratch` (LDS, 64 floats per
//      wave).  code = rne(y * (7/max)) as in quantize_act: |y * (7/max)| <= 7(1+2^-23), so the
//      clamp of the definition cannot bind and the rounding is done by adding 1.5*2^23 + 8
//      (round-to-nearest-even of the fp32 add), which leaves code+8 in the low four bits.
//      Eight codes per dword are assembled from two neighbouring lanes.  The wave that owns
//      channel 0 writes the scales.
template <int FM, int FN>
__device__ __forceinline__ void tile_epilogue_requant(const GemmArgs &g, v16i (&acc)[FM][FN], const EpiLane<FN> &e,
                                                       int m0, int row_w, int lane, int tid, int panel,
                                                       const float *sa_lds, float *scratch) {
    static_assert(FN == 4 && FM == 2, "32 rows per half wave; two lanes assemble one dword of eight codes");
    const bool gelu = g.act == W4A4_ACT_GELU;
    const bool n_ok = e.col_off != kPoison;
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
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    float t = (float)acc[i][j][q * 4 + rr] * sav[rr];
                    t = t * e.sw[j];
                    y[rr][j] = t + e.bias[j];                     // 0 without a bias: changes at most the sign of a zero
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
        if (m_c < g.M && __shfl(e.col_off, lane & 32, kWave) == 0)
            g.out_scale[m_c] = rg.S;                              // this wave holds channel 0 of the row
        scratch[(tid & ~63) + lane] = rg.inv;
        __builtin_amdgcn_wave_barrier();
    }
    // packed rows are N/2 bytes; even lanes store a dword of eight codes, everything else is
    // sent to an offset the bounds check of the descriptor drops
    const __amdgpu_buffer_rsrc_t q_rsrc = make_rsrc(g.out, (uint32_t)((long)g.M * (g.N / 2)));
    const uint32_t row_b = (uint32_t)g.N / 2;
    const uint32_t lane_q = ((lane & 1) == 0 && n_ok)
                                ? (uint32_t)(m0 + row_w + 4 * h) * row_b + (uint32_t)(e.nc >> 1) : kPoison;
    constexpr float kMagic = 12582912.0f + 8.0f;                  // 1.5 * 2^23 + 8
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 iv4 = *reinterpret_cast<const float4 *>(scratch + (tid & ~63) + h * 32 + i * 16 + q * 4);
            const float ivv[4] = {iv4.x, iv4.y, iv4.z, iv4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = q * 4 + rr;
                uint32_t packed = 0;
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    float t = __int_as_float(acc[i][j][r]) * ivv[rr];
                    float u = t + kMagic;                         // low mantissa bits = rne(t) + 8
                    packed |= (__float_as_uint(u) & 0xFu) << (4 * j);
                }
                packed ^= 0x8888u;                                // offset binary -> two's complement
                const uint32_t other = __shfl_down(packed, 1, kWave);   // the next lane holds the next four channels
                __builtin_amdgcn_raw_buffer_store_b32(packed | (other << 16), q_rsrc,
                                                      lane_q + (uint32_t)(i * 32 + 8 * q + rr) * row_b, 0, 0);
            }
        }
}

// Launchers of the kernel families (each defined in the file of its kernel).
// `variant` selects the tile shape; both return a w4a4_status.
int launch_generic(int variant, int mode, bool grouped, int out_kind, GemmArgs &g, hipStream_t st);
int launch_pipe(int variant, int out_kind, GemmArgs &g, hipStream_t st);
int launch_olay(int variant, int out_kind, GemmArgs &g, hipStream_t st);
int launch_fp6(int variant, int out_kind, GemmArgs &g, hipStream_t st);
int launch_group(int mode, int out_kind, GemmArgs &g, hipStream_t st);
int launch_small_packed(int out_kind, GemmArgs &g, hipStream_t st);
// Residency limits of the fused requantize on the current device (see the definitions)
int olay_requant_max_tiles_n(bool mfma_out);
int fp6_requant_max_tiles_n();
int pipe_requant_max_tiles();

}  // namespace w4a4
