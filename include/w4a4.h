/*
 * libw4a4 -- W4A4 quantized linear layer for AMD MI355X (gfx950), C ABI.
 *
 * The layer is the INT4-weight / INT4-activation linear of a BERT-style encoder
 * (arxiv 2301.12017): activations are quantized per token at run time, weights
 * per output channel or per K-group offline, two 4-bit codes travel per byte,
 * the contraction is an integer GEMM with int32 accumulation, and dequantize,
 * bias, GELU and the next layer's quantize are fused behind the GEMM.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronizes; each call enqueues its kernels on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *     returns.  Outputs are valid once the stream reaches that point.
 *   - Return value only (w4a4_status); no exceptions, no errno.  Argument errors
 *     are detected before anything is launched and leave the outputs untouched.
 *   - Matrices are row-major.  Packed code matrices hold element 2j of a row in
 *     bits 0..3 and element 2j+1 in bits 4..7 of byte j; signed codes are 4-bit
 *     two's complement in [-8,7], unsigned codes are in [0,15].  This is the
 *     canonical layout (W4A4_LAYOUT_CANONICAL).  Symmetric operands may instead be
 *     kept in the MFMA operand layout (W4A4_LAYOUT_MFMA, see w4a4_layout), a
 *     byte-wise bijection of the canonical one that halves the unpacking work of
 *     the GEMM.
 *   - Base pointers must be 16-byte aligned, K and N multiples of 32 and 8
 *     (row strides multiples of 16 bytes).  Anything else returns
 *     W4A4_ERR_UNSUPPORTED_SHAPE.  M is arbitrary (M == 0 is a no-op).
 *   - NaN / Inf inputs: results unspecified, never a fault.
 *   - Calls are re-entrant; two calls that share a workspace must be ordered on
 *     one stream.
 */
#ifndef W4A4_H
#define W4A4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    W4A4_OK = 0,
    W4A4_ERR_INVALID_ARG = -1,        /* null required pointer, negative size, mode mismatch ... */
    W4A4_ERR_UNSUPPORTED_SHAPE = -2,  /* alignment / divisibility contract not met */
    W4A4_ERR_WORKSPACE = -3,          /* workspace missing or smaller than w4a4_workspace_bytes() */
    W4A4_ERR_HIP = -4                 /* a launch failed (hipGetLastError) */
} w4a4_status;

/* Sec. 3.1: the symmetric mapping (signed codes, scale only) or the asymmetric
 * mapping (unsigned codes, scale and real-valued zero = the minimum). b = 4. */
typedef enum { W4A4_SYM = 0, W4A4_ASYM = 1 } w4a4_mode;

/* Sec. 4.2 packs two INT4 codes per byte and leaves the nibble encoding open.  Two encodings
 * are understood:
 *   CANONICAL  element 2j in bits 0..3, element 2j+1 in bits 4..7; symmetric codes as two's
 *              complement nibbles, unsigned (asymmetric) codes as they are.
 *   MFMA       chosen so that ONE bitwise AND per register turns packed codes into int8 MFMA
 *              operands: the int8 value of (byte & 0xF0) is 16*v for a two's-complement high
 *              nibble v, and (byte & 0x0F) is the low nibble read as an unsigned number.  The
 *              activation byte keeps element 2j in the low and element 2j+1 in the high nibble,
 *              the weight byte has its nibbles swapped, so that low(A) meets high(W) and
 *              high(A) meets low(W) in the contraction and every product carries the factor 16.
 *              The element in the HIGH nibble is stored as a two's-complement value, the one in
 *              the LOW nibble as an unsigned one:
 *                symmetric codes c in [-8,7]:  high = c,     low = c + 8
 *                    [activations: canonical byte XOR 0x08]
 *                    the contraction yields 16*P + 128*(esum[n] + osum[m]) with
 *                      osum[m] = sum of the ODD-position codes of token m,
 *                      esum[n] = sum of the EVEN-position codes of channel n;
 *                unsigned codes u in [0,15]:   high = u - 8, low = u
 *                    [activations: canonical byte XOR 0x80]
 *                    per weight K-group g the contraction yields
 *                      16*(P_g - 8*AE[m,g] - 8*WO[n,g]) with
 *                      AE[m,g] = sum of the EVEN-position codes of token m inside group g,
 *                      WO[n,g] = sum of the ODD-position codes of channel n inside group g.
 *              The sums travel beside the codes (osum / esum below) and the GEMM removes
 *              their terms again; int32 results (w4a4_gemm_i32) are exact in both layouts.
 * The MFMA layout needs K % 128 == 0 and, for symmetric codes, per-channel weight scales
 * (group == 0); for unsigned codes, weight groups that are multiples of 128 (or one group) whose
 * tables fit the kernel (K / group <= 32 at K <= 4096).  w4a4_preferred_layout tells whether
 * w4a4_linear is faster in it for a shape.
 *   FP6        not a nibble encoding: every symmetric code c in [-7, 7] (the range the quantizers
 *              produce; -8 does not exist here) is stored as the 6-bit FP6 E2M3 number of the same
 *              value (sign, two exponent bits, three mantissa bits), 3/4 byte per code, so that the
 *              GEMM runs on the FP6 form of the matrix instruction with FP32 accumulation: products
 *              and sums of such integers are exact in FP32 below 2^24, i.e. the accumulator IS the
 *              INT32 result of the integer GEMM (Sec. 4.2 counts on INT4 tensor cores at twice the
 *              INT8 rate; on gfx950 that pipe is the FP6 one).  Private to the library in every detail:
 *              - a row of K codes is K/32 operands of 32 codes = 24 bytes; operands 2b and 2b+1 form
 *                the row's 48-byte block b: operand 2b+h as 16 bytes at 16h and 8 bytes at 32 + 8h
 *                (the two 8-byte parts exchanged in storage rows 16..31 of every 32);
 *              - operand o of a row holds codes 32o .. 32o+31 in its 6-bit fields 0 .. 31 (fields
 *                little-endian in the 24 bytes), for activations and weights alike;
 *              - rows are stored in panels, block b of all rows of a panel contiguously (what lets the
 *                GEMM fetch whole kilobytes of consecutive addresses): activations in panels of 64
 *                tokens, token m in storage row m % 64 of panel m / 64; weights in panels of 128
 *                output channels, channel n in storage row (n % 4) * 32 + (n % 128) / 4 of panel
 *                n / 128; a panel is K/64 blocks of [storage row][48 bytes]; matrices are padded with
 *                zero rows to whole panels.  q therefore holds ceil(M/64)*64 (ceil(N/128)*128) rows
 *                of 3K/4 bytes; lda of such a w4a4_act is 3K/4 and is not a stride.
 * The FP6 layout needs symmetric codes, one scale per token / output channel (group == 0),
 * K % 256 == 0, K <= 10240 (the token-wise quantizer stages its rows on chip), and K >= 512 for the GEMM; no code
 * sums travel with it.
 * w4a4_quantize_act, w4a4_quantize_weight, w4a4_gemm_i32 and w4a4_linear understand it (any epilogue: a
 * requantized output in the FP6 layout is written by the GEMM kernel itself, as the next layer's operand - one
 * range per token, N % 256 == 0, N / 256 column tiles co-resident, else UNSUPPORTED_SHAPE -, one in the
 * canonical or the MFMA layout goes through the fp32 rows of the workspace), and so do w4a4_layernorm_quantize,
 * w4a4_part_linear, w4a4_ffn (a fused FFN pair with both parts in it) and w4a4_encoder_layer; the one-launch
 * small-token call w4a4_linear_f16act does not.  Padding rows of a matrix written by the GEMM kernel hold zeros of either sign
 * (the sign bit of a field may be set). */
typedef enum { W4A4_LAYOUT_CANONICAL = 0, W4A4_LAYOUT_MFMA = 1, W4A4_LAYOUT_FP6 = 2 } w4a4_layout;

/* Sec. 4.2: GELU (erf form) may sit between the GEMM and the next quantize. */
typedef enum { W4A4_ACT_NONE = 0, W4A4_ACT_GELU = 1 } w4a4_act_fn;

/* A token-wise quantized activation matrix (App. A, activation quantization). */
typedef struct {
    const uint8_t *q;      /* [M, lda] bytes, first K/2 bytes of a row are codes; layout == FP6:
                              ceil(M/64)*64 * 3K/4 bytes in panels (see w4a4_layout)       */
    const float   *scale;  /* [M]   S of each token                                       */
    const float   *zero;   /* [M]   x_zero of each token; NULL when mode == SYM           */
    const int32_t *gsum;   /* [M, ng] sum of the codes of a token inside each weight
                              K-group; required when mode == ASYM, else may be NULL      */
    int M, K;
    int lda;               /* row stride of q in BYTES (>= K/2, multiple of 16): lets a
                              GEMM read a column slice of a wider packed matrix in place;
                              layout == FP6: 3/4 byte times the row length of the matrix q
                              points into (a multiple of 48; a 64-token panel is 64*lda
                              bytes).  A column slice of whole 64-code blocks [b0, b0+K/64)
                              of a wider matrix is q = matrix + b0*3072, K = its length,
                              lda = the wider matrix's                                    */
    int group;             /* K-group length the gsum was taken over (0 = whole row)     */
    int mode;              /* w4a4_mode */
    int layout;            /* w4a4_layout of q                                           */
    const int32_t *osum;   /* layout == MFMA, SYM: osum[m*ldo] = sum of the odd-position codes
                              of the K codes of token m that this view covers.
                              layout == MFMA, ASYM: osum[g*M + m] = 128 * AE[m,g], group-major
                              [K/group, M] (ldo is ignored).  Else NULL.                  */
    int ldo;               /* SYM: stride of osum in ELEMENTS (>= 1): a column slice of a wider
                              matrix points into a [M, slices] array of partial sums     */
} w4a4_act;

/* A weight matrix quantized offline (App. A, weight quantization), row n = output
 * channel n, groups = contiguous runs of `group` elements along K. ng = K/group. */
typedef struct {
    const uint8_t *q;          /* [N, K/2]; layout == FP6: ceil(N/128)*128 * 3K/4 bytes   */
    const float   *scale;      /* [N, ng]                                                */
    const float   *zero;       /* [N, ng]; NULL when mode == SYM                         */
    const float   *rowsum_deq; /* [N] sum over k of the dequantized weight; ASYM only    */
    int N, K;
    int group;                 /* 0 = one group per output channel, else multiple of 128 */
    int mode;                  /* w4a4_mode */
    int layout;                /* w4a4_layout of q                                       */
    const int32_t *esum;       /* layout == MFMA, SYM: [N] sum of the even-position codes of a
                                  channel.  layout == MFMA, ASYM: [N, ng+1]: WO[n,g] for the ng
                                  groups of channel n, then one word with the fp32 bits of
                                  8 * sum_g scale[n,g] * (float)WO[n,g] (ascending g, every
                                  operation rounded).  Else NULL.                          */
} w4a4_weight;

/* What happens between the int32 accumulators and memory (Sec. 4.2). */
typedef struct {
    const void *bias_f16;   /* [N] fp16, may be NULL                                      */
    int act;                /* w4a4_act_fn                                                */
    int requant;            /* 0: store fp16 [M,N].  1: quantize each fp32 output row per
                               token and store packed codes [M,N/2] + scale (+ zero,gsum) */
    int requant_mode;       /* w4a4_mode of the requantized output                        */
    int requant_group;      /* K-group of the NEXT layer's weights, for out_gsum (0=row);
                               with requant_layout == MFMA: length of the column slices
                               the odd-position sums are kept for (0 = whole row, else a
                               multiple of 256 that divides N)                            */
    int requant_layout;     /* w4a4_layout of the requantized codes (MFMA and FP6 need
                               requant_mode == SYM; FP6 needs operands in the FP6 layout
                               and requant_group 0 or N, and takes no out_gsum)           */
    int schedule;           /* 0 = pick the tile schedule from the built-in shape table
                               (Sec. 4.2: schedules are pre-tuned per shape); > 0 forces
                               schedule number `schedule` (see w4a4_schedule_count)       */
} w4a4_epilogue;

const char *w4a4_version(void);
const char *w4a4_status_string(int status);

/* Number of GEMM tile schedules compiled in, and a short name of schedule i (1-based). */
int         w4a4_schedule_count(void);
const char *w4a4_schedule_name(int schedule);

/* ---- the INT8 sibling of the path (W8A8) ------------------------------------------------------
 * The paper measures its INT4 pipeline against an INT8 one built from the same pieces (Sec. 4.1,
 * Sec. 4.3).  These three calls are that sibling on this hardware, where INT4 and INT8 share the
 * int8 MFMA: Sec. 3.1's symmetric mapping with b = 8 (S = absmax / 127, one code per byte), the
 * INT8 x INT8 -> INT32 GEMM, and the symmetric per-token / per-channel epilogue of w4a4_linear.
 * All pointers are device pointers; calls are asynchronous on `stream`. */

/* Rows of X_f16 [M, ldx] (first K columns) -> q [M, K] int8, scale [M].  Token-wise for activations;
 * called on W [N, K] it is the per-output-channel weight quantizer.  K % 32 == 0, K <= 16384. */
int w8a8_quantize_rows(const void *X_f16, int M, int K, int ldx, int8_t *q, float *scale, void *stream);

/* out[M, N] fp16 = epilogue(Aq[M, K] * Wq[N, K]^T): y = ((float)P * sa[m]) * sw[n] (+ bias) (GELU).
 * lda = row stride of Aq in bytes (>= K, multiple of 16).  K % 64 == 0, K >= 128, N % 8 == 0.
 * Of `ep` only bias_f16 and act are used; ep->requant must be 0. */
int w8a8_linear(const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw,
                int N, int K, const w4a4_epilogue *ep, void *out, void *stream);

/* w8a8_quantize_rows + w8a8_linear in ONE kernel for small token counts, as w4a4_linear_f16act does it
 * for INT4 (Sec. 4.2: at small batch x sequence launch overhead and the quantize kernels decide): the
 * result equals those two calls bit for bit.  X_f16 [M, ldx] fp16, Wq [N, K] int8, sw [N]; K % 64 == 0,
 * K <= 4096, N % 8 == 0; ep->requant must be 0.  Meant for M up to a few hundred tokens. */
int w8a8_linear_f16act(const void *X_f16, int M, int K, int ldx, const int8_t *Wq, const float *sw, int N,
                       const w4a4_epilogue *ep, void *out, void *stream);

/* The int32 accumulators alone (parity export): acc [M, N]. */
int w8a8_gemm_i32(const int8_t *Aq, int lda, const float *sa, int M, const int8_t *Wq, const float *sw,
                  int N, int K, int32_t *acc, void *stream);

/* ---- per-part quantization strategy ---------------------------------------------------------
 * Sec. 4.2 (last paragraphs) builds the four linear parts of an encoder layer (QKV projection,
 * attention output, MLP intermediate, MLP output) as separate components whose INT4 quantization
 * can be switched on or off one by one, because gain and quantize overhead depend on model size,
 * input shape and hardware; Sec. 4.3 reports that on the paper's GPU the smallest inputs are
 * served best with only the MLP intermediate GEMM in INT4.  A part that is switched off runs in
 * a higher-bit type, which costs no accuracy; here that is the INT8 sibling above.  Which
 * combination is fastest is measured in the deployment environment, as the paper tunes its
 * GEMM schedules there. */
enum { W4A4_PART_QKV = 0, W4A4_PART_ATTN_OUT = 1, W4A4_PART_FFN1 = 2, W4A4_PART_FFN2 = 3, W4A4_PARTS = 4 };

/* A strategy is a bit set: bit p (1 << W4A4_PART_*) = part p runs in INT4, else in INT8.
 * W4A4_STRATEGY_FUSED_FFN (needs the FFN1 and FFN2 bits): FFN1's epilogue requantizes its fp32
 * outputs per token and hands packed codes to FFN2 (Sec. 4.2: quantize fused behind bias-add /
 * GELU); without it FFN1 stores fp16 and FFN2 quantizes that. */
#define W4A4_STRATEGY_FUSED_FFN 16
#define W4A4_STRATEGY_ALL_INT4 31

/* One linear part, its weights prepared in both precisions (device pointers, caller-owned). */
typedef struct {
    w4a4_weight   w4;        /* INT4 form, any mode / group / layout w4a4_linear accepts        */
    const int8_t *w8q;       /* INT8 form [N, K] (w8a8_quantize_rows of the same fp16 weights) */
    const float  *w8s;       /* [N]                                                            */
    const void   *bias_f16;  /* [N] or NULL                                                    */
    int           act;       /* w4a4_act_fn                                                    */
} w4a4_part;

/* Bytes of device workspace w4a4_part_linear needs for M tokens (either precision). */
size_t w4a4_part_workspace_bytes(int M, const w4a4_part *P);

/* out_f16 [M, N] = part P applied to X_f16 [M, ldx] (first K columns), in INT4 (int4 != 0:
 * steps a1..a3, in one kernel when the shape allows, else token-wise quantize + w4a4_linear) or in
 * INT8 (one kernel when the shape allows, else w8a8_quantize_rows + w8a8_linear).  The result is bit for
 * bit what those calls give.
 * Asynchronous on `stream`; the workspace (256-byte aligned) is free again when the call's work
 * has finished.  INT8 needs K % 64 == 0, K >= 128. */
int w4a4_part_linear(const void *X_f16, int M, int ldx, const w4a4_part *P, int int4, void *out_f16,
                     void *workspace, size_t workspace_bytes, void *stream);

/* FFN1 (+ its activation) followed by FFN2 under `strategy` (only the FFN1 / FFN2 / FUSED_FFN
 * bits are read).  out_f16 [M, N2].  FUSED_FFN needs symmetric FFN2 weights.  The workspace
 * holds the intermediate [M, N1] as well. */
size_t w4a4_ffn_workspace_bytes(int M, const w4a4_part *ffn1, const w4a4_part *ffn2);
int w4a4_ffn(const void *X_f16, int M, int ldx, const w4a4_part *ffn1, const w4a4_part *ffn2, int strategy,
             void *out_f16, void *workspace, size_t workspace_bytes, void *stream);

/* Measured cost of the options, in microseconds. */
typedef struct {
    float part_us[4][2];     /* [part][0] = INT8, [part][1] = INT4: the part alone, fp16 in, fp16 out */
    float ffn_fused_us;      /* FFN1 + FFN2 in INT4 with the codes handed over in the epilogue        */
} w4a4_strategy_costs;

/* The strategy of least total cost: QKV and attention output are independent choices; the FFN
 * pair costs part_us[FFN1][.] + part_us[FFN2][.], or ffn_fused_us with FUSED_FFN.  Ties go to the
 * strategy with more INT4 parts, then to the fused one.  Pure host arithmetic.  Returns the bit
 * set (never with W4A4_STRATEGY_FUSED_LN, which is not a choice between GEMM precisions), or
 * W4A4_ERR_INVALID_ARG for NULL / negative / non-finite costs. */
int w4a4_strategy_pick(const w4a4_strategy_costs *costs);

/* Measures all options for an encoder layer of this shape (hidden size h: QKV h -> 3h, attention
 * output h -> h, FFN1 h -> ffn with GELU, FFN2 ffn -> h; symmetric per-channel weights, biases)
 * on the current device with synthetic operands: `iters` timed runs per option after two warm-up
 * runs, HIP events on `stream`.  Allocates and frees its own device buffers and synchronizes the
 * stream.  Timings that differ by at most 3 % count as equal (a part's two precisions; the fused
 * pair against its two INT4 parts), so that the tie rules of w4a4_strategy_pick decide and not the
 * timing noise.  Fills *costs with the raw timings (may be NULL), remembers the picked strategy for this
 * (device, M, h, ffn) and returns it (>= 0) or a w4a4_status (< 0).  h % 64 == 0, ffn % 64 == 0, h <= 4096, ffn <= 16384. */
int w4a4_strategy_tune(int M, int hidden, int ffn, int iters, w4a4_strategy_costs *costs, void *stream);

/* The strategy remembered by w4a4_strategy_tune for this shape on the current device, else the
 * built-in table measured on MI355X (every part in INT4; FFN pair fused from 6144 tokens up at
 * hidden sizes >= 1024, from 16384 tokens up below that). */
int w4a4_strategy_lookup(int M, int hidden, int ffn);

/* ---- a whole encoder layer -----------------------------------------------------------------
 * Sec. 4.2 describes the pipeline around the four linears: attention stays in FP16 between the QKV
 * projection and the attention output, LayerNorm (with the residual) follows the attention output
 * and the MLP, and for small batch x sequence the whole sequence of launches is replayed from a
 * graph.  These calls enqueue that sequence for one post-LayerNorm (BERT) encoder layer; capturing
 * it in a HIP graph is the caller's business (every launch is capturable: counters are cleared by
 * fill kernels, nothing is allocated, no host synchronization). */

/* FP16 attention without a mask, a plain stand-in for the attention kernel the paper takes from
 * elsewhere: ctx[b*seq + i, j*64 .. j*64+63] = softmax_k(q_i . k_k / 8) V for every sequence b and
 * head j.  QKV_f16 [batch*seq, 3h], h = heads*64: queries in columns [0,h), keys in [h,2h), values
 * in [2h,3h); ctx_f16 [batch*seq, h].  fp32 arithmetic.  Head size 64 only, 1 <= seq <= 512,
 * pointers 16-byte aligned. */
int w4a4_attention_f16(const void *QKV_f16, int batch, int seq, int heads, void *ctx_f16, void *stream);

/* Strategy bit (needs the FFN1 bit): FFN1 reads the codes LayerNorm 1 produced from its fp32
 * result (Sec. 4.2: quantize fused with the LayerNorm that produces the activation) instead of
 * quantizing the fp16 copy of the residual stream. */
#define W4A4_STRATEGY_FUSED_LN 32

typedef struct {
    int hidden, heads, ffn;                 /* hidden = heads * 64                                  */
    w4a4_part qkv, attn_out, ffn1, ffn2;    /* [3h,h], [h,h], [ffn,h] (its act applies), [h,ffn];
                                               symmetric weights for ffn1 / ffn2                    */
    const void *ln1_gamma_f16, *ln1_beta_f16, *ln2_gamma_f16, *ln2_beta_f16;   /* [h] each         */
    float ln_eps;
} w4a4_encoder_layer_weights;

/* out_f16 [batch*seq, h] = LN2(x1 + ffn2(ffn1(x1))),  x1 = LN1(x + attn_out(attention(qkv(x)))),
 * every part run as `strategy` says (bits of w4a4_strategy_pick plus W4A4_STRATEGY_FUSED_LN).
 * X_f16 [batch*seq, h] dense.  Workspace 256-byte aligned, w4a4_encoder_layer_workspace_bytes
 * large; it holds every intermediate, so one call per workspace at a time. */
size_t w4a4_encoder_layer_workspace_bytes(int batch, int seq, const w4a4_encoder_layer_weights *L);
int w4a4_encoder_layer(const void *X_f16, int batch, int seq, const w4a4_encoder_layer_weights *L, int strategy,
                       void *out_f16, void *workspace, size_t workspace_bytes, void *stream);

/* Measurement hook (no passage of the paper: it serves the roofline figure).  Arms the calling
 * thread: the GEMM kernel of its NEXT w4a4_linear / w4a4_gemm_i32 call records the two HIP events
 * (hipEvent_t, created by the caller with timing enabled) at the kernel's own start and end, the
 * interval a kernel trace reports, free of the dispatch gap that events recorded around the call
 * include.  The arming is consumed by that one launch; two NULLs disarm.  Returns W4A4_OK. */
int w4a4_time_next_gemm(void *start_event, void *stop_event);

/* Measurement probes (no passage of the paper: they give the measured ceilings that a kernel's rate is read
 * against beside the nominal peaks).  Both launch one kernel on `stream`; w4a4_time_next_gemm arms them like a
 * GEMM launch, so the caller times them with the same pair of events.
 *   w4a4_probe_mfma: a register-only loop of independent v_mfma_i32_32x32x32_i8 on every SIMD of the device
 *     (two waves each, eight accumulators per wave, `iters` rounds).  operands [64 lanes][16] 32-bit words
 *     (device): per lane two A operands (words 0..3, 8..11) and two B operands (words 4..7, 12..15) of sixteen
 *     int8 each; the rate depends on their values through the clock the chip keeps (zeros: highest).  Returns
 *     the number of wave-level MFMA instructions issued (65536 integer operations each) or a w4a4_status < 0.
 *   w4a4_probe_mfma_fp6: the same loop of v_mfma_f32_32x32x64_f8f6f4 with both operands FP6 E2M3 (what the FP6
 *     operand layout runs on).  operands [64 lanes][32] words: per lane two A operands (words 0..5, 16..21) and
 *     two B operands (words 8..13, 24..29) of 32 six-bit fields each.  Returns the number of wave-level MFMA
 *     instructions issued (131072 operations each) or a w4a4_status < 0.
 *   w4a4_probe_stream: reads `bytes` (a multiple of 16, 16-byte aligned) from src with coalesced 16-byte loads
 *     and either writes them to dst (a copy) or, with dst == NULL, stores nothing.  Returns a w4a4_status.
 *   sink: one device word that the kernels never write in practice (it keeps their loops alive). */
long w4a4_probe_mfma(const uint32_t *operands, int iters, uint32_t *sink, void *stream);
long w4a4_probe_mfma_fp6(const uint32_t *operands, int iters, uint32_t *sink, void *stream);
int w4a4_probe_stream(const void *src, void *dst, size_t bytes, uint32_t *sink, void *stream);

/* The schedule number (1-based, see w4a4_schedule_name) that w4a4_linear would run this layer on with
 * ep->schedule as given (0 = the built-in shape table), or a w4a4_status < 0 if it would refuse the layer.
 * Host arithmetic only; pointers inside A and W are not read. */
int w4a4_pick_schedule(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep);

/* The layout in which w4a4_linear is fastest for a layer of this shape (Sec. 4.2: the GEMM
 * schedule, and with it the operand layout it reads, is fixed per shape ahead of time).  Both
 * operands of a layer must use the same layout; every layout a layer supports gives identical
 * results. */
int w4a4_preferred_layout(int M, int N, int K, int mode, int group);

/* Bytes of device workspace that are enough for w4a4_linear on ANY layer of this shape and
 * epilogue (0 when none is needed; M*N*4 for a requantizing epilogue). */
size_t w4a4_workspace_bytes(int M, int N, int K, const w4a4_epilogue *ep);

/* Bytes of workspace w4a4_linear needs for exactly this layer on the current device.  A symmetric,
 * per-channel layer with K % 128 == 0 that requantizes to symmetric codes without code sums
 * (want_gsum == 0) runs fused in one kernel and needs only (M + ceil(M/128) + 4) 32-bit words: the
 * column tiles of a row panel exchange per-token maxima through it (Sec. 4.2: quantize
 * fused behind bias-add / GELU).  The fused kernel's workgroups wait for each other, so it is only
 * taken when the runtime's occupancy figure for it on this device says that the tiles which wait
 * for each other are resident together; every other requantizing layer needs M*N*4 bytes: the
 * GEMM leaves fp32 rows there and a second kernel packs them.
 * Failure mode of the fused kernel: a workgroup polls a bounded number of times for its siblings
 * (about a second); if they do not arrive (for instance because kernels of OTHER streams occupy the
 * device's workgroup slots, which the occupancy figure cannot know) it sets the LAST 32-bit word of
 * this workspace and the device-wide flag behind w4a4_fused_fault_check to non-zero and finishes
 * with invalid codes.  Read either one after the stream has been synchronized. */
size_t w4a4_linear_workspace_bytes(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep,
                                   int want_gsum);

/* Waits for `stream`, then returns 1 if any fused-requantize kernel on the current device has given
 * up waiting for its sibling tiles since the last check (and clears the flag), 0 if none has, or a
 * w4a4_status < 0.  This is how callers of w4a4_ffn and w4a4_encoder_layer, whose inner w4a4_linear
 * workspaces are carved by the library, learn of that failure; the outputs of such a call are invalid.
 * Synchronizes; not for capture in a graph. */
int w4a4_fused_fault_check(void *stream);

/* Test hook for that failure path (no passage of the paper).  Fused-requantize kernels launched by the
 * calling thread from now on poll at most spin_limit times (0 = the default bound) and wait for
 * extra_arrivals more sibling tiles than a row panel has (0 = none).  With extra_arrivals > 0 every
 * workgroup gives up after spin_limit polls, raises the fault words and exits normally, so the failure
 * path can be exercised without a hang.  (0, 0) restores the defaults.  Returns W4A4_OK, or
 * W4A4_ERR_INVALID_ARG for a negative argument. */
int w4a4_debug_fused_wait(int spin_limit, int extra_arrivals);

/* Step a0 (offline): App. A weight quantization of W_f16[N,K] with the Sec. 3.1 mapping.
 * Outputs: q[N,K/2], scale[N,ng], zero[N,ng] (ASYM; may be NULL for SYM),
 * gsum[N,ng] code sums (may be NULL), rowsum_deq[N] (may be NULL; needed for ASYM layers).
 * group: 0 or a multiple of 32 that divides K.
 * layout == W4A4_LAYOUT_MFMA also needs esum ([N] for SYM with group == 0; [N, K/group + 1] for ASYM
 * with K % 128 == 0 and group % 128 == 0, see w4a4_weight); else esum is ignored.
 * layout == W4A4_LAYOUT_FP6 (SYM, group == 0, a K the layout exists for: see w4a4_layout): q receives
 * ceil(N/128)*128 rows of 3K/4 bytes (whole panels; the rows past N are written as zeros); gsum[N] = the
 * code sum of a channel. */
int w4a4_quantize_weight(const void *W_f16, int N, int K, int mode, int group,
                         uint8_t *q, float *scale, float *zero, int32_t *gsum, float *rowsum_deq,
                         int layout, int32_t *esum, void *stream);

/* Step a1: token-wise dynamic quantization (App. A) of X_f16[M,K] (row stride ldx
 * ELEMENTS) with the Sec. 3.1 mapping, packed two codes per byte (Sec. 4.2).
 * Outputs: q[M,K/2] (dense rows), scale[M], zero[M] (ASYM only, else may be NULL),
 * gsum[M, K/group] (may be NULL).  K <= 16384.
 * layout == W4A4_LAYOUT_MFMA also needs osum ([M] for SYM; [K/group, M] for ASYM with K % 128 == 0 and
 * group % 128 == 0, see w4a4_act); else osum is ignored.
 * layout == W4A4_LAYOUT_FP6 (SYM, group == 0, a K the layout exists for): q receives ceil(M/64)*64 rows of
 * 3K/4 bytes (whole panels; the rows past M are written as zeros); gsum must be NULL
 * (W4A4_ERR_UNSUPPORTED_SHAPE otherwise). */
int w4a4_quantize_act(const void *X_f16, int M, int K, int ldx, int mode, int group,
                      uint8_t *q, float *scale, float *zero, int32_t *gsum,
                      int layout, int32_t *osum, void *stream);

/* Steps a2+a3 fused: INT4 x INT4 -> INT32 GEMM (Sec. 4.1 shapes, activations [M,K],
 * weights [N,K]) with the dequantize / zero-point terms / bias / GELU epilogue and
 * either an fp16 store or a per-token requantize (Sec. 4.2) behind it.
 *   out:       fp16 [M,N] (requant == 0) or u8 [M,N/2] (requant == 1; requant_layout == FP6:
 *              ceil(M/64)*64 * 3N/4 bytes, all of them written)
 *   out_scale: [M], out_zero: [M] (requant_mode ASYM), out_gsum: [M, N/requant_group]
 *              (may be NULL; with requant_layout == MFMA it is REQUIRED and receives the
 *              odd-position code sums of each column slice); all ignored when requant == 0.
 * A->mode must equal W->mode, A->layout == W->layout, A->K == W->K, and for ASYM
 * A->group == W->group. */
int w4a4_linear(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep,
                void *out, float *out_scale, float *out_zero, int32_t *out_gsum,
                void *workspace, size_t workspace_bytes, void *stream);

/* w4a4_linear for callers that cannot allocate device memory or carry a workspace around: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * checks as w4a4_linear minus the workspace: the exchange area of the fused requantize (per-token
 * maxima, arrival counters, fault word) is a static device array inside the library, 264 208 bytes per
 * GPU, which every GPU the library has run this call on holds until the process ends.  The call
 * allocates nothing, frees nothing and does not synchronize; the array is cleared by a fill kernel on
 * `stream` before each use.
 *   - requant == 0: identical to w4a4_linear (no scratch is involved).
 *   - requant == 1: only layers whose requantize w4a4_linear fuses into the GEMM kernel on this device
 *     (w4a4_linear_workspace_bytes < M*N*4), with M <= 65536 tokens.  Anything else (an unfusable
 *     requantize would need M*N*4 bytes of fp32 rows; more tokens than the array has room for) returns
 *     W4A4_ERR_WORKSPACE before anything is launched or written.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents until the next
 *     call clears it: two requantizing calls that overlap in time on one GPU (different streams, or
 *     threads) race on it.  Order them on one stream, or use w4a4_linear with separate workspaces.
 *   - A give-up of the bounded wait is reported through w4a4_fused_fault_check only. */
int w4a4_linear_static(const w4a4_act *A, const w4a4_weight *W, const w4a4_epilogue *ep,
                       void *out, float *out_scale, float *out_zero, int32_t *out_gsum, void *stream);

/* Producer fusion (Sec. 4.2: the quantize of an activation shares a kernel with the bias-add,
 * GELU or LayerNorm that produces it): LayerNorm over the K features of every token of X (+ R),
 * then step a1 on the result, in one kernel.
 *     v = X + R;  y = (v - mean(v)) / sqrt(var(v) + eps) * gamma + beta      (fp32, biased variance)
 * y is quantized per token from its fp32 value exactly as w4a4_quantize_act quantizes a row
 * (same outputs, same meaning of mode / group / layout / gsum / osum), and stored as fp16 in
 * Y_f16 when that is not NULL (the residual stream of the encoder).
 *   X_f16, R_f16  [M, ldx] fp16 (device; R_f16 may be NULL; 16-byte aligned, ldx*2 % 16 == 0)
 *   gamma_f16, beta_f16  [K] fp16 (device, 16-byte aligned)
 *   Y_f16  [M, K] fp16 or NULL
 *   K % 32 == 0, K <= 4096; groups as for w4a4_quantize_act.  The MFMA and the FP6 operand layouts are
 *   produced for symmetric codes and one range per token only (mode == W4A4_ASYM with either returns
 *   W4A4_ERR_INVALID_ARG); the FP6 layout takes the row lengths w4a4_quantize_act takes in it, no gsum,
 *   and q of ceil(M/64)*64 * 3K/4 bytes, all of them written. */
int w4a4_layernorm_quantize(const void *X_f16, const void *R_f16, int M, int K, int ldx,
                            const void *gamma_f16, const void *beta_f16, float eps, void *Y_f16,
                            int mode, int group, uint8_t *q, float *scale, float *zero, int32_t *gsum,
                            int layout, int32_t *osum, void *stream);

/* Steps a1 + a2 + a3 in ONE kernel, for small token counts (Sec. 4.2: at small batch x
 * sequence the launch overhead and the memory-bound quantize kernels decide the latency):
 * the result equals w4a4_quantize_act(X, SYM, group 0, canonical layout) followed by
 * w4a4_linear(requant = 0) bit for bit, but the codes and scales of the activations never
 * leave the kernel.  Every workgroup re-derives the scales of its 32 tokens, so the cost grows
 * with N/32 * M * K: meant for M up to a few hundred tokens.
 *   X_f16 [M, ldx] fp16 (device, 16-byte aligned, ldx >= K elements, ldx*2 % 16 == 0)
 *   W     symmetric per-channel weights in the canonical layout (K % 64 == 0, K <= 4096,
 *         N % 8 == 0)
 *   ep    bias / activation; ep->requant must be 0
 *   out   fp16 [M, N] (device)
 * UNSUPPORTED_SHAPE for asymmetric / K-grouped / operand-layout weights and for requant. */
int w4a4_linear_f16act(const void *X_f16, int M, int K, int ldx, const w4a4_weight *W,
                       const w4a4_epilogue *ep, void *out, void *stream);

/* Step a2 alone, the INT4 x INT4 -> INT32 GEMM of Sec. 4.1 (activations [M,K] times weights [N,K]
 * transposed, the four encoder shapes) before the dequantize of Sec. 4.2 is applied: the parity /
 * debugging export.  acc[ng, M, N] int32 (device, 16-byte aligned), one plane per weight K-group
 * (App. A groups; ng == 1 for per-channel weights): acc[g,m,n] = sum over the codes k of group g of
 * qa[m,k] * qw[n,k], exact.  Operand rules as for w4a4_linear; schedule as in w4a4_epilogue.
 * Argument errors return before anything is launched. */
int w4a4_gemm_i32(const w4a4_act *A, const w4a4_weight *W, int32_t *acc, int schedule, void *stream);

/* Step a3 alone, the dequantize of Sec. 4.2 (per-token and per-channel / per-group scales of
 * Sec. 3.1 and App. A, the zero-point terms that Sec. 4.3 calls the extra bias-term work of the
 * asymmetric mapping, bias, GELU, then the fp16 store or the next layer's token-wise quantize)
 * applied to int32 accumulators acc[ng, M, N] that are already in device memory (the layout
 * w4a4_gemm_i32 writes).  A and W supply scales, zero points and code sums; their code pointers
 * are not read.  Outputs as for w4a4_linear (requantized codes in the canonical layout only).
 * Needs no workspace.  Argument errors return before anything is launched. */
int w4a4_dequant_epilogue(const int32_t *acc, const w4a4_act *A, const w4a4_weight *W,
                          const w4a4_epilogue *ep, void *out, float *out_scale, float *out_zero,
                          int32_t *out_gsum, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* W4A4_H */
