/*
 * iflow.h - C ABI of libiflow.so: block-quantized weights (Inferflow, arXiv 2401.08294, Section 3)
 * and the fused dequantize-and-multiply of the decode step, for AMD MI355X (gfx950).
 *
 * Conventions that hold for every call
 *   - W is a row-major [rows][cols] matrix (rows = outputs N, cols = reduction length K).  A
 *     quantization block is `block` consecutive elements of one row ("tensor block", Section 3).
 *   - All data pointers are DEVICE pointers owned by the caller and must be 16-byte aligned.
 *     Only `size_t *bytes` of iflow_packed_bytes and the scalar arguments live on the host.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues kernels on that stream and returns; the library allocates nothing, keeps no
 *     per-call state and never synchronises.
 *   - Arguments are validated on the host before anything is launched; a call that returns an
 *     error other than IFLOW_ERR_DEVICE has launched nothing.
 *   - fp16 values cross the ABI as uint16_t bit patterns (IEEE binary16).
 *   - Inputs are assumed finite with |w| <= 65504; otherwise the result is unspecified (no fault).
 *
 * Packed device layout, version 1 (sizes are exact: no padding anywhere)
 *   Every block stores its codes plus two fp16 numbers (remark after Table 3):
 *       scale  = fp16((max - min) / L)      offset = fp16(min)
 *   with L = 2^k - 1 for k-bit levels (Eq.1: 255, 63, 31, 15, 7, 3) and 10 for 3.5-bit (Eq.3).
 *
 *   IFLOW_Q3H_B64 - 32 bytes per block of 64 weights.  The 64 levels q0..q63 give 32 pair codes
 *     c[j] = q[2j]*11 + q[2j+1] (Eq.4, 0..120).  With S, O the 16-bit patterns of scale and offset
 *     the block is eight little-endian 32-bit words
 *       W[i] = c[4i] | c[4i+2]<<7 | ((S>>2i)&3)<<14 | c[4i+1]<<16 | c[4i+3]<<23 | ((O>>2i)&3)<<30
 *     for i = 0..7.  A row of nbk = cols/64 blocks occupies nbk*32 consecutive bytes and rows
 *     follow each other, so row r starts at byte r*nbk*32.  Inside a row, blocks are grouped
 *     into strips of 64 consecutive blocks (the last strip holds the remaining n_t <= 64).  Strip
 *     t starts at byte t*2048 of the row and is stored as two planes: words W[0..3] of each of
 *     its n_t blocks (16 bytes per block, blocks in order), followed by words W[4..7] of each
 *     block.  (One wavefront reads a plane of a full strip as 1 KiB of consecutive bytes.)
 *   IFLOW_Q4_B32 / IFLOW_Q4_B64 - first all codes, row after row, cols/2 bytes per row; then
 *     one 4-byte header {scale, offset} per block, blocks in row-major order.  The levels of
 *     eight consecutive weights v0..v7 form one little-endian 32-bit word whose nibbles, from
 *     the least significant, are v0 v2 v4 v6 v1 v3 v5 v7.
 *   IFLOW_Q8_B32 / IFLOW_Q8_B64 - first all levels as bytes in natural order (cols bytes per
 *     row); then the headers as for 4-bit.
 *   IFLOW_Q6_B64 / IFLOW_Q5_B64 / IFLOW_Q3_B32 / IFLOW_Q2_B32 - a level's bits are split over bit planes, stored one
 *     after the other (each plane: all rows, row after row); then the headers as for 4-bit.  Planes, from the level's
 *     least significant bits: 6-bit = 4 + 2 bits, 5-bit = 4 + 1, 3-bit = 2 + 1, 2-bit = 2.  A plane of width w stores
 *     cols*w/8 bytes per row as little-endian 32-bit words; a word holds the plane's bits of n = 32/w consecutive
 *     weights u0..u(n-1), u(e) at bit (e/2)*w + 16*(e%2): the even weights in the low half, the odd ones in the high
 *     half, each in order.  (For w = 4 this is the 4-bit format's nibble order.  A kernel turns a field of either half
 *     into an fp16 number with one AND-OR, so a plane costs about one instruction per weight and product.)
 */
#ifndef IFLOW_H
#define IFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Formats: names and block sizes from the header rows of Table 3.  The 2-bit format is in Section 1's list of supported
 * quantizations but not in Table 3: it takes the 3-bit format's block size here. */
typedef enum {
    IFLOW_Q8_B32 = 0,   /* 8-bit levels, block 32: 9   bits/weight */
    IFLOW_Q8_B64 = 1,   /* 8-bit levels, block 64: 8.5 bits/weight */
    IFLOW_Q4_B32 = 2,   /* 4-bit levels, block 32: 5   bits/weight */
    IFLOW_Q4_B64 = 3,   /* 4-bit levels, block 64: 4.5 bits/weight */
    IFLOW_Q3H_B64 = 4,  /* 3.5-bit ("Q3H"): 11 levels, two weights per 7-bit code, block 64: 4 bits/weight */
    IFLOW_Q6_B64 = 5,   /* 6-bit levels, block 64: 6.5 bits/weight */
    IFLOW_Q5_B64 = 6,   /* 5-bit levels, block 64: 5.5 bits/weight */
    IFLOW_Q3_B32 = 7,   /* 3-bit levels, block 32: 4   bits/weight */
    IFLOW_Q2_B32 = 8    /* 2-bit levels, block 32: 3   bits/weight */
} iflow_format_t;

typedef enum {
    IFLOW_OK = 0,
    IFLOW_ERR_NULL = 1,     /* a required pointer is NULL */
    IFLOW_ERR_FORMAT = 2,   /* unknown iflow_format_t */
    IFLOW_ERR_SHAPE = 3,    /* rows, cols or batch <= 0, cols not a multiple of the block size, or a size above 2^30 */
    IFLOW_ERR_SIZE = 4,     /* an output buffer is smaller than required */
    IFLOW_ERR_ALIGN = 5,    /* a device pointer is not 16-byte aligned */
    IFLOW_ERR_DEVICE = 6,   /* a HIP call failed; see iflow_last_hip_error() */
    IFLOW_ERR_TIMEOUT = 7   /* iflow_qgemv_chain_check: a phase of a chained launch gave up waiting for its input */
} iflow_status_t;

/* Version of the packed layout described above (1). */
int iflow_layout_version(void);

/* Static text for a status code. */
const char *iflow_status_string(iflow_status_t status);

/* hipError_t (as int) of the most recent failed HIP call made by this library on the calling thread; 0 if none. */
int iflow_last_hip_error(void);

/* Block size (32 or 64), number of levels (2^k for k-bit levels, 11 for 3.5-bit), or -1 for an unknown format.  Table 3 / Eq.1 / Eq.3. */
int iflow_format_block(iflow_format_t format);
int iflow_format_levels(iflow_format_t format);

/* Bytes of the packed matrix: rows*cols/block * (code bytes per block + 4).  This is Table 3's "actual
 * bits/weight" (9, 8.5, 6.5, 5.5, 5, 4.5, 4, 4; 3 for the 2-bit format) times rows*cols/8.  `bytes` is a host pointer. */
iflow_status_t iflow_packed_bytes(iflow_format_t format, int64_t rows, int64_t cols, size_t *bytes);

/* Eq.1 (Eq.3 for Q3H) per block, then Eq.4 packing, into the device layout.
 *   w            [rows][cols] fp32, device, read only
 *   packed       device, at least iflow_packed_bytes() bytes, fully overwritten
 *   packed_bytes capacity of `packed`
 * Per block, in IEEE fp32 without contraction: mn/mx = min/max (a zero of either sign counts as +0),
 * scale = fp16((mx - mn)/L), offset = fp16(mn), both round-to-nearest-even; with s, o the stored
 * values widened to fp32: level = clamp(round_half_away((w - o)/s), 0, L), or 0 when s == 0. */
iflow_status_t iflow_quantize(iflow_format_t format, const float *w, int64_t rows, int64_t cols,
                              void *packed, size_t packed_bytes, void *stream);

/* Eq.5 then Eq.2 with the stored pair: w16[r][k] = fp16(level*scale + offset), the exact value
 * rounded once to nearest-even (fp16 subnormals kept).  w16 is [rows][cols] fp16, device. */
iflow_status_t iflow_dequant(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                             uint16_t *w16, void *stream);

/* The decode step's product at batch 1: y[n] = sum_k w'[n][k] * x[k], w' as defined by
 * iflow_dequant, fp32 accumulation, y rounded to fp16.  The packed matrix is streamed once.
 *   x [cols] fp16, y [rows] fp16, both device. */
iflow_status_t iflow_qgemv(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                           const uint16_t *x, uint16_t *y, void *stream);

/* Several projections of ONE activation vector in one launch: y_i = W'_i x for i < count (1..8), e.g. the q, k, v
 * or the gate, up matrices of a decoder layer, which the decode step applies to the same input.  All matrices have
 * `cols` columns; matrix i has rows[i] rows, its own packed buffer packed[i] and its own output y[i] ([rows[i]] fp16).
 * `packed`, `rows` and `y` are HOST arrays of `count` entries (of device pointers / sizes); they are read during the
 * call and need not outlive it.  Results are those of `count` iflow_qgemv calls, bit for bit.  (Every format takes one
 * launch; rows of more than about 60000 columns, which the one-launch kernels of the formats other than 3.5-bit cannot
 * stage, fall back to one launch per matrix.) */
iflow_status_t iflow_qgemv_multi(iflow_format_t format, int count, const void *const *packed, const int64_t *rows,
                                 int64_t cols, const uint16_t *x, uint16_t *const *y, void *stream);

/* iflow_qgemv_multi with the modules around the linear layer fused into the same launch (every format; for the formats
 * other than the 3.5-bit one the activations of a whole row must fit in LDS: rows longer than 63488 columns, 58368 for
 * the 8-bit formats, are IFLOW_ERR_SHAPE).  Section 2 lists the normalization and activation functions among the configurable
 * modules of a decoder layer ("rms" and "silu" for the LLaMA family) and Section 5's Infer() applies them between
 * the products; fused, the small kernels between the matrix products of a decode step disappear.
 *   x_op = IFLOW_X_PLAIN:     y_i = W'_i x (+ residual_i)
 *   x_op = IFLOW_X_RMS_GAIN:  rms normalization in front of the product.  aux = gains g [cols] fp16.
 *                             y_i = fp16( (W'_i v) / sqrt(mean_k x_k^2 + eps) (+ residual_i) ), v_k = fp16(x_k g_k):
 *                             the normalization's scalar is applied to the fp32 row sums, where it commutes with the
 *                             product, so x is read once and no normalized copy of it is ever stored.
 *   x_op = IFLOW_X_SILU_MUL:  the input of a gated feed-forward's last projection.  aux = second factor [cols] fp16.
 *                             y_i = W'_i v (+ residual_i), v_k = fp16(silu(x_k) aux_k), silu(a) = a / (1 + exp(-a)),
 *                             evaluated in fp32.
 *   residual: HOST array of `count` device pointers ([rows[i]] fp16 each; entries may be null) or null for none;
 *             the sum with the residual is rounded to fp16 once.  residual[i] may equal y[i] (in-place update of a
 *             hidden state); it must not overlap x or aux.
 * eps is used by IFLOW_X_RMS_GAIN only (must be >= 0 and finite); aux must be null for IFLOW_X_PLAIN. */
typedef enum { IFLOW_X_PLAIN = 0, IFLOW_X_RMS_GAIN = 1, IFLOW_X_SILU_MUL = 2 } iflow_x_op_t;
iflow_status_t iflow_qgemv_fused(iflow_format_t format, int count, const void *const *packed, const int64_t *rows,
                                 int64_t cols, const uint16_t *x, iflow_x_op_t x_op, const uint16_t *aux, float eps,
                                 const uint16_t *const *residual, uint16_t *const *y, void *stream);

/* The two first projections of a gated feed-forward and its gate in one launch (Section 2's module table: activation
 * "silu" of the LLaMA family's feed-forward; Section 5's Infer() applies it between the products): with
 * W_gate and W_up both [rows][cols] in `format`,
 *   y_n = fp16( silu(c (W'_gate v)_n) * (c (W'_up v)_n) ),   silu(a) = a / (1 + exp(-a)) in fp32,
 * where x_op = IFLOW_X_PLAIN: v = x, c = 1 (aux must be null), or x_op = IFLOW_X_RMS_GAIN: v_k = fp16(x_k aux_k),
 * c = 1 / sqrt(mean_k x_k^2 + eps) as in iflow_qgemv_fused (IFLOW_X_SILU_MUL: IFLOW_ERR_SHAPE).  Neither projection is
 * stored or rounded on its own; the next product (the "down" projection) reads y as a plain activation vector.
 * x [cols], aux [cols], y [rows] fp16; y must not overlap x or aux.  Row-length limits as for iflow_qgemv_fused. */
iflow_status_t iflow_qgemv_gated(iflow_format_t format, const void *packed_gate, const void *packed_up, int64_t rows,
                                 int64_t cols, const uint16_t *x, iflow_x_op_t x_op, const uint16_t *aux, float eps,
                                 uint16_t *y, void *stream);

/* iflow_qgemv_fused for a small batch of activation vectors (Section 5: with dynamic batching a decode step serves several
 * queries at once; each of them is normalized, gated and carried on by itself): one matrix, 1 <= batch <= 16 vectors,
 *   Y[b][n] = fp16( c_b * sum_k w'[n][k] v[b][k]  (+ residual[b][n]) ),
 * x_op = IFLOW_X_PLAIN: v = X, c_b = 1, aux null; IFLOW_X_RMS_GAIN: v[b][k] = fp16(X[b][k] aux[k]) with the gains aux [cols],
 * c_b = 1 / sqrt(mean_k X[b][k]^2 + eps); IFLOW_X_SILU_MUL: v[b][k] = fp16(silu(X[b][k]) aux[b][k]) with aux [batch][cols],
 * c_b = 1.  X [batch][cols], residual and Y [batch][rows], fp16, device; residual may be null, or Y itself (in place); Y must
 * not overlap X or aux.  All nine formats; cols a multiple of 64; batch 1 is iflow_qgemv_fused, 2..16 run on the matrix
 * cores with the weights streamed once (the kernel of iflow_qgemm); more than 16 vectors: IFLOW_ERR_SHAPE. */
iflow_status_t iflow_qgemm_fused(iflow_format_t format, const void *packed, int64_t rows, int64_t cols, const uint16_t *X,
                                 int64_t batch, iflow_x_op_t x_op, const uint16_t *aux, float eps, const uint16_t *residual,
                                 uint16_t *Y, void *stream);

/* A chain of batch-1 products in ONE launch (every format of Table 3 and the 2-bit format): the decode step applies its projections one
 * after the other to a single token (Section 3; Section 5 calls one such pass over all layers one Infer step), and
 * at 7B sizes each product is so short that the idle time between dependent launches costs as much as a third of
 * the weight stream.  The chain is a list of `nphases` (1..IFLOW_CHAIN_MAX_PHASES) phases.  Phase p multiplies counts[p]
 * (1..IFLOW_CHAIN_MAX_GROUP) matrices, all with cols[p] columns (<= 65536; 8-bit formats <= 61440: a row's activations are staged in LDS), with the
 * activation vector x[p]; the matrices
 * of all phases are listed in order in packed / rows / y (at most IFLOW_CHAIN_MAX_MATRICES in total: a whole 32-layer
 * stack of seven matrices per layer fits several times).  x[p] is either
 *   - an input of the call: device memory that NO output of the call overlaps (workgroups run ahead of each other, so
 *     a later phase's output may be written before a slow workgroup has read an earlier phase's input), or
 *   - exactly the output y[i] of a matrix of an EARLIER phase with rows[i] == cols[p]: the phase then waits, inside
 *     the launch, until that output is complete.
 * Any other overlap of an x with a y, and any overlap between two y, is IFLOW_ERR_SHAPE.  Every y[i] receives what
 * iflow_qgemv would have written, bit for bit, so the chain equals the sequence of iflow_qgemv_multi calls it replaces.
 * The weights never change between tokens, so the chain is described once and launched many times:
 *
 *   iflow_qgemv_chain_plan    validates the chain, writes its description (one descriptor per phase and per matrix) into
 *       `plan`, zeroes `workspace` and fills *chain.  All arrays are HOST arrays read during the call; pointers in them
 *       are device pointers that must stay valid for as long as the chain is launched.  The call synchronises `stream`
 *       (it cannot be captured into a HIP graph); it allocates host memory only.
 *   iflow_qgemv_chain_launch  one kernel launch on `stream`; allocates nothing, may be captured and replayed.
 *   iflow_qgemv_chain_check   synchronises `stream`; IFLOW_ERR_TIMEOUT if a phase of an earlier launch gave up waiting
 *       for its input (its wait exceeded its bound of tens of milliseconds; the launch then still ends, its outputs are
 *       unspecified, and the record stays until the chain is planned again), IFLOW_OK otherwise.
 *
 * plan:      device memory of iflow_qgemv_chain_plan_bytes(nphases, total matrices) bytes, 16-byte aligned, owned by the
 *            caller, read-only for the launches.
 * workspace: device memory of at least iflow_qgemv_chain_workspace_bytes() bytes, 16-byte aligned, owned by the caller,
 *            left alone between launches: it carries the hand-over words and a launch counter from launch to launch.
 *            Its 32-bit words IFLOW_CHAIN_WS_CLOCKS .. +3 are a diagnostic that a caller may read after a launch has ended:
 *            the shader clock counter and the constant 100 MHz counter (low words) as the launch's first workgroup read
 *            them when it started (+0, +1) and when it ended (+2, +3); (end - start) of the first over (end - start) of
 *            the second, times 100, is the clock in MHz that the launch ran at.
 *            Launches of one chain must be ordered (one stream); a second chain needs a plan and a workspace of its own.
 * iflow_chain_t is plain data (no resources behind it): it may be copied and dropped freely.
 *
 * The launch keeps one workgroup per compute unit resident and its phases wait for each other, so it wants the
 * device to itself: if other work holds compute units for long, or two chains run at once, a wait can exceed its bound. */
#define IFLOW_CHAIN_MAX_PHASES 1024
#define IFLOW_CHAIN_MAX_GROUP 4
#define IFLOW_CHAIN_MAX_MATRICES 4096
#define IFLOW_CHAIN_WS_HEADER 4096
#define IFLOW_CHAIN_WS_CLOCKS 8
#define IFLOW_CHAIN_MAGIC 0x69464c57u
typedef struct iflow_chain_t {
    void *plan;                 /* device */
    void *workspace;            /* device */
    int32_t grid, max_strips;   /* launch geometry the plan was written for */
    uint32_t magic, fused;      /* fused: the plan uses the modules of iflow_qgemv_chain_plan_fused */
    int32_t format, lds_bytes;  /* the chain's iflow_format_t; LDS of a launch */
    int64_t max_seq;            /* iflow_decode_stack_plan: rows of the key/value caches (0 for other plans) */
} iflow_chain_t;
iflow_status_t iflow_qgemv_chain_workspace_bytes(int nmatrices, const int64_t *rows, size_t *bytes);
iflow_status_t iflow_qgemv_chain_plan_bytes(int nphases, int nmatrices, size_t *bytes);
iflow_status_t iflow_qgemv_chain_plan(iflow_format_t format, int nphases, const int *counts, const int64_t *cols,
                                      const uint16_t *const *x, const void *const *packed, const int64_t *rows,
                                      uint16_t *const *y, void *plan, size_t plan_bytes, void *workspace,
                                      size_t workspace_bytes, void *stream, iflow_chain_t *chain);
/* iflow_qgemv_chain_plan with the modules that sit between the products of a decoder layer (Section 2's module table:
 * normalization "rms", activation "silu"; Section 5's Infer() applies them between the products) inside the same launch,
 * so that a launch can run whole layers: e.g. o + residual -> rms norm -> silu(gate) * up -> down + residual -> rms norm ->
 * the next layer's q, k, v as four phases.  Arguments as iflow_qgemv_chain_plan, plus (each array may be null = none):
 *   x_op     per phase: IFLOW_X_PLAIN, or IFLOW_X_RMS_GAIN: the phase multiplies the rms-normalized input,
 *            y = (W' v) / sqrt(mean_k x_k^2 + eps[p]) with v_k = fp16(x_k aux[p]_k), as in iflow_qgemv_fused
 *            (aux[p]: the gains, [cols[p]] fp16, an input of the launch that no output overlaps).  IFLOW_X_SILU_MUL:
 *            IFLOW_ERR_SHAPE (use a gated phase).
 *   gated    per phase: nonzero = the phase has exactly two matrices of equal size, the gate and the up projection of a
 *            gated feed-forward, and ONE output y[gate] = fp16(silu(c (W'_gate v)_n) * (c (W'_up v)_n)) ([rows] fp16; c the
 *            normalization's scalar or 1), as in iflow_qgemv_gated; y[up] must be null.  Later phases may take y[gate] as input.
 *   residual per matrix: null, or a vector [rows[m]] fp16 added to the output before its one rounding to fp16: an input of
 *            the launch that no output overlaps (4-byte aligned), or exactly the output y[i] of a matrix of an earlier phase
 *            (any earlier phase: its hand-over words are read at the store, with the same bounded re-read as a phase's
 *            input).  Not for gated phases.
 * A plan without any module is the plan of iflow_qgemv_chain_plan (same kernel, same bits). */
iflow_status_t iflow_qgemv_chain_plan_fused(iflow_format_t format, int nphases, const int *counts, const int64_t *cols,
                                            const uint16_t *const *x, const iflow_x_op_t *x_op, const uint16_t *const *aux,
                                            const float *eps, const int *gated, const void *const *packed, const int64_t *rows,
                                            const uint16_t *const *residual, uint16_t *const *y, void *plan, size_t plan_bytes,
                                            void *workspace, size_t workspace_bytes, void *stream, iflow_chain_t *chain);
iflow_status_t iflow_qgemv_chain_launch(const iflow_chain_t *chain, void *stream);
iflow_status_t iflow_qgemv_chain_check(const iflow_chain_t *chain, void *stream);

/* One decode step of grouped-query attention over an fp16 key/value cache (section "Grouped-query attention":
 * head_i = Attention(Q_i, K^j, V^j), j the group of query head i; scaled dot-product attention; n_kv_heads == n_heads is
 * multi-head attention).  One query position attends to all seq_len cached positions:
 *   out[i][:] = fp16( sum_t softmax_t(scale * q[i] . K[j][t]) * V[j][t][:] ),  j = i / (n_heads / n_kv_heads).
 *   q        [n_heads][head_dim] fp16     (head_dim 64 or 128; other values: IFLOW_ERR_SHAPE)
 *   k_cache  [n_kv_heads][max_seq][head_dim] fp16, v_cache likewise; positions >= seq_len are not read
 *   out      [n_heads][head_dim] fp16
 *   n_heads a multiple of n_kv_heads, any ratio (1: multi-head; n_kv_heads == 1: multi-query; the keys and values are read
 *   once per sixteen query heads of a group); n_heads <= 512; n_kv_heads <= 64; 1 <= seq_len <= max_seq <= 2^20.
 *   workspace: device memory of iflow_attn_decode_workspace_bytes(n_heads) bytes, 16-byte aligned; scratch for the
 *     partial results of the position ranges the sequence is split into (up to 64; a second small kernel merges them),
 *     its contents before and after the call mean nothing.  Launches that share a workspace must be ordered (same stream).
 * Everything is computed in fp32 from the fp16 inputs and rounded to fp16 once; the order of the sums is fixed, so
 * the result does not vary from run to run.  All pointers are device pointers, 16-byte aligned. */
iflow_status_t iflow_attn_decode_workspace_bytes(int n_heads, size_t *bytes);
iflow_status_t iflow_attn_decode(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads,
                                 int n_kv_heads, int head_dim, int64_t seq_len, int64_t max_seq, float scale,
                                 uint16_t *out, void *workspace, size_t workspace_bytes, void *stream);

/* iflow_attn_decode for callers that cannot allocate device memory or hand a workspace over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same results, bit
 * for bit; the partial results of the position ranges go to a device array that is part of the library's code object
 * (IFLOW_ATTN_STATIC_MAX_HEADS * 130 * 64 floats = 4 259 840 bytes, held by every device the library is loaded on
 * until the process ends) instead of a workspace.  n_heads above IFLOW_ATTN_STATIC_MAX_HEADS is IFLOW_ERR_SIZE.  The call
 * allocates nothing and frees nothing.  Every call on a device shares that device's array: calls must be ordered (one
 * stream, or events between streams); calls that overlap on one device race and their outputs are unspecified.  Nothing
 * in the array has to be cleared between calls (a call reads only what it has written itself). */
#define IFLOW_ATTN_STATIC_MAX_HEADS 128
iflow_status_t iflow_attn_decode_static(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads,
                                        int n_kv_heads, int head_dim, int64_t seq_len, int64_t max_seq, float scale,
                                        uint16_t *out, void *stream);

/* Rotary position embedding for one decode step, and the step's append to the key/value cache (Section 2's table of
 * configurable modules: position_embedding = "rope"): the launch that sits between the q/k/v projections and
 * iflow_attn_decode.  Pair i (0 .. d/2 - 1) of a head's d = head_dim components at position p is rotated by the angle
 * p * base^(-2i/d): (a, b) -> (a cos - b sin, a sin + b cos); IFLOW_ROPE_ADJACENT pairs components (2i, 2i+1),
 * IFLOW_ROPE_HALVES pairs (i, i + d/2).
 *   q        [n_heads][d] fp16: rotated IN PLACE
 *   k_new    [n_kv_heads][d] fp16, this step's keys (unrotated); v_new likewise, this step's values
 *   k_cache  [n_kv_heads][max_seq][d] fp16: row `position` of every head receives the rotated keys;
 *   v_cache  likewise: row `position` receives v_new unchanged.  No other row is touched.
 *   0 <= position < max_seq <= 2^20; head_dim a multiple of 8 from 16 to 256; base > 1 (10000 for the LLaMA family).
 * Angles, sines, cosines and the rotation are computed in fp64 and rounded to fp16 once, so that positions in the
 * hundreds of thousands are as exact as position 1.  All pointers are device pointers, 16-byte aligned. */
typedef enum { IFLOW_ROPE_ADJACENT = 0, IFLOW_ROPE_HALVES = 1 } iflow_rope_pairing_t;
iflow_status_t iflow_rope_append(uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, int n_heads, int n_kv_heads,
                                 int head_dim, int64_t position, int64_t max_seq, float base, iflow_rope_pairing_t pair_mode,
                                 uint16_t *k_cache, uint16_t *v_cache, void *stream);

/* A whole decode step of a decoder stack in ONE launch (Section 5: Infer() = one pass over all layers for the step's token;
 * Section 2's module table for the LLaMA family: "rms" normalization, "rope" position embedding, "silu" activation with a gate;
 * section "Grouped-query attention").  Per layer, with h the layer's input [hidden]:
 *   q, k, v = Wq n1, Wk n1, Wv n1          n1 = rmsnorm(h; norm1, eps)
 *   q, k rotated by the rotary embedding at `position`; k, v appended to the layer's caches at row `position`
 *   t = attention(q; cached keys and values of positions 0 .. position)        (scale 1 / sqrt(head_dim))
 *   h1 = h + Wo t
 *   h2 = h1 + Wdown (silu(Wgate n2) * (Wup n2))          n2 = rmsnorm(h1; norm2, eps)
 * and h2 is the next layer's input; the last layer's h2 is h_out.  The products are the chained launch above with its modules
 * (iflow_qgemv_chain_plan_fused), the attention runs as two more phases of the same launch; every vector is rounded to fp16
 * exactly where the separate calls (iflow_qgemv_fused, iflow_rope_append, iflow_attn_decode, iflow_qgemv_gated) round it, and
 * all intermediate vectors are left in `scratch` (per layer, each rounded up to 128 elements: q [hidden], k, v
 * [n_kv_heads * 128] as the products leave them (not rotated: the rotated key goes to the cache), t [hidden], h1 [hidden],
 * silu(gate) * up [ffn], h2 [hidden]; the last layer's h2 goes to h_out instead).
 *   format: a format of the chained launch; head_dim must be 128, hidden = n_heads * 128, n_heads a multiple of n_kv_heads
 *   with 1 or an even number of query heads per key/value head; hidden and ffn multiples of 64.
 *   layers: HOST array of n_layers entries (1 .. 128); every pointer in it a device pointer, 16-byte aligned.
 *   h_in, h_out, scratch: device; h_in is not written and must not overlap h_out or scratch.  Every layer has caches of its
 *   own; caches, gains, h_in, h_out and scratch must not overlap each other (IFLOW_ERR_SHAPE).
 * iflow_decode_stack_sizes gives the bytes of scratch, plan and workspace for a description (pointers in it are not read).
 * iflow_decode_stack_plan is iflow_qgemv_chain_plan for this chain (same rules: synchronises, allocates host memory only);
 * iflow_decode_stack_launch runs one step at 0 <= position < max_seq (IFLOW_ERR_SHAPE otherwise): one kernel launch,
 * allocates nothing, may be captured; iflow_qgemv_chain_check reports a wait that gave up. */
typedef struct iflow_decode_layer_t {
    const void *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down;    /* packed matrices */
    const uint16_t *norm1, *norm2;                              /* rms gains [hidden] fp16 */
    uint16_t *k_cache, *v_cache;                                /* [n_kv_heads][max_seq][128] fp16 */
} iflow_decode_layer_t;
typedef struct iflow_decode_stack_t {
    iflow_format_t format;
    int32_t n_layers, hidden, ffn, n_heads, n_kv_heads, head_dim;
    int64_t max_seq;
    float eps, rope_base;
    int32_t rope_pairing;                                       /* iflow_rope_pairing_t */
    const iflow_decode_layer_t *layers;
    const uint16_t *h_in;
    uint16_t *h_out;
    uint16_t *scratch;
} iflow_decode_stack_t;
iflow_status_t iflow_decode_stack_sizes(const iflow_decode_stack_t *stack, size_t *scratch_bytes, size_t *plan_bytes, size_t *workspace_bytes);
iflow_status_t iflow_decode_stack_plan(const iflow_decode_stack_t *stack, void *plan, size_t plan_bytes, void *workspace,
                                       size_t workspace_bytes, void *stream, iflow_chain_t *chain);
iflow_status_t iflow_decode_stack_launch(const iflow_chain_t *chain, int64_t position, void *stream);

/* Y = X * W'^T for a batch of activations (dynamic batching makes batch > 1 the served case,
 * Section 5): Y[b][n] = sum_k w'[n][k] * X[b][k].
 *   X [batch][cols] fp16, Y [batch][rows] fp16, both device.
 * One backend, chosen by batch: 1 is iflow_qgemv; 2 (8-bit formats: up to 4) runs on the vector units with the
 * activation vectors side by side; up to 31 the weights stream once per sixteen vectors and the multiply runs on the
 * matrix cores (16x16x16 tiles, weights dequantized in registers); from 32 on (and cols a multiple of 64) 128 x 64
 * output tiles run on the matrix cores from dequantized fp16 tiles in LDS - or, up to 256 vectors, further passes of
 * sixteen where a cost model of the two says those are cheaper (few vectors against long rows).  Which kernel runs
 * depends on the shapes, the format and the device only.  Results of one call do not depend on
 * how busy the device is (all sums are taken in a fixed order). */
iflow_status_t iflow_qgemm(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                           const uint16_t *X, int64_t batch, uint16_t *Y, void *stream);

/* Test helper: the device layout read back into plain arrays, so that a check of the quantizer does
 * not depend on the layout.  levels [rows][cols] uint8 (Eq.5 already applied for Q3H);
 * scale16 / offset16 [rows][cols/block] fp16 bit patterns.  All device. */
iflow_status_t iflow_unpack_logical(iflow_format_t format, const void *packed, int64_t rows, int64_t cols,
                                    uint8_t *levels, uint16_t *scale16, uint16_t *offset16, void *stream);

/* Test helper, 3.5-bit format only (others: IFLOW_ERR_FORMAT): the stored pair codes themselves, before Eq.5 takes them
 * apart - codes [rows][cols/2] uint8, code i of a row = 11 q[2i] + q[2i+1] (Eq.4), each below 121.  Device, 16-byte aligned. */
iflow_status_t iflow_unpack_pair_codes(iflow_format_t format, const void *packed, int64_t rows, int64_t cols, uint8_t *codes,
                                       void *stream);

/* Measurement helper (no counterpart in the paper): a plain device copy of `bytes` bytes (a positive multiple of
 * 16; src and dst device, 16-byte aligned, not overlapping) made of the same 16-byte-per-lane nontemporal loads as
 * the weight stream.  Profilers scale their bytes-per-dispatch counters by what they report for this transfer of
 * exactly known size. */
iflow_status_t iflow_calibration_copy(const void *src, void *dst, size_t bytes, void *stream);

/* Measurement helper (no counterpart in the paper): the loads of iflow_calibration_copy without its stores - a
 * kernel that only reads `bytes` bytes (a positive multiple of 16) from `src`.  Timed over the packed weights it
 * gives the rate the memory system delivers to a pure read of them, the ceiling for any kernel that streams them.
 * `sink` is a device word (16-byte aligned) that is written only for one data pattern that real weights do not
 * produce; it exists so that the loads are kept. */
iflow_status_t iflow_calibration_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IFLOW_H */
