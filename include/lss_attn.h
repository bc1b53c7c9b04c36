/*
 * lss_attn.h -- C ABI of the MI355X (gfx950) segment-attention library.
 *
 * The operation is one GPU's share of the distributed self-attention of the
 * LSS Transformer (Section 3, Principle 3): a contiguous segment Q_i of
 * l_s = l_x / N query rows attends to the full, replicated K and V of l_x rows,
 *     E_i = softmax(Q_i K^T / sqrt(d_k)) V                      (Eq. 2)
 * whose row-concatenation over segments is Eq. 1.  d_k is read as the per-head
 * width d; heads are independent column slices of the E_m = H*d columns.  The
 * models are decoder-only (Section 5.1), so with causal != 0 the query at global
 * position g = seg_offset + r sees keys j <= g; masked pairs have weight 0.
 * The headline entry points apply no dropout to the weights; the *_dropout
 * pair below does.
 *
 * The backward pass is the gradient of Eq. 2.  Each segment produces dQ_i and
 * its own contribution ("partial") to dK and dV; the sum of the partials over
 * segments is the full gradient -- the arithmetic of the reduce-scatter that is
 * the backward of the all-gather (Section 3, Principle 4, Fig. 2(v)).
 *
 * Around that operation the header also declares, further down, the rest of a
 * layer as one GPU computes it for its segment: the projections in the
 * fused-communication form with their input and weight gradients (Principle 3,
 * Fig. 2(ii)), and the operations that act on a segment's rows alone
 * (Principles 1 and 2): positional-embedding rows, residual connection with
 * dropout, layer normalisation, GeLU and general linear maps.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     neither frees nor retains them.  They must be 16-byte aligned.
 *   - Activations are [B, L, H, d] contiguous, d fastest (token-major rows of
 *     E_m columns); L = l_s for q_seg/out/dO/dq and l_x for k/v/partials.
 *     lse is [B, H, l_s] float: natural log of the sum of exp(scaled score)
 *     over the visible keys.
 *   - d must be 64 or 128.  0 <= seg_offset, seg_offset + l_s <= l_x, l_x >= 1.
 *     Segments need not be equal.  l_s == 0 or B == 0 is a valid empty call.
 *     B*H <= 65535.  seg_offset does not enter the arithmetic when causal == 0.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work
 *     is enqueued on it; no call synchronises with the host.
 *   - Return value: LSS_OK (0) or a negative lss_status.  On error nothing has
 *     been launched and no output was touched; lss_last_error() describes it.
 *   - Scratch memory comes from the caller: lss_set_workspace() registers one
 *     buffer per GPU, which every call made with that GPU current uses; the *_ex
 *     entry points take a buffer of their own instead.  Kernels launched by one
 *     call use the buffer until they finish, so calls that overlap in time on one
 *     GPU (different streams) must be given different buffers through *_ex.
 *   - Results are bit-reproducible run to run: no atomics, every reduction has a
 *     fixed order.
 */
#ifndef LSS_ATTN_H
#define LSS_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lss_status {
    LSS_OK = 0,
    LSS_ERR_NULL = -1,          /* a required pointer is NULL */
    LSS_ERR_SHAPE = -2,         /* negative size, l_x < 1, B*H too large */
    LSS_ERR_UNSUPPORTED_D = -3, /* d is not 64 or 128 */
    LSS_ERR_ALIGN = -4,         /* a pointer is not 16-byte aligned */
    LSS_ERR_RANGE = -5,         /* seg_offset < 0 or seg_offset + l_s > l_x */
    LSS_ERR_WORKSPACE = -6,     /* workspace missing or smaller than lss_workspace_bytes() */
    LSS_ERR_LAUNCH = -7         /* the HIP runtime refused a launch */
} lss_status;

/* Library version: major * 10000 + minor * 100 + patch. */
int lss_version(void);

/* Message for the last error returned on the calling thread ("" if none). Host pointer, static storage. */
const char *lss_last_error(void);

/*
 * Bytes of device scratch that one forward or backward call of this shape may use
 * (split-KV partial outputs, the row terms D = rowsum(dO * out), partial dQ).
 * Depends on the shape only, not on seg_offset or causal.  Returns 0 for an
 * empty or invalid shape.  `elem_bytes` is 2 (bf16 entry points) or 4 (f32).
 */
size_t lss_workspace_bytes(int64_t l_s, int64_t l_x, int64_t B, int64_t H, int64_t d, int elem_bytes);

/*
 * Hands the library a device buffer (16-byte aligned) to use as scratch from now
 * on by calls made, from any thread, while the GPU that is current now is current.
 * One registration per GPU (at most 64 GPUs).  The caller keeps ownership and
 * must keep the buffer alive until the last call that uses it has finished on the
 * GPU.  (NULL, 0) clears this GPU's registration.
 */
int lss_set_workspace(void *device_ptr, size_t bytes);

/*
 * Forward of Eq. 2 for one segment, bf16 storage, fp32 accumulation.
 *   q_seg [B, l_s, H, d] bf16; k, v [B, l_x, H, d] bf16
 *   out   [B, l_s, H, d] bf16 (written); lse [B, H, l_s] float (written)
 * Scores and P*V products run on bf16 matrix cores; softmax is online over key
 * tiles in fp32; key tiles that the causal mask hides entirely are skipped.
 */
int lss_segment_attn_fwd(const void *q_seg, const void *k, const void *v,
                         int64_t seg_offset, int64_t l_s, int64_t l_x,
                         int64_t B, int64_t H, int64_t d, int causal,
                         void *out, float *lse, void *stream);

/*
 * Backward of Eq. 2 for one segment (gradient described above), bf16 storage.
 *   out, lse: what the forward call wrote;  dO [B, l_s, H, d] bf16
 *   dq [B, l_s, H, d] bf16 (written)
 *   dk_partial, dv_partial [B, l_x, H, d] float (every row written; with
 *   causal != 0 the rows >= seg_offset + l_s are exactly 0)
 */
int lss_segment_attn_bwd(const void *q_seg, const void *k, const void *v,
                         int64_t seg_offset, int64_t l_s, int64_t l_x,
                         int64_t B, int64_t H, int64_t d, int causal,
                         const void *out, const float *lse, const void *dO,
                         void *dq, float *dk_partial, float *dv_partial, void *stream);

/*
 * lss_segment_attn_bwd for callers that cannot allocate or register memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same results bit for bit; the scratch (the rows' start
 * values -D and -lse*sqrt(d), split partial dQ) lives in a buffer of
 * LSS_NOALLOC_SCRATCH_BYTES bytes that is part of the library's device image: every GPU
 * the library runs on holds one until the process ends.  The call allocates and frees
 * nothing and ignores lss_set_workspace().  Shapes whose backward scratch exceeds the
 * buffer are rejected with LSS_ERR_WORKSPACE: that scratch is the part of
 * lss_workspace_bytes(l_s, l_x, B, H, d, 2) that is not the forward's split partial
 * results -- 12 bytes per query row and head, plus 4 B l_s H d bytes per key split of dQ
 * (at most 16; none once B H l_s / 128 reaches 512) -- and lss_last_error() names it.  Nothing in
 * the buffer has to be cleared between calls (every value is written before it is read),
 * but all calls on one GPU share it: calls that overlap in time on one GPU (different
 * streams, different threads) race.  The first call on a GPU looks the buffer's address up
 * (hipGetSymbolAddress), so make it before a capture begins.
 */
#define LSS_NOALLOC_SCRATCH_BYTES (64u << 20)
int lss_segment_attn_bwd_noalloc(const void *q_seg, const void *k, const void *v,
                                 int64_t seg_offset, int64_t l_s, int64_t l_x,
                                 int64_t B, int64_t H, int64_t d, int causal,
                                 const void *out, const float *lse, const void *dO,
                                 void *dq, float *dk_partial, float *dv_partial, void *stream);

/*
 * Single-precision twins (the paper's runs are single precision, Section 5.2):
 * q_seg, k, v, out, dO, dq are float; products run on fp32 matrix cores.
 */
int lss_segment_attn_fwd_f32(const void *q_seg, const void *k, const void *v,
                             int64_t seg_offset, int64_t l_s, int64_t l_x,
                             int64_t B, int64_t H, int64_t d, int causal,
                             void *out, float *lse, void *stream);
int lss_segment_attn_bwd_f32(const void *q_seg, const void *k, const void *v,
                             int64_t seg_offset, int64_t l_s, int64_t l_x,
                             int64_t B, int64_t H, int64_t d, int causal,
                             const void *out, const float *lse, const void *dO,
                             void *dq, float *dk_partial, float *dv_partial, void *stream);

/*
 * Forward and backward with dropout on the attention weights.  Section 2.2 names
 * a dropout next to the softmax in the normalisation of the scores; read as: the
 * softmax row A_w is computed, each weight is kept with probability 1 - p_drop and kept
 * weights are divided by 1 - p_drop, and E_i = dropout(A_w) V.  lse is still the
 * logsumexp of the scores.  The keep decision of a weight depends only on
 * (seed, batch*head, GLOBAL query position seg_offset + r, key position): a
 * segment drops exactly what the sequential computation drops at those
 * positions, so segment outputs still concatenate to the full-sequence result
 * and the partials still add up (Section 3, Principles 3 and 4).  The backward
 * call must be given the same p_drop and seed as the forward call.
 *   p_drop      in [0, 1) (LSS_ERR_RANGE otherwise); 0 is exactly the plain call
 *   seed        any 64-bit value
 *   elem_bytes  2: q_seg, k, v, out, dO, dq are bf16;  4: float
 * All other arguments as in lss_segment_attn_fwd / lss_segment_attn_bwd.
 * With p_drop > 0 the bf16 calls run dropout variants of the tuned kernels; the
 * float case uses the library's general kernels.
 */
int lss_segment_attn_fwd_dropout(const void *q_seg, const void *k, const void *v,
                                 int64_t seg_offset, int64_t l_s, int64_t l_x,
                                 int64_t B, int64_t H, int64_t d, int causal,
                                 double p_drop, uint64_t seed, int elem_bytes,
                                 void *out, float *lse, void *stream);
int lss_segment_attn_bwd_dropout(const void *q_seg, const void *k, const void *v,
                                 int64_t seg_offset, int64_t l_s, int64_t l_x,
                                 int64_t B, int64_t H, int64_t d, int causal,
                                 double p_drop, uint64_t seed, int elem_bytes,
                                 const void *out, const float *lse, const void *dO,
                                 void *dq, float *dk_partial, float *dv_partial, void *stream);

/*
 * General forms of the forward and backward calls: everything the entry points
 * above take, plus per-call flags and a per-call scratch buffer.  With flags = 0,
 * workspace = NULL they are lss_segment_attn_fwd_dropout / _bwd_dropout.
 *   flags      LSS_FLAG_SKIP_MASKED_TAIL (backward, causal != 0): the 128-row key
 *              tiles of dk_partial / dv_partial that lie entirely at or beyond row
 *              seg_offset + l_s -- keys no query of the segment sees, by default
 *              filled with zeros -- are left UNWRITTEN.  For callers whose only use
 *              of the partials is lss_reduce_partials() with rows_valid[i] =
 *              seg_offset + l_s, which never reads those rows: short segments of
 *              long sequences then stop paying for l_x rows of zeros per call (the
 *              segment sum of Section 3, Principle 4 only needs the rows a segment
 *              contributes to).  Other bits must be 0 (LSS_ERR_RANGE).
 *   workspace  DEVICE buffer of at least lss_workspace_bytes() bytes, 16-byte
 *              aligned, used instead of the one registered with lss_set_workspace();
 *              NULL: the registered one.  Calls that overlap in time on one GPU
 *              need a buffer each.
 */
#define LSS_FLAG_SKIP_MASKED_TAIL 1u
int lss_segment_attn_fwd_ex(const void *q_seg, const void *k, const void *v,
                            int64_t seg_offset, int64_t l_s, int64_t l_x,
                            int64_t B, int64_t H, int64_t d, int causal,
                            double p_drop, uint64_t seed, int elem_bytes, unsigned flags,
                            void *workspace, size_t workspace_bytes,
                            void *out, float *lse, void *stream);
int lss_segment_attn_bwd_ex(const void *q_seg, const void *k, const void *v,
                            int64_t seg_offset, int64_t l_s, int64_t l_x,
                            int64_t B, int64_t H, int64_t d, int causal,
                            double p_drop, uint64_t seed, int elem_bytes, unsigned flags,
                            void *workspace, size_t workspace_bytes,
                            const void *out, const float *lse, const void *dO,
                            void *dq, float *dk_partial, float *dv_partial, void *stream);

/*
 * Segment sum of partials (Fig. 2(v): what the reduce-scatter adds up):
 *     out = parts[0] + parts[1] + ... + parts[n-1]   elementwise, in that order.
 *   parts       HOST array of n DEVICE pointers, each [B, l_x, H, d] float
 *   rows_valid  HOST array of n row counts, or NULL.  Rows >= rows_valid[i] of
 *               parts[i] are taken as 0 without being read (for a causal
 *               segment, seg_offset + l_s).  NULL means l_x for every part.
 *   out         DEVICE [B, l_x, H, d] float (written); may alias parts[0] only.
 * 1 <= n; the host arrays are read before the call returns.
 */
int lss_reduce_partials(const float *const *parts, int n, const int64_t *rows_valid,
                        int64_t l_x, int64_t B, int64_t H, int64_t d,
                        float *out, void *stream);

/*
 * The linear maps in front of the attention, in the fused-communication form
 * (Section 3, Principle 3; Fig. 2(ii), (iii)): a segment computes its query from
 * its own rows of the layer input, and key and value from the gathered sequence,
 *     Q_i = x_i W_q,    K = x W_k,    V = x W_v.
 * Section 2.2 gives Q, K and V as linear maps of x with the shape of x: read
 * here as square E_m x E_m weights (E_m = H*d) and no bias.
 *   x      [B, l_x, E_m] bf16, the gathered sequence; x_i is its rows
 *          seg_offset .. seg_offset + l_s - 1
 *   w_q    [E_m, E_m] bf16 row-major;  w_kv [E_m, 2 E_m] bf16 row-major holds
 *          W_k in columns 0 .. E_m-1 and W_v in columns E_m .. 2 E_m-1
 *   q_seg  [B, l_s, H, d] bf16 (written);  k, v [B, l_x, H, d] bf16 (written)
 * bf16 matrix cores, fp32 accumulation, one rounding to bf16 at the end.
 * E_m must be a multiple of 128 and at most 65536 (LSS_ERR_SHAPE otherwise).
 * Uses no workspace.
 */
int lss_project_qkv(const void *x, const void *w_q, const void *w_kv,
                    int64_t seg_offset, int64_t l_s, int64_t l_x,
                    int64_t B, int64_t H, int64_t d,
                    void *q_seg, void *k, void *v, void *stream);

/*
 * Backward of those maps with respect to their inputs (Fig. 2(v)):
 *     dx_q       = dQ_i W_q^T                         [B, l_s, E_m] float (written)
 *     dx_partial = dK_part W_k^T + dV_part W_v^T      [B, l_x, E_m] float (written)
 * dx_q is the gradient that reaches the segment's own rows x_i through the query;
 * dx_partial is this segment's contribution to the gradient of the gathered x,
 * the quantity the reduce-scatter adds over segments: sum it with
 * lss_reduce_partials(parts, n, rows_valid, l_x, B, 1, E_m, ...).
 *   dq          [B, l_s, H, d] bf16;  dk_partial, dv_partial [B, l_x, H, d] float,
 *               as lss_segment_attn_bwd wrote them
 *   rows_valid  leading rows (per batch entry) of the partials that hold data:
 *               l_x, or seg_offset + l_s for a causal segment.  Later rows are not
 *               read; those rows of dx_partial are written as zeros
 *               (lss_project_bwd_ex with LSS_FLAG_SKIP_MASKED_TAIL: 256-row tiles
 *               entirely past rows_valid are left unwritten instead; other flag
 *               bits must be 0).
 * The partials are rounded to bf16 as matrix-core operands; accumulation is fp32.
 * Same restrictions as lss_project_qkv.
 */
int lss_project_bwd(const void *dq, const float *dk_partial, const float *dv_partial,
                    const void *w_q, const void *w_kv,
                    int64_t l_s, int64_t l_x, int64_t rows_valid,
                    int64_t B, int64_t H, int64_t d,
                    float *dx_q, float *dx_partial, void *stream);
int lss_project_bwd_ex(const void *dq, const float *dk_partial, const float *dv_partial,
                       const void *w_q, const void *w_kv,
                       int64_t l_s, int64_t l_x, int64_t rows_valid,
                       int64_t B, int64_t H, int64_t d, unsigned flags,
                       float *dx_q, float *dx_partial, void *stream);

/*
 * One segment's share of the gradients of the projection weights (the gradient
 * averaging over the sequence-parallel group, Section 4, adds the segments'):
 *     dw_q  [E_m, E_m]   = sum_b x_i^T dQ_i                        float (written)
 *     dw_kv [E_m, 2 E_m] = sum_b x^T [dK_part | dV_part]           float (written)
 * the second over the leading rows_valid rows of every batch entry (the segment
 * projected K and V of the whole gathered x itself, Fig. 2(ii)).
 *   x           [B, l_x, E_m] bf16;  dq [B, l_s, H, d] bf16
 *   dk_partial, dv_partial  [B, l_x, H, d] float as lss_segment_attn_bwd wrote them;
 *               rows >= rows_valid are not read.  Rounded to bf16 as matrix-core
 *               operands; accumulation and results are fp32.
 *   scratch     DEVICE buffer of lss_project_bwd_weight_scratch_bytes(l_s, l_x, B, H, d)
 *               bytes (enough for any rows_valid), caller-owned, overwritten.  Rows are
 *               divided into chunks whose partial results are added in chunk
 *               order: bit-reproducible, no atomics.
 * Same restrictions as lss_project_qkv.  l_s = 0 or rows_valid = 0 writes zeros to
 * the gradient concerned.
 */
size_t lss_project_bwd_weight_scratch_bytes(int64_t l_s, int64_t l_x, int64_t B,
                                            int64_t H, int64_t d);
int lss_project_bwd_weight(const void *x, const void *dq, const float *dk_partial,
                           const float *dv_partial, int64_t seg_offset,
                           int64_t l_s, int64_t l_x, int64_t rows_valid,
                           int64_t B, int64_t H, int64_t d,
                           float *dw_q, float *dw_kv,
                           void *scratch, size_t scratch_bytes, void *stream);

/*
 * The segment-local remainder of a layer (Section 3, Principles 1 and 2): each of
 * these works on the rows of one segment alone, with no communication.  bf16
 * activations, fp32 arithmetic, one rounding to bf16 per output.  All pointers are
 * DEVICE pointers, 16-byte aligned; E_m a multiple of 8.  None uses the workspace.
 *
 * Positional embedding (Principle 2): a segment adds only its own contiguous rows
 * of the lookup table,
 *     x[b, r, :] = tok[b, r, :] + pe_table[seg_offset + r, :],
 * and the gradient of those table rows is the sum over the batch, b increasing:
 *     dpe_rows[r, :] = sum_b dx[b, r, :].
 *   tok, x, dx  [B, l_s, E_m] bf16;  pe_table [l_x, E_m] bf16;  dpe_rows [l_s, E_m] float
 * 0 <= seg_offset, seg_offset + l_s <= l_x (LSS_ERR_RANGE otherwise).
 */
int lss_embed_pe_fwd(const void *tok, const void *pe_table, int64_t seg_offset,
                     int64_t l_s, int64_t l_x, int64_t B, int64_t E_m,
                     void *x, void *stream);
int lss_embed_pe_bwd(const void *dx, int64_t l_s, int64_t B, int64_t E_m,
                     float *dpe_rows, void *stream);

/*
 * Residual connection with dropout on the branch (Principle 1 counts dropout among
 * the operations that act on each segment independently):
 *     out = x + dropout(delta),   dropout: keep with probability 1 - p_drop, kept
 *                                 elements times 1 / (1 - p_drop).
 * Element (b, r, c) is decided by the generator of lss_segment_attn_fwd_dropout with
 * (batch*head, row, key) := (b, seg_offset + r, c): a function of the position in
 * the whole sequence, so the segments' results concatenate to the sequential one.
 * The backward of the branch is the same call on the gradient: d delta =
 * lss_residual_dropout_add(NULL, d out, ...) with the same seg_offset, p_drop, seed.
 *   x      [B, l_s, E_m] bf16, or NULL (taken as zeros)
 *   delta, out  [B, l_s, E_m] bf16; out may alias x or delta
 * p_drop in [0, 1) (LSS_ERR_RANGE otherwise); 0 is the plain sum.
 */
int lss_residual_dropout_add(const void *x, const void *delta, int64_t seg_offset,
                             int64_t l_s, int64_t B, int64_t E_m,
                             double p_drop, uint64_t seed, void *out, void *stream);

/*
 * Layer normalisation of each row over its E_m columns (the encoder/decoder blocks
 * of Section 2.2; the paper gives no formula: the usual one, biased variance):
 *     y = (x - mean) * rstd * gamma + beta,   rstd = 1 / sqrt(var + eps).
 *   x, y    [rows, E_m] bf16;  gamma, beta [E_m] float;  mean, rstd [rows] float
 *           (written by the forward, read by the backward)
 * Backward: dx [rows, E_m] bf16, dgamma, dbeta [E_m] float; the sums over rows are
 * taken in a fixed order (within blocks of 32 rows, then over the blocks), through
 *   scratch  DEVICE buffer of lss_layernorm_bwd_scratch_bytes(rows, E_m) bytes,
 *            caller-owned, overwritten.
 * E_m <= 4096 (LSS_ERR_SHAPE otherwise); rows = 0 writes zeros to dgamma, dbeta.
 */
int lss_layernorm_fwd(const void *x, const float *gamma, const float *beta, double eps,
                      int64_t rows, int64_t E_m, void *y, float *mean, float *rstd,
                      void *stream);
size_t lss_layernorm_bwd_scratch_bytes(int64_t rows, int64_t E_m);
int lss_layernorm_bwd(const void *x, const float *gamma, const float *mean,
                      const float *rstd, const void *dy, int64_t rows, int64_t E_m,
                      void *dx, float *dgamma, float *dbeta,
                      void *scratch, size_t scratch_bytes, void *stream);

/*
 * Feed-forward unit (Section 2.2), read as y = GeLU(h W1) W2 without biases, GeLU
 * exact (u Phi(u)), built from three calls forward and three backward:
 *     u = lss_linear_fwd(h, W1);  g = lss_gelu_fwd(u);  y = lss_linear_fwd(g, W2)
 *     dg = lss_linear_bwd_input(dy, W2);  du = lss_gelu_bwd(u, dg);
 *     dh = lss_linear_bwd_input(du, W1)
 *   lss_linear_fwd        c[rows, N] = a[rows, K] w[K, N]
 *   lss_linear_bwd_input  da[rows, K] = dc[rows, N] w[K, N]^T
 *   lss_gelu_fwd / _bwd   elementwise over n elements, n a multiple of 8;
 *                         du = dg * (Phi(u) + u phi(u))
 * a, c, dc, da, u, g, dg, du bf16 row-major; w bf16 row-major.  K and N multiples of
 * 128, at most 65536; rows < 2^31 (LSS_ERR_SHAPE otherwise).  bf16 matrix cores,
 * fp32 accumulation.
 * Weight gradient over a segment's rows (one segment's contribution: the gradient
 * averaging over the sequence-parallel group, Section 4, adds the segments'):
 *   lss_linear_bwd_weight  dw[K, N] = a[rows, K]^T dc[rows, N], float (written)
 *     scratch  DEVICE buffer of lss_linear_bwd_weight_scratch_bytes(rows, K, N)
 *              bytes (0 for few rows: may then be NULL), caller-owned, overwritten.
 *              Rows are divided into chunks whose partial results are added in
 *              chunk order: bit-reproducible, no atomics.  rows = 0 writes zeros.
 * Two fused forms save the GeLU's own passes over memory and give bit-identical
 * results to the calls they replace:
 *   lss_linear_gelu_fwd        u = a w  and  g = GeLU(u)   (u, g [rows, N])
 *   lss_linear_bwd_input_gelu  du = (dc w^T) * GeLU'(u)    (u, du [rows, K])
 */
int lss_linear_fwd(const void *a, const void *w, int64_t rows, int64_t K, int64_t N,
                   void *c, void *stream);
int lss_linear_bwd_input(const void *dc, const void *w, int64_t rows, int64_t K, int64_t N,
                         void *da, void *stream);
size_t lss_linear_bwd_weight_scratch_bytes(int64_t rows, int64_t K, int64_t N);
int lss_linear_bwd_weight(const void *a, const void *dc, int64_t rows, int64_t K, int64_t N,
                          float *dw, void *scratch, size_t scratch_bytes, void *stream);
int lss_linear_gelu_fwd(const void *a, const void *w, int64_t rows, int64_t K, int64_t N,
                        void *u, void *g, void *stream);
int lss_linear_bwd_input_gelu(const void *dc, const void *w, const void *u,
                              int64_t rows, int64_t K, int64_t N, void *du, void *stream);
int lss_gelu_fwd(const void *u, int64_t n, void *g, void *stream);
int lss_gelu_bwd(const void *u, const void *dg, int64_t n, void *du, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LSS_ATTN_H */
