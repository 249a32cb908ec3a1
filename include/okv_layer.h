/*
 * okv_layer -- the linear layers of a decoder layer in the decode stage, for one MI355X.
 *
 * Next to the attention, the paper counts 8 h1^2 + 4 h1 h2 flops per generated token and
 * layer (§IV-D): four h1 x h1 projections and the two matrices of the feed-forward
 * block.  With a decode batch of a few dozen tokens every weight is read once per step
 * and used BS times, so these products are bound by reading the weights from HBM, like
 * the attention is by reading the KV cache.  The entry points below are those products
 * and the layer norm between them; together with kv_append / decode_attn (okv.h) they
 * make a whole decoder layer of the models the paper runs (OPT: layer norm before the
 * attention and before the feed-forward block, ReLU, biases, residual connections).
 *
 * Conventions as in okv.h: C ABI, every pointer DEVICE unless labelled, fp16 tensors
 * row-major and 16-byte aligned, the caller owns all memory, calls enqueue on `stream` (a hipStream_t, NULL
 * = the default stream) and return at once; OKV_OK or a negative OKV_E* code;
 * okv_last_error(NULL) has the message.
 */
#ifndef OKV_LAYER_H
#define OKV_LAYER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OKV_LINEAR_MAX_ROWS 128     /* rows that one launch of the product kernels takes whatever the shape   */
#define OKV_LINEAR_MAX_ROWS_STAGED 192  /* ... and when n_in is a multiple of 256 and the workspace is there    */
#define OKV_LINEAR_MAX_BATCH 4096   /* rows per call: beyond that a call issues several launches              */

struct okv_ctx;   /* okv.h */

/* Rearranges a weight matrix for okv_linear.
 *   src  fp16 [n_out][n_in] row-major (the layout of a framework's linear layer:
 *        out = x * src^T)
 *   dst  fp16, n_out * n_in elements: 16 output features x 32 inputs at a time, stored as
 *        the 64 x 16-byte pieces a wavefront loads with one instruction and feeds to the
 *        matrix cores: piece (lane) of block (n / 16, k / 32) holds
 *        src[16 * (n / 16) + lane % 16][32 * (k / 32) + 8 * (lane / 16) .. + 7]
 * n_out must be a multiple of 16 and n_in of 32.  dst and src must not overlap. */
int okv_pack_linear_weight(void *dst, const void *src, int32_t n_out, int32_t n_in, void *stream);

/* out = act(x * W^T + bias) + residual for a batch of m <= OKV_LINEAR_MAX_BATCH rows
 * (paper §IV-D: the linear layers of the decode stage, 2 n_out n_in flops per row).  Up to
 * OKV_LINEAR_MAX_ROWS rows are one launch, in which every weight is read once, and up to
 * OKV_LINEAR_MAX_ROWS_STAGED when the input width is a multiple of 256 (and the workspace of
 * okv_linear_workspace_bytes is passed); more rows are cut into the fewest launches of nearly
 * equal size, each of which reads the weights again.
 *   x         fp16 [m][n_in]
 *   w_packed  fp16, as okv_pack_linear_weight leaves it
 *   bias      fp16 [n_out] or NULL
 *   residual  fp16 [m][n_out] or NULL (added after the activation; n_seg must be 1)
 *   out       HOST array of n_seg DEVICE pointers: the n_out output features are cut into
 *             n_seg equal runs (1 <= n_seg <= 3, n_out / n_seg a multiple of 16) and run s
 *             is written as fp16 [m][n_out / n_seg] to out[s] -- one product for the query,
 *             key and value projections, each landing in a tensor of its own
 *   relu      1: act = max(., 0); 0: act = identity
 *   workspace DEVICE scratch memory of at least okv_linear_workspace_bytes(m, n_out, n_in)
 *             bytes (workspace_bytes says how much there is); its contents before and
 *             after the call mean nothing.  Calls that may run at the same time (different
 *             streams) need workspaces of their own.  With more than 8 rows and n_in a
 *             multiple of 256 the fast kernel runs: where that fills the GPU better the
 *             input dimension is cut across workgroups, their fp32 shares go through the
 *             workspace and a second small kernel adds them in a fixed order (results do
 *             not vary from run to run).  With fewer rows or another n_in, or when a cut
 *             is wanted and the workspace is NULL or too small, a simpler kernel runs that
 *             needs no workspace.
 * Products accumulate in fp32 on the matrix cores; the result is rounded to fp16 once.
 * residual may alias out[0] (each element is read before it is written, by the same lane). */
int okv_linear(const void *x, const void *w_packed, const void *bias, const void *residual,
               void *const *out, int32_t n_seg, int32_t m, int32_t n_out, int32_t n_in,
               int32_t relu, void *workspace, int64_t workspace_bytes, void *stream);

/* The stacked query / key / value projection of a layer with grouped heads: okv_linear with
 * three output tensors of which the first is q_cols wide and the other two kv_cols
 * (W is [q_cols + 2 kv_cols][n_in] before packing, rows in the order q, k, v; no ReLU, no
 * residual).  With q_cols = kv_cols this is okv_linear with n_seg = 3.
 *   q  fp16 [m][q_cols];  k, v  fp16 [m][kv_cols]   (the shapes kv_append / decode_attn take:
 *      q_cols = n_q_heads * head_dim, kv_cols = n_kv_heads * head_dim)
 * Workspace as for okv_linear(m, q_cols + 2 kv_cols, n_in). */
int okv_linear_qkv(const void *x, const void *w_packed, const void *bias, void *q, void *k, void *v,
                   int32_t m, int32_t q_cols, int32_t kv_cols, int32_t n_in, void *workspace,
                   int64_t workspace_bytes, void *stream);

/* okv_linear (one output tensor) followed by okv_layernorm of its result:
 *   out      = act(x * W^T + bias) + residual          fp16 [m][n_out]
 *   out_norm = LayerNorm(out) with gamma, beta, eps    fp16 [m][n_out], a buffer other than out
 * -- the output projection feeding the second norm of a decoder layer, the feed-forward
 * block feeding the next layer's first norm.  The norm is taken of `out` as stored (after
 * its rounding to fp16), so `out` is bit for bit what okv_linear gives and out_norm what
 * okv_layernorm gives up to the rounding of its fp32 arithmetic; when the fast
 * kernel runs and the workspace holds okv_linear_workspace_bytes, the norm rides on the
 * kernel that adds the shares and one launch and one pass over the rows are saved.
 * n_out at most 16384; other arguments as for okv_linear. */
int okv_linear_layernorm(const void *x, const void *w_packed, const void *bias,
                         const void *residual, void *out, const void *gamma, const void *beta,
                         float eps, void *out_norm, int32_t m, int32_t n_out, int32_t n_in,
                         int32_t relu, void *workspace, int64_t workspace_bytes, void *stream);

/* Bytes of workspace okv_linear wants for this shape on the current device (0 if it
 * would not use one); < 0 on a bad shape. */
int64_t okv_linear_workspace_bytes(int32_t m, int32_t n_out, int32_t n_in);

/* out[i] = (x[i] - mean_i) / sqrt(var_i + eps) * gamma + beta for each of m rows of h
 * numbers (population variance; statistics in fp32).
 *   x, out  fp16 [m][h] (may be the same buffer);  gamma, beta  fp16 [h]
 * h must be a multiple of 8 and at most 16384. */
int okv_layernorm(const void *x, const void *gamma, const void *beta, void *out, int32_t m,
                  int32_t h, float eps, void *stream);

/* One decoder layer's parameters for okv_decoder_step: matrices as okv_pack_linear_weight leaves
 * them, biases and layer-norm vectors fp16.  w_qkv stacks the query, key and value projections
 * ([h1 + 2 kv][h1] before packing, h1 = n_q_heads * head_dim, kv = n_kv_heads * head_dim), w_o is
 * [h1][h1], w_ff1 [h2][h1], w_ff2 [h1][h2]. */
typedef struct {
  const void *ln1_gamma, *ln1_beta;   /* [h1]: the norm before the attention           */
  const void *w_qkv, *b_qkv;          /* [(h1 + 2 kv) x h1] packed, [h1 + 2 kv]         */
  const void *w_o, *b_o;              /* [h1 x h1] packed, [h1]                         */
  const void *ln2_gamma, *ln2_beta;   /* [h1]: the norm before the feed-forward block   */
  const void *w_ff1, *b_ff1;          /* [h2 x h1] packed, [h2]                         */
  const void *w_ff2, *b_ff2;          /* [h1 x h2] packed, [h1]                         */
} okv_decoder_layer;

/* Bytes of scratch that okv_decoder_step needs for a batch of m rows: the layer's intermediate
 * tensors (normed input, q, k, v, attention output, two residual streams, feed-forward hidden). */
int64_t okv_decoder_scratch_bytes(const struct okv_ctx *ctx, int32_t m, int32_t h2);

/* One decode step through n_layers = the context's layers of whole decoder layers (paper §IV-D:
 * per token and layer the attention over the cache plus 8 h1^2 + 4 h1 h2 flops of linear layers),
 * issued from inside the library on the context's compute stream: okv_step_begin, then per layer
 *   a = LayerNorm1(x); q, k, v = a W_qkv^T + b; kv_append(k, v); t = decode_attn(q);
 *   y = x + t W_o^T + b_o;  z = LayerNorm2(y);  u = relu(z W_ff1^T + b_ff1);  x = y + u W_ff2^T + b_ff2
 * and okv_step_end.  The same launches, in the same order, as the calls one by one; what this
 * saves is the caller's time per call (a Python caller spends longer on the six calls of a layer
 * than a small layer runs on the GPU).
 *   layers     HOST array [n_layers]
 *   x          fp16 [B][h1], B = the batch of okv_set_batch (<= OKV_LINEAR_MAX_BATCH); overwritten
 *              with the output of the last layer
 *   scratch    >= okv_decoder_scratch_bytes(ctx, B, h2) bytes, 256-byte aligned
 *   workspace  >= the largest okv_linear_workspace_bytes of the four products
 *   eps        of both layer norms
 * Errors as the calls it stands for; OKV_EINVAL also when the context's out_dtype is not fp16. */
int okv_decoder_step(struct okv_ctx *ctx, const okv_decoder_layer *layers, int32_t n_layers, int32_t h2, void *x,
                     float eps, void *scratch, int64_t scratch_bytes, void *workspace, int64_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* OKV_LAYER_H */
