/*
 * libstreambp - StreamBP hot path for AMD MI355X (gfx950): the sequence-chunked,
 * layer-wise exact backward pass of a decoder-only transformer.
 *
 * For every chunk of the sequence the library recomputes that chunk's forward
 * and runs its backward; weight gradients, the prefix dK/dV and the input
 * gradient accumulate across chunks, so full-sequence activations and logits are
 * never stored (paper Sec. 3.1, Eq. 1: the full chain-rule product is the sum of
 * the per-chunk products over any partition of the module's output).
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - All tensor pointers are DEVICE pointers owned by the caller; config and
 *    weight-table structs are HOST memory, read before the call returns.
 *  - The library never allocates, frees or synchronises.  Work is enqueued on
 *    `hip_stream` (a hipStream_t passed as void*; NULL = the default stream) and is
 *    complete when that stream is.  Scratch memory comes from the caller through
 *    `workspace`; the matching *_workspace_bytes() call gives the size needed.
 *    Workspace must be 256-byte aligned.  Two calls may not share a workspace
 *    unless they are ordered on one stream.
 *  - Tensors are dense row-major.  Matrices are stored [out, in] (y = x W^T).
 *  - `dtype` selects the storage type of activations and weights (fp32 or bf16);
 *    arithmetic accumulates in fp32.  Weight-gradient accumulators, dK/dV and
 *    the loss are always fp32.
 *  - "+=" arguments are accumulated into (the caller zeroes them before the
 *    first call - "initialised from zero", Sec. 3.2.1); "out" arguments are
 *    overwritten.  Inputs are never modified.
 *  - Return value: 0 on success; negative on error, in which case nothing has
 *    been enqueued (except SBP_ERR_HIP, which can surface mid-sequence).
 *    streambp_last_error() returns a thread-local message for the last failure.
 *  - chunk need not divide seq_len (the last chunk is shorter); chunk >= seq_len
 *    means a single chunk (Sec. 4.4, partition-size ablation).
 */
#ifndef STREAMBP_H
#define STREAMBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SBP_F32 = 0, SBP_BF16 = 1 };

enum {
  SBP_OK = 0,
  SBP_ERR_NULL = -1,       /* a required pointer is NULL                        */
  SBP_ERR_SHAPE = -2,      /* bad shape / config value                          */
  SBP_ERR_UNSUPPORTED = -3,/* dtype / objective / alignment not supported       */
  SBP_ERR_WORKSPACE = -4,  /* workspace too small or misaligned                 */
  SBP_ERR_HIP = -5         /* HIP runtime error (see streambp_last_error)       */
};

enum { SBP_OBJ_SFT = 0, SBP_OBJ_GRPO = 1, SBP_OBJ_DPO = 2 };

/* ---------------------------------------------------------------- layer -- */

/* One pre-norm decoder layer (Sec. 3.2.2; the paper's display leaves out the
 * norms, heads, residuals and W_o, which are present here):
 *   a = RMSNorm(x; g1); q,k,v = a Wq^T, a Wk^T, a Wv^T; RoPE(q), RoPE(k)
 *   o = causal softmax(q k^T / sqrt(head_dim)) v   (query head h uses KV head
 *       h / (n_q_heads / n_kv_heads))
 *   h1 = x + o Wo^T;  m = RMSNorm(h1; g2)
 *   y = h1 + (silu(m Wgate^T) * (m Wup^T)) Wdown^T
 * RoPE pairs element j with j + head_dim/2, angle (t + pos_offset) * rope_theta^(-2j/head_dim). */
typedef struct {
  int32_t dtype;        /* SBP_F32 or SBP_BF16: x, dy, dx, y and the weights  */
  int32_t batch;        /* B independent sequences of equal length            */
  int32_t seq_len;      /* T                                                  */
  int32_t chunk;        /* c: rows of the output processed per partition      */
  int32_t hidden;       /* d                                                  */
  int32_t n_q_heads, n_kv_heads, head_dim;  /* head_dim even                  */
  int32_t mlp_width;    /* F                                                  */
  float rms_eps;        /* e.g. 1e-6                                          */
  float rope_theta;     /* e.g. 1e4                                           */
  int32_t pos_offset;   /* RoPE position of row 0                             */
  int32_t grad_dtype;   /* element type of the weight-gradient matrices:
                           SBP_F32 (0, default) or SBP_BF16 (needs dtype ==
                           SBP_BF16; App. D (experiment setup) of the paper uses bf16
                           weights and gradients).  A bf16 gradient is read,
                           added to in fp32 and rounded once per pass over it. */
  int32_t dw_group_rows; /* rows of chunk operands kept alive so that one pass over
                           the weight gradients adds several chunks' products
                           (Eq. 1: the summands may be added in any grouping):
                           the group is min(8, max(1, dw_group_rows / chunk))
                           chunks.  0 = default (8192).  More rows: fewer passes
                           over every dW, more workspace (one more copy of a
                           chunk's ten GEMM operand buffers per chunk of the group) */
  int32_t window;       /* attention mask (Sec. 3.2.2 allows a general mask M, "padding /
                           sliding window"): 0 = plain causal; > 0 = the token at row t
                           attends to rows t - window < u <= t only                 */
  const int32_t *seq_first; /* HOST array [batch] or NULL: rows of sequence b before
                           seq_first[b] are padding in front of the sequence - never
                           attended to; as queries they attend to nothing, so their
                           attention output is zero (the rest of the layer still maps
                           them row by row).  0 <= seq_first[b] <= seq_len.  Read
                           before the call returns.                                  */
} sbp_layer_cfg;

/* wq [Hq*dh, d]; wk, wv [Hkv*dh, d]; wo [d, Hq*dh]; wgate, wup [F, d];
 * wdown [d, F]; g1, g2 [d].  Element type = cfg.dtype. */
typedef struct {
  const void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown, *g1, *g2;
} sbp_layer_weights;

/* Same shapes, accumulated into.  The seven matrices have element type
 * cfg.grad_dtype; the gradients of the two norm gains are always fp32. */
typedef struct {
  void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown;
  float *g1, *g2;
} sbp_layer_grads;

/* Bytes of workspace streambp_layer_backward / streambp_layer_forward need for
 * this config (0 if the config is invalid).  The figure is
 *   alpha * min(chunk, T) + beta * T * n_kv_heads * head_dim + const:
 * it has no term in T * mlp_width, T * hidden or T^2 (Sec. 3.2.2, memory
 * efficiency: K and V are cached for the whole sequence, everything else is
 * per chunk). */
size_t streambp_layer_workspace_bytes(const sbp_layer_cfg *cfg);

/* StreamBP of one layer (Sec. 3.2.2): K and V are computed once for the whole
 * sequence and cached in the workspace; then for every chunk of rows the
 * chunk's forward is recomputed against the prefix K/V only and its backward
 * is run, with dW += per-chunk term (Eq. 1), dK/dV of the prefix accumulated in
 * fp32 in the workspace and dx rows written as soon as they are final.
 *   x  [B, T, d] in  : layer input (the gradient checkpoint)
 *   dy [B, T, d] in  : gradient of the loss wrt the layer output
 *   dx [B, T, d] out : gradient wrt the layer input (may not alias x or dy)
 *   dw          +=   : weight gradients, summed over chunks and sequences */
int32_t streambp_layer_backward(const sbp_layer_cfg *cfg, const sbp_layer_weights *w,
                                const void *x, const void *dy, void *dx,
                                const sbp_layer_grads *dw,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* Adapter mode (App. D, experiment setup: the largest model is trained with rank-32 low-rank adapters and only the
 * adapter gradients are computed).  An adapted matrix acts as y = x W^T + s (x A^T) B^T = x (W + s B A)^T with W
 * frozen.  Matrices in the order wq, wk, wv, wo, wgate, wup, wdown; a[i] == b[i] == NULL: matrix i has no adapter. */
typedef struct {
  int32_t rank;          /* r, 1 .. 256                                              */
  float scale;           /* s (usually alpha / r)                                    */
  const void *a[7];      /* A_i [r, in_i]   device, cfg.dtype                        */
  const void *b[7];      /* B_i [out_i, r]  device, cfg.dtype                        */
} sbp_lora_adapters;
typedef struct {
  float *da[7];          /* [r, in_i]  fp32 device, +=  (NULL where not adapted)     */
  float *db[7];          /* [out_i, r] fp32 device, +=                               */
} sbp_lora_grads;

size_t streambp_layer_lora_workspace_bytes(const sbp_layer_cfg *cfg, const sbp_lora_adapters *ad);

/* StreamBP of one layer in adapter mode: the same chunk loop as streambp_layer_backward on the effective matrices
 * W + s B A (built once per call in the workspace: one extra copy of the adapted matrices), but no gradient of W,
 * g1 or g2 is formed; per chunk and adapted matrix the Eq. 1 summands dB += s dY^T (X A^T) and dA += s (dY B)^T X are
 * accumulated (the chain rule through B A, without forming dW).  dx [B, T, d] out.  cfg.grad_dtype must be SBP_F32;
 * cfg.dw_group_rows is ignored (there are no passes over weight gradients to group). */
int32_t streambp_layer_lora_backward(const sbp_layer_cfg *cfg, const sbp_layer_weights *w,
                                     const sbp_lora_adapters *ad, const void *x, const void *dy, void *dx,
                                     const sbp_lora_grads *dad, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/* Chunked forward of the same layer with the same kernels (used to produce the
 * per-layer checkpoints of a stack): y [B, T, d] out. */
int32_t streambp_layer_forward(const sbp_layer_cfg *cfg, const sbp_layer_weights *w,
                               const void *x, void *y,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* --------------------------------------------------------------- LM head -- */

/* logits = h W^T (Sec. 3.2.1); the objective is a sum of independent
 * per-position terms, so logits exist only for one chunk of rows at a time. */
typedef struct {
  int32_t dtype;        /* SBP_F32 or SBP_BF16: h, w, dh                       */
  int32_t batch, seq_len;
  int32_t chunk;        /* rows of logits alive at once                        */
  int32_t hidden, vocab;
  int32_t objective;    /* SBP_OBJ_SFT, SBP_OBJ_GRPO or SBP_OBJ_DPO            */
  float loss_scale;     /* SFT: L = -loss_scale * sum_active log p(target).
                           1 = the paper's un-normalised sum; 1/n_active = mean */
  float clip_eps;       /* GRPO: ratio clip                                    */
  float kl_beta;        /* GRPO: weight of the KL term; DPO: beta              */
  int32_t kl_mode;      /* GRPO: 0 = log(pi/pi_ref) (the paper's compact form),
                           1 = exp(ref-logp) - (ref-logp) - 1                  */
  int32_t grad_dtype;   /* element type of dw: SBP_F32 (0, default) or SBP_BF16
                           (needs dtype == SBP_BF16)                            */
  int32_t dw_group_rows; /* as in sbp_layer_cfg: dz and the gathered h rows of
                           min(8, max(1, dw_group_rows / chunk)) chunks stay alive
                           and dw is added to once per group.  0 = default (16384) */
} sbp_head_cfg;

size_t streambp_lmhead_workspace_bytes(const sbp_head_cfg *cfg);

/* StreamBP of the LM head + objective (Sec. 3.2.1).  Per chunk of rows:
 * logits chunk -> row log-sum-exp and log p(target) -> dz = coef * (onehot -
 * softmax) -> dh rows = dz W, dw += dz^T h.
 *   w [V, d] in; h [B, T, d] in
 *   targets [B, T] int32 in: id the row must predict (labels already shifted
 *       by the caller); negative = ignored row (its dh row is exactly zero).
 *       An id >= vocab is a caller error that only the device can see: such rows
 *       are treated as ignored (the id is never used as an index) and the call
 *       reports them through n_active
 *   old_logp [B, T] fp32 or NULL (GRPO; NULL = on-policy, ratio 1)
 *   ref_logp [B, T] fp32 (GRPO, DPO; NULL for SFT)
 *   advantages [B] fp32 (GRPO; NULL otherwise)
 *   dh [B, T, d] out (cfg.dtype);  dw [V, d] (cfg.grad_dtype) +=
 *   loss: device fp32 scalar, +=.   n_active: device int64 scalar, out: the
 *       number of rows with 0 <= target < vocab - or, if any target is >= vocab,
 *       minus the number of such targets (the gradients then cover the valid rows only).
 * GRPO: L = -(1/B) sum_j (1/T_o,j) sum_{t active in j} f(j,t) with T_o,j the
 * number of active rows of sequence j.
 * DPO (batch must be 2: row 0 chosen, row 1 rejected): gradients are first
 * accumulated with coefficient +-beta, then scaled in place by
 * sigmoid(beta*ell) - 1 once ell is complete, as the paper prescribes; dw must
 * therefore hold only this call's contribution (zero on entry). */
int32_t streambp_lmhead_ce_backward(const sbp_head_cfg *cfg, const void *w, const void *h,
                                    const int32_t *targets, const float *old_logp,
                                    const float *ref_logp, const float *advantages,
                                    void *dh, void *dw, float *loss, int64_t *n_active,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------- chunk attention -- */

/* Causal attention of one chunk of queries against the cached prefix
 * (Sec. 3.2.2, partitioned attention; Property 3.1).  Query row t sits at global
 * position q_start + t and sees keys 0 .. q_start + t. */
typedef struct {
  int32_t dtype;                 /* q, k, v, o, d_o, dq                       */
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t q_start;               /* s: global position of the chunk's row 0   */
  int32_t q_len;                 /* c                                         */
  float scale;                   /* usually 1/sqrt(head_dim); must be positive and finite */
  int32_t window;                /* 0 = plain causal; > 0 = the query at position p sees
                                    keys p - window < u <= p only (sliding window)   */
  int32_t kv_first;              /* key positions before this one are padding in front of
                                    the sequence: never visible.  A query that sees no key
                                    gets o = 0, lse = -inf and no gradient             */
} sbp_attn_cfg;

size_t streambp_attn_workspace_bytes(const sbp_attn_cfg *cfg);

/* q [c, Hq, dh] (rotated); k, v [>= s + c, Hkv, dh]; o [c, Hq, dh] out;
 * lse [Hq, c] fp32 out (natural log-sum-exp of the scaled masked scores). */
int32_t streambp_attn_chunk_forward(const sbp_attn_cfg *cfg, const void *q, const void *k,
                                    const void *v, void *o, float *lse, void *hip_stream);

/* d_o [c, Hq, dh] in; dq [c, Hq, dh] out; dk, dv [>= s + c, Hkv, dh] fp32 +=
 * (rows 0 .. s + c - 1 are touched; contributions of the query heads that
 * share a KV head are summed). */
int32_t streambp_attn_chunk_backward(const sbp_attn_cfg *cfg, const void *q, const void *k,
                                     const void *v, const void *o, const float *lse,
                                     const void *d_o, void *dq, float *dk, float *dv,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same backward for callers that cannot allocate device memory and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Identical arguments, kernels and results,
 * but the scratch (2 floats per (query, head) pair) is a fixed array inside the library's own device image - 2 MiB
 * that every GPU the library runs on holds until the process ends - so the call takes no workspace and makes no
 * allocation of any kind.  Limit: q_len * n_q_heads <= 262144 (e.g. 2048 queries x 128 heads); larger chunks return
 * SBP_ERR_WORKSPACE and must use the call above.  All calls on one GPU share that array: calls that overlap on one
 * GPU (two streams, two threads) race and must be ordered by the caller; nothing in it has to be cleared between calls
 * (every element a call reads it has written first).  The first call on a device looks the array's address up (a symbol
 * query, no allocation): make that call outside stream capture. */
int32_t streambp_attn_chunk_backward_noalloc(const sbp_attn_cfg *cfg, const void *q, const void *k,
                                             const void *v, const void *o, const float *lse,
                                             const void *d_o, void *dq, float *dk, float *dv,
                                             void *hip_stream);

/* ------------------------------------------------ stack glue (Sec. 2, 3.1) -- */

/* Final RMSNorm between the layer stack and the LM head, and the embedding
 * lookup in front of the stack: rows x [n, d] (dtype), gain g [d].
 * forward:  y = RMSNorm(x; g).   backward: dx out (dtype), dg fp32 +=; needs
 * streambp_rmsnorm_workspace_bytes(n_rows, hidden) bytes of workspace. */
size_t streambp_rmsnorm_workspace_bytes(int64_t n_rows, int32_t hidden);
int32_t streambp_rmsnorm_forward(int32_t dtype, int64_t n_rows, int32_t hidden, float eps,
                                 const void *x, const void *g, void *y, void *hip_stream);
int32_t streambp_rmsnorm_backward(int32_t dtype, int64_t n_rows, int32_t hidden, float eps,
                                  const void *x, const void *g, const void *dy, void *dx,
                                  float *dg, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);
/* x[t] = emb[ids[t]] ; demb[ids[t]] += dx[t] (fp32 accumulators, atomic adds).  An id outside [0, vocab) is never
 * used as an index: its row of x is zero and its row of dx is dropped. */
int32_t streambp_embedding_forward(int32_t dtype, int64_t n_rows, int32_t hidden, int32_t vocab,
                                   const int32_t *ids, const void *emb, void *x, void *hip_stream);
int32_t streambp_embedding_backward(int32_t dtype, int64_t n_rows, int32_t hidden, int32_t vocab,
                                    const int32_t *ids, const void *dx, float *demb, void *hip_stream);

/* ----------------------------------------------------------------- stack -- */

/* Layer-wise StreamBP through a stack of identical-shape layers from per-layer
 * checkpoints (Sec. 2: checkpointed layer inputs; Sec. 3.1: the gradient of a
 * layer's output is the input of the backward of the layer before it):
 *   x_0 = emb[ids];  x_{l+1} = layer_l(x_l);  h = RMSNorm(x_L; g_final);
 *   L = objective(h W_head^T, targets).
 * ckpt[l] (l = 0..L) are caller-owned [B, T, d] buffers: ckpt[l] holds the
 * input of layer l, ckpt[L] the output of the last layer. */
typedef struct {
  sbp_layer_cfg layer;      /* shape of every layer; its chunk is the layer chunk */
  int32_t n_layers;
  int32_t vocab;
  int32_t head_chunk;       /* rows of logits alive at once                       */
  int32_t objective;        /* as in sbp_head_cfg                                 */
  float loss_scale, clip_eps, kl_beta;
  int32_t kl_mode;
  float final_eps;          /* eps of the final RMSNorm                           */
} sbp_stack_cfg;

size_t streambp_stack_workspace_bytes(const sbp_stack_cfg *cfg);

/* Chunked forward that fills the checkpoints.  emb [V, d] and ids [B, T] may both
 * be NULL, in which case ckpt[0] must already hold the stack input. */
int32_t streambp_stack_forward(const sbp_stack_cfg *cfg, const sbp_layer_weights *layers /*[L]*/,
                               const void *emb, const int32_t *ids, void *const *ckpt /*[L+1]*/,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward: LM head + objective on RMSNorm(ckpt[L]), final norm, then layers
 * L-1 .. 0, each by streambp_layer_backward on its checkpoint.
 *   dlayers [L] (+=; matrices in layer.grad_dtype), dg_final [d] fp32 (+=),
 *   dw_head [V, d] in layer.grad_dtype (+=; DPO: zero on entry),
 *   demb [V, d] fp32 (+=, may be NULL together with ids), loss (+=), n_active (out);
 *   dx0 [B, T, d] out (may be NULL): gradient wrt the stack input. */
int32_t streambp_stack_backward(const sbp_stack_cfg *cfg, const sbp_layer_weights *layers,
                                const void *g_final, const void *w_head, void *const *ckpt,
                                const int32_t *ids, const int32_t *targets, const float *old_logp,
                                const float *ref_logp, const float *advantages,
                                const sbp_layer_grads *dlayers, float *dg_final, void *dw_head,
                                float *demb, void *dx0, float *loss, int64_t *n_active,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------ misc -- */

const char *streambp_version(void);
const char *streambp_last_error(void);
/* Which kernels a configuration gets (host arithmetic only).  1: every GEMM and the attention of the configuration
 * run on the bf16 MFMA kernels (needs bf16 storage, head_dim 128 and hidden, n_q_heads*head_dim, n_kv_heads*head_dim,
 * mlp_width - for the head: hidden and vocab - multiples of 64, 16-byte aligned tensors; widths that are not multiples
 * of the 256-wide output tile, such as a 151936-word vocabulary, run with a masked last tile).  0: some of it runs on the
 * shape-agnostic fp32-ALU kernels, a correctness path that is orders of magnitude slower (streambp_last_error() says
 * which dimension is the reason); nothing is refused.  Negative: the configuration itself is invalid. */
int32_t streambp_layer_fast_path(const sbp_layer_cfg *cfg);
int32_t streambp_lmhead_fast_path(const sbp_head_cfg *cfg);
/* Number of bf16 GEMM / attention launches, since the library was loaded, that ran on the shape-agnostic kernels because
 * the MFMA kernels could not take their shape or alignment.  A caller that expects the fast path checks that this does
 * not move across its calls. */
int64_t streambp_generic_launches(void);
/* Number of (query tile, key tile) pairs the attention kernels visit for a
 * chunk, and the tile sizes; host arithmetic only, for the causal-skip check
 * (Sec. 3.2.2, computational efficiency: about (1+D)/(2D) of the full square). */
int64_t streambp_attn_tile_pairs(int32_t q_start, int32_t q_len, int32_t *tile_q, int32_t *tile_k);

#ifdef __cplusplus
}
#endif
#endif /* STREAMBP_H */
