// Host-side launchers of the HIP kernels.  Every function only enqueues work on
// `st`; none allocates or synchronises.  Shapes are validated by the callers in
// api.hip before anything is launched.
#pragma once
#include "common.h"

namespace sbp {

// C[M,N] (=|+=) sum_k A(m,k) * B(k,n), fp32 accumulation.
//   A(m,k) = ta ? A[k*lda + m] : A[m*lda + k]
//   B(k,n) = tb ? B[n*ldb + k] : B[k*ldb + n]
// in_dt: element type of A and B; out_dt: element type of C; acc: C += (fp32 C only).
struct GemmArgs {
  const void* A; const void* B; void* C;
  int M, N, K;
  int64_t lda, ldb, ldc;
  bool ta, tb;
  int in_dt, out_dt;
  bool acc;
  float* scratch = nullptr;      // optional fp32 scratch for split-K partial tiles
  size_t scratch_bytes = 0;
  // Optional device-side count of valid "rows" (the M dimension of NT / NN problems, the K dimension of the
  // dW form): the kernels read it at run time and skip the work beyond it; the host-side M (resp. K) is the
  // upper bound the launch is sized for.
  const int* rows_dev = nullptr;
  // Optional second operand pair of the same shapes and leading dimensions: C (=|+=) A B + A2 B2 in one launch
  // (the two products become the two slices of a split-K launch; falls back to two launches where that does not fit).
  const void* A2 = nullptr;
  const void* B2 = nullptr;
  // Optional row statistics of the output (store form C = A B^T with fp32 C, MFMA kernel only: ask
  // gemm_row_stats_supported first): row_stats[m * ceil(N / GEMM_STAT_COLS) + t] = (max, sum of exp(c - max)) of row m
  // over the columns [t * GEMM_STAT_COLS, (t + 1) * GEMM_STAT_COLS), taken from the fp32 accumulators.
  float2* row_stats = nullptr;
  // Optional "softmax numerators" form of the row-statistics store (C bf16, MFMA kernel only: ask
  // gemm_numerators_supported first).  C does not receive the product c but exp(c - max), max being the row's maximum
  // over the element's block of GEMM_STAT_COLS columns - the same (max, sum of exp) pairs go to row_stats, the sums
  // taken from the unrounded fp32 values - and the product's value in column numer_targets[r] of row m goes to
  // numer_target_value[m] (fp32), r = numer_row_index ? numer_row_index[m] : m; a target outside [0, N) matches no
  // column and leaves the entry untouched.  What a softmax over the row needs is then all there in half the bytes:
  // softmax(c)[n] = C[m, n] * exp(max_block(n) - lse(m)).
  const int32_t* numer_targets = nullptr;
  const int32_t* numer_row_index = nullptr;
  float* numer_target_value = nullptr;
  // Optional fused SwiGLU adjoint (store form C = A B with the same row-major [M, N] layout and leading dimension for
  // C, gate, up and act; bf16): the product is the gradient wrt act = silu(gate) * up and is never stored; instead the
  // epilogue reads the tile's gate and up values and writes act (what the forward would have produced; optional),
  // gate <- d gate and up <- d up in place.  Where the MFMA kernel cannot take the problem the dispatcher runs the
  // plain product into C followed by the elementwise kernel - same results up to the rounding of the product to bf16.
  void* swiglu_gate = nullptr;
  void* swiglu_up = nullptr;
  void* swiglu_act = nullptr;
};
constexpr int GEMM_STAT_COLS = 256;
bool gemm_row_stats_supported(const GemmArgs& g);
bool gemm_numerators_supported(const GemmArgs& g);
// upper bound of the scratch a GEMM with M <= max_m rows and N <= max_n columns may use
size_t gemm_scratch_bytes(int max_m, int max_n, int max_splits);
hipError_t gemm(const GemmArgs& g, hipStream_t st);
// n independent GEMMs (distinct outputs); one grouped launch when the MFMA kernel can take them all
// group_small: take the grouped launch also when the problems together have few output tiles (skinny problems)
hipError_t gemm_batch(const GemmArgs* gs, int n, hipStream_t st, bool group_small = false);
// true when the bf16 MFMA kernel can take this problem (used by tests / tile accounting)
bool gemm_uses_mfma(const GemmArgs& g);
// force the generic kernel (debug / A-B tests)
void gemm_set_force_generic(bool on);
// which of the optional fusions the entry points use (A/B measurements): bit 0 = SwiGLU adjoint in the epilogue of the
// dact GEMM, bit 1 = rotary embedding of q / its adjoint on dq inside the attention kernels, bit 2 = the LM head's logits
// GEMM stores bf16 softmax numerators (and the target logits) instead of fp32 logits
enum { FUSE_SWIGLU = 1, FUSE_ROPE_Q = 2, FUSE_NUMERATORS = 4 };
int fusion_mask();
void set_fusion_mask(int mask);
// bf16 problems that have run on the shape-agnostic kernels since the library was loaded
long long generic_bf16_launches();
void note_generic_bf16_launch();

// ---- optional per-launch timing (off unless streambp_debug_profile_begin was called) ----
namespace prof {
// kinds 0..11: gemm_mfma_k<layout, mode> with layout NT=0, NN=1, TN=2 and mode 0..3; 12..23: the grouped kernel;
// then the shape-agnostic GEMM, the attention forward / backward launch sequences, the segmented weight-gradient GEMM and the
// store form with row statistics (gemm_mfma_k<NT, 5>), the input-gradient form with the fused SwiGLU adjoint (gemm_mfma_k<NN, 6>)
// and the softmax-numerator store (gemm_mfma_k<NT, 7>)
enum { GEMM_SINGLE = 0, GEMM_GROUP = 12, GEMM_GENERIC = 24, ATTN_FWD = 25, ATTN_BWD = 26, GEMM_SEG = 27, GEMM_STATS = 28, GEMM_SWIGLU = 29,
       GEMM_NUMER = 30, N_KIND = 31 };
struct Scope {
  hipStream_t st; bool active = false; int kind = 0; double work = 0; bool bounded = false; hipEvent_t e0{}, e1{};
  // bounded: `work` was computed from a host-side upper bound of a run-time row count
  Scope(int kind, double work, bool bounded, hipStream_t st);
  ~Scope();
};
}  // namespace prof

// ---- elementwise / row kernels (dt = storage type of the T-typed tensors) ----
// cos/sin table [n_pos, dh/2] (float2), angles evaluated in fp64.
hipError_t rope_table(float2* tab, int n_pos, int dh, float theta, int pos_offset, hipStream_t st);
// in-place rotation of x [rows, H, dh]; tab points at the row of position 0 of these rows.
hipError_t rope_apply(int dt, void* x, const float2* tab, int rows, int H, int dh, bool inverse, hipStream_t st);
// out = g * (x + add) * rstd ; sum_out = x + add (fp32, optional) ; rstd per row
hipError_t rmsnorm_fwd(int dt, const void* x, const float* add, const void* g, void* out, float* sum_out,
                       float* rstd, int rows, int d, float eps, hipStream_t st);
// adjoint: dnorm [rows,d] fp32 is the gradient wrt the normalised output.
//   xin: the tensor that was normalised (x_is_f32 ? fp32 : dt);  res: gradient flowing around the norm
//   (res_is_f32 ? fp32 : dt);  out_f32 / out_t (either may be NULL) = res + dx_norm;
//   dg += column sums of dnorm * xin * rstd (two-stage, deterministic; `partial` >= cdiv(rows,8)*d floats)
hipError_t rmsnorm_bwd(int dt, const float* dnorm, const void* xin, bool x_is_f32, const void* g,
                       const float* rstd, const void* res, bool res_is_f32, float* out_f32, void* out_t,
                       float* dg, float* partial, int rows, int d, hipStream_t st);
size_t rmsnorm_bwd_partial_floats(int rows, int d);
// dy, x, dx in dt; no residual branch
hipError_t rmsnorm_bwd_plain(int dt, const void* dy, const void* x, const void* g, const float* rstd, void* dx,
                             float* dg, float* partial, int rows, int d, hipStream_t st);
// recompute rstd only (used when the statistic was not kept): not needed by the layer path
hipError_t swiglu_fwd(int dt, const void* gate, const void* up, void* act, int64_t n, hipStream_t st);
// in place: gate <- dgate, up <- dup, given dact; act (optional) <- silu(gate) * up of the incoming values, the same
// numbers swiglu_fwd writes (for callers that need act only in the backward)
hipError_t swiglu_bwd(int dt, void* gate, void* up, const void* dact, void* act, int64_t n, hipStream_t st);
// y = T(a + b) with a, b fp32
hipError_t add_store(int dt, const float* a, const float* b, void* y, int64_t n, hipStream_t st);
// dkc = T(RoPE^T(dK rows)), dvc = T(dV rows);  dK, dV fp32 [rows, H, dh]
hipError_t kv_grad_finish(int dt, const float* dK, const float* dV, const float2* tab, void* dkc, void* dvc,
                          int rows, int H, int dh, hipStream_t st);
hipError_t fill_zero(void* p, size_t bytes, hipStream_t st);
// MFMA rate probe: operands = 32768 bf16 values on the device, sink = workgroups * 512 floats; lds_reads = 0, 6 or 8 of the
// eight A fragments of a round re-read from LDS
hipError_t mfma_rate_probe(const void* operands, float* sink, int workgroups, int iters, int lds_reads, hipStream_t st);
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t st);     // 16-byte aligned, bytes % 16 == 0 fast path
// dst [R2, C2] (dt, dense) = zero-padded scale * src, src [R, C] (dt, dense) or its transpose (src [C, R]) - small matrices
hipError_t pad_matrix(int dt, const void* src, int R, int C, bool transposed, float scale, void* dst, int R2, int C2, hipStream_t st);
// dst [R, C] fp32 (dense) += scale * src[i * ld + j]
hipError_t add_scaled_block(const float* src, int64_t ld, float scale, float* dst, int R, int C, hipStream_t st);
// ids outside [0, vocab) are never used as an index: their x row is zero, their dx row is dropped
hipError_t embedding_fwd(int dt, const int32_t* ids, const void* emb, void* x, int64_t rows, int d, int vocab, hipStream_t st);
hipError_t embedding_bwd(int dt, const int32_t* ids, const void* dx, float* demb, int64_t rows, int d, int vocab, hipStream_t st);

// ---- chunk attention ----
struct AttnArgs {
  int dt;
  int Hq, Hkv, dh;
  int q_start, q_len;
  float scale;
  int window = 0;          // > 0: a query at position t sees only keys t - window < u <= t
  int kv_first = 0;        // key positions before this one are padding: never visible
  const void *q, *k, *v;   // q [c,Hq,dh]; k,v [>=s+c,Hkv,dh]
  void* o; float* lse;     // o [c,Hq,dh]; lse [Hq,c]
  const void* d_o; void* dq; float *dk, *dv;
  float* delta;            // [2,Hq,c] scratch (backward): delta, then the log2-domain log-sum-exp
  // Optional rotary embedding of the chunk's queries folded into the attention kernels: cos/sin rows [c, dh/2] of the
  // chunk's positions.  Forward: q arrives un-rotated, is rotated on load and written back rotated (q must then be
  // writable); backward: q is the rotated tensor the forward left, and dq leaves the kernel already rotated back
  // (the adjoint rotation), i.e. as the gradient wrt the un-rotated projection.
  const float2* rope_q = nullptr;
};
hipError_t attn_forward(const AttnArgs& a, hipStream_t st);
hipError_t attn_backward(const AttnArgs& a, hipStream_t st);
bool attn_uses_mfma(int dt, int dh, int Hq, int Hkv);
void attn_set_force_generic(bool on);
constexpr int ATTN_TILE_Q = 256;   // rows of queries per workgroup in the MFMA kernels (8 waves x 32 rows)
constexpr int ATTN_WAVE_Q = 32;    // rows of queries per wave: the granularity at which key tiles are skipped
constexpr int ATTN_TILE_K = 64;    // keys per inner step

// ---- LM head rows ----
struct HeadRowArgs {
  int dt;                   // type of dz
  int objective;            // 0 SFT, 1 GRPO, 2 DPO
  const float* z;           // [rows, V] fp32 logits of the chunk (unused in the numerator form)
  void* dz;                 // [rows, V] dt; numerator form (target_logit != NULL): holds exp(z - block max) on entry
  const int32_t* targets;   // [rows] (already offset to the chunk)
  const float* old_logp;    // [rows] or NULL
  const float* ref_logp;    // [rows] or NULL
  const float* advantages;  // [B] or NULL
  const float* seq_weight;  // [B] GRPO: 1/(B*T_o,j); NULL otherwise
  int64_t row0;             // global row index of the chunk's first row (row / T = sequence)
  const int32_t* row_index; // optional: original row of each chunk row (compacted chunks); then targets / old_logp /
                            // ref_logp are indexed by it and row0 is ignored
  const int* rows_dev;      // optional device-side count of valid chunk rows (<= rows)
  const float2* stats;      // optional [rows, n_stat]: per row and column block (max, sum of exp(z - max)) from the logits
  int n_stat;               // GEMM; the kernel then reads z once instead of twice
  const float* target_logit; // optional [rows]: z[row, target] from the logits GEMM's numerator form (needs stats, bf16 dz)
  int rows, V, T;
  float loss_scale, clip_eps, kl_beta; int kl_mode;
  float* row_loss;          // [rows] scratch: per-row loss term (DPO: per-row signed log-ratio)
};
hipError_t head_rows(const HeadRowArgs& a, hipStream_t st);
// loss += sum(row_loss[0..rows)) in a fixed order
hipError_t reduce_add(const float* v, int n, float* out, hipStream_t st, const int* n_dev = nullptr);
// per-sequence active counts (0 <= target < V) -> seq_weight[j] = 1/(B*T_o,j) (0 if empty), n_active total - or minus the
// number of targets >= V if there is any
hipError_t count_active(const int32_t* targets, int B, int T, int V, float* seq_weight, int64_t* n_active, hipStream_t st);
// index[0..n_active) = rows with 0 <= target < V in increasing order; chunk_rows[i] = clamp(n_active - i*chunk, 0, chunk)
hipError_t compact_active(const int32_t* targets, int64_t rows, int chunk, int V, int32_t* index, int32_t* chunk_rows, int n_chunks,
                          hipStream_t st);
// dst[r,:] = src[index[r],:] for r < *rows_dev, zero rows after;  scatter: dst[index[r],:] = src[r,:] for r < *rows_dev
hipError_t gather_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t st);
hipError_t scatter_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t st);
// DPO fix-up: factor = sigmoid(beta*ell)-1 ; scales dh (dt) and dw (fp32) in place, loss += -log sigmoid(beta*ell)
hipError_t dpo_finish(int dt, const float* ell, float beta, void* dh, int64_t n_dh, void* dw, int dw_dt, int64_t n_dw,
                      float* loss, hipStream_t st);

}  // namespace sbp
