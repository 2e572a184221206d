// C ABI of libstreambp and the host-side chunk loops (paper Sec. 3.2.1, 3.2.2).
// Host code only validates, carves the caller's workspace and enqueues kernels
// on the caller's stream; it never allocates or synchronises.
#include "../../include/streambp.h"
#include "launch.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

using namespace sbp;

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIPCHK(expr)                                                                       \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return fail(SBP_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

// Bump allocator over the caller's workspace (256-byte granularity).
struct Carver {
  char* base; size_t off = 0;
  explicit Carver(void* p) : base((char*)p) {}
  template <typename T> T* take(size_t n_elems) { return (T*)take_bytes(n_elems * sizeof(T)); }
  void* take_bytes(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

bool valid_dtype(int32_t dt) { return dt == SBP_F32 || dt == SBP_BF16; }
// weight gradients: fp32, or bf16 next to bf16 weights
int32_t check_grad_dtype(int32_t dt, int32_t grad_dt) {
  if (!valid_dtype(grad_dt)) return fail(SBP_ERR_UNSUPPORTED, "grad_dtype %d not supported", grad_dt);
  if (grad_dt == SBP_BF16 && dt != SBP_BF16) return fail(SBP_ERR_UNSUPPORTED, "bf16 gradients need dtype == SBP_BF16");
  return SBP_OK;
}

// Weight gradients are added once per group of chunks (one read-modify-write pass over every dW per group instead of
// one per chunk): as many chunks as it takes to reach dw_group_rows rows, at most MAX_DW_GROUP (the GEMM kernels take
// up to eight reduction segments per output).  The operands of the group's chunks stay alive until the launch.
constexpr int MAX_DW_GROUP = 8;
// Defaults (dw_group_rows == 0).  Measured at 7B widths, chunk 2048: the head's dW pass (2.2 GB read-modify-written) still
// gains from eight chunks per pass over four; the layer's seven dW (0.93 GB) do not, so the layer keeps four.
constexpr int DW_GROUP_ROWS_LAYER = 8192;
constexpr int DW_GROUP_ROWS_HEAD = 16384;
int dw_group_for(size_t chunk_rows, int32_t cfg_rows, int default_rows) {   // cfg_rows: the config's dw_group_rows (0 = default)
  const size_t rows = cfg_rows > 0 ? (size_t)cfg_rows : (size_t)default_rows;
  return (int)std::max<size_t>(1, std::min<size_t>(MAX_DW_GROUP, rows / std::max<size_t>(chunk_rows, 1)));
}

// ------------------------------------------------------------- layer ------
struct LayerWs {
  void *K, *V;                 // [T, Hkv*dh] dt   cached for the whole sequence
  float *dK, *dV;              // [T, Hkv*dh] fp32 prefix accumulators
  float2* rope;                // [T, dh/2] cos/sin
  void *a, *q, *o, *m, *gate, *up, *act, *dact, *dh1_t, *d_o, *dq, *dkc, *dvc;   // per chunk, dt
  float *h1, *dm, *dh1, *da, *proj;                                       // per chunk, fp32 [c, d]
  float *rstd1, *rstd2, *lse, *delta, *partial;
  float* gemm_scratch; size_t gemm_scratch_bytes;
  // Further copies of the operands of the chunk's weight-gradient GEMMs (a, o, m, gate, up, act, dh1_t, dq, dkc, dvc):
  // the weight gradients of dw_group consecutive chunks are added in one launch, so a chunk's operands stay alive
  // while the next chunks are processed.
  int dw_group;
  void* alt[MAX_DW_GROUP - 1][10];
  size_t bytes;
};
// The workspace view a chunk uses: set 0 = the primary operand buffers, sets 1.. the further copies.
LayerWs chunk_view(const LayerWs& s, int set) {
  LayerWs v = s;
  if (set > 0) {
    void** ptrs[10] = {&v.a, &v.o, &v.m, &v.gate, &v.up, &v.act, &v.dh1_t, &v.dq, &v.dkc, &v.dvc};
    for (int i = 0; i < 10; ++i) *ptrs[i] = s.alt[set - 1][i];
  }
  return v;
}

int32_t check_layer_cfg(const sbp_layer_cfg* c) {
  if (!c) return fail(SBP_ERR_NULL, "cfg is NULL");
  if (!valid_dtype(c->dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype %d not supported", c->dtype);
  if (int32_t rc = check_grad_dtype(c->dtype, c->grad_dtype)) return rc;
  if (c->dw_group_rows < 0) return fail(SBP_ERR_SHAPE, "dw_group_rows must be >= 0");
  if (c->batch < 1 || c->seq_len < 1 || c->chunk < 1) return fail(SBP_ERR_SHAPE, "batch, seq_len and chunk must be >= 1");
  if (c->hidden < 1 || c->mlp_width < 1) return fail(SBP_ERR_SHAPE, "hidden and mlp_width must be >= 1");
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads != 0)
    return fail(SBP_ERR_SHAPE, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", c->n_q_heads, c->n_kv_heads);
  if (c->head_dim < 2 || (c->head_dim & 1) || c->head_dim > 256)
    return fail(SBP_ERR_SHAPE, "head_dim must be even and in [2, 256]");
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(SBP_ERR_SHAPE, "rms_eps must be >= 0 and rope_theta > 0");
  if (c->window < 0) return fail(SBP_ERR_SHAPE, "window must be >= 0");
  if (c->seq_first)
    for (int b = 0; b < c->batch; ++b)
      if (c->seq_first[b] < 0 || c->seq_first[b] > c->seq_len)
        return fail(SBP_ERR_SHAPE, "seq_first[%d] = %d is outside [0, seq_len]", b, c->seq_first[b]);
  return SBP_OK;
}

LayerWs carve_layer(const sbp_layer_cfg* c, void* ws) {
  const size_t es = dtype_size(c->dtype);
  const size_t T = c->seq_len, cm = (size_t)std::min(c->chunk, c->seq_len);
  const size_t d = c->hidden, F = c->mlp_width, qd = (size_t)c->n_q_heads * c->head_dim, kd = (size_t)c->n_kv_heads * c->head_dim;
  Carver cv(ws);
  LayerWs w;
  w.K = cv.take_bytes(T * kd * es);
  w.V = cv.take_bytes(T * kd * es);
  w.dK = cv.take<float>(T * kd);
  w.dV = cv.take<float>(T * kd);
  w.rope = cv.take<float2>(T * (c->head_dim / 2));
  w.a = cv.take_bytes(cm * d * es);
  w.q = cv.take_bytes(cm * qd * es);
  w.o = cv.take_bytes(cm * qd * es);
  w.m = cv.take_bytes(cm * d * es);
  w.gate = cv.take_bytes(cm * F * es);
  w.up = cv.take_bytes(cm * F * es);
  w.act = cv.take_bytes(cm * F * es);
  w.dact = cv.take_bytes(cm * F * es);
  w.dh1_t = cv.take_bytes(cm * d * es);
  w.d_o = cv.take_bytes(cm * qd * es);
  w.dq = cv.take_bytes(cm * qd * es);
  w.dkc = cv.take_bytes(cm * kd * es);
  w.dvc = cv.take_bytes(cm * kd * es);
  w.h1 = cv.take<float>(cm * d);
  w.dm = cv.take<float>(cm * d);
  w.dh1 = cv.take<float>(cm * d);
  w.da = cv.take<float>(cm * d);
  w.proj = cv.take<float>(cm * d);
  w.rstd1 = cv.take<float>(cm);
  w.rstd2 = cv.take<float>(cm);
  w.lse = cv.take<float>(cm * c->n_q_heads);
  w.delta = cv.take<float>(2 * cm * c->n_q_heads);
  w.partial = cv.take<float>(rmsnorm_bwd_partial_floats((int)cm, (int)d));
  w.gemm_scratch_bytes = c->dtype == SBP_BF16 ? gemm_scratch_bytes((int)cm, (int)std::max(d, qd), 4) : 0;
  w.gemm_scratch = (float*)cv.take_bytes(w.gemm_scratch_bytes);
  {
    const size_t sizes[10] = {cm * d * es, cm * qd * es, cm * d * es, cm * F * es, cm * F * es, cm * F * es,
                              cm * d * es, cm * qd * es, cm * kd * es, cm * kd * es};   // a, o, m, gate, up, act, dh1_t, dq, dkc, dvc
    w.dw_group = dw_group_for(cm, c->dw_group_rows, DW_GROUP_ROWS_LAYER);
    for (int g = 1; g < w.dw_group; ++g)
      for (int i = 0; i < 10; ++i) w.alt[g - 1][i] = cv.take_bytes(sizes[i]);
  }
  w.bytes = cv.off;
  return w;
}

// split-K scratch of the entry point currently running on this host thread
thread_local float* t_gemm_scratch = nullptr;
thread_local size_t t_gemm_scratch_bytes = 0;

GemmArgs mk(const void* A, const void* B, void* C, int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
            bool ta, bool tb, int in_dt, int out_dt, bool acc) {
  GemmArgs g{A, B, C, M, N, K, lda, ldb, ldc, ta, tb, in_dt, out_dt, acc};
  g.scratch = t_gemm_scratch;
  g.scratch_bytes = t_gemm_scratch_bytes;
  return g;
}
// Y[M,N] = X[M,K] W[N,K]^T
GemmArgs fwd_gemm(const void* X, const void* W, void* Y, int M, int N, int K, int dt, int out_dt) {
  return mk(X, W, Y, M, N, K, K, K, N, false, true, dt, out_dt, false);
}
// dX[M,K] (=|+=) dY[M,N] W[N,K]
GemmArgs dx_gemm(const void* dY, const void* W, void* dX, int M, int N, int K, int dt, int out_dt, bool acc) {
  return mk(dY, W, dX, M, K, N, N, K, K, false, false, dt, out_dt, acc);
}
// dW[N,K] += dY[M,N]^T X[M,K]
GemmArgs dw_gemm(const void* dY, const void* X, void* dW, int M, int N, int K, int dt, int grad_dt) {
  return mk(dY, X, dW, N, K, M, N, K, K, true, false, dt, grad_dt, true);
}

const char* at(const void* p, size_t row, size_t width, size_t es) { return (const char*)p + row * width * es; }
char* at(void* p, size_t row, size_t width, size_t es) { return (char*)p + row * width * es; }

int32_t check_layer_ptrs(const sbp_layer_weights* w) {
  if (!w) return fail(SBP_ERR_NULL, "weights table is NULL");
  const void* ps[] = {w->wq, w->wk, w->wv, w->wo, w->wgate, w->wup, w->wdown, w->g1, w->g2};
  for (const void* p : ps) if (!p) return fail(SBP_ERR_NULL, "a weight pointer is NULL");
  return SBP_OK;
}

// K and V of the whole sequence, once (cached for all chunks of the layer).  The pass runs in row blocks as large as
// the chunk buffers that are idle at this point allow (gate, up, act, dact are contiguous: 4 c F elements hold the
// normalised rows of 4 c F / d positions), so that the two projections are GEMMs with enough output tiles to fill
// the chip on their own; nothing proportional to T is added to the workspace.
int32_t kv_prepass(const sbp_layer_cfg* c, const sbp_layer_weights* w, const LayerWs& s, const char* xb, hipStream_t st) {
  const int dt = c->dtype;
  const size_t es = dtype_size(dt);
  const int T = c->seq_len, cm = std::min(c->chunk, T), d = c->hidden;
  const int kd = c->n_kv_heads * c->head_dim;
  void* a_rows = s.a;
  int block = cm;
  const size_t idle_rows = (size_t)((const char*)s.dh1_t - (const char*)s.gate) / ((size_t)d * es);
  if (idle_rows > (size_t)cm) {
    a_rows = s.gate;
    block = (int)std::min<size_t>((size_t)T, idle_rows);
  }
  for (int r0 = 0; r0 < T; r0 += block) {
    const int n = std::min(block, T - r0);
    HIPCHK(rmsnorm_fwd(dt, at(xb, r0, d, es), nullptr, w->g1, a_rows, nullptr, nullptr, n, d, c->rms_eps, st));
    const GemmArgs kv[2] = {fwd_gemm(a_rows, w->wk, at(s.K, r0, kd, es), n, kd, d, dt, dt),
                            fwd_gemm(a_rows, w->wv, at(s.V, r0, kd, es), n, kd, d, dt, dt)};
    HIPCHK(gemm_batch(kv, 2, st));
    HIPCHK(rope_apply(dt, at(s.K, r0, kd, es), s.rope + (size_t)r0 * (c->head_dim / 2), n, c->n_kv_heads, c->head_dim, false, st));
  }
  return SBP_OK;
}

// Partitioned reforward of rows [r0, r0+n): fills a, q, o, lse, h1, m, gate, up, act.
// with_act = false leaves s.act unwritten: the backward gets it from swiglu_bwd, which reads gate and up anyway
int32_t chunk_reforward(const sbp_layer_cfg* c, const sbp_layer_weights* w, const LayerWs& s, const char* xb,
                        int r0, int n, int kv_first, bool with_act, hipStream_t st) {
  const int dt = c->dtype;
  const size_t es = dtype_size(dt);
  const int d = c->hidden, F = c->mlp_width, qd = c->n_q_heads * c->head_dim;
  const char* xc = at(xb, r0, d, es);
  HIPCHK(rmsnorm_fwd(dt, xc, nullptr, w->g1, s.a, nullptr, s.rstd1, n, d, c->rms_eps, st));
  HIPCHK(gemm(fwd_gemm(s.a, w->wq, s.q, n, qd, d, dt, dt), st));
  AttnArgs aa{};
  aa.dt = dt; aa.Hq = c->n_q_heads; aa.Hkv = c->n_kv_heads; aa.dh = c->head_dim;
  aa.q_start = r0; aa.q_len = n; aa.scale = 1.0f / std::sqrt((float)c->head_dim);
  aa.window = c->window; aa.kv_first = kv_first;
  aa.q = s.q; aa.k = s.K; aa.v = s.V; aa.o = s.o; aa.lse = s.lse;
  if (fusion_mask() & FUSE_ROPE_Q) aa.rope_q = s.rope + (size_t)r0 * (c->head_dim / 2);   // RoPE(q) inside the attention kernel, which leaves s.q rotated
  else HIPCHK(rope_apply(dt, s.q, s.rope + (size_t)r0 * (c->head_dim / 2), n, c->n_q_heads, c->head_dim, false, st));
  HIPCHK(attn_forward(aa, st));
  HIPCHK(gemm(fwd_gemm(s.o, w->wo, s.proj, n, d, qd, dt, DT_F32), st));
  HIPCHK(rmsnorm_fwd(dt, xc, s.proj, w->g2, s.m, s.h1, s.rstd2, n, d, c->rms_eps, st));
  {
    const GemmArgs gu[2] = {fwd_gemm(s.m, w->wgate, s.gate, n, F, d, dt, dt), fwd_gemm(s.m, w->wup, s.up, n, F, d, dt, dt)};
    HIPCHK(gemm_batch(gu, 2, st));
  }
  if (with_act) HIPCHK(swiglu_fwd(dt, s.gate, s.up, s.act, (int64_t)n * F, st));
  return SBP_OK;
}

}  // namespace

extern "C" {

const char* streambp_version(void) { return "streambp-mi355x 0.1 (gfx950)"; }
const char* streambp_last_error(void) { return g_err; }

size_t streambp_layer_workspace_bytes(const sbp_layer_cfg* cfg) {
  if (check_layer_cfg(cfg) != SBP_OK) return 0;
  return carve_layer(cfg, nullptr).bytes;
}

// Low-rank adapter mode of the layer backward (App. D, experiment setup: rank-32 adapters, adapter gradients only).
// The chunk loop runs on the effective matrices W + s B A (built once per call); instead of the seven weight gradients
// of a chunk it forms, per adapted matrix, P = X A^T, Q = dY B (chunk x rank, the rank rounded up to a multiple of 8) and
// accumulates dB += dY^T P, dA += Q^T X - the chain rule through B A without ever forming dW.
constexpr int LORA_MAX_RANK = 256;
struct LoraCtx {
  int n;                           // adapted matrices
  int pad;                         // adapter rank rounded up to a multiple of 8 (the GEMMs' 16-byte granule); the
                                   // MFMA GEMMs take such widths with a masked ragged tile
  int which[7];                    // index into the order wq, wk, wv, wo, wgate, wup, wdown
  int out_dim[7], in_dim[7];
  void *a_pad[7], *b_pad[7];       // [pad, in], [out, pad] in the storage type, zero beyond the rank
  float *da_pad[7], *db_pad[7];    // fp32 accumulators of the same shapes
  void *P[7], *Q[7];               // [chunk, pad] per adapted matrix
  float* dg_sink;                  // the norm gains are frozen: their gradient goes nowhere
};
} // extern "C"

namespace {
int32_t layer_backward_impl(const sbp_layer_cfg* c, const sbp_layer_weights* w, const void* x, const void* dy, void* dx,
                            const sbp_layer_grads* g, const LoraCtx* lora, const LayerWs& s_all, hipStream_t st) {
  int32_t rc;
  t_gemm_scratch = s_all.gemm_scratch; t_gemm_scratch_bytes = s_all.gemm_scratch_bytes;
  const int dt = c->dtype, gdt = c->grad_dtype;
  const size_t es = dtype_size(dt);
  const int T = c->seq_len, cm = std::min(c->chunk, T), d = c->hidden, F = c->mlp_width;
  const int qd = c->n_q_heads * c->head_dim, kd = c->n_kv_heads * c->head_dim, half = c->head_dim / 2;
  float* dg1 = lora ? lora->dg_sink : g->g1;
  float* dg2 = lora ? lora->dg_sink + d : g->g2;

  HIPCHK(rope_table(s_all.rope, T, c->head_dim, c->rope_theta, c->pos_offset, st));
  for (int b = 0; b < c->batch; ++b) {
    const char* xb = at(x, (size_t)b * T, d, es);
    const char* dyb = at(dy, (size_t)b * T, d, es);
    char* dxb = at(dx, (size_t)b * T, d, es);
    const int kv_first = c->seq_first ? c->seq_first[b] : 0;      // rows before it are padding in front of the sequence
    if ((rc = kv_prepass(c, w, s_all, xb, st))) return rc;
    HIPCHK(fill_zero(s_all.dK, (size_t)T * kd * sizeof(float), st));
    HIPCHK(fill_zero(s_all.dV, (size_t)T * kd * sizeof(float), st));
    // Chunks run last to first: rows of dK/dV belonging to chunk i are final once
    // chunks >= i are done (later queries are the only other readers of those
    // keys), so the K/V-side gradient and dx of the chunk can be finished at once.
    const int n_chunks = (int)cdiv(T, cm);
    GemmArgs dws[7 * MAX_DW_GROUP];   // weight-gradient GEMMs waiting for their launch (a group of chunks' worth)
    int n_dws = 0;
    for (int ci = n_chunks - 1; ci >= 0; --ci) {
      const int r0 = ci * cm, n = std::min(cm, T - r0);
      const LayerWs s = chunk_view(s_all, ci % s_all.dw_group);
      if ((rc = chunk_reforward(c, w, s, xb, r0, n, kv_first, false, st))) return rc;
      const char* dyc = at(dyb, r0, d, es);
      // ---- MLP backward (the weight-gradient GEMMs of the chunk are deferred to one grouped launch below)
      {   // dact = dy W_d, then the SwiGLU adjoint: gate <- dgate, up <- dup, act <- silu(gate) up.  The adjoint can run as
          // the GEMM's epilogue (dact is then never stored); measured slower than the elementwise pass, so off by default.
        GemmArgs gd = dx_gemm(dyc, w->wdown, s.dact, n, d, F, dt, dt, false);
        if (fusion_mask() & FUSE_SWIGLU) {
          gd.swiglu_gate = s.gate; gd.swiglu_up = s.up; gd.swiglu_act = s.act;
          HIPCHK(gemm(gd, st));
        } else {
          HIPCHK(gemm(gd, st));
          HIPCHK(swiglu_bwd(dt, s.gate, s.up, s.dact, s.act, (int64_t)n * F, st));
        }
      }
      {   // dm = dgate W_g + dup W_u: two operand pairs, one launch
        GemmArgs gm = dx_gemm(s.gate, w->wgate, s.dm, n, F, d, dt, DT_F32, false);
        gm.A2 = s.up; gm.B2 = w->wup;
        HIPCHK(gemm(gm, st));
      }
      HIPCHK(rmsnorm_bwd(dt, s.dm, s.h1, true, w->g2, s.rstd2, dyc, false, s.dh1, s.dh1_t, dg2, s.partial, n, d, st));
      // ---- attention-side backward
      HIPCHK(gemm(dx_gemm(s.dh1_t, w->wo, s.d_o, n, d, qd, dt, dt, false), st));
      AttnArgs aa{};
      aa.dt = dt; aa.Hq = c->n_q_heads; aa.Hkv = c->n_kv_heads; aa.dh = c->head_dim;
      aa.q_start = r0; aa.q_len = n; aa.scale = 1.0f / std::sqrt((float)c->head_dim);
      aa.window = c->window; aa.kv_first = kv_first;
      aa.q = s.q; aa.k = s.K; aa.v = s.V; aa.o = s.o; aa.lse = s.lse;
      aa.d_o = s.d_o; aa.dq = s.dq; aa.dk = s.dK; aa.dv = s.dV; aa.delta = s.delta;
      if (fusion_mask() & FUSE_ROPE_Q) aa.rope_q = s.rope + (size_t)r0 * half;   // dq leaves the kernel rotated back (RoPE's adjoint)
      HIPCHK(attn_backward(aa, st));
      if (!(fusion_mask() & FUSE_ROPE_Q)) HIPCHK(rope_apply(dt, s.dq, s.rope + (size_t)r0 * half, n, c->n_q_heads, c->head_dim, true, st));
      HIPCHK(gemm(dx_gemm(s.dq, w->wq, s.da, n, qd, d, dt, DT_F32, false), st));
      // ---- K/V side of rows [r0, r0+n): final now
      HIPCHK(kv_grad_finish(dt, s.dK + (size_t)r0 * kd, s.dV + (size_t)r0 * kd, s.rope + (size_t)r0 * half, s.dkc, s.dvc,
                            n, c->n_kv_heads, c->head_dim, st));
      {   // da += dkc W_k + dvc W_v: same output, one launch with two reduction segments
        const GemmArgs kv[2] = {dx_gemm(s.dkc, w->wk, s.da, n, kd, d, dt, DT_F32, true),
                                dx_gemm(s.dvc, w->wv, s.da, n, kd, d, dt, DT_F32, true)};
        HIPCHK(gemm_batch(kv, 2, st));
      }
      if (!lora) {
        // ---- the seven weight gradients of the chunk, dW += dY^T X (Eq. 1 summand): queued, and launched together
        //      with those of the other chunks of the group (one pass over every dW for the group's rows)
        const GemmArgs mine[7] = {dw_gemm(dyc, s.act, g->wdown, n, d, F, dt, gdt),  dw_gemm(s.gate, s.m, g->wgate, n, F, d, dt, gdt),
                                  dw_gemm(s.up, s.m, g->wup, n, F, d, dt, gdt),    dw_gemm(s.dh1_t, s.o, g->wo, n, d, qd, dt, gdt),
                                  dw_gemm(s.dq, s.a, g->wq, n, qd, d, dt, gdt),    dw_gemm(s.dkc, s.a, g->wk, n, kd, d, dt, gdt),
                                  dw_gemm(s.dvc, s.a, g->wv, n, kd, d, dt, gdt)};
        for (int i = 0; i < 7; ++i) dws[n_dws++] = mine[i];
        if (n_dws == 7 * s_all.dw_group || ci == 0) {
          HIPCHK(gemm_batch(dws, n_dws, st));
          n_dws = 0;
        }
      } else {
        // ---- adapter gradients of the chunk (Eq. 1 summands of dA and dB): four grouped launches of skinny GEMMs
        const void* dYs[7] = {s.dq, s.dkc, s.dvc, s.dh1_t, s.gate, s.up, dyc};     // order wq, wk, wv, wo, wgate, wup, wdown
        const void* Xs[7] = {s.a, s.a, s.a, s.o, s.m, s.m, s.act};
        GemmArgs gp[7], gq[7], gb[7], ga[7];
        const int rp = lora->pad;
        for (int j = 0; j < lora->n; ++j) {
          const int i = lora->which[j], out = lora->out_dim[j], in = lora->in_dim[j];
          gp[j] = fwd_gemm(Xs[i], lora->a_pad[j], lora->P[j], n, rp, in, dt, dt);                                   // P = X A^T
          gq[j] = mk(dYs[i], lora->b_pad[j], lora->Q[j], n, rp, out, out, rp, rp, false, false, dt, dt, false);    // Q = dY B
          gb[j] = dw_gemm(dYs[i], lora->P[j], lora->db_pad[j], n, out, rp, dt, DT_F32);                             // dB += dY^T P
          ga[j] = dw_gemm(lora->Q[j], Xs[i], lora->da_pad[j], n, rp, in, dt, DT_F32);                               // dA += Q^T X
        }
        // P and Q are chunk x rank: a handful of output tiles each.  Those with a long reduction (the MLP width) go out
        // alone, where the dispatcher splits the reduction over the chip; the short ones share one grouped launch.
        auto launch_skinny = [&](const GemmArgs* gs, int cnt) -> int32_t {
          GemmArgs shortk[7];
          int n_short = 0;
          for (int j = 0; j < cnt; ++j) {
            if (gs[j].K >= 8192) HIPCHK(gemm(gs[j], st));
            else shortk[n_short++] = gs[j];
          }
          if (n_short == 1) HIPCHK(gemm(shortk[0], st));
          else if (n_short > 1) HIPCHK(gemm_batch(shortk, n_short, st, true));
          return SBP_OK;
        };
        if ((rc = launch_skinny(gp, lora->n))) return rc;
        if ((rc = launch_skinny(gq, lora->n))) return rc;
        if (lora->n == 1) {
          HIPCHK(gemm(gb[0], st)); HIPCHK(gemm(ga[0], st));
        } else {
          HIPCHK(gemm_batch(gb, lora->n, st, true));
          HIPCHK(gemm_batch(ga, lora->n, st, true));
        }
      }
      HIPCHK(rmsnorm_bwd(dt, s.da, at(xb, r0, d, es), false, w->g1, s.rstd1, s.dh1, true, nullptr, at(dxb, r0, d, es),
                         dg1, s.partial, n, d, st));
    }
  }
  return SBP_OK;
}
}  // namespace

extern "C" {

int32_t streambp_layer_backward(const sbp_layer_cfg* c, const sbp_layer_weights* w, const void* x, const void* dy,
                                void* dx, const sbp_layer_grads* g, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  int32_t rc = check_layer_cfg(c);
  if (rc) return rc;
  if ((rc = check_layer_ptrs(w))) return rc;
  if (!x || !dy || !dx || !g || !workspace) return fail(SBP_ERR_NULL, "x, dy, dx, dw and workspace must be non-NULL");
  {
    const void* ps[] = {g->wq, g->wk, g->wv, g->wo, g->wgate, g->wup, g->wdown, g->g1, g->g2};
    for (const void* p : ps) if (!p) return fail(SBP_ERR_NULL, "a gradient pointer is NULL");
  }
  if (dx == x || dx == dy) return fail(SBP_ERR_SHAPE, "dx may not alias x or dy");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const LayerWs s_all = carve_layer(c, workspace);
  if (workspace_bytes < s_all.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, s_all.bytes);
  return layer_backward_impl(c, w, x, dy, dx, g, nullptr, s_all, (hipStream_t)hip_stream);
}

// ---- adapter mode ---------------------------------------------------------------------------------------------
namespace {
int32_t check_lora(const sbp_layer_cfg* c, const sbp_lora_adapters* ad) {
  if (!ad) return fail(SBP_ERR_NULL, "adapters table is NULL");
  if (ad->rank < 1 || ad->rank > LORA_MAX_RANK) return fail(SBP_ERR_SHAPE, "adapter rank must be in [1, %d]", LORA_MAX_RANK);
  if (!std::isfinite(ad->scale)) return fail(SBP_ERR_SHAPE, "adapter scale must be finite");
  if (c->grad_dtype != SBP_F32) return fail(SBP_ERR_UNSUPPORTED, "adapter gradients are fp32");
  int n = 0;
  for (int i = 0; i < 7; ++i) {
    if ((ad->a[i] == nullptr) != (ad->b[i] == nullptr)) return fail(SBP_ERR_NULL, "adapter %d: A and B must be given together", i);
    n += ad->a[i] != nullptr;
  }
  if (n == 0) return fail(SBP_ERR_NULL, "no matrix is adapted");
  return SBP_OK;
}
struct LoraWs { LoraCtx ctx; sbp_layer_weights w_eff; void* bt[7]; sbp_layer_cfg layer_cfg; void* layer_ws; size_t layer_bytes; size_t bytes; };
LoraWs carve_lora(const sbp_layer_cfg* c, const sbp_layer_weights* w, const sbp_lora_adapters* ad, void* ws) {
  const size_t es = dtype_size(c->dtype);
  const int d = c->hidden, F = c->mlp_width, qd = c->n_q_heads * c->head_dim, kd = c->n_kv_heads * c->head_dim;
  const int outs[7] = {qd, kd, kd, d, F, F, d}, ins[7] = {d, d, d, qd, d, d, F};
  const size_t cm = (size_t)std::min(c->chunk, c->seq_len);
  Carver cv(ws);
  LoraWs L{};
  if (w) L.w_eff = *w;
  const void** eff[7] = {&L.w_eff.wq, &L.w_eff.wk, &L.w_eff.wv, &L.w_eff.wo, &L.w_eff.wgate, &L.w_eff.wup, &L.w_eff.wdown};
  LoraCtx& x = L.ctx;
  x.n = 0;
  x.pad = (ad->rank + 7) & ~7;
  const size_t rp = (size_t)x.pad;
  for (int i = 0; i < 7; ++i) {
    if (!ad->a[i]) continue;
    const int j = x.n++;
    x.which[j] = i; x.out_dim[j] = outs[i]; x.in_dim[j] = ins[i];
    *eff[i] = cv.take_bytes((size_t)outs[i] * ins[i] * es);                      // W + s B A
    x.a_pad[j] = cv.take_bytes(rp * ins[i] * es);
    x.b_pad[j] = cv.take_bytes((size_t)outs[i] * rp * es);
    L.bt[j] = cv.take_bytes((size_t)ad->rank * outs[i] * es);                    // s B^T, the merge GEMM's operand
    x.da_pad[j] = cv.take<float>(rp * ins[i]);
    x.db_pad[j] = cv.take<float>((size_t)outs[i] * rp);
    x.P[j] = cv.take_bytes(cm * rp * es);
    x.Q[j] = cv.take_bytes(cm * rp * es);
  }
  x.dg_sink = cv.take<float>((size_t)2 * d);
  L.layer_cfg = *c;
  L.layer_cfg.dw_group_rows = 1;          // no weight-gradient passes to group: one set of chunk buffers
  L.layer_ws = cv.take_bytes(0);
  L.layer_bytes = carve_layer(&L.layer_cfg, nullptr).bytes;
  L.bytes = cv.off + L.layer_bytes;
  return L;
}
}  // namespace

size_t streambp_layer_lora_workspace_bytes(const sbp_layer_cfg* cfg, const sbp_lora_adapters* ad) {
  if (check_layer_cfg(cfg) != SBP_OK || check_lora(cfg, ad) != SBP_OK) return 0;
  return carve_lora(cfg, nullptr, ad, nullptr).bytes;
}

int32_t streambp_layer_lora_backward(const sbp_layer_cfg* c, const sbp_layer_weights* w, const sbp_lora_adapters* ad,
                                     const void* x, const void* dy, void* dx, const sbp_lora_grads* g, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  int32_t rc = check_layer_cfg(c);
  if (rc) return rc;
  if ((rc = check_layer_ptrs(w))) return rc;
  if ((rc = check_lora(c, ad))) return rc;
  if (!x || !dy || !dx || !g || !workspace) return fail(SBP_ERR_NULL, "x, dy, dx, the gradient table and workspace must be non-NULL");
  for (int i = 0; i < 7; ++i)
    if (ad->a[i] && (!g->da[i] || !g->db[i])) return fail(SBP_ERR_NULL, "adapter %d: da and db must be non-NULL", i);
  if (dx == x || dx == dy) return fail(SBP_ERR_SHAPE, "dx may not alias x or dy");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const LoraWs L = carve_lora(c, w, ad, workspace);
  if (workspace_bytes < L.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.bytes);
  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c->dtype;
  const size_t es = dtype_size(dt);
  const void* base[7] = {w->wq, w->wk, w->wv, w->wo, w->wgate, w->wup, w->wdown};
  const void* eff[7] = {L.w_eff.wq, L.w_eff.wk, L.w_eff.wv, L.w_eff.wo, L.w_eff.wgate, L.w_eff.wup, L.w_eff.wdown};
  const LoraCtx& X = L.ctx;
  t_gemm_scratch = nullptr; t_gemm_scratch_bytes = 0;
  for (int j = 0; j < X.n; ++j) {
    const int i = X.which[j], out = X.out_dim[j], in = X.in_dim[j], r = ad->rank;
    // operands with the rank rounded up to a multiple of 8, and the effective matrix W + s B A: a copy of W, then one pass that reads
    // it, adds the rank-r product in fp32 and rounds once
    HIPCHK(pad_matrix(dt, ad->a[i], r, in, false, 1.0f, X.a_pad[j], X.pad, in, st));
    HIPCHK(pad_matrix(dt, ad->b[i], out, r, false, 1.0f, X.b_pad[j], out, X.pad, st));
    HIPCHK(pad_matrix(dt, ad->b[i], r, out, true, ad->scale, L.bt[j], r, out, st));
    HIPCHK(copy_bytes((void*)eff[i], base[i], (size_t)out * in * es, st));
    HIPCHK(gemm(mk(L.bt[j], X.a_pad[j], (void*)eff[i], out, in, r, out, in, in, true, false, dt, dt, true), st));
    HIPCHK(fill_zero(X.da_pad[j], (size_t)X.pad * in * sizeof(float), st));
    HIPCHK(fill_zero(X.db_pad[j], (size_t)out * X.pad * sizeof(float), st));
  }
  const LayerWs s_all = carve_layer(&L.layer_cfg, L.layer_ws);
  if ((rc = layer_backward_impl(&L.layer_cfg, &L.w_eff, x, dy, dx, nullptr, &X, s_all, st))) return rc;
  for (int j = 0; j < X.n; ++j) {
    const int i = X.which[j];
    HIPCHK(add_scaled_block(X.da_pad[j], X.in_dim[j], ad->scale, g->da[i], ad->rank, X.in_dim[j], st));
    HIPCHK(add_scaled_block(X.db_pad[j], X.pad, ad->scale, g->db[i], X.out_dim[j], ad->rank, st));
  }
  return SBP_OK;
}

int32_t streambp_layer_forward(const sbp_layer_cfg* c, const sbp_layer_weights* w, const void* x, void* y,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  int32_t rc = check_layer_cfg(c);
  if (rc) return rc;
  if ((rc = check_layer_ptrs(w))) return rc;
  if (!x || !y || !workspace) return fail(SBP_ERR_NULL, "x, y and workspace must be non-NULL");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const LayerWs s = carve_layer(c, workspace);
  if (workspace_bytes < s.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, s.bytes);
  hipStream_t st = (hipStream_t)hip_stream;
  t_gemm_scratch = s.gemm_scratch; t_gemm_scratch_bytes = s.gemm_scratch_bytes;
  const int dt = c->dtype;
  const size_t es = dtype_size(dt);
  const int T = c->seq_len, cm = std::min(c->chunk, T), d = c->hidden, F = c->mlp_width;
  HIPCHK(rope_table(s.rope, T, c->head_dim, c->rope_theta, c->pos_offset, st));
  for (int b = 0; b < c->batch; ++b) {
    const char* xb = at(x, (size_t)b * T, d, es);
    char* yb = at(y, (size_t)b * T, d, es);
    const int kv_first = c->seq_first ? c->seq_first[b] : 0;
    if ((rc = kv_prepass(c, w, s, xb, st))) return rc;
    for (int r0 = 0; r0 < T; r0 += cm) {
      const int n = std::min(cm, T - r0);
      if ((rc = chunk_reforward(c, w, s, xb, r0, n, kv_first, true, st))) return rc;
      HIPCHK(gemm(fwd_gemm(s.act, w->wdown, s.proj, n, d, F, dt, DT_F32), st));
      HIPCHK(add_store(dt, s.h1, s.proj, at(yb, r0, d, es), (int64_t)n * d, st));
    }
  }
  return SBP_OK;
}

// --------------------------------------------------------------- LM head --
static int32_t check_head_cfg(const sbp_head_cfg* c) {
  if (!c) return fail(SBP_ERR_NULL, "cfg is NULL");
  if (!valid_dtype(c->dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype %d not supported", c->dtype);
  if (int32_t rc = check_grad_dtype(c->dtype, c->grad_dtype)) return rc;
  if (c->dw_group_rows < 0) return fail(SBP_ERR_SHAPE, "dw_group_rows must be >= 0");
  if (c->batch < 1 || c->seq_len < 1 || c->chunk < 1 || c->hidden < 1 || c->vocab < 1)
    return fail(SBP_ERR_SHAPE, "batch, seq_len, chunk, hidden and vocab must be >= 1");
  if (c->objective < SBP_OBJ_SFT || c->objective > SBP_OBJ_DPO) return fail(SBP_ERR_UNSUPPORTED, "objective %d not supported", c->objective);
  if (c->objective == SBP_OBJ_DPO && c->batch != 2) return fail(SBP_ERR_SHAPE, "DPO needs batch == 2 (chosen, rejected)");
  return SBP_OK;
}

// The weight gradient of the head is accumulated once per group of chunks (dw_group_for): dz and the gathered h rows of that
// many chunks stay alive and one GEMM with a segmented reduction adds them into dW, so the 8 bytes per element of
// read-modify-write traffic on dW (the largest tensor of the path) are paid once per group instead of once per
// chunk.  The fp32 logits - the dominant term - still exist for one chunk only.
struct HeadWs {
  int dw_group;
  float* z; void* dz[MAX_DW_GROUP]; float *row_loss, *target_logit, *seq_weight, *ell;
  float2* stats; int n_stat;          // per row and 256-column block of the chunk's logits: (max, sum of exp), written by the logits GEMM
  int32_t *index, *chunk_rows; void *hc[MAX_DW_GROUP], *dhc;   // active-row compaction: row list, rows per chunk, gathered h / dh rows
  float* gemm_scratch; size_t gemm_scratch_bytes; size_t bytes;
};
static HeadWs carve_head(const sbp_head_cfg* c, void* ws) {
  const int64_t rows = (int64_t)c->batch * c->seq_len;
  const size_t cm = (size_t)std::min<int64_t>(c->chunk, rows);
  Carver cv(ws);
  HeadWs h;
  h.z = cv.take<float>(cm * c->vocab);
  h.dw_group = dw_group_for(cm, c->dw_group_rows, DW_GROUP_ROWS_HEAD);
  for (int g = 0; g < h.dw_group; ++g) h.dz[g] = cv.take_bytes(cm * c->vocab * dtype_size(c->dtype));
  h.row_loss = cv.take<float>(cm);
  h.target_logit = cv.take<float>(cm);
  h.n_stat = (int)cdiv(c->vocab, GEMM_STAT_COLS);
  h.stats = cv.take<float2>(cm * (size_t)h.n_stat);
  h.seq_weight = cv.take<float>(c->batch);
  h.ell = cv.take<float>(1);
  h.index = cv.take<int32_t>((size_t)rows);
  h.chunk_rows = cv.take<int32_t>((size_t)cdiv(rows, (int64_t)cm));
  for (int g = 0; g < h.dw_group; ++g) h.hc[g] = cv.take_bytes(cm * c->hidden * dtype_size(c->dtype));
  h.dhc = cv.take_bytes(cm * c->hidden * dtype_size(c->dtype));
  h.gemm_scratch_bytes = c->dtype == SBP_BF16 ? gemm_scratch_bytes((int)cm, c->hidden, 4) : 0;
  h.gemm_scratch = (float*)cv.take_bytes(h.gemm_scratch_bytes);
  h.bytes = cv.off;
  return h;
}

size_t streambp_lmhead_workspace_bytes(const sbp_head_cfg* cfg) {
  if (check_head_cfg(cfg) != SBP_OK) return 0;
  return carve_head(cfg, nullptr).bytes;
}

int32_t streambp_lmhead_ce_backward(const sbp_head_cfg* c, const void* w, const void* h, const int32_t* targets,
                                    const float* old_logp, const float* ref_logp, const float* advantages, void* dh,
                                    void* dw, float* loss, int64_t* n_active, void* workspace, size_t workspace_bytes,
                                    void* hip_stream) {
  int32_t rc = check_head_cfg(c);
  if (rc) return rc;
  if (!w || !h || !targets || !dh || !dw || !loss || !n_active || !workspace)
    return fail(SBP_ERR_NULL, "w, h, targets, dh, dw, loss, n_active and workspace must be non-NULL");
  if (c->objective == SBP_OBJ_GRPO && (!ref_logp || !advantages)) return fail(SBP_ERR_NULL, "GRPO needs ref_logp and advantages");
  if (c->objective == SBP_OBJ_DPO && !ref_logp) return fail(SBP_ERR_NULL, "DPO needs ref_logp");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const HeadWs s = carve_head(c, workspace);
  if (workspace_bytes < s.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, s.bytes);

  hipStream_t st = (hipStream_t)hip_stream;
  const int dt = c->dtype;
  const size_t es = dtype_size(dt);
  t_gemm_scratch = s.gemm_scratch; t_gemm_scratch_bytes = s.gemm_scratch_bytes;
  const int64_t rows = (int64_t)c->batch * c->seq_len;
  const int cm = (int)std::min<int64_t>(c->chunk, rows);
  const int d = c->hidden, V = c->vocab;

  HIPCHK(count_active(targets, c->batch, c->seq_len, V, s.seq_weight, n_active, st));
  if (c->objective == SBP_OBJ_DPO) HIPCHK(fill_zero(s.ell, sizeof(float), st));
  // Rows with an ignored target contribute nothing (dz = 0): only the active rows are pushed through the
  // GEMMs.  Positions are independent (Sec. 3.2.1), so the active rows of all sequences are chunked as one
  // flat list; the list and the per-chunk row counts live on the device (no host synchronisation), and the
  // kernels of a chunk read their row count at run time.
  const int n_chunks = (int)cdiv(rows, (int64_t)cm);
  HIPCHK(compact_active(targets, rows, cm, V, s.index, s.chunk_rows, n_chunks, st));
  HIPCHK(fill_zero(dh, (size_t)rows * d * es, st));          // ignored rows of dh: exact zeros
  GemmArgs pending[MAX_DW_GROUP];
  int n_pending = 0;
  for (int ci = 0; ci < n_chunks; ++ci) {
    const int32_t* idx = s.index + (size_t)ci * cm;
    const int* n_dev = s.chunk_rows + ci;
    const int n = (int)std::min<int64_t>(cm, rows - (int64_t)ci * cm);      // upper bound of the chunk's rows
    void* hc = s.hc[n_pending];
    void* dz = s.dz[n_pending];
    HIPCHK(gather_rows(dt, h, idx, n_dev, hc, n, d, st));
    // The logits: fp32 with (max, sum of exp) per row and 256-column block out of the GEMM's epilogue where the MFMA kernel
    // takes the problem - or, better, never as logits at all: the numerator form leaves exp(z - block max) in bf16 directly in
    // the chunk's dz buffer plus the target logits, and the row kernel finishes dz in place.
    GemmArgs gz = fwd_gemm(hc, w, s.z, n, V, d, dt, DT_F32);
    gz.rows_dev = n_dev;
    gz.row_stats = s.stats;
    bool numer = false;
    if ((fusion_mask() & FUSE_NUMERATORS) && dt == DT_BF16 && s.n_stat > 0) {
      GemmArgs gn = fwd_gemm(hc, w, dz, n, V, d, dt, DT_BF16);
      gn.rows_dev = n_dev; gn.row_stats = s.stats;
      gn.numer_targets = targets; gn.numer_row_index = idx; gn.numer_target_value = s.target_logit;
      if (gemm_numerators_supported(gn)) { gz = gn; numer = true; }
    }
    const bool stats = numer || (s.n_stat > 0 && gemm_row_stats_supported(gz));   // the LSE statistics come out of the GEMM's epilogue
    if (!stats) gz.row_stats = nullptr;
    HIPCHK(gemm(gz, st));
    HeadRowArgs a{};
    a.stats = stats ? s.stats : nullptr; a.n_stat = s.n_stat;
    a.target_logit = numer ? s.target_logit : nullptr;
    a.dt = dt; a.objective = c->objective; a.z = s.z; a.dz = dz; a.targets = targets;
    a.old_logp = old_logp; a.ref_logp = ref_logp;
    a.advantages = advantages; a.seq_weight = s.seq_weight; a.row0 = 0; a.row_index = idx; a.rows_dev = n_dev;
    a.rows = n; a.V = V; a.T = c->seq_len;
    a.loss_scale = c->loss_scale; a.clip_eps = c->clip_eps; a.kl_beta = c->kl_beta; a.kl_mode = c->kl_mode;
    a.row_loss = s.row_loss;
    HIPCHK(head_rows(a, st));
    HIPCHK(reduce_add(s.row_loss, n, c->objective == SBP_OBJ_DPO ? s.ell : loss, st, n_dev));
    GemmArgs gh = dx_gemm(dz, w, s.dhc, n, V, d, dt, dt, false);
    gh.rows_dev = n_dev;
    HIPCHK(gemm(gh, st));
    HIPCHK(scatter_rows(dt, s.dhc, idx, n_dev, dh, n, d, st));
    pending[n_pending] = dw_gemm(dz, hc, dw, n, V, d, dt, c->grad_dtype);
    pending[n_pending].rows_dev = n_dev;
    if (++n_pending == s.dw_group || ci + 1 == n_chunks) {
      HIPCHK(gemm_batch(pending, n_pending, st));
      n_pending = 0;
    }
  }
  if (c->objective == SBP_OBJ_DPO)
    HIPCHK(dpo_finish(dt, s.ell, c->kl_beta, dh, rows * d, dw, c->grad_dtype, (int64_t)V * d, loss, st));
  return SBP_OK;
}

// -------------------------------------------------------- chunk attention --
static int32_t check_attn_cfg(const sbp_attn_cfg* c) {
  if (!c) return fail(SBP_ERR_NULL, "cfg is NULL");
  if (!valid_dtype(c->dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype %d not supported", c->dtype);
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads != 0)
    return fail(SBP_ERR_SHAPE, "n_q_heads must be a positive multiple of n_kv_heads");
  if (c->head_dim < 1 || c->head_dim > 256) return fail(SBP_ERR_SHAPE, "head_dim must be in [1, 256]");
  if (c->q_start < 0 || c->q_len < 0) return fail(SBP_ERR_SHAPE, "q_start and q_len must be >= 0");
  if ((int64_t)c->q_start + c->q_len > INT32_MAX) return fail(SBP_ERR_SHAPE, "q_start + q_len overflows");
  // the kernels take row maxima of the raw scores before scaling them, which is only right for a positive finite scale
  if (!(c->scale > 0.f) || !std::isfinite(c->scale)) return fail(SBP_ERR_SHAPE, "scale must be positive and finite");
  if (c->window < 0 || c->kv_first < 0) return fail(SBP_ERR_SHAPE, "window and kv_first must be >= 0");
  return SBP_OK;
}

size_t streambp_attn_workspace_bytes(const sbp_attn_cfg* cfg) {
  if (check_attn_cfg(cfg) != SBP_OK) return 0;
  return align_up((size_t)2 * std::max(cfg->q_len, 1) * cfg->n_q_heads * sizeof(float), 256);
}

int32_t streambp_attn_chunk_forward(const sbp_attn_cfg* c, const void* q, const void* k, const void* v, void* o,
                                    float* lse, void* hip_stream) {
  int32_t rc = check_attn_cfg(c);
  if (rc) return rc;
  if (c->q_len == 0) return SBP_OK;   // empty chunk: nothing to do
  if (!q || !k || !v || !o || !lse) return fail(SBP_ERR_NULL, "q, k, v, o and lse must be non-NULL");
  AttnArgs a{};
  a.dt = c->dtype; a.Hq = c->n_q_heads; a.Hkv = c->n_kv_heads; a.dh = c->head_dim;
  a.q_start = c->q_start; a.q_len = c->q_len; a.scale = c->scale; a.window = c->window; a.kv_first = c->kv_first;
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
  HIPCHK(attn_forward(a, (hipStream_t)hip_stream));
  return SBP_OK;
}

int32_t streambp_attn_chunk_backward(const sbp_attn_cfg* c, const void* q, const void* k, const void* v, const void* o,
                                     const float* lse, const void* d_o, void* dq, float* dk, float* dv,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  int32_t rc = check_attn_cfg(c);
  if (rc) return rc;
  if (c->q_len == 0) return SBP_OK;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
    return fail(SBP_ERR_NULL, "all tensor pointers and workspace must be non-NULL");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < streambp_attn_workspace_bytes(c)) return fail(SBP_ERR_WORKSPACE, "workspace too small");
  AttnArgs a{};
  a.dt = c->dtype; a.Hq = c->n_q_heads; a.Hkv = c->n_kv_heads; a.dh = c->head_dim;
  a.q_start = c->q_start; a.q_len = c->q_len; a.scale = c->scale; a.window = c->window; a.kv_first = c->kv_first;
  a.q = q; a.k = k; a.v = v; a.o = (void*)o; a.lse = (float*)lse;
  a.d_o = d_o; a.dq = dq; a.dk = dk; a.dv = dv; a.delta = (float*)workspace;
  HIPCHK(attn_backward(a, (hipStream_t)hip_stream));
  return SBP_OK;
}

// Which kernels a configuration gets.  The bf16 MFMA GEMMs need every matrix dimension of the layer (hidden, the q and
// k/v widths, mlp_width - resp. hidden and vocab for the head) to be a multiple of 64 (the reduction step; output tiles
// are 256 wide with a masked ragged last tile), the MFMA attention head_dim 128; anything else runs on the
// shape-agnostic fp32-ALU kernels, which are a correctness path and orders of magnitude slower.
int32_t streambp_layer_fast_path(const sbp_layer_cfg* c) {
  if (int32_t rc = check_layer_cfg(c)) return rc;
  if (c->dtype != SBP_BF16) return fail(0, "fp32 storage: the shape-agnostic kernels are the only path"), 0;
  const int qd = c->n_q_heads * c->head_dim, kd = c->n_kv_heads * c->head_dim;
  if (c->head_dim != 128) return fail(0, "head_dim %d: the MFMA attention kernels take 128 only", c->head_dim), 0;
  const int dims[4] = {c->hidden, qd, kd, c->mlp_width};
  const char* names[4] = {"hidden", "n_q_heads*head_dim", "n_kv_heads*head_dim", "mlp_width"};
  for (int i = 0; i < 4; ++i)   // every width is the reduction length of some GEMM of the layer
    if (dims[i] % 64) return fail(0, "%s = %d is not a multiple of 64: its GEMMs leave the MFMA kernels", names[i], dims[i]), 0;
  return 1;
}
int32_t streambp_lmhead_fast_path(const sbp_head_cfg* c) {
  if (int32_t rc = check_head_cfg(c)) return rc;
  if (c->dtype != SBP_BF16) return fail(0, "fp32 storage: the shape-agnostic kernels are the only path"), 0;
  if (c->hidden % 64) return fail(0, "hidden = %d is not a multiple of 64: the head's GEMMs leave the MFMA kernels", c->hidden), 0;
  if (c->vocab % 64) return fail(0, "vocab = %d is not a multiple of 64: the head's GEMMs leave the MFMA kernels", c->vocab), 0;
  return 1;
}
int64_t streambp_generic_launches(void) { return (int64_t)generic_bf16_launches(); }

// ---- the same backward for callers that cannot allocate ------------------------------------------------------
// The per-call scratch of the attention backward (delta and the log2-domain log-sum-exp, 2 floats per (query, head)
// pair) lives in device memory that belongs to the library's code object instead of a caller workspace.  Every GPU
// the library runs on holds its own copy of the array at its own address; the address is looked up once per device
// (a symbol query, not an allocation) and only that pointer - never the array's name, which on the host is a stand-in
// and not a device address - is handed to kernels.
constexpr int64_t STATIC_SCRATCH_PAIRS = 1 << 18;            // q_len * n_q_heads <= 262144 (2 MiB of scratch)
static __device__ __align__(256) float g_static_scratch[2 * STATIC_SCRATCH_PAIRS];
constexpr int STATIC_MAX_DEVICES = 64;
static float* g_static_scratch_ptr[STATIC_MAX_DEVICES];      // per device, filled on the first call on that device
static std::mutex g_static_scratch_mu;

int32_t streambp_attn_chunk_backward_noalloc(const sbp_attn_cfg* c, const void* q, const void* k, const void* v, const void* o,
                                             const float* lse, const void* d_o, void* dq, float* dk, float* dv,
                                             void* hip_stream) {
  int32_t rc = check_attn_cfg(c);
  if (rc) return rc;
  if (c->q_len == 0) return SBP_OK;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return fail(SBP_ERR_NULL, "all tensor pointers must be non-NULL");
  const int64_t pairs = (int64_t)c->q_len * c->n_q_heads;
  if (pairs > STATIC_SCRATCH_PAIRS)
    return fail(SBP_ERR_WORKSPACE, "q_len * n_q_heads = %lld exceeds the %lld pairs the built-in scratch holds; use "
                "streambp_attn_chunk_backward with a caller workspace", (long long)pairs, (long long)STATIC_SCRATCH_PAIRS);
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(SBP_ERR_UNSUPPORTED, "device index %d out of range", dev);
  float* scratch;
  {
    std::lock_guard<std::mutex> lock(g_static_scratch_mu);
    if (!g_static_scratch_ptr[dev]) {
      void* p = nullptr;
      HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
      if (!p) return fail(SBP_ERR_HIP, "hipGetSymbolAddress returned a null address for the built-in scratch");
      g_static_scratch_ptr[dev] = (float*)p;
    }
    scratch = g_static_scratch_ptr[dev];
  }
  AttnArgs a{};
  a.dt = c->dtype; a.Hq = c->n_q_heads; a.Hkv = c->n_kv_heads; a.dh = c->head_dim;
  a.q_start = c->q_start; a.q_len = c->q_len; a.scale = c->scale; a.window = c->window; a.kv_first = c->kv_first;
  a.q = q; a.k = k; a.v = v; a.o = (void*)o; a.lse = (float*)lse;
  a.d_o = d_o; a.dq = dq; a.dk = dk; a.dv = dv; a.delta = scratch;
  HIPCHK(attn_backward(a, (hipStream_t)hip_stream));
  return SBP_OK;
}

int64_t streambp_attn_tile_pairs(int32_t q_start, int32_t q_len, int32_t* tile_q, int32_t* tile_k) {
  // Work is skipped per wave: a wave owns ATTN_WAVE_Q query rows and walks key tiles of ATTN_TILE_K.
  if (tile_q) *tile_q = ATTN_WAVE_Q;
  if (tile_k) *tile_k = ATTN_TILE_K;
  if (q_start < 0 || q_len <= 0) return 0;
  int64_t pairs = 0;
  for (int64_t t0 = 0; t0 < q_len; t0 += ATTN_WAVE_Q) {
    const int64_t last_q = q_start + std::min<int64_t>(t0 + ATTN_WAVE_Q, q_len) - 1;   // last query position of the wave
    pairs += last_q / ATTN_TILE_K + 1;                                                 // key tiles that start at or before it
  }
  return pairs;
}

// ------------------------------------------------------------ stack loop --
namespace {
struct StackWs { void *h, *dh, *ga, *gb; void* sub; size_t sub_bytes; size_t bytes; };
sbp_head_cfg stack_head_cfg(const sbp_stack_cfg* c) {
  sbp_head_cfg h{};
  h.dtype = c->layer.dtype; h.batch = c->layer.batch; h.seq_len = c->layer.seq_len; h.chunk = c->head_chunk;
  h.hidden = c->layer.hidden; h.vocab = c->vocab; h.objective = c->objective; h.loss_scale = c->loss_scale;
  h.clip_eps = c->clip_eps; h.kl_beta = c->kl_beta; h.kl_mode = c->kl_mode; h.grad_dtype = c->layer.grad_dtype; h.dw_group_rows = c->layer.dw_group_rows;
  return h;
}
int32_t check_stack_cfg(const sbp_stack_cfg* c) {
  if (!c) return fail(SBP_ERR_NULL, "cfg is NULL");
  int32_t rc = check_layer_cfg(&c->layer);
  if (rc) return rc;
  if (c->n_layers < 1) return fail(SBP_ERR_SHAPE, "n_layers must be >= 1");
  if (!(c->final_eps >= 0.f)) return fail(SBP_ERR_SHAPE, "final_eps must be >= 0");
  const sbp_head_cfg h = stack_head_cfg(c);
  return check_head_cfg(&h);
}
StackWs carve_stack(const sbp_stack_cfg* c, void* ws) {
  const size_t rows = (size_t)c->layer.batch * c->layer.seq_len, d = c->layer.hidden, es = dtype_size(c->layer.dtype);
  const sbp_head_cfg h = stack_head_cfg(c);
  Carver cv(ws);
  StackWs s;
  s.h = cv.take_bytes(rows * d * es);      // RMSNorm(ckpt[L])
  s.dh = cv.take_bytes(rows * d * es);     // gradient wrt h
  s.ga = cv.take_bytes(rows * d * es);     // running dL/dx, ping
  s.gb = cv.take_bytes(rows * d * es);     // pong
  s.sub_bytes = std::max(std::max(streambp_layer_workspace_bytes(&c->layer), streambp_lmhead_workspace_bytes(&h)),
                         streambp_rmsnorm_workspace_bytes((int64_t)rows, (int32_t)d));
  s.sub = cv.take_bytes(s.sub_bytes);
  s.bytes = cv.off;
  return s;
}
}  // namespace

extern "C" size_t streambp_stack_workspace_bytes(const sbp_stack_cfg* cfg) {
  if (check_stack_cfg(cfg) != SBP_OK) return 0;
  return carve_stack(cfg, nullptr).bytes;
}

extern "C" int32_t streambp_stack_forward(const sbp_stack_cfg* c, const sbp_layer_weights* layers, const void* emb,
                                          const int32_t* ids, void* const* ckpt, void* workspace, size_t workspace_bytes,
                                          void* hip_stream) {
  int32_t rc = check_stack_cfg(c);
  if (rc) return rc;
  if (!layers || !ckpt || !workspace) return fail(SBP_ERR_NULL, "layers, ckpt and workspace must be non-NULL");
  if ((emb == nullptr) != (ids == nullptr)) return fail(SBP_ERR_NULL, "emb and ids must be given together");
  for (int l = 0; l <= c->n_layers; ++l) if (!ckpt[l]) return fail(SBP_ERR_NULL, "ckpt[%d] is NULL", l);
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const StackWs s = carve_stack(c, workspace);
  if (workspace_bytes < s.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, s.bytes);
  const int64_t rows = (int64_t)c->layer.batch * c->layer.seq_len;
  if (emb && (rc = streambp_embedding_forward(c->layer.dtype, rows, c->layer.hidden, c->vocab, ids, emb, ckpt[0], hip_stream))) return rc;
  for (int l = 0; l < c->n_layers; ++l)
    if ((rc = streambp_layer_forward(&c->layer, &layers[l], ckpt[l], ckpt[l + 1], s.sub, s.sub_bytes, hip_stream))) return rc;
  return SBP_OK;
}

extern "C" int32_t streambp_stack_backward(const sbp_stack_cfg* c, const sbp_layer_weights* layers, const void* g_final,
                                           const void* w_head, void* const* ckpt, const int32_t* ids, const int32_t* targets,
                                           const float* old_logp, const float* ref_logp, const float* advantages,
                                           const sbp_layer_grads* dlayers, float* dg_final, void* dw_head, float* demb,
                                           void* dx0, float* loss, int64_t* n_active, void* workspace,
                                           size_t workspace_bytes, void* hip_stream) {
  int32_t rc = check_stack_cfg(c);
  if (rc) return rc;
  if (!layers || !g_final || !w_head || !ckpt || !targets || !dlayers || !dg_final || !dw_head || !loss || !n_active || !workspace)
    return fail(SBP_ERR_NULL, "a required pointer is NULL");
  if ((demb == nullptr) != (ids == nullptr)) return fail(SBP_ERR_NULL, "demb and ids must be given together");
  for (int l = 0; l <= c->n_layers; ++l) if (!ckpt[l]) return fail(SBP_ERR_NULL, "ckpt[%d] is NULL", l);
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const StackWs s = carve_stack(c, workspace);
  if (workspace_bytes < s.bytes) return fail(SBP_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, s.bytes);
  const int64_t rows = (int64_t)c->layer.batch * c->layer.seq_len;
  const int d = c->layer.hidden, dt = c->layer.dtype;
  const sbp_head_cfg hc = stack_head_cfg(c);
  const int L = c->n_layers;
  // head on h = RMSNorm(x_L), then the final norm's adjoint
  if ((rc = streambp_rmsnorm_forward(dt, rows, d, c->final_eps, ckpt[L], g_final, s.h, hip_stream))) return rc;
  if ((rc = streambp_lmhead_ce_backward(&hc, w_head, s.h, targets, old_logp, ref_logp, advantages, s.dh, dw_head, loss, n_active,
                                        s.sub, s.sub_bytes, hip_stream))) return rc;
  if ((rc = streambp_rmsnorm_backward(dt, rows, d, c->final_eps, ckpt[L], g_final, s.dh, s.ga, dg_final, s.sub, s.sub_bytes, hip_stream))) return rc;
  // layers L-1 .. 0: dL/dx of layer l is dL/dy of layer l-1 (Sec. 3.1)
  void* gin = s.ga;
  void* gout = s.gb;
  for (int l = L - 1; l >= 0; --l) {
    void* dst = (l == 0 && dx0) ? dx0 : gout;
    if ((rc = streambp_layer_backward(&c->layer, &layers[l], ckpt[l], gin, dst, &dlayers[l], s.sub, s.sub_bytes, hip_stream))) return rc;
    gout = gin;
    gin = dst;
  }
  if (demb && (rc = streambp_embedding_backward(dt, rows, d, c->vocab, ids, gin, demb, hip_stream))) return rc;
  return SBP_OK;
}

// ------------------------------------------------------------ stack glue --
size_t streambp_rmsnorm_workspace_bytes(int64_t n_rows, int32_t hidden) {
  if (n_rows < 0 || n_rows > INT32_MAX || hidden < 1) return 0;
  return align_up((size_t)std::max<int64_t>(n_rows, 1) * sizeof(float), 256) +
         align_up(rmsnorm_bwd_partial_floats((int)n_rows, hidden) * sizeof(float) + 256, 256);
}
int32_t streambp_rmsnorm_forward(int32_t dtype, int64_t n_rows, int32_t hidden, float eps, const void* x, const void* g,
                                 void* y, void* hip_stream) {
  if (!valid_dtype(dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype %d not supported", dtype);
  if (n_rows < 0 || n_rows > INT32_MAX || hidden < 1 || !(eps >= 0.f)) return fail(SBP_ERR_SHAPE, "bad shape");
  if (!x || !g || !y) return fail(SBP_ERR_NULL, "x, g and y must be non-NULL");
  HIPCHK(rmsnorm_fwd(dtype, x, nullptr, g, y, nullptr, nullptr, (int)n_rows, hidden, eps, (hipStream_t)hip_stream));
  return SBP_OK;
}
int32_t streambp_rmsnorm_backward(int32_t dtype, int64_t n_rows, int32_t hidden, float eps, const void* x, const void* g,
                                  const void* dy, void* dx, float* dg, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
  if (!valid_dtype(dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype %d not supported", dtype);
  if (n_rows < 0 || n_rows > INT32_MAX || hidden < 1 || !(eps >= 0.f)) return fail(SBP_ERR_SHAPE, "bad shape");
  if (!x || !g || !dy || !dx || !dg || !workspace) return fail(SBP_ERR_NULL, "x, g, dy, dx, dg and workspace must be non-NULL");
  if ((uintptr_t)workspace & 255) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < streambp_rmsnorm_workspace_bytes(n_rows, hidden)) return fail(SBP_ERR_WORKSPACE, "workspace too small");
  Carver cv(workspace);
  float* rstd = cv.take<float>((size_t)std::max<int64_t>(n_rows, 1));
  float* partial = cv.take<float>(rmsnorm_bwd_partial_floats((int)n_rows, hidden) + 64);
  hipStream_t st = (hipStream_t)hip_stream;
  HIPCHK(rmsnorm_fwd(dtype, x, nullptr, g, nullptr, nullptr, rstd, (int)n_rows, hidden, eps, st));
  HIPCHK(rmsnorm_bwd_plain(dtype, dy, x, g, rstd, dx, dg, partial, (int)n_rows, hidden, st));
  return SBP_OK;
}
int32_t streambp_embedding_forward(int32_t dtype, int64_t n_rows, int32_t hidden, int32_t vocab, const int32_t* ids,
                                   const void* emb, void* x, void* hip_stream) {
  if (!valid_dtype(dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype");
  if (n_rows < 0 || hidden < 1 || vocab < 1 || n_rows > INT32_MAX) return fail(SBP_ERR_SHAPE, "bad shape");
  if (!ids || !emb || !x) return fail(SBP_ERR_NULL, "NULL pointer");
  HIPCHK(embedding_fwd(dtype, ids, emb, x, n_rows, hidden, vocab, (hipStream_t)hip_stream));
  return SBP_OK;
}
int32_t streambp_embedding_backward(int32_t dtype, int64_t n_rows, int32_t hidden, int32_t vocab, const int32_t* ids,
                                    const void* dx, float* demb, void* hip_stream) {
  if (!valid_dtype(dtype)) return fail(SBP_ERR_UNSUPPORTED, "dtype");
  if (n_rows < 0 || hidden < 1 || vocab < 1 || n_rows > INT32_MAX) return fail(SBP_ERR_SHAPE, "bad shape");
  if (!ids || !dx || !demb) return fail(SBP_ERR_NULL, "NULL pointer");
  HIPCHK(embedding_bwd(dtype, ids, dx, demb, n_rows, hidden, vocab, (hipStream_t)hip_stream));
  return SBP_OK;
}

}  // extern "C"
