// Host stand-ins for every kernel launcher declared in csrc/launch.h.  Nothing is computed: each launcher touches the
// first and the last byte of every operand extent its kernels would read or write, so that the address sanitizer
// sees exactly the memory ranges the C-ABI layer (workspace carving, chunk offsets, leading dimensions, ragged last
// chunks) hands to the kernels.  An extent that leaves its allocation is a heap-buffer-overflow report.
#include "launch.h"

#include <algorithm>
#include <atomic>
#include <cstdio>

namespace sbp {

static std::atomic<long long> g_touches{0};
long long stub_touches() { return g_touches.load(); }

static void rd(const void* p, size_t bytes) {
  if (!p || bytes == 0) return;
  volatile const unsigned char* c = (volatile const unsigned char*)p;
  (void)c[0];
  (void)c[bytes - 1];
  ++g_touches;
}
static void wr(void* p, size_t bytes) {
  if (!p || bytes == 0) return;
  volatile unsigned char* c = (volatile unsigned char*)p;
  c[0] = c[0];
  c[bytes - 1] = c[bytes - 1];
  ++g_touches;
}
static size_t es(int dt) { return dtype_size(dt); }

static void touch_gemm(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return;
  const size_t a_el = g.ta ? (size_t)(g.K - 1) * g.lda + g.M : (size_t)(g.M - 1) * g.lda + g.K;
  const size_t b_el = g.tb ? (size_t)(g.N - 1) * g.ldb + g.K : (size_t)(g.K - 1) * g.ldb + g.N;
  const size_t c_el = (size_t)(g.M - 1) * g.ldc + g.N;
  rd(g.A, a_el * es(g.in_dt)); rd(g.B, b_el * es(g.in_dt));
  if (g.A2) { rd(g.A2, a_el * es(g.in_dt)); rd(g.B2, b_el * es(g.in_dt)); }
  if (g.swiglu_gate) {
    wr(g.swiglu_gate, c_el * es(g.out_dt)); wr(g.swiglu_up, c_el * es(g.out_dt)); wr(g.swiglu_act, c_el * es(g.out_dt));
  } else {
    wr(g.C, c_el * es(g.out_dt));
  }
  if (g.row_stats) wr(g.row_stats, (size_t)g.M * cdiv(g.N, GEMM_STAT_COLS) * sizeof(float2));
  if (g.numer_targets) { wr(g.numer_target_value, (size_t)g.M * 4); if (g.numer_row_index) rd(g.numer_row_index, (size_t)g.M * 4); }
  if (g.rows_dev) rd(g.rows_dev, sizeof(int));
  // split-K partial slices: at most what gemm_scratch_bytes promises for 4 slices of a dense C
  if (g.scratch && g.ldc == g.N) wr(g.scratch, std::min(g.scratch_bytes, (size_t)4 * g.M * g.N * sizeof(float)));
}
bool gemm_row_stats_supported(const GemmArgs& g) { return g.in_dt == DT_BF16 && !g.ta && g.tb && g.out_dt == DT_F32 && g.N % 8 == 0 && g.K % 64 == 0; }
bool gemm_numerators_supported(const GemmArgs& g) {
  return g.in_dt == DT_BF16 && !g.ta && g.tb && g.out_dt == DT_BF16 && g.N % 8 == 0 && g.K % 64 == 0 && g.row_stats && g.numer_targets && g.numer_target_value;
}
size_t gemm_scratch_bytes(int max_m, int max_n, int max_splits) { return (size_t)std::min(max_splits, 8) * max_m * max_n * sizeof(float); }
hipError_t gemm(const GemmArgs& g, hipStream_t) { touch_gemm(g); return hipSuccess; }
hipError_t gemm_batch(const GemmArgs* gs, int n, hipStream_t, bool) { for (int i = 0; i < n; ++i) touch_gemm(gs[i]); return hipSuccess; }
bool gemm_uses_mfma(const GemmArgs& g) { return g.in_dt == DT_BF16; }
void gemm_set_force_generic(bool) {}
static int g_mask = FUSE_ROPE_Q | FUSE_NUMERATORS;
int fusion_mask() { return g_mask; }
void set_fusion_mask(int m) { g_mask = m; }
long long generic_bf16_launches() { return 0; }
void note_generic_bf16_launch() {}
namespace prof { Scope::Scope(int, double, bool, hipStream_t s) : st(s) {} Scope::~Scope() {} }

hipError_t rope_table(float2* tab, int n_pos, int dh, float, int, hipStream_t) { wr(tab, (size_t)n_pos * (dh / 2) * sizeof(float2)); return hipSuccess; }
hipError_t rope_apply(int dt, void* x, const float2* tab, int rows, int H, int dh, bool, hipStream_t) {
  wr(x, (size_t)rows * H * dh * es(dt)); rd(tab, (size_t)rows * (dh / 2) * sizeof(float2)); return hipSuccess;
}
size_t rmsnorm_bwd_partial_floats(int rows, int d) { return (size_t)cdiv(rows, 8) * (size_t)d; }
hipError_t rmsnorm_fwd(int dt, const void* x, const float* add, const void* g, void* out, float* sum_out, float* rstd, int rows, int d, float, hipStream_t) {
  const size_t n = (size_t)rows * d;
  rd(x, n * es(dt)); rd(add, n * 4); rd(g, (size_t)d * es(dt)); wr(out, n * es(dt)); wr(sum_out, n * 4); wr(rstd, (size_t)rows * 4);
  return hipSuccess;
}
hipError_t rmsnorm_bwd(int dt, const float* dnorm, const void* xin, bool x_is_f32, const void* g, const float* rstd, const void* res,
                       bool res_is_f32, float* out_f32, void* out_t, float* dg, float* partial, int rows, int d, hipStream_t) {
  const size_t n = (size_t)rows * d;
  rd(dnorm, n * 4); rd(xin, n * (x_is_f32 ? 4 : es(dt))); rd(g, (size_t)d * es(dt)); rd(rstd, (size_t)rows * 4);
  rd(res, n * (res_is_f32 ? 4 : es(dt))); wr(out_f32, n * 4); wr(out_t, n * es(dt)); wr(dg, (size_t)d * 4);
  wr(partial, rmsnorm_bwd_partial_floats(rows, d) * 4);
  return hipSuccess;
}
hipError_t rmsnorm_bwd_plain(int dt, const void* dy, const void* x, const void* g, const float* rstd, void* dx, float* dg, float* partial,
                             int rows, int d, hipStream_t) {
  const size_t n = (size_t)rows * d;
  rd(dy, n * es(dt)); rd(x, n * es(dt)); rd(g, (size_t)d * es(dt)); rd(rstd, (size_t)rows * 4); wr(dx, n * es(dt)); wr(dg, (size_t)d * 4);
  wr(partial, rmsnorm_bwd_partial_floats(rows, d) * 4);
  return hipSuccess;
}
hipError_t swiglu_fwd(int dt, const void* gate, const void* up, void* act, int64_t n, hipStream_t) {
  rd(gate, n * es(dt)); rd(up, n * es(dt)); wr(act, n * es(dt)); return hipSuccess;
}
hipError_t swiglu_bwd(int dt, void* gate, void* up, const void* dact, void* act, int64_t n, hipStream_t) {
  wr(gate, n * es(dt)); wr(up, n * es(dt)); rd(dact, n * es(dt)); wr(act, n * es(dt)); return hipSuccess;
}
hipError_t add_store(int dt, const float* a, const float* b, void* y, int64_t n, hipStream_t) { rd(a, n * 4); rd(b, n * 4); wr(y, n * es(dt)); return hipSuccess; }
hipError_t kv_grad_finish(int dt, const float* dK, const float* dV, const float2* tab, void* dkc, void* dvc, int rows, int H, int dh, hipStream_t) {
  const size_t n = (size_t)rows * H * dh;
  rd(dK, n * 4); rd(dV, n * 4); rd(tab, (size_t)rows * (dh / 2) * sizeof(float2)); wr(dkc, n * es(dt)); wr(dvc, n * es(dt)); return hipSuccess;
}
hipError_t fill_zero(void* p, size_t bytes, hipStream_t) { wr(p, bytes); return hipSuccess; }
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t) { wr(dst, bytes); rd(src, bytes); return hipSuccess; }
hipError_t pad_matrix(int dt, const void* src, int R, int C, bool, float, void* dst, int R2, int C2, hipStream_t) {
  rd(src, (size_t)R * C * es(dt)); wr(dst, (size_t)R2 * C2 * es(dt)); return hipSuccess;
}
hipError_t add_scaled_block(const float* src, int64_t ld, float, float* dst, int R, int C, hipStream_t) {
  if (R > 0 && C > 0) { rd(src, ((size_t)(R - 1) * ld + C) * 4); wr(dst, (size_t)R * C * 4); }
  return hipSuccess;
}
hipError_t embedding_fwd(int dt, const int32_t* ids, const void* emb, void* x, int64_t rows, int d, int vocab, hipStream_t) {
  rd(ids, rows * 4); rd(emb, (size_t)vocab * d * es(dt)); wr(x, (size_t)rows * d * es(dt)); return hipSuccess;
}
hipError_t embedding_bwd(int dt, const int32_t* ids, const void* dx, float* demb, int64_t rows, int d, int vocab, hipStream_t) {
  rd(ids, rows * 4); rd(dx, (size_t)rows * d * es(dt)); wr(demb, (size_t)vocab * d * 4); return hipSuccess;
}

static void touch_attn(const AttnArgs& a, bool bwd) {
  const size_t qn = (size_t)a.q_len * a.Hq * a.dh, kn = (size_t)(a.q_start + a.q_len) * a.Hkv * a.dh;
  if (a.rope_q && !bwd) wr((void*)a.q, qn * es(a.dt)); else rd(a.q, qn * es(a.dt));
  rd(a.k, kn * es(a.dt)); rd(a.v, kn * es(a.dt));
  if (a.rope_q) rd(a.rope_q, (size_t)a.q_len * (a.dh / 2) * sizeof(float2));
  if (!bwd) { wr(a.o, qn * es(a.dt)); wr(a.lse, (size_t)a.Hq * a.q_len * 4); return; }
  rd(a.o, qn * es(a.dt)); rd(a.lse, (size_t)a.Hq * a.q_len * 4); rd(a.d_o, qn * es(a.dt)); wr(a.dq, qn * es(a.dt));
  wr(a.dk, kn * 4); wr(a.dv, kn * 4); wr(a.delta, (size_t)2 * a.Hq * a.q_len * 4);
}
hipError_t attn_forward(const AttnArgs& a, hipStream_t) { if (a.q_len > 0) touch_attn(a, false); return hipSuccess; }
hipError_t attn_backward(const AttnArgs& a, hipStream_t) { if (a.q_len > 0) touch_attn(a, true); return hipSuccess; }
bool attn_uses_mfma(int dt, int dh, int Hq, int Hkv) { return dt == DT_BF16 && dh == 128 && Hq % Hkv == 0; }
void attn_set_force_generic(bool) {}

hipError_t head_rows(const HeadRowArgs& a, hipStream_t) {
  const size_t n = (size_t)a.rows * a.V;
  if (a.target_logit) { rd(a.target_logit, (size_t)a.rows * 4); rd(a.dz, n * es(a.dt)); } else rd(a.z, n * 4);
  wr(a.dz, n * es(a.dt)); wr(a.row_loss, (size_t)a.rows * 4);
  if (a.stats) rd(a.stats, (size_t)a.rows * a.n_stat * sizeof(float2));
  if (a.row_index) rd(a.row_index, (size_t)a.rows * 4);
  if (a.rows_dev) rd(a.rows_dev, 4);
  return hipSuccess;
}
hipError_t reduce_add(const float* v, int n, float* out, hipStream_t, const int* n_dev) { rd(v, (size_t)n * 4); wr(out, 4); rd(n_dev, 4); return hipSuccess; }
hipError_t count_active(const int32_t* targets, int B, int T, int, float* seq_weight, int64_t* n_active, hipStream_t) {
  rd(targets, (size_t)B * T * 4); wr(seq_weight, (size_t)B * 4); wr(n_active, 8); return hipSuccess;
}
hipError_t compact_active(const int32_t* targets, int64_t rows, int, int, int32_t* index, int32_t* chunk_rows, int n_chunks, hipStream_t) {
  rd(targets, rows * 4); wr(index, rows * 4); wr(chunk_rows, (size_t)n_chunks * 4); return hipSuccess;
}
hipError_t gather_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t) {
  (void)src; rd(index, (size_t)max_rows * 4); rd(rows_dev, 4); wr(dst, (size_t)max_rows * d * es(dt)); return hipSuccess;
}
hipError_t scatter_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t) {
  (void)dst; rd(src, (size_t)max_rows * d * es(dt)); rd(index, (size_t)max_rows * 4); rd(rows_dev, 4); return hipSuccess;
}
hipError_t dpo_finish(int dt, const float* ell, float, void* dh, int64_t n_dh, void* dw, int dw_dt, int64_t n_dw, float* loss, hipStream_t) {
  rd(ell, 4); wr(dh, n_dh * es(dt)); wr(dw, n_dw * es(dw_dt)); wr(loss, 4); return hipSuccess;
}

}  // namespace sbp
