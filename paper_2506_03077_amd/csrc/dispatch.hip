// Kernel selection: bf16 MFMA kernels when the problem fits their tiling, the
// shape-agnostic kernels otherwise.
#include "../../include/streambp_debug.h"
#include "launch.h"

#include <algorithm>
#include <atomic>
#include <vector>

namespace sbp {

hipError_t gemm_generic(const GemmArgs& g, hipStream_t st);
hipError_t gemm_mfma(const GemmArgs& g, hipStream_t st);
bool gemm_mfma_eligible(const GemmArgs& g);
bool gemm_mfma_pair_ok(const GemmArgs& g);
bool gemm_mfma_stats_ok(const GemmArgs& g);
bool gemm_mfma_swiglu_ok(const GemmArgs& g);
bool gemm_mfma_numer_ok(const GemmArgs& g);
bool gemm_mfma_group_eligible(const GemmArgs* gs, int n, bool small_ok);
hipError_t gemm_mfma_group(const GemmArgs* gs, int n, hipStream_t st);
bool gemm_mfma_seg_eligible(const GemmArgs* gs, int n);
hipError_t gemm_mfma_seg(const GemmArgs* gs, int n, hipStream_t st);
hipError_t attn_forward_generic(const AttnArgs& a, hipStream_t st);
hipError_t attn_backward_generic(const AttnArgs& a, hipStream_t st);
hipError_t attn_forward_mfma(const AttnArgs& a, hipStream_t st);
hipError_t attn_backward_mfma(const AttnArgs& a, hipStream_t st);
bool attn_mfma_eligible(int dt, int dh, int Hq, int Hkv);
bool attn_mfma_aligned(const AttnArgs& a, bool backward);

static std::atomic<bool> g_force_generic_gemm{false};
static std::atomic<bool> g_force_generic_attn{false};
// bf16 problems that ran on the shape-agnostic fp32-ALU kernels (shape or alignment outside what the MFMA kernels take)
static std::atomic<long long> g_generic_bf16_launches{0};
long long generic_bf16_launches() { return g_generic_bf16_launches.load(); }
void note_generic_bf16_launch() { ++g_generic_bf16_launches; }
static std::atomic<int> g_fusion_mask{FUSE_ROPE_Q | FUSE_NUMERATORS};
int fusion_mask() { return g_fusion_mask.load(); }
void set_fusion_mask(int mask) { g_fusion_mask.store(mask); }

void gemm_set_force_generic(bool on) { g_force_generic_gemm = on; }
void attn_set_force_generic(bool on) { g_force_generic_attn = on; }

bool gemm_uses_mfma(const GemmArgs& g) { return !g_force_generic_gemm && gemm_mfma_eligible(g); }
bool gemm_row_stats_supported(const GemmArgs& g) { return gemm_uses_mfma(g) && gemm_mfma_stats_ok(g); }
bool gemm_numerators_supported(const GemmArgs& g) { return gemm_uses_mfma(g) && gemm_mfma_numer_ok(g); }
bool attn_uses_mfma(int dt, int dh, int Hq, int Hkv) { return !g_force_generic_attn && attn_mfma_eligible(dt, dh, Hq, Hkv); }

// ---- optional per-launch timing (off by default; events are created when profiling is switched on,
// never inside an entry point) -------------------------------------------------------------------
namespace prof {
struct Rec { int kind; double work; bool bounded; hipEvent_t e0, e1; };
static std::atomic<bool> g_on{false};
static std::vector<hipEvent_t> g_pool;
static std::vector<Rec> g_recs;
static size_t g_next = 0;

Scope::Scope(int kind_, double work_, bool bounded_, hipStream_t s) : st(s), kind(kind_), work(work_), bounded(bounded_) {
  if (!g_on || g_next + 2 > g_pool.size()) return;
  e0 = g_pool[g_next++]; e1 = g_pool[g_next++];
  active = hipEventRecord(e0, st) == hipSuccess;
}
Scope::~Scope() {
  if (active && hipEventRecord(e1, st) == hipSuccess) g_recs.push_back(Rec{kind, work, bounded, e0, e1});
}
}  // namespace prof

static double causal_pairs(const AttnArgs& a) {   // visible (query, key) pairs of the chunk, all query heads
  const double c = a.q_len, s = a.q_start;
  if (a.window == 0 && a.kv_first == 0) return (double)a.Hq * (c * s + c * (c + 1.0) / 2.0);
  double pairs = 0.0;
  for (int t = 0; t < a.q_len; ++t) {
    const int p = a.q_start + t, lo = std::max(a.kv_first, a.window > 0 ? p - a.window + 1 : 0);
    pairs += std::max(0, p - lo + 1);
  }
  return (double)a.Hq * pairs;
}

hipError_t gemm(const GemmArgs& g, hipStream_t st) {
  if (g.numer_targets) {
    if (!gemm_numerators_supported(g)) return hipErrorInvalidValue;               // only the MFMA store form has them
  } else if (g.row_stats && !gemm_row_stats_supported(g)) return hipErrorInvalidValue;   // only the MFMA store form emits them
  if (g.swiglu_gate && !(gemm_uses_mfma(g) && gemm_mfma_swiglu_ok(g))) {   // no fused epilogue for this problem: product, then the elementwise kernel
    GemmArgs plain = g;
    plain.swiglu_gate = plain.swiglu_up = plain.swiglu_act = nullptr;
    hipError_t e = gemm(plain, st);
    return e != hipSuccess ? e : swiglu_bwd(g.out_dt, g.swiglu_gate, g.swiglu_up, g.C, g.swiglu_act, (int64_t)g.M * g.N, st);
  }
  if (g.A2 && !(gemm_uses_mfma(g) && gemm_mfma_pair_ok(g))) {   // two operand pairs, no single launch for them: one after the other
    GemmArgs first = g, second = g;
    first.A2 = first.B2 = nullptr;
    second.A = g.A2; second.B = g.B2; second.A2 = second.B2 = nullptr; second.acc = true;
    hipError_t e = gemm(first, st);
    return e != hipSuccess ? e : gemm(second, st);
  }
  if (gemm_uses_mfma(g)) return gemm_mfma(g, st);      // times itself (it knows which kernel variant it launches)
  if (g.in_dt == DT_BF16) ++g_generic_bf16_launches;
  prof::Scope sc(prof::GEMM_GENERIC, 2.0 * g.M * g.N * g.K, g.rows_dev != nullptr, st);
  return gemm_generic(g, st);
}
hipError_t gemm_batch(const GemmArgs* gs, int n, hipStream_t st, bool group_small) {
  if (!g_force_generic_gemm && gemm_mfma_seg_eligible(gs, n)) return gemm_mfma_seg(gs, n, st);   // same C: one pass over it
  if (!g_force_generic_gemm && gemm_mfma_group_eligible(gs, n, group_small)) {
    return gemm_mfma_group(gs, n, st);
  }
  for (int i = 0; i < n; ++i) {
    hipError_t e = gemm(gs[i], st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
hipError_t attn_forward(const AttnArgs& a, hipStream_t st) {
  prof::Scope sc(prof::ATTN_FWD, 4.0 * a.dh * causal_pairs(a), false, st);
  if (attn_uses_mfma(a.dt, a.dh, a.Hq, a.Hkv) && attn_mfma_aligned(a, false)) return attn_forward_mfma(a, st);
  if (a.dt == DT_BF16) ++g_generic_bf16_launches;
  AttnArgs b = a;
  b.rope_q = nullptr;            // the shape-agnostic kernels take rotated queries: rotate in place first
  if (a.rope_q) {
    hipError_t e = rope_apply(a.dt, (void*)a.q, a.rope_q, a.q_len, a.Hq, a.dh, false, st);
    if (e != hipSuccess) return e;
  }
  return attn_forward_generic(b, st);
}
hipError_t attn_backward(const AttnArgs& a, hipStream_t st) {
  prof::Scope sc(prof::ATTN_BWD, 10.0 * a.dh * causal_pairs(a), false, st);
  if (attn_uses_mfma(a.dt, a.dh, a.Hq, a.Hkv) && attn_mfma_aligned(a, true)) return attn_backward_mfma(a, st);
  if (a.dt == DT_BF16) ++g_generic_bf16_launches;
  AttnArgs b = a;
  b.rope_q = nullptr;
  hipError_t e = attn_backward_generic(b, st);
  if (e != hipSuccess || !a.rope_q) return e;
  return rope_apply(a.dt, a.dq, a.rope_q, a.q_len, a.Hq, a.dh, true, st);   // dq back through the rotation
}

}  // namespace sbp

extern "C" void streambp_debug_set_fusions(int mask) { sbp::set_fusion_mask(mask); }
extern "C" int streambp_debug_get_fusions(void) { return sbp::fusion_mask(); }

extern "C" void streambp_debug_force_generic(int gemm_on, int attn_on) {
  sbp::gemm_set_force_generic(gemm_on != 0);
  sbp::attn_set_force_generic(attn_on != 0);
}

// Direct access to the GEMM dispatcher for unit tests and kernel timing (declared in include/streambp_debug.h).
extern "C" int streambp_debug_gemm(int M, int N, int K, int ta, int tb, int in_dt, int out_dt, int acc, const void* A,
                                   const void* B, void* C, long long lda, long long ldb, long long ldc, void* scratch,
                                   size_t scratch_bytes, void* stream, const void* A2, const void* B2, void* row_stats) {
  sbp::GemmArgs g{A, B, C, M, N, K, lda, ldb, ldc, ta != 0, tb != 0, in_dt, out_dt, acc != 0};
  g.scratch = (float*)scratch;
  g.scratch_bytes = scratch_bytes;
  g.A2 = A2;      // optional second operand pair (both or neither)
  g.B2 = B2;
  g.row_stats = (float2*)row_stats;   // optional [M, N/256] (max, sum of exp) pairs
  hipError_t e = sbp::gemm(g, (hipStream_t)stream);
  return e == hipSuccess ? (sbp::gemm_uses_mfma(g) ? 1 : 0) : -5;
}

// Weight-gradient form over several reduction segments through gemm_batch: C[M,N] += sum_s A_s^T B_s with
// A_s [K_s, M], B_s [K_s, N] (row counts optionally limited by device integers), C fp32 or bf16 (out_dt).  Returns 1 if
// the segmented MFMA kernel took it, 0 if it ran as separate launches.
extern "C" int streambp_debug_gemm_dw_segments(int n, int M, int N, const int* K, const void* const* A, const void* const* B,
                                               const int* const* rows_dev, void* C, long long lda, long long ldb,
                                               long long ldc, int in_dt, int out_dt, void* stream) {
  if (n < 1 || n > 8) return -2;
  sbp::GemmArgs gs[8];
  for (int i = 0; i < n; ++i) {
    gs[i] = sbp::GemmArgs{A[i], B[i], C, M, N, K[i], lda, ldb, ldc, true, false, in_dt, out_dt, true};
    gs[i].rows_dev = rows_dev ? rows_dev[i] : nullptr;
  }
  const bool seg = !sbp::g_force_generic_gemm.load() && sbp::gemm_mfma_seg_eligible(gs, n);
  hipError_t e = sbp::gemm_batch(gs, n, (hipStream_t)stream);
  return e == hipSuccess ? (seg ? 1 : 0) : -5;
}

extern "C" int streambp_debug_gemm_numerators(int M, int N, int K, const void* A, const void* B, void* E, long long lda, long long ldb,
                                              long long lde, void* stats, const int32_t* targets, const int32_t* row_index,
                                              float* target_value, void* stream) {
  sbp::GemmArgs g{A, B, E, M, N, K, lda, ldb, lde, false, true, sbp::DT_BF16, sbp::DT_BF16, false};
  g.row_stats = (float2*)stats;
  g.numer_targets = targets; g.numer_row_index = row_index; g.numer_target_value = target_value;
  if (!sbp::gemm_numerators_supported(g)) return 0;
  return sbp::gemm(g, (hipStream_t)stream) == hipSuccess ? 1 : -5;
}

extern "C" int streambp_debug_mfma_rate(const void* operands, float* sink, int workgroups, int iters, int lds_reads, void* stream) {
  if (!operands || !sink) return -1;
  if (lds_reads != 0 && lds_reads != 6 && lds_reads != 8) return -2;
  return sbp::mfma_rate_probe(operands, sink, workgroups, iters, lds_reads, (hipStream_t)stream) == hipSuccess ? 0 : -5;
}

// Per-launch timing with HIP events recorded on the launch stream around each GEMM kernel / attention launch
// sequence.  begin: creates 2*max_records events and switches recording on.  end: synchronises the events and
// returns per kind (see prof:: in launch.h; N_KIND entries) the launch count, the summed duration in ms, the
// summed work of launches with host-known sizes and the summed (upper-bound) work of launches whose row count
// was read on the device; then destroys the events.
extern "C" int streambp_debug_profile_kinds(void) { return sbp::prof::N_KIND; }
extern "C" int streambp_debug_profile_begin(int max_records) {
  using namespace sbp::prof;
  if (g_on) return -1;
  g_pool.resize((size_t)max_records * 2);
  for (auto& e : g_pool)
    if (hipEventCreate(&e) != hipSuccess) return -5;
  g_recs.clear();
  g_recs.reserve(max_records);
  g_next = 0;
  g_on = true;
  return 0;
}
extern "C" int streambp_debug_profile_end(long long* count, double* ms, double* work, double* work_bounded) {
  using namespace sbp::prof;
  if (!g_on) return -1;
  g_on = false;
  for (int k = 0; k < N_KIND; ++k) { count[k] = 0; ms[k] = 0.0; work[k] = 0.0; work_bounded[k] = 0.0; }
  int rc = 0;
  for (const Rec& r : g_recs) {
    float t = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) { rc = -5; continue; }
    count[r.kind] += 1; ms[r.kind] += t;
    (r.bounded ? work_bounded : work)[r.kind] += r.work;
  }
  for (auto& e : g_pool) (void)hipEventDestroy(e);
  g_pool.clear();
  g_recs.clear();
  return rc;
}
