// Kernel selection: bf16 MFMA kernels when the problem fits their tiling, the
// shape-agnostic kernels otherwise.
#include "launch.h"

#include <vector>

namespace sbp {

hipError_t gemm_generic(const GemmArgs& g, hipStream_t st);
hipError_t gemm_mfma(const GemmArgs& g, hipStream_t st);
bool gemm_mfma_eligible(const GemmArgs& g);
bool gemm_mfma_group_eligible(const GemmArgs* gs, int n);
hipError_t gemm_mfma_group(const GemmArgs* gs, int n, hipStream_t st);
hipError_t attn_forward_generic(const AttnArgs& a, hipStream_t st);
hipError_t attn_backward_generic(const AttnArgs& a, hipStream_t st);
hipError_t attn_forward_mfma(const AttnArgs& a, hipStream_t st);
hipError_t attn_backward_mfma(const AttnArgs& a, hipStream_t st);
bool attn_mfma_eligible(int dt, int dh, int Hq, int Hkv);

static bool g_force_generic_gemm = false;
static bool g_force_generic_attn = false;

void gemm_set_force_generic(bool on) { g_force_generic_gemm = on; }
void attn_set_force_generic(bool on) { g_force_generic_attn = on; }

bool gemm_uses_mfma(const GemmArgs& g) { return !g_force_generic_gemm && gemm_mfma_eligible(g); }
bool attn_uses_mfma(int dt, int dh, int Hq, int Hkv) { return !g_force_generic_attn && attn_mfma_eligible(dt, dh, Hq, Hkv); }

// ---- optional per-launch timing (off by default; events are created when profiling is switched on,
// never inside an entry point) -------------------------------------------------------------------
namespace prof {
enum Kind { GEMM_NT = 0, GEMM_NN, GEMM_TN, GEMM_GENERIC, ATTN_FWD, ATTN_BWD, N_KIND };
struct Rec { int kind; double work; hipEvent_t e0, e1; };
static bool g_on = false;
static std::vector<hipEvent_t> g_pool;
static std::vector<Rec> g_recs;
static size_t g_next = 0;

struct Scope {
  hipStream_t st; bool active = false; Rec rec{};
  Scope(int kind, double work, hipStream_t s) : st(s) {
    if (!g_on || g_next + 2 > g_pool.size()) return;
    rec.kind = kind; rec.work = work; rec.e0 = g_pool[g_next++]; rec.e1 = g_pool[g_next++];
    active = hipEventRecord(rec.e0, st) == hipSuccess;
  }
  ~Scope() {
    if (active && hipEventRecord(rec.e1, st) == hipSuccess) g_recs.push_back(rec);
  }
};
}  // namespace prof

static double causal_pairs(const AttnArgs& a) {   // visible (query, key) pairs of the chunk, all query heads
  const double c = a.q_len, s = a.q_start;
  return (double)a.Hq * (c * s + c * (c + 1.0) / 2.0);
}

hipError_t gemm(const GemmArgs& g, hipStream_t st) {
  const bool mfma = gemm_uses_mfma(g);
  const int kind = !mfma ? prof::GEMM_GENERIC : (g.ta ? prof::GEMM_TN : (g.tb ? prof::GEMM_NT : prof::GEMM_NN));
  prof::Scope sc(kind, 2.0 * g.M * g.N * g.K, st);
  return mfma ? gemm_mfma(g, st) : gemm_generic(g, st);
}
hipError_t gemm_batch(const GemmArgs* gs, int n, hipStream_t st) {
  if (!g_force_generic_gemm && gemm_mfma_group_eligible(gs, n)) {
    double work = 0.0;
    for (int i = 0; i < n; ++i) work += 2.0 * gs[i].M * gs[i].N * gs[i].K;
    const int kind = gs[0].ta ? prof::GEMM_TN : (gs[0].tb ? prof::GEMM_NT : prof::GEMM_NN);
    prof::Scope sc(kind, work, st);
    return gemm_mfma_group(gs, n, st);
  }
  for (int i = 0; i < n; ++i) {
    hipError_t e = gemm(gs[i], st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
hipError_t attn_forward(const AttnArgs& a, hipStream_t st) {
  prof::Scope sc(prof::ATTN_FWD, 4.0 * a.dh * causal_pairs(a), st);
  return attn_uses_mfma(a.dt, a.dh, a.Hq, a.Hkv) ? attn_forward_mfma(a, st) : attn_forward_generic(a, st);
}
hipError_t attn_backward(const AttnArgs& a, hipStream_t st) {
  prof::Scope sc(prof::ATTN_BWD, 10.0 * a.dh * causal_pairs(a), st);
  return attn_uses_mfma(a.dt, a.dh, a.Hq, a.Hkv) ? attn_backward_mfma(a, st) : attn_backward_generic(a, st);
}

}  // namespace sbp

extern "C" void streambp_debug_force_generic(int gemm_on, int attn_on) {
  sbp::gemm_set_force_generic(gemm_on != 0);
  sbp::attn_set_force_generic(attn_on != 0);
}

// Direct access to the GEMM dispatcher for unit tests and kernel timing (not part of the public header).
extern "C" int streambp_debug_gemm(int M, int N, int K, int ta, int tb, int in_dt, int out_dt, int acc, const void* A,
                                   const void* B, void* C, long long lda, long long ldb, long long ldc, void* scratch,
                                   size_t scratch_bytes, void* stream) {
  sbp::GemmArgs g{A, B, C, M, N, K, lda, ldb, ldc, ta != 0, tb != 0, in_dt, out_dt, acc != 0};
  g.scratch = (float*)scratch;
  g.scratch_bytes = scratch_bytes;
  hipError_t e = sbp::gemm(g, (hipStream_t)stream);
  return e == hipSuccess ? (sbp::gemm_uses_mfma(g) ? 1 : 0) : -5;
}

// Per-launch timing of the GEMM / attention dispatchers with HIP events on the launch stream.
// begin: creates 2*max_records events and switches recording on.  end: synchronises the events, returns per
// kind (NT, NN, TN, generic GEMM, attention forward, attention backward) the launch count, the summed
// duration in ms and the summed algorithmic flops, then destroys the events.
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
extern "C" int streambp_debug_profile_end(long long* count, double* ms, double* work) {
  using namespace sbp::prof;
  if (!g_on) return -1;
  g_on = false;
  for (int k = 0; k < N_KIND; ++k) { count[k] = 0; ms[k] = 0.0; work[k] = 0.0; }
  int rc = 0;
  for (const Rec& r : g_recs) {
    float t = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) { rc = -5; continue; }
    count[r.kind] += 1; ms[r.kind] += t; work[r.kind] += r.work;
  }
  for (auto& e : g_pool) hipEventDestroy(e);
  g_pool.clear();
  g_recs.clear();
  return rc;
}
