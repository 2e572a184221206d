// Kernel selection: bf16 MFMA kernels when the problem fits their tiling, the
// shape-agnostic kernels otherwise.
#include "launch.h"

namespace sbp {

hipError_t gemm_generic(const GemmArgs& g, hipStream_t st);
hipError_t gemm_mfma(const GemmArgs& g, hipStream_t st);
bool gemm_mfma_eligible(const GemmArgs& g);
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

hipError_t gemm(const GemmArgs& g, hipStream_t st) {
  return gemm_uses_mfma(g) ? gemm_mfma(g, st) : gemm_generic(g, st);
}
hipError_t attn_forward(const AttnArgs& a, hipStream_t st) {
  return attn_uses_mfma(a.dt, a.dh, a.Hq, a.Hkv) ? attn_forward_mfma(a, st) : attn_forward_generic(a, st);
}
hipError_t attn_backward(const AttnArgs& a, hipStream_t st) {
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
