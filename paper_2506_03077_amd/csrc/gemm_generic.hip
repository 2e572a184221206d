// Shape-agnostic GEMM: any M, N, K, any of the three operand layouts, fp32 or
// bf16 storage, fp32 FMA accumulation.  This is the correctness path for the
// fp32 configuration and for shapes the MFMA kernel does not take (widths that
// are not multiples of its tile); it is not a performance path.
#include "launch.h"
#include "device.h"

namespace sbp {

constexpr int GT = 64;   // output tile GT x GT per workgroup
constexpr int GK = 16;   // reduction slice

template <typename TI, typename TO, bool ACC>
__global__ __launch_bounds__(256) void gemm_generic_k(const TI* __restrict__ A, const TI* __restrict__ B,
                                                      TO* __restrict__ C, int M, int N, int K,
                                                      int64_t lda, int64_t ldb, int64_t ldc, int ta, int tb,
                                                      const int* __restrict__ rows_dev) {
  if (rows_dev) {   // run-time row count (M for NT / NN, the reduction K for the dW form)
    const int rows = max(0, *rows_dev);
    if (ta) K = min(K, rows); else M = min(M, rows);
  }
  __shared__ float As[GK][GT + 1];
  __shared__ float Bs[GK][GT + 1];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += GK) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int idx = tid + 256 * r;
      int mm, kk;
      if (ta) { mm = idx % GT; kk = idx / GT; } else { kk = idx % GK; mm = idx / GK; }
      const int m = m0 + mm, k = k0 + kk;
      float v = 0.f;
      if (m < M && k < K) v = ldf(A + (ta ? (int64_t)k * lda + m : (int64_t)m * lda + k));
      As[kk][mm] = v;
      int nn, kb;
      if (tb) { kb = idx % GK; nn = idx / GK; } else { nn = idx % GT; kb = idx / GT; }
      const int n = n0 + nn, k2 = k0 + kb;
      float w = 0.f;
      if (n < N && k2 < K) w = ldf(B + (tb ? (int64_t)n * ldb + k2 : (int64_t)k2 * ldb + n));
      Bs[kb][nn] = w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      TO* p = C + (int64_t)m * ldc + n;
      if (ACC) stf(p, ldf(p) + acc[i][j]); else stf(p, acc[i][j]);
    }
  }
}

hipError_t gemm_generic(const GemmArgs& g, hipStream_t st) {
  if (g.M == 0 || g.N == 0) return hipSuccess;
  dim3 grid((unsigned)cdiv(g.N, GT), (unsigned)cdiv(g.M, GT));
#define GG(TI, TO, ACC)                                                                                 \
  gemm_generic_k<TI, TO, ACC><<<grid, 256, 0, st>>>((const TI*)g.A, (const TI*)g.B, (TO*)g.C, g.M, g.N, g.K, \
                                                    g.lda, g.ldb, g.ldc, g.ta ? 1 : 0, g.tb ? 1 : 0, g.rows_dev)
  if (g.in_dt == DT_BF16) {
    if (g.out_dt == DT_BF16 && g.acc) GG(bf16_t, bf16_t, true);
    else if (g.out_dt == DT_BF16) GG(bf16_t, bf16_t, false);
    else if (g.acc) GG(bf16_t, float, true);
    else GG(bf16_t, float, false);
  } else {
    if (g.acc) GG(float, float, true);
    else GG(float, float, false);
  }
#undef GG
  return hipGetLastError();
}

}  // namespace sbp
