// LM-head row kernels: per-row log-sum-exp over the chunk's logits, the
// per-token objective coefficient (SFT / GRPO / DPO, paper Sec. 3.2.1) and
// dz = coef * (onehot(target) - softmax(z)).  One workgroup per row, two passes
// over the row (statistics, then dz); the label gather z[target] and the ignore
// mask are integer-indexed and exact.
#include "launch.h"
#include <algorithm>

namespace sbp {

constexpr int HR_THREADS = 512;

template <typename T>
__global__ __launch_bounds__(HR_THREADS) void head_rows_k(HeadRowArgs a) {
  __shared__ float red[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float* z = a.z + (int64_t)row * a.V;
  T* dz = (T*)a.dz + (int64_t)row * a.V;
  const int tgt = a.targets[row];
  if (tgt < 0) {   // ignored row: exact zeros, no loss term
    const int64_t row_bytes = (int64_t)a.V * sizeof(T);
    if ((row_bytes & 15) == 0) {
      uint4* p16 = (uint4*)dz;
      for (int v = tid; v < row_bytes / 16; v += HR_THREADS) p16[v] = make_uint4(0, 0, 0, 0);
    } else {
      for (int v = tid; v < a.V; v += HR_THREADS) stf(dz + v, 0.f);
    }
    if (tid == 0) a.row_loss[row] = 0.f;
    return;
  }
  // One pass for the statistics: every thread keeps a running (max, sum of exp) pair over its elements
  // and rescales the sum when its max moves; the pairs are then merged across the workgroup.
  float mx = -INFINITY, se = 0.f;
  const bool vec = (a.V & 3) == 0;
  if (vec) {
    const float4* z4 = (const float4*)z;
    for (int v = tid; v < a.V / 4; v += HR_THREADS) {
      const float4 t = z4[v];
      const float m4 = fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w));
      if (m4 > mx) { se *= __expf(mx - m4); mx = m4; }
      se += __expf(t.x - mx) + __expf(t.y - mx) + __expf(t.z - mx) + __expf(t.w - mx);
    }
  } else {
    for (int v = tid; v < a.V; v += HR_THREADS) {
      const float t = z[v];
      if (t > mx) { se *= __expf(mx - t); mx = t; }
      se += __expf(t - mx);
    }
  }
  {
    const float gmx = block_max(mx, red);
    se = block_sum(mx == -INFINITY ? 0.f : se * __expf(mx - gmx), red);
    mx = gmx;
  }
  const float lse = mx + logf(se);
  const float logp = z[tgt] - lse;

  float coef, loss_term;
  if (a.objective == 0) {                     // SFT: L = -scale * sum logp
    coef = -a.loss_scale;
    loss_term = -a.loss_scale * logp;
  } else if (a.objective == 1) {              // GRPO
    const int64_t seq = (a.row0 + row) / a.T;
    const float wgt = a.seq_weight[seq], adv = a.advantages[seq];
    const float r = a.old_logp ? expf(logp - a.old_logp[row]) : 1.0f;
    const float unclipped = r * adv;
    const float clipped = fminf(fmaxf(r, 1.0f - a.clip_eps), 1.0f + a.clip_eps) * adv;
    const float surr = fminf(unclipped, clipped);
    const float dsurr = (unclipped <= clipped) ? unclipped : 0.0f;
    const float ref = a.ref_logp[row];
    float kl, dkl;
    if (a.kl_mode == 0) { kl = logp - ref; dkl = 1.0f; }
    else { const float e = expf(ref - logp); kl = e - (ref - logp) - 1.0f; dkl = 1.0f - e; }
    loss_term = -wgt * (surr - a.kl_beta * kl);
    coef = -wgt * (dsurr - a.kl_beta * dkl);
  } else {                                    // DPO, before the final in-place correction
    const int64_t seq = (a.row0 + row) / a.T;
    const float sign = (seq == 0) ? 1.0f : -1.0f;
    coef = a.kl_beta * sign;
    loss_term = sign * (logp - a.ref_logp[row]);   // summand of ell
  }
  if (tid == 0) a.row_loss[row] = loss_term;
  if (vec && sizeof(T) == 2) {
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    const float4* z4 = (const float4*)z;
    bf16x4* dz4 = (bf16x4*)dz;
    for (int v = tid; v < a.V / 4; v += HR_THREADS) {
      const float4 t = z4[v];
      const int v0 = v * 4;
      bf16x4 o;
      o[0] = (bf16_t)(coef * ((v0 + 0 == tgt ? 1.0f : 0.0f) - __expf(t.x - lse)));
      o[1] = (bf16_t)(coef * ((v0 + 1 == tgt ? 1.0f : 0.0f) - __expf(t.y - lse)));
      o[2] = (bf16_t)(coef * ((v0 + 2 == tgt ? 1.0f : 0.0f) - __expf(t.z - lse)));
      o[3] = (bf16_t)(coef * ((v0 + 3 == tgt ? 1.0f : 0.0f) - __expf(t.w - lse)));
      dz4[v] = o;
    }
  } else {
    for (int v = tid; v < a.V; v += HR_THREADS) {
      const float sm = __expf(z[v] - lse);
      stf(dz + v, coef * ((v == tgt ? 1.0f : 0.0f) - sm));
    }
  }
}

hipError_t head_rows(const HeadRowArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  if (a.dt == DT_BF16) head_rows_k<bf16_t><<<a.rows, HR_THREADS, 0, st>>>(a);
  else head_rows_k<float><<<a.rows, HR_THREADS, 0, st>>>(a);
  return hipGetLastError();
}

// out += sum(v[0..n)) with a fixed summation tree (one workgroup).
__global__ __launch_bounds__(256) void reduce_add_k(const float* __restrict__ v, int n, float* __restrict__ out) {
  __shared__ float red[16];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) *out += s;
}
hipError_t reduce_add(const float* v, int n, float* out, hipStream_t st) {
  if (n == 0) return hipSuccess;
  reduce_add_k<<<1, 256, 0, st>>>(v, n, out);
  return hipGetLastError();
}

__global__ __launch_bounds__(1024) void count_active_k(const int32_t* __restrict__ targets, int B, int T,
                                                       float* __restrict__ seq_weight, int64_t* __restrict__ n_active) {
  __shared__ int red[16];
  int64_t total = 0;
  for (int j = 0; j < B; ++j) {
    int cnt = 0;
    for (int t = threadIdx.x; t < T; t += 1024) cnt += targets[(int64_t)j * T + t] >= 0 ? 1 : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, WAVE);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = cnt;
    __syncthreads();
    int tot = 0;
    for (int i = 0; i < 16; ++i) tot += red[i];
    if (threadIdx.x == 0 && seq_weight) seq_weight[j] = tot > 0 ? 1.0f / ((float)B * (float)tot) : 0.0f;
    total += tot;
  }
  if (threadIdx.x == 0) *n_active = total;
}
hipError_t count_active(const int32_t* targets, int B, int T, float* seq_weight, int64_t* n_active, hipStream_t st) {
  count_active_k<<<1, 1024, 0, st>>>(targets, B, T, seq_weight, n_active);
  return hipGetLastError();
}

template <typename T>
__global__ void dpo_finish_k(const float* __restrict__ ell, float beta, T* __restrict__ dh, int64_t n_dh,
                             float* __restrict__ dw, int64_t n_dw, float* __restrict__ loss) {
  const float x = beta * (*ell);
  const float sig = 1.0f / (1.0f + expf(-x));
  const float factor = sig - 1.0f;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  if (i == 0) *loss += (x > -30.f) ? log1pf(expf(-x)) : -x;
  for (; i < n_dh + n_dw; i += stride) {
    if (i < n_dh) stf(dh + i, ldf(dh + i) * factor);
    else dw[i - n_dh] *= factor;
  }
}
hipError_t dpo_finish(int dt, const float* ell, float beta, void* dh, int64_t n_dh, float* dw, int64_t n_dw,
                      float* loss, hipStream_t st) {
  unsigned grid = (unsigned)std::min<int64_t>(cdiv(n_dh + n_dw, 256), 256 * 16);
  if (dt == DT_BF16) dpo_finish_k<bf16_t><<<grid, 256, 0, st>>>(ell, beta, (bf16_t*)dh, n_dh, dw, n_dw, loss);
  else dpo_finish_k<float><<<grid, 256, 0, st>>>(ell, beta, (float*)dh, n_dh, dw, n_dw, loss);
  return hipGetLastError();
}

}  // namespace sbp
