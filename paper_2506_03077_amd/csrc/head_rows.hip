// LM-head row kernels: per-row log-sum-exp over the chunk's logits, the
// per-token objective coefficient (SFT / GRPO / DPO, paper Sec. 3.2.1) and
// dz = coef * (onehot(target) - softmax(z)).  One workgroup per row, two passes
// over the row (statistics, then dz) - or one, when the logits GEMM has already
// reduced every 256-column block of the row to a (max, sum of exp) pair; the label
// gather z[target] and the ignore mask are integer-indexed and exact.
#include "launch.h"
#include "device.h"
#include <algorithm>

namespace sbp {

constexpr int HR_THREADS = 512;

// Per-token coefficient of (onehot - softmax) in dz and the row's loss term, from the log-probability of the target
// (Sec. 3.2.1: SFT, GRPO; DPO before its final correction).
__device__ __forceinline__ void objective_terms(const HeadRowArgs& a, float logp, int64_t orig, int64_t aux, float& coef, float& loss_term) {
  if (a.objective == 0) {                     // SFT: L = -scale * sum logp
    coef = -a.loss_scale;
    loss_term = -a.loss_scale * logp;
  } else if (a.objective == 1) {              // GRPO
    const int64_t seq = orig / a.T;
    const float wgt = a.seq_weight[seq], adv = a.advantages[seq];
    const float r = a.old_logp ? expf(logp - a.old_logp[aux]) : 1.0f;
    const float unclipped = r * adv;
    const float clipped = fminf(fmaxf(r, 1.0f - a.clip_eps), 1.0f + a.clip_eps) * adv;
    const float surr = fminf(unclipped, clipped);
    const float dsurr = (unclipped <= clipped) ? unclipped : 0.0f;
    const float ref = a.ref_logp[aux];
    float kl, dkl;
    if (a.kl_mode == 0) { kl = logp - ref; dkl = 1.0f; }
    else { const float e = expf(ref - logp); kl = e - (ref - logp) - 1.0f; dkl = 1.0f - e; }
    loss_term = -wgt * (surr - a.kl_beta * kl);
    coef = -wgt * (dsurr - a.kl_beta * dkl);
  } else {                                    // DPO, before the final in-place correction
    const int64_t seq = orig / a.T;
    const float sign = (seq == 0) ? 1.0f : -1.0f;
    coef = a.kl_beta * sign;
    loss_term = sign * (logp - a.ref_logp[aux]);   // summand of ell
  }
}

template <typename T>
__global__ __launch_bounds__(HR_THREADS) void head_rows_k(HeadRowArgs a) {
  __shared__ float red[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  if (a.rows_dev && row >= *a.rows_dev) return;                 // beyond the valid rows of a compacted chunk
  const float* z = a.z + (int64_t)row * a.V;
  T* dz = (T*)a.dz + (int64_t)row * a.V;
  const int64_t orig = a.row_index ? (int64_t)a.row_index[row] : a.row0 + row;   // row in the caller's [B*T] order
  const int64_t aux = a.row_index ? orig : (int64_t)row;        // index into targets / old_logp / ref_logp as passed
  const int tgt = a.targets[aux];
  if (tgt < 0 || tgt >= a.V) {   // ignored row (or an id outside the vocabulary, which is never used as an index): exact zeros, no loss term
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
  if (a.stats) {   // the logits GEMM left (max, sum of exp) per column block: merge those instead of reading the row
    const float2* ps = a.stats + (int64_t)row * a.n_stat;
    for (int t = tid; t < a.n_stat; t += HR_THREADS) {
      const float2 p = ps[t];
      const float m2 = fmaxf(mx, p.x);
      se = se * __expf(mx - m2) + p.y * __expf(p.x - m2);
      mx = m2;
    }
  } else if (vec) {
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
  objective_terms(a, logp, orig, aux, coef, loss_term);
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

// Numerator form: the logits GEMM left exp(z - block max) in dz (bf16), the (max, sum) pair of every 256-column block in
// stats and z[target] in target_logit.  One pass, in place: dz = coef * (onehot - numerator * exp(block max - lse)) -
// one multiply per element, the factor changes once per block.
typedef bf16_t bf16x8h __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(HR_THREADS) void head_rows_numer_k(HeadRowArgs a) {
  __shared__ float red[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  if (a.rows_dev && row >= *a.rows_dev) return;
  bf16x8h* dz8 = (bf16x8h*)((bf16_t*)a.dz + (int64_t)row * a.V);
  const int64_t orig = a.row_index ? (int64_t)a.row_index[row] : a.row0 + row;
  const int64_t aux = a.row_index ? orig : (int64_t)row;
  const int tgt = a.targets[aux];
  const int n8 = a.V / 8;
  if (tgt < 0 || tgt >= a.V) {   // ignored row: exact zeros, no loss term
    bf16x8h zero;
#pragma unroll
    for (int k = 0; k < 8; ++k) zero[k] = (bf16_t)0.0f;
    for (int v = tid; v < n8; v += HR_THREADS) dz8[v] = zero;
    if (tid == 0) a.row_loss[row] = 0.f;
    return;
  }
  const float2* ps = a.stats + (int64_t)row * a.n_stat;
  float mx = -INFINITY, se = 0.f;
  for (int t = tid; t < a.n_stat; t += HR_THREADS) {
    const float2 p = ps[t];
    const float m2 = fmaxf(mx, p.x);
    se = se * __expf(mx - m2) + p.y * __expf(p.x - m2);
    mx = m2;
  }
  {
    const float gmx = block_max(mx, red);
    se = block_sum(mx == -INFINITY ? 0.f : se * __expf(mx - gmx), red);
    mx = gmx;
  }
  const float lse = mx + logf(se);
  const float logp = a.target_logit[row] - lse;
  float coef, loss_term;
  objective_terms(a, logp, orig, aux, coef, loss_term);
  if (tid == 0) a.row_loss[row] = loss_term;
  for (int v = tid; v < n8; v += HR_THREADS) {
    const int v0 = v * 8;
    const float f = coef * __expf(ps[v0 / GEMM_STAT_COLS].x - lse);   // 8 | 256: the eight elements share a block
    const bf16x8h e = dz8[v];
    bf16x8h o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = (bf16_t)((v0 + k == tgt ? coef : 0.0f) - (float)e[k] * f);
    dz8[v] = o;
  }
}

hipError_t head_rows(const HeadRowArgs& a, hipStream_t st) {
  if (a.rows == 0) return hipSuccess;
  if (a.target_logit) {
    if (a.dt != DT_BF16 || !a.stats || a.V % 8 != 0 || ((uintptr_t)a.dz & 15)) return hipErrorInvalidValue;
    head_rows_numer_k<<<a.rows, HR_THREADS, 0, st>>>(a);
    return hipGetLastError();
  }
  if (a.dt == DT_BF16) head_rows_k<bf16_t><<<a.rows, HR_THREADS, 0, st>>>(a);
  else head_rows_k<float><<<a.rows, HR_THREADS, 0, st>>>(a);
  return hipGetLastError();
}

// out += sum(v[0..n)) with a fixed summation tree (one workgroup).
__global__ __launch_bounds__(256) void reduce_add_k(const float* __restrict__ v, int n, float* __restrict__ out,
                                                    const int* __restrict__ n_dev) {
  __shared__ float red[16];
  if (n_dev) n = min(n, max(0, *n_dev));
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) *out += s;
}
hipError_t reduce_add(const float* v, int n, float* out, hipStream_t st, const int* n_dev) {
  if (n == 0) return hipSuccess;
  reduce_add_k<<<1, 256, 0, st>>>(v, n, out, n_dev);
  return hipGetLastError();
}

// Stable compaction of the active rows (target >= 0) by one workgroup: per-thread counts over a contiguous
// slice, an exclusive scan of the 1024 counts in LDS, then each thread writes its slice's indices in order.
__global__ __launch_bounds__(1024) void compact_active_k(const int32_t* __restrict__ targets, int64_t rows, int chunk, int V,
                                                         int32_t* __restrict__ index, int32_t* __restrict__ chunk_rows,
                                                         int n_chunks) {
  __shared__ int cnt[1024];
  const int tid = threadIdx.x;
  const int64_t per = (rows + 1023) / 1024;
  const int64_t b = min(rows, (int64_t)tid * per), e = min(rows, b + per);
  int c = 0;
  for (int64_t r = b; r < e; ++r) c += (uint32_t)targets[r] < (uint32_t)V ? 1 : 0;   // 0 <= target < V
  cnt[tid] = c;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {       // inclusive Hillis-Steele scan
    const int v = tid >= off ? cnt[tid - off] : 0;
    __syncthreads();
    cnt[tid] += v;
    __syncthreads();
  }
  int pos = cnt[tid] - c;
  for (int64_t r = b; r < e; ++r)
    if ((uint32_t)targets[r] < (uint32_t)V) index[pos++] = (int32_t)r;
  const int total = cnt[1023];
  for (int i = tid; i < n_chunks; i += 1024) chunk_rows[i] = min(chunk, max(0, total - i * chunk));
}
hipError_t compact_active(const int32_t* targets, int64_t rows, int chunk, int V, int32_t* index, int32_t* chunk_rows, int n_chunks,
                          hipStream_t st) {
  compact_active_k<<<1, 1024, 0, st>>>(targets, rows, chunk, V, index, chunk_rows, n_chunks);
  return hipGetLastError();
}

template <typename T, bool SCATTER>
__global__ __launch_bounds__(256) void move_rows_k(const T* __restrict__ src, const int32_t* __restrict__ index,
                                                   const int* __restrict__ rows_dev, T* __restrict__ dst, int d) {
  const int r = blockIdx.x;
  const bool valid = r < *rows_dev;
  if (SCATTER) {
    if (!valid) return;
    const int64_t o = index[r];
    for (int j = threadIdx.x; j < d; j += 256) dst[o * d + j] = src[(int64_t)r * d + j];
  } else {
    const int64_t o = valid ? index[r] : 0;
    for (int j = threadIdx.x; j < d; j += 256) dst[(int64_t)r * d + j] = valid ? src[o * d + j] : (T)0.0f;
  }
}
hipError_t gather_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t st) {
  if (max_rows == 0) return hipSuccess;
  if (dt == DT_BF16) move_rows_k<bf16_t, false><<<max_rows, 256, 0, st>>>((const bf16_t*)src, index, rows_dev, (bf16_t*)dst, d);
  else move_rows_k<float, false><<<max_rows, 256, 0, st>>>((const float*)src, index, rows_dev, (float*)dst, d);
  return hipGetLastError();
}
hipError_t scatter_rows(int dt, const void* src, const int32_t* index, const int* rows_dev, void* dst, int max_rows, int d, hipStream_t st) {
  if (max_rows == 0) return hipSuccess;
  if (dt == DT_BF16) move_rows_k<bf16_t, true><<<max_rows, 256, 0, st>>>((const bf16_t*)src, index, rows_dev, (bf16_t*)dst, d);
  else move_rows_k<float, true><<<max_rows, 256, 0, st>>>((const float*)src, index, rows_dev, (float*)dst, d);
  return hipGetLastError();
}

// Active rows are those with 0 <= target < V.  A target >= V is a caller error the host cannot see (the ids live on
// the device): such rows are treated as ignored everywhere - the id is never used as an index - and the call reports
// them by writing minus their number to n_active instead of the count of active rows.
__global__ __launch_bounds__(1024) void count_active_k(const int32_t* __restrict__ targets, int B, int T, int V,
                                                       float* __restrict__ seq_weight, int64_t* __restrict__ n_active) {
  __shared__ int red[16], red_bad[16];
  int64_t total = 0, total_bad = 0;
  for (int j = 0; j < B; ++j) {
    int cnt = 0, bad = 0;
    for (int t = threadIdx.x; t < T; t += 1024) {
      const int tg = targets[(int64_t)j * T + t];
      cnt += (uint32_t)tg < (uint32_t)V ? 1 : 0;
      bad += tg >= V ? 1 : 0;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { cnt += __shfl_xor(cnt, off, WAVE); bad += __shfl_xor(bad, off, WAVE); }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = cnt; red_bad[threadIdx.x >> 6] = bad; }
    __syncthreads();
    int tot = 0, tot_bad = 0;
    for (int i = 0; i < 16; ++i) { tot += red[i]; tot_bad += red_bad[i]; }
    if (threadIdx.x == 0 && seq_weight) seq_weight[j] = tot > 0 ? 1.0f / ((float)B * (float)tot) : 0.0f;
    total += tot;
    total_bad += tot_bad;
  }
  if (threadIdx.x == 0) *n_active = total_bad > 0 ? -total_bad : total;
}
hipError_t count_active(const int32_t* targets, int B, int T, int V, float* seq_weight, int64_t* n_active, hipStream_t st) {
  count_active_k<<<1, 1024, 0, st>>>(targets, B, T, V, seq_weight, n_active);
  return hipGetLastError();
}

template <typename T, typename TW>
__global__ void dpo_finish_k(const float* __restrict__ ell, float beta, T* __restrict__ dh, int64_t n_dh,
                             TW* __restrict__ dw, int64_t n_dw, float* __restrict__ loss) {
  const float x = beta * (*ell);
  const float sig = 1.0f / (1.0f + expf(-x));
  const float factor = sig - 1.0f;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  if (i == 0) *loss += (x > -30.f) ? log1pf(expf(-x)) : -x;
  for (; i < n_dh + n_dw; i += stride) {
    if (i < n_dh) stf(dh + i, ldf(dh + i) * factor);
    else stf(dw + (i - n_dh), ldf(dw + (i - n_dh)) * factor);
  }
}
hipError_t dpo_finish(int dt, const float* ell, float beta, void* dh, int64_t n_dh, void* dw, int dw_dt, int64_t n_dw,
                      float* loss, hipStream_t st) {
  unsigned grid = (unsigned)std::min<int64_t>(cdiv(n_dh + n_dw, 256), 256 * 16);
  if (dt == DT_BF16 && dw_dt == DT_BF16) dpo_finish_k<bf16_t, bf16_t><<<grid, 256, 0, st>>>(ell, beta, (bf16_t*)dh, n_dh, (bf16_t*)dw, n_dw, loss);
  else if (dt == DT_BF16) dpo_finish_k<bf16_t, float><<<grid, 256, 0, st>>>(ell, beta, (bf16_t*)dh, n_dh, (float*)dw, n_dw, loss);
  else dpo_finish_k<float, float><<<grid, 256, 0, st>>>(ell, beta, (float*)dh, n_dh, (float*)dw, n_dw, loss);
  return hipGetLastError();
}

}  // namespace sbp
