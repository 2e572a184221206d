// Shape-agnostic chunk attention (any head_dim <= 256, fp32 or bf16 storage):
// the correctness path for the fp32 configuration and for head sizes the MFMA
// kernels do not take.  Query row t of the chunk sits at global position
// q_start + t and sees keys 0 .. q_start + t; the causal mask is an integer
// comparison of positions, never a stored tensor, and so are the two optional
// rules: a sliding window (keys t - window < u <= t) and padding in front of the
// sequence (keys before kv_first hidden).  A query that sees no key gets o = 0,
// lse = -inf and sends no gradient.  No atomics: every output element has
// exactly one owner, so results are reproducible.
#include "launch.h"
#include "device.h"

namespace sbp {

constexpr int AG_THREADS = 256;

template <typename T>
__global__ __launch_bounds__(AG_THREADS) void attn_fwd_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                                 const T* __restrict__ v, T* __restrict__ o,
                                                                 float* __restrict__ lse, int Hq, int Hkv, int dh,
                                                                 int q_start, int c, float scale, int window, int kv_first) {
  __shared__ float qs[256];
  __shared__ float p[AG_THREADS];
  __shared__ float red[16];
  const int t = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int kvh = h / (Hq / Hkv);
  const int n_keys = q_start + t + 1;
  const int lo = max(kv_first, window > 0 ? q_start + t - window + 1 : 0);   // first visible key
  const int64_t kv_stride = (int64_t)Hkv * dh;
  if (tid < dh) qs[tid] = ldf(q + ((int64_t)t * Hq + h) * dh + tid) * scale;
  __syncthreads();
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int u0 = lo; u0 < n_keys; u0 += AG_THREADS) {
    const int u = u0 + tid;
    float sc = -INFINITY;
    if (u < n_keys) {
      const T* kr = k + (int64_t)u * kv_stride + (int64_t)kvh * dh;
      float s = 0.f;
      for (int j = 0; j < dh; ++j) s = fmaf(qs[j], ldf(kr + j), s);
      sc = s;
    }
    const float m_new = fmaxf(m_run, block_max(sc, red));
    const float pe = (u < n_keys) ? expf(sc - m_new) : 0.f;
    const float tile_sum = block_sum(pe, red);
    const float corr = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    l_run = l_run * corr + tile_sum;
    p[tid] = pe;
    __syncthreads();
    if (tid < dh) {
      const int lim = min(AG_THREADS, n_keys - u0);
      float a = acc * corr;
      const T* vr = v + (int64_t)u0 * kv_stride + (int64_t)kvh * dh + tid;
      for (int i = 0; i < lim; ++i) a = fmaf(p[i], ldf(vr + (int64_t)i * kv_stride), a);
      acc = a;
    }
    m_run = m_new;
    __syncthreads();
  }
  if (tid < dh) stf(o + ((int64_t)t * Hq + h) * dh + tid, l_run > 0.f ? acc / l_run : 0.f);
  if (tid == 0) lse[(int64_t)h * c + t] = l_run > 0.f ? m_run + logf(l_run) : -INFINITY;
}

// delta[h, t] = sum_j d_o[t,h,j] * o[t,h,j]
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_k(const T* __restrict__ o, const T* __restrict__ d_o,
                                                   float* __restrict__ delta, int Hq, int dh, int c) {
  const int t = blockIdx.x, h = blockIdx.y;
  const int64_t base = ((int64_t)t * Hq + h) * dh;
  float s = 0.f;
  for (int j = threadIdx.x; j < dh; j += 64) s += ldf(o + base + j) * ldf(d_o + base + j);
  s = wave_sum(s);
  if (threadIdx.x == 0) delta[(int64_t)h * c + t] = s;
}

template <typename T>
__global__ __launch_bounds__(AG_THREADS) void attn_dq_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                                const T* __restrict__ v, const T* __restrict__ d_o,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta, T* __restrict__ dq,
                                                                int Hq, int Hkv, int dh, int q_start, int c, float scale,
                                                                int window, int kv_first) {
  __shared__ float qs[256];
  __shared__ float dos[256];
  __shared__ float dsv[AG_THREADS];
  const int t = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int kvh = h / (Hq / Hkv);
  const int n_keys = q_start + t + 1;
  const int64_t kv_stride = (int64_t)Hkv * dh;
  const int64_t qbase = ((int64_t)t * Hq + h) * dh;
  if (tid < dh) { qs[tid] = ldf(q + qbase + tid); dos[tid] = ldf(d_o + qbase + tid); }
  __syncthreads();
  const float L = lse[(int64_t)h * c + t], D = delta[(int64_t)h * c + t];
  const int lo = max(kv_first, window > 0 ? q_start + t - window + 1 : 0);
  float acc = 0.f;
  for (int u0 = lo; u0 < n_keys; u0 += AG_THREADS) {
    const int u = u0 + tid;
    float ds = 0.f;
    if (u < n_keys) {
      const T* kr = k + (int64_t)u * kv_stride + (int64_t)kvh * dh;
      const T* vr = v + (int64_t)u * kv_stride + (int64_t)kvh * dh;
      float s = 0.f, dp = 0.f;
      for (int j = 0; j < dh; ++j) { s = fmaf(qs[j], ldf(kr + j), s); dp = fmaf(dos[j], ldf(vr + j), dp); }
      const float pr = expf(s * scale - L);
      ds = pr * (dp - D) * scale;
    }
    dsv[tid] = ds;
    __syncthreads();
    if (tid < dh) {
      const int lim = min(AG_THREADS, n_keys - u0);
      const T* kr = k + (int64_t)u0 * kv_stride + (int64_t)kvh * dh + tid;
      float a = acc;
      for (int i = 0; i < lim; ++i) a = fmaf(dsv[i], ldf(kr + (int64_t)i * kv_stride), a);
      acc = a;
    }
    __syncthreads();
  }
  if (tid < dh) stf(dq + qbase + tid, acc);
}

// One workgroup owns key u of KV head kvh and walks the (query row, query head)
// pairs that see it: rows t >= u - q_start, heads of the group.
template <typename T>
__global__ __launch_bounds__(AG_THREADS) void attn_dkv_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                                 const T* __restrict__ v, const T* __restrict__ d_o,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 float* __restrict__ dk, float* __restrict__ dv,
                                                                 int Hq, int Hkv, int dh, int q_start, int c, float scale,
                                                                 int window, int kv_first) {
  __shared__ float ks[256];
  __shared__ float vs[256];
  __shared__ float ps[AG_THREADS];
  __shared__ float dss[AG_THREADS];
  const int u = blockIdx.x, kvh = blockIdx.y, tid = threadIdx.x;
  const int G = Hq / Hkv;
  const int64_t kbase = ((int64_t)u * Hkv + kvh) * dh;
  if (tid < dh) { ks[tid] = ldf(k + kbase + tid); vs[tid] = ldf(v + kbase + tid); }
  __syncthreads();
  const int t_min = max(0, u - q_start);
  int t_end = c;                                                 // rows [t_min, t_end) see key u
  if (window > 0) t_end = min(c, u + window - q_start);         // position <= u + window - 1
  if (u < kv_first) t_end = t_min;
  const int n_pairs = max(0, t_end - t_min) * G;
  float acc_k = 0.f, acc_v = 0.f;
  for (int i0 = 0; i0 < n_pairs; i0 += AG_THREADS) {
    const int i = i0 + tid;
    float pr = 0.f, ds = 0.f;
    if (i < n_pairs) {
      const int t = t_min + i / G, h = kvh * G + i % G;
      const int64_t qb = ((int64_t)t * Hq + h) * dh;
      float s = 0.f, dp = 0.f;
      for (int j = 0; j < dh; ++j) { s = fmaf(ldf(q + qb + j), ks[j], s); dp = fmaf(ldf(d_o + qb + j), vs[j], dp); }
      pr = expf(s * scale - lse[(int64_t)h * c + t]);
      ds = pr * (dp - delta[(int64_t)h * c + t]) * scale;
    }
    ps[tid] = pr; dss[tid] = ds;
    __syncthreads();
    if (tid < dh) {
      const int lim = min(AG_THREADS, n_pairs - i0);
      for (int ii = 0; ii < lim; ++ii) {
        const int i2 = i0 + ii;
        const int t = t_min + i2 / G, h = kvh * G + i2 % G;
        const int64_t qb = ((int64_t)t * Hq + h) * dh + tid;
        acc_v = fmaf(ps[ii], ldf(d_o + qb), acc_v);
        acc_k = fmaf(dss[ii], ldf(q + qb), acc_k);
      }
    }
    __syncthreads();
  }
  if (tid < dh) { dk[kbase + tid] += acc_k; dv[kbase + tid] += acc_v; }
}

hipError_t attn_forward_generic(const AttnArgs& a, hipStream_t st) {
  if (a.q_len == 0) return hipSuccess;
  dim3 grid(a.q_len, a.Hq);
  if (a.dt == DT_BF16)
    attn_fwd_generic_k<bf16_t><<<grid, AG_THREADS, 0, st>>>((const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v,
                                                           (bf16_t*)a.o, a.lse, a.Hq, a.Hkv, a.dh, a.q_start, a.q_len, a.scale,
                                                           a.window, a.kv_first);
  else
    attn_fwd_generic_k<float><<<grid, AG_THREADS, 0, st>>>((const float*)a.q, (const float*)a.k, (const float*)a.v,
                                                          (float*)a.o, a.lse, a.Hq, a.Hkv, a.dh, a.q_start, a.q_len, a.scale,
                                                          a.window, a.kv_first);
  return hipGetLastError();
}

template <typename T>
static hipError_t attn_backward_generic_t(const AttnArgs& a, hipStream_t st) {
  dim3 gq(a.q_len, a.Hq);
  attn_delta_k<T><<<gq, 64, 0, st>>>((const T*)a.o, (const T*)a.d_o, a.delta, a.Hq, a.dh, a.q_len);
  attn_dq_generic_k<T><<<gq, AG_THREADS, 0, st>>>((const T*)a.q, (const T*)a.k, (const T*)a.v, (const T*)a.d_o, a.lse,
                                                  a.delta, (T*)a.dq, a.Hq, a.Hkv, a.dh, a.q_start, a.q_len, a.scale, a.window,
                                                  a.kv_first);
  dim3 gk(a.q_start + a.q_len, a.Hkv);
  attn_dkv_generic_k<T><<<gk, AG_THREADS, 0, st>>>((const T*)a.q, (const T*)a.k, (const T*)a.v, (const T*)a.d_o, a.lse,
                                                   a.delta, a.dk, a.dv, a.Hq, a.Hkv, a.dh, a.q_start, a.q_len, a.scale, a.window,
                                                   a.kv_first);
  return hipGetLastError();
}

hipError_t attn_backward_generic(const AttnArgs& a, hipStream_t st) {
  if (a.q_len == 0) return hipSuccess;
  return a.dt == DT_BF16 ? attn_backward_generic_t<bf16_t>(a, st) : attn_backward_generic_t<float>(a, st);
}

}  // namespace sbp
