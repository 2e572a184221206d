// Row-statistic and elementwise kernels: RMSNorm (forward / adjoint), RoPE,
// SwiGLU, residual adds, dK/dV finishing, embedding gather / scatter-add.
// All are HBM-bound: one pass over their operands, 128-bit accesses where the
// row width allows, fp32 arithmetic with wavefront (64-lane) reductions.
#include "launch.h"
#include "device.h"
#include <algorithm>

namespace sbp {

#define DISPATCH_DT(dt, T, ...)                      \
  do {                                               \
    if ((dt) == DT_BF16) { using T = bf16_t; __VA_ARGS__; } \
    else { using T = float; __VA_ARGS__; }           \
  } while (0)

// ------------------------------------------------------------------ RoPE --
// Rotate-half pairing (j, j + dh/2), angle (t + pos_offset) * theta^(-2j/dh).
// Angles go through fp64: an fp32 product pos*inv_freq has an absolute error of
// ~2e-3 rad at position 32768, which the fp32 path's tolerance cannot absorb.
__global__ void rope_table_k(float2* tab, int n_pos, int half, double theta, int pos_offset) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)n_pos * half) return;
  int t = (int)(i / half), j = (int)(i % half);
  double inv_freq = pow(theta, -(double)j / (double)half);   // theta^(-2j/dh)
  double ang = ((double)t + (double)pos_offset) * inv_freq;
  double s, c;
  sincos(ang, &s, &c);
  tab[i] = make_float2((float)c, (float)s);
}

hipError_t rope_table(float2* tab, int n_pos, int dh, float theta, int pos_offset, hipStream_t st) {
  int half = dh / 2;
  int64_t n = (int64_t)n_pos * half;
  if (n == 0) return hipSuccess;
  rope_table_k<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(tab, n_pos, half, (double)theta, pos_offset);
  return hipGetLastError();
}

template <typename T>
__global__ void rope_apply_k(T* x, const float2* tab, int64_t n_pairs, int H, int half, int inverse) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pairs) return;
  int j = (int)(i % half);
  int64_t rh = i / half;              // row * H + head
  int64_t row = rh / H;
  float2 cs = tab[row * half + j];
  float sn = inverse ? -cs.y : cs.y;
  T* p = x + rh * (2 * half);
  float a = ldf(p + j), b = ldf(p + j + half);
  stf(p + j, a * cs.x - b * sn);
  stf(p + j + half, b * cs.x + a * sn);
}

hipError_t rope_apply(int dt, void* x, const float2* tab, int rows, int H, int dh, bool inverse, hipStream_t st) {
  int64_t n = (int64_t)rows * H * (dh / 2);
  if (n == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (rope_apply_k<T><<<(unsigned)cdiv(n, 256), 256, 0, st>>>((T*)x, tab, n, H, dh / 2, inverse ? 1 : 0)));
  return hipGetLastError();
}

// --------------------------------------------------------------- RMSNorm --
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  typedef bf16_t bf16x8_t __attribute__((ext_vector_type(8)));
  const bf16x8_t a = *(const bf16x8_t*)p;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
  *(float4*)(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  typedef bf16_t bf16x8_t __attribute__((ext_vector_type(8)));
  bf16x8_t a;
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = (bf16_t)v[e];
  *(bf16x8_t*)p = a;
}
constexpr int RV_MAX_IT = 8;    // 64 lanes x 8 elements x 8 = 4096 columns (the backward's 4 x d floats of LDS stay under 64 KiB)
// Vectorised form for d % 8 == 0, d <= 4096: one wave per row, 8 elements per lane per access, the row stays in
// registers between the sum of squares and the scaling (one read of x instead of two).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_vec_k(const T* __restrict__ x, const float* __restrict__ add,
                                                         const T* __restrict__ g, T* __restrict__ out,
                                                         float* __restrict__ sum_out, float* __restrict__ rstd,
                                                         int rows, int d, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int n_it = (d + 511) / 512;
  float v[RV_MAX_IT][8];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < RV_MAX_IT; ++it) {
    const int j = it * 512 + lane * 8;
    if (it < n_it && j < d) {
      load8(x + row * d + j, v[it]);
      if (add) {
        float a[8];
        load8(add + row * d + j, a);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[it][e] += a[e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[it][e] * v[it][e];
    }
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  if (lane == 0 && rstd) rstd[row] = r;
  if (!out) return;
#pragma unroll
  for (int it = 0; it < RV_MAX_IT; ++it) {
    const int j = it * 512 + lane * 8;
    if (it < n_it && j < d) {
      float gv[8], o[8];
      load8(g + j, gv);
      if (sum_out) store8(sum_out + row * d + j, v[it]);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = gv[e] * v[it][e] * r;
      store8(out + row * d + j, o);
    }
  }
}

// One workgroup per row.  r = 1/sqrt(mean(v^2) + eps) with v = x (+ add).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_k(const T* __restrict__ x, const float* __restrict__ add,
                                                     const T* __restrict__ g, T* __restrict__ out,
                                                     float* __restrict__ sum_out, float* __restrict__ rstd,
                                                     int d, float eps) {
  __shared__ float red[16];
  const int64_t row = blockIdx.x;
  const T* xr = x + row * d;
  const float* ar = add ? add + row * d : nullptr;
  float ss = 0.f;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    float v = ldf(xr + j) + (ar ? ar[j] : 0.f);
    ss += v * v;
  }
  ss = block_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  if (threadIdx.x == 0 && rstd) rstd[row] = r;
  if (!out) return;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    float v = ldf(xr + j) + (ar ? ar[j] : 0.f);
    if (sum_out) sum_out[row * d + j] = v;
    stf(out + row * d + j, ldf(g + j) * v * r);
  }
}

hipError_t rmsnorm_fwd(int dt, const void* x, const float* add, const void* g, void* out, float* sum_out,
                       float* rstd, int rows, int d, float eps, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  const bool vec = d % 8 == 0 && d <= 512 * RV_MAX_IT && al(x) && al(add) && al(g) && al(out) && al(sum_out);
  DISPATCH_DT(dt, T, {
    if (vec) rmsnorm_fwd_vec_k<T><<<(unsigned)cdiv(rows, 4), 256, 0, st>>>((const T*)x, add, (const T*)g, (T*)out, sum_out, rstd, rows, d, eps);
    else rmsnorm_fwd_k<T><<<rows, 256, 0, st>>>((const T*)x, add, (const T*)g, (T*)out, sum_out, rstd, d, eps);
  });
  return hipGetLastError();
}

// Adjoint.  With u = dnorm * g and dot = <u, x>:  dx = u*r - x * r^3 * dot / d.
// A workgroup owns RB consecutive rows so that it can emit one partial row of
// dg = sum_rows dnorm * x * r; a second kernel adds the partial rows in a fixed
// order (no atomics: the result is reproducible run to run).
constexpr int RB = 8;
template <typename T, typename XT, typename RT, typename DN = float>
__global__ __launch_bounds__(256) void rmsnorm_bwd_k(const DN* __restrict__ dnorm, const XT* __restrict__ xin,
                                                     const T* __restrict__ g, const float* __restrict__ rstd,
                                                     const RT* __restrict__ res, float* __restrict__ out_f32,
                                                     T* __restrict__ out_t, float* __restrict__ partial,
                                                     int rows, int d) {
  __shared__ float red[16];
  __shared__ float dots[RB];
  const int64_t row0 = (int64_t)blockIdx.x * RB;
  const int nr = (int)min((int64_t)RB, (int64_t)rows - row0);
  for (int r = 0; r < nr; ++r) {
    const int64_t row = row0 + r;
    float acc = 0.f;
    for (int j = threadIdx.x; j < d; j += blockDim.x)
      acc += ldf(dnorm + row * d + j) * ldf(g + j) * ldf(xin + row * d + j);
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) dots[r] = acc;
  }
  __syncthreads();
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    const float gj = ldf(g + j);
    float dgj = 0.f;
    for (int r = 0; r < nr; ++r) {
      const int64_t row = row0 + r;
      const float rs = rstd[row];
      const float xv = ldf(xin + row * d + j);
      const float dn = ldf(dnorm + row * d + j);
      dgj += dn * xv * rs;
      const float v = (res ? ldf(res + row * d + j) : 0.f) + dn * gj * rs - xv * rs * rs * rs * dots[r] / (float)d;
      if (out_f32) out_f32[row * d + j] = v;
      if (out_t) stf(out_t + row * d + j, v);
    }
    partial[(int64_t)blockIdx.x * d + j] = dgj;
  }
}

// Vectorised form for d % 8 == 0, d <= 4096: one wave per row, 8 elements (128 or 256 bits) per lane per access;
// a workgroup of 4 waves takes RB rows (2 per wave), each wave keeps its share of dg in registers across its rows
// and the four waves' shares meet in LDS in a fixed order.  Same arithmetic and the same partial-sum layout as the
// plain kernel above.
template <typename T, typename XT, typename RT, typename DN>
__global__ __launch_bounds__(256) void rmsnorm_bwd_vec_k(const DN* __restrict__ dnorm, const XT* __restrict__ xin,
                                                         const T* __restrict__ g, const float* __restrict__ rstd,
                                                         const RT* __restrict__ res, float* __restrict__ out_f32,
                                                         T* __restrict__ out_t, float* __restrict__ partial,
                                                         int rows, int d) {
  extern __shared__ float sdg[];   // [4][d]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * RB;
  const int n_it = (d + 511) / 512;
  float dg[RV_MAX_IT][8];
#pragma unroll
  for (int it = 0; it < RV_MAX_IT; ++it)
#pragma unroll
    for (int e = 0; e < 8; ++e) dg[it][e] = 0.f;
  for (int r = wave; r < RB; r += 4) {
    const int64_t row = row0 + r;
    if (row >= rows) break;
    const float rs = rstd[row];
    float dot = 0.f;
#pragma unroll
    for (int it = 0; it < RV_MAX_IT; ++it) {
      const int j = it * 512 + lane * 8;
      if (it < n_it && j < d) {
        float dn[8], gv[8], xv[8];
        load8(dnorm + row * d + j, dn); load8(g + j, gv); load8(xin + row * d + j, xv);
#pragma unroll
        for (int e = 0; e < 8; ++e) dot += dn[e] * gv[e] * xv[e];
      }
    }
    dot = wave_sum(dot);
    const float coef = rs * rs * rs * dot / (float)d;
#pragma unroll
    for (int it = 0; it < RV_MAX_IT; ++it) {
      const int j = it * 512 + lane * 8;
      if (it < n_it && j < d) {
        float dn[8], gv[8], xv[8], rv[8], o[8];
        load8(dnorm + row * d + j, dn); load8(g + j, gv); load8(xin + row * d + j, xv);
        if (res) load8(res + row * d + j, rv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          dg[it][e] += dn[e] * xv[e] * rs;
          o[e] = (res ? rv[e] : 0.f) + dn[e] * gv[e] * rs - xv[e] * coef;
        }
        if (out_f32) store8(out_f32 + row * d + j, o);
        if (out_t) store8(out_t + row * d + j, o);
      }
    }
  }
#pragma unroll
  for (int it = 0; it < RV_MAX_IT; ++it) {
    const int j = it * 512 + lane * 8;
    if (it < n_it && j < d) store8(sdg + (int64_t)wave * d + j, dg[it]);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < d; j += blockDim.x)
    partial[(int64_t)blockIdx.x * d + j] = (sdg[j] + sdg[d + j]) + (sdg[2 * d + j] + sdg[3 * d + j]);
}
static bool rmsnorm_bwd_vec_ok(int d, const void* a, const void* b, const void* c, const void* e, const void* f, const void* h) {
  auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  return d % 8 == 0 && d <= 512 * RV_MAX_IT && al(a) && al(b) && al(c) && al(e) && al(f) && al(h);
}

// dg[j] += sum_b partial[b][j]: 64 columns per workgroup, the partial rows dealt to 4 waves, fixed summation order.
__global__ __launch_bounds__(256) void colsum_accum_k(const float* __restrict__ partial, float* __restrict__ dg, int nblk, int d) {
  __shared__ float red[4][64];
  const int j = blockIdx.x * 64 + (threadIdx.x & 63), part = threadIdx.x >> 6;
  float s = 0.f;
  if (j < d)
    for (int b = part; b < nblk; b += 4) s += partial[(int64_t)b * d + j];
  red[part][threadIdx.x & 63] = s;
  __syncthreads();
  if (part == 0 && j < d) dg[j] += (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

size_t rmsnorm_bwd_partial_floats(int rows, int d) { return (size_t)cdiv(rows, RB) * (size_t)d; }

hipError_t rmsnorm_bwd(int dt, const float* dnorm, const void* xin, bool x_is_f32, const void* g,
                       const float* rstd, const void* res, bool res_is_f32, float* out_f32, void* out_t,
                       float* dg, float* partial, int rows, int d, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  const int nblk = (int)cdiv(rows, RB);
  const bool vec = rmsnorm_bwd_vec_ok(d, dnorm, xin, g, res, out_f32, out_t);
  const size_t shm = (size_t)4 * d * sizeof(float);
#define RB_LAUNCH(T, XT, RT)                                                                                     \
  do {                                                                                                           \
    if (vec)                                                                                                     \
      rmsnorm_bwd_vec_k<T, XT, RT, float><<<nblk, 256, shm, st>>>(dnorm, (const XT*)xin, (const T*)g, rstd,      \
                                                                  (const RT*)res, out_f32, (T*)out_t, partial, rows, d); \
    else                                                                                                         \
      rmsnorm_bwd_k<T, XT, RT><<<nblk, 256, 0, st>>>(dnorm, (const XT*)xin, (const T*)g, rstd, (const RT*)res,   \
                                                     out_f32, (T*)out_t, partial, rows, d);                      \
  } while (0)
  DISPATCH_DT(dt, T, {
    if (x_is_f32 && res_is_f32) RB_LAUNCH(T, float, float);
    else if (x_is_f32) RB_LAUNCH(T, float, T);
    else if (res_is_f32) RB_LAUNCH(T, T, float);
    else RB_LAUNCH(T, T, T);
  });
#undef RB_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  colsum_accum_k<<<(unsigned)cdiv(d, 64), 256, 0, st>>>(partial, dg, nblk, d);
  return hipGetLastError();
}

// Stand-alone norm adjoint with the incoming gradient in the storage type and no
// residual branch (the final norm between the layer stack and the LM head).
hipError_t rmsnorm_bwd_plain(int dt, const void* dy, const void* x, const void* g, const float* rstd, void* dx,
                             float* dg, float* partial, int rows, int d, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  const int nblk = (int)cdiv(rows, RB);
  const bool vec = rmsnorm_bwd_vec_ok(d, dy, x, g, nullptr, nullptr, dx);
  const size_t shm = (size_t)4 * d * sizeof(float);
  DISPATCH_DT(dt, T, {
    if (vec)
      rmsnorm_bwd_vec_k<T, T, T, T><<<nblk, 256, shm, st>>>((const T*)dy, (const T*)x, (const T*)g, rstd, (const T*)nullptr,
                                                            nullptr, (T*)dx, partial, rows, d);
    else
      rmsnorm_bwd_k<T, T, T, T><<<nblk, 256, 0, st>>>((const T*)dy, (const T*)x, (const T*)g, rstd, (const T*)nullptr,
                                                      nullptr, (T*)dx, partial, rows, d);
  });
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  colsum_accum_k<<<(unsigned)cdiv(d, 64), 256, 0, st>>>(partial, dg, nblk, d);
  return hipGetLastError();
}

// ---------------------------------------------------------------- SwiGLU --
__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

template <typename T>
__global__ void swiglu_fwd_k(const T* __restrict__ gate, const T* __restrict__ up, T* __restrict__ act, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float z = ldf(gate + i);
    stf(act + i, z * sigmoidf_(z) * ldf(up + i));
  }
}
template <typename T>
__global__ void swiglu_bwd_k(T* __restrict__ gate, T* __restrict__ up, const T* __restrict__ dact, T* __restrict__ act, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float z = ldf(gate + i), u = ldf(up + i), da = ldf(dact + i);
    float sg = sigmoidf_(z);
    if (act) stf(act + i, z * sg * u);
    stf(gate + i, da * u * sg * (1.0f + z * (1.0f - sg)));
    stf(up + i, da * z * sg);
  }
}
// 8 bf16 per lane (128-bit) variants for the wide MLP tensors
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
__global__ void swiglu_fwd_bf16x8_k(const bf16x8* __restrict__ gate, const bf16x8* __restrict__ up,
                                    bf16x8* __restrict__ act, int64_t n8) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n8; i += stride) {
    bf16x8 g = gate[i], u = up[i], a;
#pragma unroll
    for (int j = 0; j < 8; ++j) { float z = (float)g[j]; a[j] = (bf16_t)(z * sigmoidf_(z) * (float)u[j]); }
    act[i] = a;
  }
}
template <bool WITH_ACT>
__global__ void swiglu_bwd_bf16x8_k(bf16x8* __restrict__ gate, bf16x8* __restrict__ up,
                                    const bf16x8* __restrict__ dact, bf16x8* __restrict__ act, int64_t n8) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n8; i += stride) {
    bf16x8 g = gate[i], u = up[i], da = dact[i], dg, du, a;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float z = (float)g[j], uu = (float)u[j], d = (float)da[j];
      float sg = sigmoidf_(z);
      if (WITH_ACT) a[j] = (bf16_t)(z * sg * uu);
      dg[j] = (bf16_t)(d * uu * sg * (1.0f + z * (1.0f - sg)));
      du[j] = (bf16_t)(d * z * sg);
    }
    if (WITH_ACT) act[i] = a;
    gate[i] = dg; up[i] = du;
  }
}

static inline unsigned ew_grid(int64_t n) { return (unsigned)std::min<int64_t>(cdiv(n, 256), 256 * 16); }

hipError_t swiglu_fwd(int dt, const void* gate, const void* up, void* act, int64_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  if (dt == DT_BF16 && n % 8 == 0) {
    swiglu_fwd_bf16x8_k<<<ew_grid(n / 8), 256, 0, st>>>((const bf16x8*)gate, (const bf16x8*)up, (bf16x8*)act, n / 8);
  } else {
    DISPATCH_DT(dt, T, (swiglu_fwd_k<T><<<ew_grid(n), 256, 0, st>>>((const T*)gate, (const T*)up, (T*)act, n)));
  }
  return hipGetLastError();
}
hipError_t swiglu_bwd(int dt, void* gate, void* up, const void* dact, void* act, int64_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  if (dt == DT_BF16 && n % 8 == 0) {
    if (act) swiglu_bwd_bf16x8_k<true><<<ew_grid(n / 8), 256, 0, st>>>((bf16x8*)gate, (bf16x8*)up, (const bf16x8*)dact, (bf16x8*)act, n / 8);
    else swiglu_bwd_bf16x8_k<false><<<ew_grid(n / 8), 256, 0, st>>>((bf16x8*)gate, (bf16x8*)up, (const bf16x8*)dact, nullptr, n / 8);
  } else {
    DISPATCH_DT(dt, T, (swiglu_bwd_k<T><<<ew_grid(n), 256, 0, st>>>((T*)gate, (T*)up, (const T*)dact, (T*)act, n)));
  }
  return hipGetLastError();
}

// ------------------------------------------------------------ small glue --
template <typename T>
__global__ void add_store_k(const float* __restrict__ a, const float* __restrict__ b, T* __restrict__ y, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) stf(y + i, a[i] + b[i]);
}
hipError_t add_store(int dt, const float* a, const float* b, void* y, int64_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (add_store_k<T><<<ew_grid(n), 256, 0, st>>>(a, b, (T*)y, n)));
  return hipGetLastError();
}

template <typename T>
__global__ void kv_grad_finish_k(const float* __restrict__ dK, const float* __restrict__ dV,
                                 const float2* __restrict__ tab, T* __restrict__ dkc, T* __restrict__ dvc,
                                 int64_t n_pairs, int H, int half) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pairs) return;
  int j = (int)(i % half);
  int64_t rh = i / half;
  int64_t row = rh / H;
  float2 cs = tab[row * half + j];
  int64_t base = rh * (2 * half);
  float a = dK[base + j], b = dK[base + j + half];
  stf(dkc + base + j, a * cs.x + b * cs.y);            // rotation by the negative angle
  stf(dkc + base + j + half, b * cs.x - a * cs.y);
  stf(dvc + base + j, dV[base + j]);
  stf(dvc + base + j + half, dV[base + j + half]);
}
hipError_t kv_grad_finish(int dt, const float* dK, const float* dV, const float2* tab, void* dkc, void* dvc,
                          int rows, int H, int dh, hipStream_t st) {
  int64_t n = (int64_t)rows * H * (dh / 2);
  if (n == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (kv_grad_finish_k<T><<<(unsigned)cdiv(n, 256), 256, 0, st>>>(dK, dV, tab, (T*)dkc, (T*)dvc, n, H, dh / 2)));
  return hipGetLastError();
}

__global__ void fill_zero_k(uint4* p, int64_t n16) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}
__global__ void fill_zero_bytes_k(unsigned char* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}
// A fill kernel rather than a memset node, so that callers may capture the stream into a graph.
hipError_t fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16, tail = bytes - n16 * 16;
  if (((uintptr_t)p & 15) != 0) { n16 = 0; tail = bytes; }
  if (n16) fill_zero_k<<<ew_grid((int64_t)n16), 256, 0, st>>>((uint4*)p, (int64_t)n16);
  if (tail) fill_zero_bytes_k<<<(unsigned)cdiv((int64_t)tail, 256), 256, 0, st>>>((unsigned char*)p + n16 * 16, (int64_t)tail);
  return hipGetLastError();
}

// An id outside [0, vocab) is never used as an index: its row of x is zero and its row of dx is dropped.
__global__ void copy16_k(uint4* __restrict__ d, const uint4* __restrict__ s, int64_t n16) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) d[i] = s[i];
}
__global__ void copy1_k(unsigned char* __restrict__ d, const unsigned char* __restrict__ s, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = s[i];
}
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16, tail = bytes - n16 * 16;
  if ((((uintptr_t)dst | (uintptr_t)src) & 15) != 0) { n16 = 0; tail = bytes; }
  if (n16) copy16_k<<<ew_grid((int64_t)n16), 256, 0, st>>>((uint4*)dst, (const uint4*)src, (int64_t)n16);
  if (tail) copy1_k<<<(unsigned)cdiv((int64_t)tail, 256), 256, 0, st>>>((unsigned char*)dst + n16 * 16, (const unsigned char*)src + n16 * 16, (int64_t)tail);
  return hipGetLastError();
}

template <typename T>
__global__ void pad_matrix_k(const T* __restrict__ src, int R, int C, int transposed, float scale, T* __restrict__ dst, int R2, int C2) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)R2 * C2) return;
  const int r = (int)(i / C2), c = (int)(i % C2);
  float v = 0.f;
  if (r < R && c < C) v = scale * ldf(transposed ? src + (int64_t)c * R + r : src + (int64_t)r * C + c);
  stf(dst + i, v);
}
hipError_t pad_matrix(int dt, const void* src, int R, int C, bool transposed, float scale, void* dst, int R2, int C2, hipStream_t st) {
  const int64_t n = (int64_t)R2 * C2;
  if (n == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (pad_matrix_k<T><<<(unsigned)cdiv(n, 256), 256, 0, st>>>((const T*)src, R, C, transposed ? 1 : 0, scale, (T*)dst, R2, C2)));
  return hipGetLastError();
}
__global__ void add_scaled_block_k(const float* __restrict__ src, int64_t ld, float scale, float* __restrict__ dst, int R, int C) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)R * C) return;
  const int r = (int)(i / C), c = (int)(i % C);
  dst[i] += scale * src[(int64_t)r * ld + c];
}
hipError_t add_scaled_block(const float* src, int64_t ld, float scale, float* dst, int R, int C, hipStream_t st) {
  const int64_t n = (int64_t)R * C;
  if (n == 0) return hipSuccess;
  add_scaled_block_k<<<(unsigned)cdiv(n, 256), 256, 0, st>>>(src, ld, scale, dst, R, C);
  return hipGetLastError();
}

template <typename T>
__global__ void embedding_fwd_k(const int32_t* __restrict__ ids, const T* __restrict__ emb, T* __restrict__ x, int d, int vocab) {
  const int64_t row = blockIdx.x;
  const int64_t id = ids[row];
  const bool ok = id >= 0 && id < vocab;
  for (int j = threadIdx.x; j < d; j += blockDim.x) x[row * d + j] = ok ? emb[id * d + j] : (T)0.0f;
}
template <typename T>
__global__ void embedding_bwd_k(const int32_t* __restrict__ ids, const T* __restrict__ dx, float* __restrict__ demb, int d, int vocab) {
  const int64_t row = blockIdx.x;
  const int64_t id = ids[row];
  if (id < 0 || id >= vocab) return;
  for (int j = threadIdx.x; j < d; j += blockDim.x) atomicAdd(demb + id * d + j, ldf(dx + row * d + j));
}
hipError_t embedding_fwd(int dt, const int32_t* ids, const void* emb, void* x, int64_t rows, int d, int vocab, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (embedding_fwd_k<T><<<(unsigned)rows, 256, 0, st>>>(ids, (const T*)emb, (T*)x, d, vocab)));
  return hipGetLastError();
}
hipError_t embedding_bwd(int dt, const int32_t* ids, const void* dx, float* demb, int64_t rows, int d, int vocab, hipStream_t st) {
  if (rows == 0) return hipSuccess;
  DISPATCH_DT(dt, T, (embedding_bwd_k<T><<<(unsigned)rows, 256, 0, st>>>(ids, (const T*)dx, demb, d, vocab)));
  return hipGetLastError();
}

}  // namespace sbp
