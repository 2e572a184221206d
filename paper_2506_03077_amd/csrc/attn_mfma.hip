// bf16 MFMA chunk attention for gfx950 (head_dim 128): forward, dQ and dK/dV.
//
// Query row t of the chunk sits at global position q_start + t and sees keys
// 0 .. q_start + t of the cached prefix (paper Sec. 3.2.2, partitioned attention;
// Property 3.1).  Key tiles that lie entirely above the diagonal are skipped,
// tiles on the diagonal are masked by an integer comparison of positions, rows
// past q_start + q_len of K/V are never read.  Two more mask rules are index
// arithmetic of the same kind (the paper's mask M covers "padding / sliding
// window"): window > 0 limits a query at position t to the keys t - window < u <= t,
// and kv_first hides the key positions before it (padding in front of the
// sequence); key tiles wholly outside a wave's range are skipped on the left edge
// just as on the right one, and a query that sees no key gets o = 0, lse = -inf
// and sends no gradient.
//
// All three kernels use the "transposed score" formulation on the 32x32x16
// MFMA: S^T[key, query] = K Q^T.  The accumulator layout then gives every lane
// ONE query (column l%32) and 16 keys per 32-key block, so row max / row sum
// are in-register plus one cross-half exchange, and exp(S^T) is already in the
// register layout of the B operand of the next product (P^T as [key, query]
// with keys as the reduction index) - probabilities never touch LDS.  The
// reduction-index permutation this implies (slot j of half h <-> key
// 16*ks + 8*(j>>2) + 4*h + (j&3)) is matched on the A side by the transposing
// LDS load (ds_read_b64_tr_b16) that fetches V^T / K^T / Q^T / dO^T fragments
// from tiles kept in their natural [row][head_dim] layout.
//
//  forward : workgroup = 256 queries of one query head, 8 waves x 32 queries;
//            K and V tiles of 64 keys stream HBM -> LDS (direct-to-LDS, double
//            buffered); online softmax in the exp2 domain.
//  dQ      : same decomposition; recomputes P from the saved log-sum-exp;
//            dQ^T += K^T dS^T.
//  dK/dV   : workgroup = 128 keys of one KV head, 4 key blocks x 2 roles: one wave of
//            a block computes P and dV^T += dO^T P, its partner dP, dS and
//            dK^T += Q^T dS (P crosses through LDS); loops over the query tiles at
//            or below the diagonal and over the query heads of the group, Q and dO
//            tiles of 64 queries stream through LDS; results are added to the fp32
//            prefix accumulators (every element has one owner: no atomics,
//            reproducible).
#include "launch.h"
#include "device.h"

#include <type_traits>

#include <algorithm>

namespace sbp {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LDS_AS(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int DH = 128;                  // head_dim of the MFMA path
constexpr int ROW_BYTES = DH * 2;        // 256 B per tile row
constexpr int AT_THREADS = 512;          // 8 waves (forward, dQ): 2 per SIMD
constexpr int TQ = ATTN_TILE_Q;          // queries per workgroup (fwd, dQ): 8 waves x 32
constexpr int TK = ATTN_TILE_K;          // 64 keys per step (fwd, dQ)
constexpr int KV_TILE = 128;             // keys per workgroup (dK/dV): 4 key blocks x 2 roles = 8 waves
constexpr int KV_THREADS = 512;
constexpr int QT = 64;                   // queries per step (dK/dV)
constexpr int TILE64_BYTES = 64 * ROW_BYTES;   // 16 KiB
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// LDS tile [rows][128 bf16], 16 chunks of 16 B per row, chunk ^= f(row) with
// f(row) = ((row&3)<<2)|((row>>2)&3): conflict-free both for 128-bit row-fragment
// reads (16 consecutive rows, same chunk) and for the transposing 64-bit reads
// (4 consecutive rows x 32 B).
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * ROW_BYTES + ((chunk ^ swz(row)) << 4); }

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int ks) {
  bf16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (bf16_t)v[8 * ks + j];
  return o;
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// ---- address work hoisted out of the tile loops --------------------------------------------------------------
// In the tile loops every vector-ALU instruction competes with the softmax arithmetic for the SIMD's VALU issue
// slots, so nothing there computes an address: the per-lane byte offsets of the fragment reads inside a 64-row
// tile and of the direct-to-LDS loads are computed once per kernel, every tile / row block / stage is reached
// with immediate offsets, and the global side is an SGPR base plus those per-lane offsets.
struct FragPre {
  uint32_t rows[8];   // frag_rows: k16 step ks of row block 0            (row block b: + b * 32 * ROW_BYTES)
  uint32_t tr[8];     // frag_cols_tr: [i * 2 + hi], head_dim block i, tile rows +0 / +8, row_base 0 (+ row_base * ROW_BYTES)
};
__device__ __forceinline__ FragPre frag_pre(uint32_t lds_base /* LDS address of tile 0 */) {
  const int l = threadIdx.x & 63;
  FragPre f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) f.rows[ks] = pin(lds_base + (uint32_t)tile_off(l & 31, ks * 2 + (l >> 5)));
  const int p = l & 15, g = l >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int col = i * 32 + 16 * (g & 1) + 4 * (p & 3);
      const int row = 4 * (g >> 1) + (p >> 2) + 8 * hi;
      f.tr[i * 2 + hi] = pin(lds_base + (uint32_t)(tile_off(row, col >> 3) + ((col & 7) << 1)));
    }
  return f;
}
__device__ __forceinline__ bf16x8 lds_b128(uint32_t addr) {
  return *(const bf16x8*)(__attribute__((address_space(3))) const char*)(uintptr_t)addr;
}
__device__ __forceinline__ bf16x8 lds_tr(uint32_t lo_addr, uint32_t hi_addr) {
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(uintptr_t)lo_addr);
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(uintptr_t)hi_addr);
  short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

// Direct-to-LDS load of a 64-row tile by NT threads: rows 0..63 of a [*, stride] bf16 matrix starting at `g`
// (uniform pointer to the tile's first row, first of its 128 columns).  rows_valid = rows that exist from `g` on:
// a tile that runs past the end (only the last one) clamps its row indices so that nothing out of range is read.
template <int NT>
struct TileLoad { uint32_t voff[1024 / NT]; };
template <int NT>
__device__ __forceinline__ uint32_t tile_load_offset(int i, int64_t stride, int rows_valid) {
  const int id = i * NT + (int)threadIdx.x;
  const int row = id >> 4, pc = id & 15;
  const int chunk = pc ^ swz(row);
  return (uint32_t)(((int64_t)min(row, rows_valid - 1) * stride + chunk * 8) * 2);
}
template <int NT>
__device__ __forceinline__ TileLoad<NT> tile_load_pre(int64_t stride) {
  TileLoad<NT> t;
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) t.voff[i] = pin(tile_load_offset<NT>(i, stride, 64));
  return t;
}
template <int NT>
__device__ __forceinline__ void dma_tile64(const TileLoad<NT>& t, const bf16_t* g, int64_t stride, int rows_valid, uint32_t lds_tile) {
  const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile + (uint32_t)(threadIdx.x & ~63) * 16u);
  if (rows_valid >= 64) {
#pragma unroll
    for (int i = 0; i < 1024 / NT; ++i) dma16((const char*)g, t.voff[i], dst + (uint32_t)(i * NT * 16));
  } else {
#pragma unroll
    for (int i = 0; i < 1024 / NT; ++i) dma16((const char*)g, tile_load_offset<NT>(i, stride, rows_valid), dst + (uint32_t)(i * NT * 16));
  }
}

// A chain of N MFMAs whose A operands come from LDS: the fragment of step i+DEPTH is requested before the MFMA of
// step i issues (ring of DEPTH+1 fragments), and scheduling barriers keep that order - left alone, the compiler
// sinks every LDS read to just before its MFMA and the wave eats one LDS latency per MFMA.
template <int N, int DEPTH = 3, typename LoadF, typename MmaF>
__device__ __forceinline__ void mfma_chain(LoadF load, MmaF mma) {
  bf16x8 f[DEPTH + 1];
#pragma unroll
  for (int i = 0; i < DEPTH && i < N; ++i) f[i] = load(i);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + DEPTH < N) f[(i + DEPTH) % (DEPTH + 1)] = load(i + DEPTH);
    __builtin_amdgcn_sched_barrier(0);
    mma(i, f[i % (DEPTH + 1)]);
    __builtin_amdgcn_sched_barrier(0);
  }
}
#define WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0f70)

// row index (within a 32-row accumulator block) held in register r of a lane in half h
__device__ __forceinline__ int acc_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// ------------------------------------------------------------------ forward --
// 8 waves x 32 queries; K/V tiles of 64 keys stream through two LDS stages.  The softmax denominator is taken from
// the matrix pipe as well (one extra MFMA per k16 step against an all-ones operand sums the rounded probabilities
// of each query), which takes 32 additions per tile off the vector ALU - the busier of the two units here.
__global__ __launch_bounds__(AT_THREADS) void attn_fwd_mfma_k(bf16_t* q, const bf16_t* __restrict__ k,
                                                                 const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                                 float* __restrict__ lse, int Hq, int Hkv, int q_start,
                                                                 int c, float scale, const float2* __restrict__ rope,
                                                                 int window, int kv_first) {
  __shared__ __attribute__((aligned(1024))) char sT[4][TILE64_BYTES];   // stage st: K = sT[2 st], V = sT[2 st + 1]

  const int q0 = blockIdx.x * TQ, h = blockIdx.y, kvh = h / (Hq / Hkv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int qw0 = q0 + wave * 32;
  const int my_q = qw0 + (lane & 31);
  const bool q_valid = my_q < c;
  const int q_row = min(my_q, c - 1);
  const int qpos = q_start + q_row;
  const int64_t kv_stride = (int64_t)Hkv * DH;
  const bf16_t* kbase = k + (int64_t)kvh * DH;
  const bf16_t* vbase = v + (int64_t)kvh * DH;
  const int n_total = q_start + c;                                    // rows of K/V that exist for this chunk
  const int n_keys = q_start + min(q0 + TQ, c);                       // keys visible to the workgroup
  const int n_tiles = (n_keys + TK - 1) / TK;
  const int wave_last_key = q_start + min(qw0 + 32, c) - 1;           // last key any query of this wave sees
  const int wave_first_qpos = q_start + qw0;
  // left edge of the visible range: first visible key of a query at position p
  auto first_key = [&](int p) { return max(kv_first, window > 0 ? p - window + 1 : 0); };
  const int lo_q = first_key(qpos);                                   // of this lane's query
  const int wave_lo_min = first_key(wave_first_qpos);                 // lowest first key in the wave (its first query)
  const int wave_lo_max = first_key(wave_last_key);                   // highest one (its last query)
  const int kt0 = first_key(q_start + q0) / TK;                       // first key tile any query of the workgroup sees

  const uint32_t lds0 = lds_addr(&sT[0][0]);
  const FragPre fp = frag_pre(lds0);
  const TileLoad<AT_THREADS> tl = tile_load_pre<AT_THREADS>(kv_stride);

  bf16x8 bq[8];
  {
    bf16_t* qp = q + ((int64_t)q_row * Hq + h) * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) bq[ks] = *(const bf16x8*)(qp + ks * 16);
    if (rope) {
      // Rotary embedding of the query on load: the lane holds elements ks*16 + half*8 + e of its query, and the
      // rotate-half partner of element j < 64 is j + 64, i.e. the same e of fragment ks + 4 of the same lane.  The
      // rotated row is written back so that the backward kernels, which read q through LDS, find it rotated.
      const float2* tr = rope + (int64_t)q_row * (DH / 2) + half * 8;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 cs = tr[ks * 16 + e];
          const float x1 = (float)bq[ks][e], x2 = (float)bq[ks + 4][e];
          bq[ks][e] = (bf16_t)(x1 * cs.x - x2 * cs.y);
          bq[ks + 4][e] = (bf16_t)(x2 * cs.x + x1 * cs.y);
        }
      if (q_valid) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) *(bf16x8*)(qp + ks * 16) = bq[ks];
      }
    }
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)1.0f;
  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc_o[i] = zero16();
  f32x16 acc_l = zero16();      // every register of a lane: sum over the keys so far of the probabilities of its query
  float m_run = -INFINITY;
  const float sl = scale * LOG2E;

  auto step = [&](int kt, auto stage) {
    constexpr uint32_t oK = decltype(stage)::value * 2 * TILE64_BYTES, oV = oK + TILE64_BYTES;
    const int k0 = kt * TK;
    if (qw0 >= c || k0 > wave_last_key || k0 + TK - 1 < wave_lo_min) return;   // nothing visible to this wave in the tile
    f32x16 s[2];
    s[0] = zero16();
    s[1] = zero16();
    mfma_chain<16>([&](int i) { return lds_b128(fp.rows[i & 7] + oK + (i >> 3) * 32 * ROW_BYTES); },
                   [&](int i, const bf16x8& f) { s[i >> 3] = MFMA(f, bq[i & 7], s[i >> 3]); });
    const bool diag = k0 + TK - 1 > wave_first_qpos || k0 < wave_lo_max;   // some (query, key) pair of the wave is masked
    if (diag) {                                           // wave-uniform: only tiles on an edge of the visible range pay for the mask
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + b * 32 + acc_row(r, half);
          if (key > qpos || key < lo_q) s[b][r] = -INFINITY;
        }
    }
    float mx = s[0][0];                                   // max of the raw scores (scale > 0 keeps the order)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sl;
    // The running max (and with it the rescale of O) only moves when some query of the wave sees a new maximum.
    if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);   // a query that has seen no key yet keeps its zeros
      m_run = m_new;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_l[r] *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
    }
    const float m_sub = m_run == -INFINITY ? 0.0f : m_run;    // all scores so far masked: exp2(-inf - 0) = 0, not exp2(-inf + inf)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[b][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], sl, -m_sub));
    bf16x8 pb[4];     // P^T of the tile as four B operands: index = block * 2 + k16 step
#pragma unroll
    for (int j = 0; j < 4; ++j) pb[j] = pack8(s[j >> 1], j & 1);
    mfma_chain<16>([&](int i) { return lds_tr(fp.tr[(i & 3) * 2] + oV + (i >> 2) * 16 * ROW_BYTES, fp.tr[(i & 3) * 2 + 1] + oV + (i >> 2) * 16 * ROW_BYTES); },
                   [&](int i, const bf16x8& f) {
                     acc_o[i & 3] = MFMA(f, pb[i >> 2], acc_o[i & 3]);
                     if ((i & 3) == 3) acc_l = MFMA(ones, pb[i >> 2], acc_l);
                   });
  };
  auto issue = [&](int kt, int st) {
    const int64_t row0 = (int64_t)kt * TK;
    dma_tile64(tl, kbase + row0 * kv_stride, kv_stride, n_total - kt * TK, lds0 + (uint32_t)(st * 2 * TILE64_BYTES));
    dma_tile64(tl, vbase + row0 * kv_stride, kv_stride, n_total - kt * TK, lds0 + (uint32_t)((st * 2 + 1) * TILE64_BYTES));
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  if (kt0 < n_tiles) issue(kt0, 0);
  for (int kt = kt0; kt < n_tiles; kt += 2) {
    WAIT_VM0();
    __syncthreads();
    if (kt + 1 < n_tiles) issue(kt + 1, 1);
    step(kt, S0{});
    if (kt + 1 < n_tiles) {
      WAIT_VM0();
      __syncthreads();
      if (kt + 2 < n_tiles) issue(kt + 2, 0);
      step(kt + 1, S1{});
    }
  }

  const float l_tot = acc_l[0];
  if (q_valid) {
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.0f;      // a query that saw no key: o = 0, lse = -inf
    bf16_t* op = o + ((int64_t)my_q * Hq + h) * DH;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(acc_o[i][4 * a + e] * inv);
        *(bf16x4*)(op + i * 32 + 8 * a + 4 * half) = w;
      }
    if (half == 0) lse[(int64_t)h * c + my_q] = l_tot > 0.f ? (m_run + log2f(l_tot)) * LN2 : -INFINITY;
  }
}

// ----------------------------------------------------------------------- dQ --
__global__ __launch_bounds__(AT_THREADS) void attn_bwd_dq_mfma_k(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                                    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
                                                                    const float* __restrict__ lse, const float* __restrict__ delta,
                                                                    bf16_t* __restrict__ dq, int Hq, int Hkv, int q_start, int c,
                                                                    float scale, const float2* __restrict__ rope, int window,
                                                                    int kv_first) {
  __shared__ __attribute__((aligned(1024))) char sT[4][TILE64_BYTES];   // stage st: K = sT[2 st], V = sT[2 st + 1]

  const int q0 = blockIdx.x * TQ, h = blockIdx.y, kvh = h / (Hq / Hkv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int qw0 = q0 + wave * 32;
  const int my_q = qw0 + (lane & 31);
  const bool q_valid = my_q < c;
  const int q_row = min(my_q, c - 1);
  const int qpos = q_start + q_row;
  const int64_t kv_stride = (int64_t)Hkv * DH;
  const bf16_t* kbase = k + (int64_t)kvh * DH;
  const bf16_t* vbase = v + (int64_t)kvh * DH;
  const int n_total = q_start + c;
  const int n_keys = q_start + min(q0 + TQ, c);
  const int n_tiles = (n_keys + TK - 1) / TK;
  const int wave_last_key = q_start + min(qw0 + 32, c) - 1;
  const int wave_first_qpos = q_start + qw0;
  auto first_key = [&](int p) { return max(kv_first, window > 0 ? p - window + 1 : 0); };   // left edge of the visible range
  const int lo_q = first_key(qpos);
  const int wave_lo_min = first_key(wave_first_qpos), wave_lo_max = first_key(wave_last_key);
  const int kt0 = first_key(q_start + q0) / TK;

  const uint32_t lds0 = lds_addr(&sT[0][0]);
  const FragPre fp = frag_pre(lds0);
  const TileLoad<AT_THREADS> tl = tile_load_pre<AT_THREADS>(kv_stride);

  bf16x8 bq[8], bdo[8];
  {
    const int64_t off = ((int64_t)q_row * Hq + h) * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) { bq[ks] = *(const bf16x8*)(q + off + ks * 16); bdo[ks] = *(const bf16x8*)(d_o + off + ks * 16); }
  }
  const float lse_q = lse[(int64_t)h * c + q_row];
  const float lse2 = lse_q == -INFINITY ? 0.0f : lse_q * LOG2E;    // a query that saw no key: every score is masked, p = exp2(-inf) = 0
  const float dlt = delta[(int64_t)h * c + q_row];
  const float sl = scale * LOG2E;
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = zero16();

  auto step = [&](int kt, auto stage) {
    constexpr uint32_t oK = decltype(stage)::value * 2 * TILE64_BYTES, oV = oK + TILE64_BYTES;
    const int k0 = kt * TK;
    if (qw0 >= c || k0 > wave_last_key || k0 + TK - 1 < wave_lo_min) return;
    const bool diag = k0 + TK - 1 > wave_first_qpos || k0 < wave_lo_max;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      f32x16 s = zero16(), dp = zero16();
      mfma_chain<16>([&](int i) { return lds_b128(fp.rows[i & 7] + (i < 8 ? oK : oV) + b * 32 * ROW_BYTES); },
                     [&](int i, const bf16x8& f) { if (i < 8) s = MFMA(f, bq[i], s); else dp = MFMA(f, bdo[i - 8], dp); });
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + b * 32 + acc_row(r, half);
          if (key > qpos || key < lo_q) s[r] = -INFINITY;     // exp2(-inf) = 0
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], sl, -lse2));
        s[r] = p * (dp[r] - dlt);                              // dS^T (the factor `scale` is applied at the end)
      }
      bf16x8 db[2];
      db[0] = pack8(s, 0);
      db[1] = pack8(s, 1);
      mfma_chain<8>([&](int i) { return lds_tr(fp.tr[(i & 3) * 2] + oK + (b * 32 + (i >> 2) * 16) * ROW_BYTES, fp.tr[(i & 3) * 2 + 1] + oK + (b * 32 + (i >> 2) * 16) * ROW_BYTES); },
                    [&](int i, const bf16x8& f) { acc[i & 3] = MFMA(f, db[i >> 2], acc[i & 3]); });
    }
  };
  auto issue = [&](int kt, int st) {
    const int64_t row0 = (int64_t)kt * TK;
    dma_tile64(tl, kbase + row0 * kv_stride, kv_stride, n_total - kt * TK, lds0 + (uint32_t)(st * 2 * TILE64_BYTES));
    dma_tile64(tl, vbase + row0 * kv_stride, kv_stride, n_total - kt * TK, lds0 + (uint32_t)((st * 2 + 1) * TILE64_BYTES));
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  if (kt0 < n_tiles) issue(kt0, 0);
  for (int kt = kt0; kt < n_tiles; kt += 2) {
    WAIT_VM0();
    __syncthreads();
    if (kt + 1 < n_tiles) issue(kt + 1, 1);
    step(kt, S0{});
    if (kt + 1 < n_tiles) {
      WAIT_VM0();
      __syncthreads();
      if (kt + 2 < n_tiles) issue(kt + 2, 0);
      step(kt + 1, S1{});
    }
  }

  if (q_valid) {
    bf16_t* op = dq + ((int64_t)my_q * Hq + h) * DH;
    if (rope) {
      // adjoint of the rotary embedding on the way out: element j < 64 (accumulator block i < 2) pairs with j + 64
      // (block i + 2, same register of the same lane); rotation by the negative angle
      const float2* tr = rope + (int64_t)my_q * (DH / 2) + 4 * half;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          bf16x4 w1, w2;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float2 cs = tr[i * 32 + 8 * a + e];
            const float d1 = acc[i][4 * a + e] * scale, d2 = acc[i + 2][4 * a + e] * scale;
            w1[e] = (bf16_t)(d1 * cs.x + d2 * cs.y);
            w2[e] = (bf16_t)(d2 * cs.x - d1 * cs.y);
          }
          *(bf16x4*)(op + i * 32 + 8 * a + 4 * half) = w1;
          *(bf16x4*)(op + (i + 2) * 32 + 8 * a + 4 * half) = w2;
        }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(acc[i][4 * a + e] * scale);
          *(bf16x4*)(op + i * 32 + 8 * a + 4 * half) = w;
        }
    }
  }
}

// -------------------------------------------------------------------- dK/dV --
// Workgroup = 128 keys of one KV head, 8 waves = 4 key blocks of 32 x 2 roles, so that each SIMD holds the two
// waves of one key block:
//   role P (waves 0-3): S = Q K^T -> P = exp2(S*sl - lse) (masked), rounded to bf16 -> leaves P in LDS for its
//                       partner -> dV^T += dO^T P
//   role S (waves 4-7): dP = dO V^T -> takes P -> dS = P * (dP - delta) -> dK^T += Q^T dS
// Each role keeps only its own operand fragments (K or V) and its own accumulator (dV or dK) in registers:
// half the registers of a do-everything wave, so two waves fit per SIMD.  Role S runs one tile behind role P:
// in step j role P works on tile j while role S works on tile j-1, whose P is already in LDS, so inside a step
// the two waves of a SIMD never wait for each other and the exponentials of one overlap the MFMAs of the other.
// That takes three stages of the Q / dO tiles (tile j+1 in flight, j and j-1 in use) and two of P.
// The loop walks the query tiles at or below the diagonal and, for each, the query heads of the group.
constexpr int KV_STAGES = 3;

__global__ __launch_bounds__(KV_THREADS) void attn_bwd_dkv_mfma_k(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                                  const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
                                                                  const float* __restrict__ lse2, const float* __restrict__ delta,
                                                                  float* __restrict__ dk, float* __restrict__ dv, int Hq, int Hkv,
                                                                  int q_start, int c, float scale, int window, int kv_first,
                                                                  int key_block0) {
  __shared__ __attribute__((aligned(1024))) char sQD[KV_STAGES][2][TILE64_BYTES];   // [stage][Q | dO]
  __shared__ __attribute__((aligned(16))) bf16x8 sP[2][4][4][64];   // [tile parity][key block][query block * 2 + k16 step][lane]
  __shared__ __attribute__((aligned(16))) float sL[KV_STAGES][QT];  // log2-domain log-sum-exp of the tile's queries
  __shared__ __attribute__((aligned(16))) float sDl[KV_STAGES][QT]; // delta of the tile's queries

  const int G = Hq / Hkv;
  const int key0 = (key_block0 + (int)blockIdx.x) * KV_TILE, kvh = blockIdx.y;   // key blocks before key_block0 are visible to no query
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int kb = wave & 3;
  const bool role_p = wave < 4;
  const int n_total = q_start + c;
  const int kw0 = key0 + kb * 32;
  const int my_key = kw0 + (lane & 31);
  const int key_row = min(my_key, n_total - 1);
  const int64_t kv_stride = (int64_t)Hkv * DH;
  const int64_t q_stride = (int64_t)Hq * DH;

  // Fragment addresses: one set reaches 64 KiB (stages 0 and 1), a second one stage 2.  Role P reads Q row-wise and
  // dO transposed, role S the other way round; only the half of each set that the role uses stays live.
  const uint32_t lds0 = lds_addr(&sQD[0][0][0]);
  const FragPre f0 = frag_pre(lds0 + (role_p ? 0 : TILE64_BYTES));                 // row-wise operand: Q (P) / dO (S)
  const FragPre g0 = frag_pre(lds0 + (role_p ? TILE64_BYTES : 0));                 // transposed operand: dO (P) / Q (S)
  const FragPre f2 = frag_pre(lds0 + 2 * 2 * TILE64_BYTES + (role_p ? 0 : TILE64_BYTES));
  const FragPre g2 = frag_pre(lds0 + 2 * 2 * TILE64_BYTES + (role_p ? TILE64_BYTES : 0));
  const TileLoad<KV_THREADS> tl = tile_load_pre<KV_THREADS>(q_stride);
  const uint32_t sp_lane = pin(lds_addr(&sP[0][kb][0][lane]));                      // + parity * 8192 + (b * 2 + ks) * 1024
  const uint32_t stat_lane = pin(lds_addr(role_p ? &sL[0][4 * half] : &sDl[0][4 * half]));   // + stage * 256 + (b * 32 + 8 a) * 4

  bf16x8 breg[8];   // B operand of the first product: K rows (role P) or V rows (role S) of my key
  {
    const bf16_t* src = (role_p ? k : v) + (int64_t)key_row * kv_stride + (int64_t)kvh * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) breg[ks] = *(const bf16x8*)(src + ks * 16);
  }
  const float sl = scale * LOG2E;

  // query tiles that can see at least one key of this workgroup: query position >= key0
  // ... and, under a sliding window, query position <= last key of the workgroup + window - 1
  const int qt_first = max(0, key0 - q_start) / QT;
  int n_qt = (c + QT - 1) / QT;
  if (window > 0) n_qt = min(n_qt, max(0, key0 + KV_TILE - 1 + window - 1 - q_start) / QT + 1);
  const int n_iter = max(0, n_qt - qt_first) * G;

  auto issue = [&](int it, int stage) {
    const int qt = qt_first + it / G, hh = kvh * G + it % G;
    const int64_t corner = (int64_t)qt * QT * q_stride + (int64_t)hh * DH;
    dma_tile64(tl, q + corner, q_stride, c - qt * QT, lds0 + (uint32_t)(stage * 2 * TILE64_BYTES));
    dma_tile64(tl, d_o + corner, q_stride, c - qt * QT, lds0 + (uint32_t)((stage * 2 + 1) * TILE64_BYTES));
    if (wave < 2) {   // 64 log-sum-exp values (wave 0) and 64 deltas (wave 1), 4 B per lane, also direct to LDS
      const int row = min(qt * QT + lane, c - 1);
      dma4(uniform_ptr((wave == 0 ? lse2 : delta) + (int64_t)hh * c), (uint32_t)row * 4u,
           __builtin_amdgcn_readfirstlane(lds_addr(wave == 0 ? &sL[stage][0] : &sDl[stage][0])));
    }
  };
  // One 64-query tile = two 32-query blocks.  `active`: the wave has a valid key and some query of the tile is
  // at or after its first key (the same answer for both waves of a key block).
  auto tile_active = [&](int qbase) {
    return kw0 < n_total && q_start + min(qbase + QT, c) - 1 >= kw0 && kw0 + 31 >= kv_first &&
           (window == 0 || q_start + qbase - window < kw0 + 31);     // the tile's first query still reaches the wave's last key
  };
  auto lds_f4 = [](uint32_t addr) { return *(const float4*)(__attribute__((address_space(3))) const char*)(uintptr_t)addr; };

  auto p_step = [&](f32x16 (&acc)[4], int it, auto stage_c, int par) __attribute__((always_inline)) {
    constexpr int stage = decltype(stage_c)::value;
    constexpr uint32_t so = (stage & 1) * 2 * TILE64_BYTES;        // offset of the stage from its address set
    const FragPre& fr = stage < 2 ? f0 : f2;
    const FragPre& gt = stage < 2 ? g0 : g2;
    const int qbase = (qt_first + it / G) * QT;
    if (!tile_active(qbase)) return;
    const bool diag = (q_start + qbase < kw0 + 31) || (qbase + QT > c) || kw0 < kv_first ||   // some pair masked, or ragged query tile
                      (window > 0 && q_start + qbase + QT - 1 - window >= kw0);
    const uint32_t sp = sp_lane + (uint32_t)par * (uint32_t)sizeof(sP[0]);
#pragma unroll
    for (int b = 0; b < 2; ++b) {      // one 32-query block at a time: fewer live registers
      f32x16 t = zero16();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) t = MFMA(lds_b128(fr.rows[ks] + so + b * 32 * ROW_BYTES), breg[ks], t);
      // accumulator: column = my key, rows = queries qbase + b*32 + acc_row(r, half)
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qi = qbase + b * 32 + acc_row(r, half);
          if (qi >= c || my_key > q_start + qi || my_key < kv_first || (window > 0 && my_key <= q_start + qi - window))
            t[r] = -INFINITY;                                          // exp2(-inf) = 0
        }
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const float4 l4 = lds_f4(stat_lane + stage * QT * 4 + (b * 32 + 8 * a) * 4);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) t[4 * a + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(t[4 * a + e], sl, -lv[e]));
      }
      bf16x8 pb[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        pb[ks] = pack8(t, ks);
        *(bf16x8*)(__attribute__((address_space(3))) char*)(uintptr_t)(sp + (b * 2 + ks) * 1024) = pb[ks];
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i] = MFMA(lds_tr(gt.tr[i * 2] + so + (b * 32 + ks * 16) * ROW_BYTES, gt.tr[i * 2 + 1] + so + (b * 32 + ks * 16) * ROW_BYTES),
                        pb[ks], acc[i]);
    }
  };

  auto s_step = [&](f32x16 (&acc)[4], int it, auto stage_c, int par) __attribute__((always_inline)) {
    constexpr int stage = decltype(stage_c)::value;
    constexpr uint32_t so = (stage & 1) * 2 * TILE64_BYTES;
    const FragPre& fr = stage < 2 ? f0 : f2;
    const FragPre& gt = stage < 2 ? g0 : g2;
    const int qbase = (qt_first + it / G) * QT;
    if (!tile_active(qbase)) return;
    const uint32_t sp = sp_lane + (uint32_t)par * (uint32_t)sizeof(sP[0]);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      f32x16 t = zero16();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) t = MFMA(lds_b128(fr.rows[ks] + so + b * 32 * ROW_BYTES), breg[ks], t);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const float4 d0 = lds_f4(stat_lane + stage * QT * 4 + (b * 32 + 16 * ks) * 4);
        const float4 d1 = lds_f4(stat_lane + stage * QT * 4 + (b * 32 + 16 * ks + 8) * 4);
        const float dl[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
        const bf16x8 p8 = lds_b128(sp + (b * 2 + ks) * 1024);
#pragma unroll
        for (int j = 0; j < 8; ++j)     // dS (the softmax scale is applied once at the end)
          t[8 * ks + j] = (float)p8[j] * (t[8 * ks + j] - dl[j]);
        const bf16x8 db = pack8(t, ks);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i] = MFMA(lds_tr(gt.tr[i * 2] + so + (b * 32 + ks * 16) * ROW_BYTES, gt.tr[i * 2 + 1] + so + (b * 32 + ks * 16) * ROW_BYTES), db, acc[i]);
      }
    }
  };

  // Step j: tile j+1 goes in flight, role P takes tile j, role S takes tile j-1.  The barrier at the top says:
  // tile j has landed for everyone, P of tile j-1 is written, and the stage and the P slot about to be
  // overwritten (those of tile j-2) are no longer read.  Tile j lives in stage j % 3; the loop is unrolled by three
  // so that every stage offset is an immediate.
  // The whole loop exists once per role (the role is a compile-time constant inside it): with one loop and a role
  // branch in its body the register allocator gives the accumulator different homes in the two branches and copies
  // all 64 registers in and out at every step.  Both copies execute the same number of barriers.
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  using S2 = std::integral_constant<int, 2>;
  auto run = [&](auto role_c) __attribute__((always_inline)) {
    constexpr bool RP = decltype(role_c)::value;
    f32x16 acc[4];   // dV^T (role P) or dK^T (role S): rows = head_dim, column = my key
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = zero16();
    auto body = [&](int j, auto st_p, auto st_s, int st_next) __attribute__((always_inline)) {
      WAIT_VM0();
      __syncthreads();
      if (j + 1 < n_iter) issue(j + 1, st_next);
      if constexpr (RP) {
        if (j < n_iter) p_step(acc, j, st_p, j & 1);
      } else {
        if (j > 0 && j <= n_iter) s_step(acc, j - 1, st_s, (j - 1) & 1);
      }
    };
    if (n_iter > 0) {
      issue(0, 0);
      // always whole groups of three steps (a step past the last tile is a barrier and nothing else): a loop with
      // exits between the unrolled steps makes the compiler shuttle the accumulator between register sets
      for (int j = 0; j <= n_iter; j += 3) {
        body(j, S0{}, S2{}, 1);
        body(j + 1, S1{}, S0{}, 2);
        body(j + 2, S2{}, S1{}, 0);
      }
    }
    if (my_key < n_total) {
      float* out = (RP ? dv : dk) + (int64_t)my_key * kv_stride + (int64_t)kvh * DH;
      const float f = RP ? 1.0f : scale;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const int d0 = i * 32 + 8 * a + 4 * half;
          float4 u = *(float4*)(out + d0);
          u.x += acc[i][4 * a + 0] * f; u.y += acc[i][4 * a + 1] * f; u.z += acc[i][4 * a + 2] * f; u.w += acc[i][4 * a + 3] * f;
          *(float4*)(out + d0) = u;
        }
    }
  };
  if (role_p) run(std::true_type{});
  else run(std::false_type{});
}

// delta[h, t] = sum_j d_o[t,h,j] * o[t,h,j]  (one wave per (t, h))
// also lse2[h, t] = lse[h, t] * log2(e), the form the dK/dV kernel's exp2 wants (one multiply per (t, h) here
// instead of one per score there)
__global__ __launch_bounds__(256) void attn_delta_mfma_k(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o,
                                                         const float* __restrict__ lse, float* __restrict__ delta,
                                                         float* __restrict__ lse2, int Hq, int c) {
  const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // t * Hq + h
  if (pair >= (int64_t)c * Hq) return;
  const int lane = threadIdx.x & 63;
  const int t = (int)(pair / Hq), h = (int)(pair % Hq);
  const int64_t base = pair * DH + lane * 2;
  float s = (float)o[base] * (float)d_o[base] + (float)o[base + 1] * (float)d_o[base + 1];
  s = wave_sum(s);
  if (lane == 0) {
    delta[(int64_t)h * c + t] = s;
    const float l = lse[(int64_t)h * c + t];
    lse2[(int64_t)h * c + t] = l == -INFINITY ? 0.0f : l * LOG2E;   // a query that saw no key: its scores are all masked anyway
  }
}

bool attn_mfma_eligible(int dt, int dh, int Hq, int Hkv) { return dt == DT_BF16 && dh == DH && Hq % Hkv == 0; }

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// the MFMA kernels move 16 bytes per lane: every tensor they touch must be 16-byte aligned
bool attn_mfma_aligned(const AttnArgs& a, bool backward) {
  if (!aligned16(a.q) || !aligned16(a.k) || !aligned16(a.v) || !aligned16(a.o) || ((uintptr_t)a.rope_q & 7)) return false;
  return !backward || (aligned16(a.d_o) && aligned16(a.dq) && aligned16(a.dk) && aligned16(a.dv));
}

hipError_t attn_forward_mfma(const AttnArgs& a, hipStream_t st) {
  if (a.q_len == 0) return hipSuccess;
  dim3 grid((unsigned)cdiv(a.q_len, TQ), a.Hq);
  attn_fwd_mfma_k<<<grid, AT_THREADS, 0, st>>>((bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, (bf16_t*)a.o, a.lse,
                                               a.Hq, a.Hkv, a.q_start, a.q_len, a.scale, a.rope_q, a.window, a.kv_first);
  return hipGetLastError();
}

hipError_t attn_backward_mfma(const AttnArgs& a, hipStream_t st) {
  if (a.q_len == 0) return hipSuccess;
  const int64_t pairs = (int64_t)a.q_len * a.Hq;
  float* lse2 = a.delta + pairs;   // second half of the [2, Hq, c] scratch
  attn_delta_mfma_k<<<(unsigned)cdiv(pairs, 4), 256, 0, st>>>((const bf16_t*)a.o, (const bf16_t*)a.d_o, a.lse, a.delta, lse2, a.Hq,
                                                              a.q_len);
  dim3 gq((unsigned)cdiv(a.q_len, TQ), a.Hq);
  attn_bwd_dq_mfma_k<<<gq, AT_THREADS, 0, st>>>((const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, (const bf16_t*)a.d_o,
                                                a.lse, a.delta, (bf16_t*)a.dq, a.Hq, a.Hkv, a.q_start, a.q_len, a.scale, a.rope_q,
                                                a.window, a.kv_first);
  // key blocks that no query of the chunk can see (before the padding ends, or older than the first query's window)
  // are not launched: their dK/dV contribution is zero
  const int first_visible = std::max(a.kv_first, a.window > 0 ? a.q_start - a.window + 1 : 0);
  const int kb0 = std::max(0, first_visible) / KV_TILE, kb1 = (int)cdiv(a.q_start + a.q_len, KV_TILE);
  if (kb1 > kb0) {
    dim3 gk((unsigned)(kb1 - kb0), a.Hkv);
    attn_bwd_dkv_mfma_k<<<gk, KV_THREADS, 0, st>>>((const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, (const bf16_t*)a.d_o,
                                                   lse2, a.delta, a.dk, a.dv, a.Hq, a.Hkv, a.q_start, a.q_len, a.scale,
                                                   a.window, a.kv_first, kb0);
  }
  return hipGetLastError();
}

}  // namespace sbp
