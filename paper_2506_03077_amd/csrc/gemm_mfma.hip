// bf16 MFMA GEMM for gfx950, fp32 accumulation, three operand layouts:
//   NT  C[M,N] = A[M,K] B[N,K]^T     (forward projections: both operands K-contiguous)
//   NN  C[M,N] = A[M,K] B[K,N]       (input gradients dX = dY W)
//   TN  C[M,N] = A[K,M]^T B[K,N]     (weight gradients dW += dY^T X; K = chunk rows)
//
// Design (CDNA4):
//  * 256x256 output tile per workgroup, 8 wavefronts (2 x 4), each wave owns a
//    128x64 sub-tile = 4x2 v_mfma_f32_32x32x16_bf16 accumulators (128 registers).
//  * Operand tiles (256 x 64 bf16 each) go HBM -> LDS with 128-bit direct-to-LDS
//    loads (no VGPR staging), double-buffered: tile kt+1 streams in while tile kt
//    is consumed; one barrier per K step.
//  * K-contiguous operands are read from LDS with ds_read_b128; operands whose
//    reduction index is the slow dimension in memory are kept in their natural
//    [k][m|n] layout in LDS and fetched with the transposing LDS load
//    (ds_read_b64_tr_b16), so no transposed copy ever exists in HBM.
//  * The main loop contains no vector ALU instructions: a VALU instruction of one wave queues behind the MFMAs
//    of the SIMD's other wave, so per-load address arithmetic would stretch the issue of a tile's loads
//    several-fold.  Global addresses are an SGPR base (scalar adds per K step) + per-lane 32-bit offsets
//    computed once; LDS fragment addresses are computed once per stage and reached with immediate offsets.
//  * Both LDS layouts are XOR-swizzled (at 16-byte / 64-byte granularity) so that
//    the fragment reads are bank-conflict free; because a direct-to-LDS load
//    writes lane-linear, the swizzle is applied on the global-address side.
//  * Workgroups are renumbered so that each XCD (own L2) works on a contiguous
//    band of output tiles that share operand panels.
//  * Ragged M (last chunk) and ragged N (an output width that is a multiple of 8 but not of 256, e.g. a 151936-word
//    vocabulary) are handled by clamping loads and masking stores;
//    ragged K in the TN form (chunk rows) by clamping loads and zeroing the A
//    fragments of the out-of-range reduction rows.
//  * Optional split-K (a power of two, for outputs with too few tiles to fill the chip): partial tiles go to an
//    fp32 scratch and a small kernel sums them in a fixed order (deterministic) into C; each K slice is pinned to
//    its own group of XCDs.
//  * Weight gradients: C += by no-return fp32 atomic adds (one add per element per launch), or into a bf16 C by
//    paired loads / stores; several reduction segments (operand pairs) per output tile; grouped launches.
#include "launch.h"
#include "device.h"

#include <algorithm>

namespace sbp {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LDS_AS(p) ((__attribute__((address_space(3))) void*)(p))


constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NSTAGE = 2;                              // LDS ring of operand tiles; NSTAGE-1 tiles are in flight
constexpr int NWAVE_M = 2, NWAVE_N = 4;
constexpr int NTHREADS = NWAVE_M * NWAVE_N * 64;      // 512
constexpr int WTM = BM / NWAVE_M, WTN = BN / NWAVE_N;  // 128 x 64 per wave
constexpr int FM = WTM / 32, FN = WTN / 32;            // 4 x 2 MFMA tiles
constexpr int TILE_BYTES = BM * BK * 2;                // 32 KiB per operand tile
constexpr int LOADS_PER_THREAD = TILE_BYTES / 16 / NTHREADS;   // 4 x 16 B per operand
constexpr int LOADS_PER_TILE = 2 * LOADS_PER_THREAD;           // wave-level VMEM instructions per k-tile

// ---- K-contiguous operand: LDS [rows][BK], 128 B per row = 8 chunks of 16 B, chunk ^= (row>>1)&7:
//      16 consecutive rows at one logical chunk cover all 64 banks exactly once.
constexpr int CPR = BK / 8;                            // 16-byte chunks per row
__device__ __forceinline__ int kmaj_swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int kmaj_off(int row, int chunk) { return row * (BK * 2) + ((chunk ^ kmaj_swz(row)) << 4); }

// ---- reduction-major operand: LDS [BK][rows], 512 B per k-row, 64-byte groups ^= krow&7
__device__ __forceinline__ int mnmaj_off(int krow, int col /*element*/) {
  const int c16 = col >> 3;
  const int p16 = ((((c16 >> 2) ^ (krow & 7)) << 2) | (c16 & 3));
  return krow * (BM * 2) + (p16 << 4) + ((col & 7) << 1);
}

// Byte offset, relative to the tile's corner element, of load i (0..LOADS_PER_THREAD-1) of this thread's share.
//   KMAJ : corner = (row r0, column k0); rows clamped so that r0 + row <= r_max
//   MNMAJ: corner = (k-row k0, column r0); k-rows clamped so that k0 + krow <= k_max, columns so that r0 + col <= r_max
template <bool MNMAJ>
__device__ __forceinline__ uint32_t load_offset(int i, int64_t ld, int r0, int r_max, int k0, int k_max) {
  const int id = i * NTHREADS + (int)threadIdx.x;   // 16-byte slot in the tile, lane-linear within a wave
  if (!MNMAJ) {
    const int row = id / CPR, pc = id % CPR;
    const int chunk = pc ^ kmaj_swz(row);
    return (uint32_t)(((int64_t)(min(r0 + row, r_max) - r0) * ld + chunk * 8) * 2);
  } else {
    const int krow = id >> 5, p16 = id & 31;
    const int c16 = ((((p16 >> 2) ^ (krow & 7)) << 2) | (p16 & 3));
    // columns past the operand's last one (a ragged last tile; widths are multiples of 8) re-read its last 8 columns:
    // finite duplicates whose products land in rows / columns of C that the epilogue masks
    const int col = min(c16 * 8, r_max - r0 - 7);
    return (uint32_t)(((int64_t)(min(k0 + krow, k_max) - k0) * ld + col) * 2);
  }
}

// LDS byte offset (within an operand tile) of this lane's fragment read, for a 32-row block starting at row_base
// and k16 step kk.  K-major: one 128-bit read.  Reduction-major: two transposing 64-bit reads (k-rows +0 and +4).
__device__ __forceinline__ uint32_t frag_off_kmaj(int row_base, int kk) {
  const int l = threadIdx.x & 63;
  return (uint32_t)kmaj_off(row_base + (l & 31), kk * 2 + (l >> 5));
}
__device__ __forceinline__ uint32_t frag_off_mnmaj(int row_base, int kk, int hi) {
  const int l = threadIdx.x & 63;
  const int p = l & 15, g = l >> 4;
  const int col = row_base + 16 * (g & 1) + 4 * (p & 3);
  const int krow = kk * 16 + 8 * (g >> 1) + (p >> 2) + 4 * hi;
  return (uint32_t)mnmaj_off(krow, col);
}
typedef short short8v __attribute__((ext_vector_type(8)));
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
  return *(const bf16x8*)(__attribute__((address_space(3))) const char*)(uintptr_t)addr;
}
__device__ __forceinline__ bf16x8 lds_read_tr(uint32_t lo_addr, uint32_t hi_addr) {
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(uintptr_t)lo_addr);
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(uintptr_t)hi_addr);
  short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

// Tile id -> (tile_m, tile_n): walk tiles in column bands of group_m row tiles so that the workgroups resident
// together share A row panels and B column panels in their XCD's L2.
__device__ __forceinline__ void band_coords(int id, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
  const int band = group_m * tiles_n;
  const int g = id / band;
  const int first_m = g * group_m;
  const int gsz = min(tiles_m - first_m, group_m);
  const int r = id % band;
  tm = first_m + r % gsz;
  tn = r / gsz;
}
// Band height.  With XCD-contiguous ids each XCD works on a run of n_tiles/8 consecutive ids, i.e. a block of
// group_m rows x run/group_m columns of tiles; the fabric traffic of that XCD is proportional to rows + columns,
// so the block is made as square as the problem allows.  (Interleaved ids, used by the accumulate form, give
// every XCD one row of each band and all columns; 8 rows per band suit that.)
__device__ __forceinline__ int band_height_for_run(int tiles_m, int run) {
  int h = (int)(sqrtf((float)max(1, run)) + 0.5f);
  return max(1, min(h, min(tiles_m, 8)));
}
__device__ __forceinline__ int band_height(int tiles_m, int n_tiles, bool xcd_contiguous) {
  if (!xcd_contiguous) return 8;
  return band_height_for_run(tiles_m, n_tiles / 8);
}
// Hardware deals consecutive workgroups round-robin to the 8 XCDs (each with its own L2); undo that so each
// XCD gets a contiguous run of tile ids.  Measured: +3-4% for the store-only forms; the accumulate form (atomic adds
// into C) is 8% faster with the hardware's interleaved order, so it keeps that.
__device__ __forceinline__ int xcd_contiguous_id(int id, int n_tiles) {
  constexpr int NXCD = 8;
  const int x = id % NXCD, q = n_tiles / NXCD, r = n_tiles % NXCD;   // XCD x owns q (+1 if x < r) consecutive ids
  return x * q + min(x, r) + id / NXCD;
}

// vmcnt(n) with expcnt / lgkmcnt left unconstrained
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

// One 256x256 output tile: K range [k_begin, k_end).
// MODE: 0 = store fp32, 1 = store bf16, 2 = accumulate fp32 (C +=), 3 = split-K partial (fp32 store, C already offset),
//       4 = accumulate into a bf16 C (read, add in fp32, round once; weight-gradient form only),
//       5 = store fp32 and emit per-row (max, sum of exp) pairs over the tile's columns (`stats`)
//       6 = C is not stored: the tile is the gradient wrt act = silu(gate) * up and the epilogue writes act, d gate, d up
//       7 = like 5, but C (bf16) receives exp(c - block max) instead of c, and the value of each row's target column is kept
constexpr bool mode_accumulates(int mode) { return mode == 2 || mode == 4; }
constexpr bool mode_swaps_operands(int mode) { return mode == 5 || mode == 6 || mode == 7; }   // accumulators hold C^T blocks
struct SwigluFuse { bf16_t* gate; bf16_t* up; bf16_t* act; };
struct NumerFuse { const int32_t* targets; const int32_t* row_index; float* target_value; };
//
// The main loop is written so that it contains no vector ALU instructions at all: global addresses are an SGPR base
// (advanced with scalar adds) plus per-lane offsets computed once, LDS fragment addresses are computed once per
// stage and reached with immediate offsets, and the two LDS stages are unrolled.  Only the last K step of a ragged
// reduction (weight-gradient form) takes a slower path with clamped addresses and zeroed fragments.
// The reduction may come in several segments (operand pairs of the same shape and leading dimensions whose products
// are summed into the same output tile): one accumulator, one epilogue.
constexpr int MAX_SEG = 8;
struct KSegments {
  const bf16_t* A[MAX_SEG];
  const bf16_t* B[MAX_SEG];
  int K[MAX_SEG];         // reduction length of the segment (clamp for the loads)
  int k_begin[MAX_SEG];   // range of the segment this tile works on
  int k_end[MAX_SEG];
  int n;
};

template <bool TA, bool TB, int MODE>
__device__ __forceinline__ void gemm_tile(const KSegments& segs, void* __restrict__ Cv, int M, int N, int64_t lda,
                                          int64_t ldb, int64_t ldc, int tm, int tn, char (&smem)[NSTAGE][2][TILE_BYTES],
                                          float2* __restrict__ stats = nullptr, SwigluFuse sw = SwigluFuse{nullptr, nullptr, nullptr},
                                          NumerFuse nf = NumerFuse{nullptr, nullptr, nullptr}) {
  static_assert(NSTAGE == 2, "the main loop is unrolled over two LDS stages");
  constexpr bool AMN = TA, BMN = !TB;     // operand kept reduction-major in LDS (B stored [N,K] is the K-contiguous case)
  const int m0 = tm * BM, n0 = tn * BN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm0 = (wave / NWAVE_N) * WTM, wn0 = (wave % NWAVE_N) * WTN;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- global side: per-lane byte offsets (rows clamped once); the uniform 64-bit bases walk along K
  const int64_t stepA = (AMN ? (int64_t)BK * lda : (int64_t)BK) * 2, stepB = (BMN ? (int64_t)BK * ldb : (int64_t)BK) * 2;
  uint32_t offA[LOADS_PER_THREAD], offB[LOADS_PER_THREAD];
#pragma unroll
  for (int i = 0; i < LOADS_PER_THREAD; ++i) {
    // the unclamped k range (k_max = INT_MAX) is right for every full K step
    offA[i] = pin(load_offset<AMN>(i, lda, m0, M - 1, 0, 0x7fffffff));
    offB[i] = pin(load_offset<BMN>(i, ldb, n0, N - 1, 0, 0x7fffffff));
  }
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_addr(&smem[0][0][0]) + (uint32_t)(threadIdx.x & ~63) * 16u);

  // ---- LDS side: fragment addresses per stage, computed once
  constexpr int NA = AMN ? 2 * FM : BK / 16, NB = BMN ? 2 * FN : BK / 16;
  uint32_t fa[NSTAGE][NA], fb[NSTAGE][NB];
#pragma unroll
  for (int st = 0; st < NSTAGE; ++st) {
    const uint32_t sa = lds_addr(&smem[st][0][0]), sb = lds_addr(&smem[st][1][0]);
#pragma unroll
    for (int x = 0; x < NA; ++x) fa[st][x] = pin(sa + (AMN ? frag_off_mnmaj(wm0 + (x >> 1) * 32, 0, x & 1) : frag_off_kmaj(wm0, x)));
#pragma unroll
    for (int x = 0; x < NB; ++x) fb[st][x] = pin(sb + (BMN ? frag_off_mnmaj(wn0 + (x >> 1) * 32, 0, x & 1) : frag_off_kmaj(wn0, x)));
  }
  // fragment (block i, k16 step kk) of stage st: K-major blocks are 32 rows = 4096 B apart (the swizzle repeats every
  // 16 rows); reduction-major k16 steps are 16 k-rows = 8192 B apart (the swizzle repeats every 8 k-rows)
  auto frag_a = [&](int st, int i, int kk) {
    if (AMN) return lds_read_tr(fa[st][2 * i] + kk * 16 * BM * 2, fa[st][2 * i + 1] + kk * 16 * BM * 2);
    else return lds_read_b128(fa[st][kk] + i * 32 * BK * 2);
  };
  auto frag_b = [&](int st, int j, int kk) {
    if (BMN) return lds_read_tr(fb[st][2 * j] + kk * 16 * BN * 2, fb[st][2 * j + 1] + kk * 16 * BN * 2);
    else return lds_read_b128(fb[st][kk] + j * 32 * BK * 2);
  };

  // One K step on stage st.  Fragments are double-buffered in registers: the LDS reads of k16 step kk+1 are in
  // flight while the MFMAs of step kk issue.
  auto compute = [&](int st, int k_valid) {
    bf16x8 a[2][FM], b[2][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) a[0][i] = frag_a(st, i, 0);
#pragma unroll
    for (int j = 0; j < FN; ++j) b[0][j] = frag_b(st, j, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < FM; ++i) a[nxt][i] = frag_a(st, i, kk + 1);
#pragma unroll
        for (int j = 0; j < FN; ++j) b[nxt][j] = frag_b(st, j, kk + 1);
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the prefetch above the MFMAs (the scheduler would sink it to its use)
      if (TA && k_valid < BK) {   // zero reduction rows past the end (A only: B rows are finite duplicates)
        const int kbase = kk * 16 + 8 * (lane >> 5);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (kbase + e >= k_valid) a[cur][i][e] = (bf16_t)0.0f;
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = mode_swaps_operands(MODE) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[cur][j], a[cur][i], acc[i][j], 0, 0, 0)   // C^T blocks
                                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Two stages: at step kt wait for tile kt, barrier (every wave's share has landed and everyone is done reading
  // the other stage), refill the other stage with tile kt+1, compute.
#pragma unroll      // constant segment indices: the segment table stays in scalar registers
  for (int sg = 0; sg < MAX_SEG; ++sg) {
    if (sg >= segs.n) break;
    const int K = segs.K[sg], k_begin = segs.k_begin[sg], k_end = segs.k_end[sg];
    const int nk = (k_end - k_begin + BK - 1) / BK;
    if (nk <= 0) continue;
    const char* gA = uniform_ptr(segs.A[sg] + (AMN ? (int64_t)k_begin * lda + m0 : (int64_t)m0 * lda + k_begin));
    const char* gB = uniform_ptr(segs.B[sg] + (BMN ? (int64_t)k_begin * ldb + n0 : (int64_t)n0 * ldb + k_begin));
    auto issue = [&](int kt, int st) {
      const char* a_base = gA + (int64_t)kt * stepA;
      const char* b_base = gB + (int64_t)kt * stepB;
      const uint32_t la = lds_wave + (uint32_t)(st * 2 * TILE_BYTES), lb = la + TILE_BYTES;
      const int k0 = k_begin + kt * BK;
      if ((AMN || BMN) && k0 + BK > K) {    // ragged last K step: clamp the k-rows (slow path, once per tile)
#pragma unroll
        for (int i = 0; i < LOADS_PER_THREAD; ++i) {
          dma16(a_base, AMN ? load_offset<AMN>(i, lda, m0, M - 1, k0, K - 1) : offA[i], la + (uint32_t)(i * NTHREADS * 16));
          dma16(b_base, BMN ? load_offset<BMN>(i, ldb, n0, N - 1, k0, K - 1) : offB[i], lb + (uint32_t)(i * NTHREADS * 16));
        }
      } else {
#pragma unroll
        for (int i = 0; i < LOADS_PER_THREAD; ++i) {
          dma16(a_base, offA[i], la + (uint32_t)(i * NTHREADS * 16));
          dma16(b_base, offB[i], lb + (uint32_t)(i * NTHREADS * 16));
        }
      }
    };
    if (sg > 0) __syncthreads();     // everyone is done reading the stages of the previous segment
    issue(0, 0);
    for (int kt = 0; kt < nk; kt += 2) {
      WAIT_VMCNT(0);
      __syncthreads();
      if (kt + 1 < nk) issue(kt + 1, 1);
      compute(0, k_end - (k_begin + kt * BK));
      if (kt + 1 < nk) {
        WAIT_VMCNT(0);
        __syncthreads();
        if (kt + 2 < nk) issue(kt + 2, 0);
        compute(1, k_end - (k_begin + (kt + 1) * BK));
      }
    }
  }

  // Epilogue.  Accumulator register r of lane l: row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  float* Cf = (float*)Cv;
  bf16_t* Cb = (bf16_t*)Cv;
  if constexpr (MODE == 4) {
    // bf16 C += acc, two columns (4 bytes) per lane and access: neighbouring lanes hold neighbouring columns, so for each
    // register pair (r, r+1) the even lane takes row r of both columns and the odd lane row r+1 of both (one lane
    // swap).  Every element has exactly one owner per launch: plain loads and stores, the sum is formed in fp32 and
    // rounded once.  All loads of a 32-row block are issued before the first store so that the wave waits for C once
    // per block, not once per element.
    typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
    const bool odd = lane & 1;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      float lo[8][FN], hi[8][FN];
      bf16x2 old[8][FN];
#pragma unroll
      for (int rp = 0; rp < 8; ++rp) {
        const int r = 2 * rp;
        const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3) + (odd ? 1 : 0);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          float a0 = acc[i][j][r], a1 = acc[i][j][r + 1];
          asm volatile("" : "+v"(a0), "+v"(a1));     // two plain registers: the select below stays a single v_cndmask
          const float keep = odd ? a1 : a0;
          const float send = odd ? a0 : a1;
          const float got = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, false));
          lo[rp][j] = odd ? got : keep;
          hi[rp][j] = odd ? keep : got;
          const int col = n0 + wn0 + j * 32 + (lane & 31) - (odd ? 1 : 0);     // even column of the pair (N is a multiple of 8)
          const int64_t idx = (int64_t)row * ldc + col;
          if (row < M && col < N) old[rp][j] = *(const bf16x2*)(Cb + idx);
        }
      }
#pragma unroll
      for (int rp = 0; rp < 8; ++rp) {
        const int r = 2 * rp;
        const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3) + (odd ? 1 : 0);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int col = n0 + wn0 + j * 32 + (lane & 31) - (odd ? 1 : 0);
          const int64_t idx = (int64_t)row * ldc + col;
          bf16x2 v;
          v[0] = (bf16_t)((float)old[rp][j][0] + lo[rp][j]);
          v[1] = (bf16_t)((float)old[rp][j][1] + hi[rp][j]);
          if (row < M && col < N) *(bf16x2*)(Cb + idx) = v;
        }
      }
    }
    return;
  }
  if constexpr (MODE == 5) {
    // Row statistics for a softmax over the columns of C: every row of the tile gets (max, sum of exp(c - max)) over
    // the tile's 256 columns.  The products were formed with the operands swapped, so the accumulators hold C^T
    // blocks: a lane owns one row of C (l % 32 inside the 32-row block) and 32 of its columns - per column block j
    // and register quad q the four columns 8q + 4(l / 32) .. +3 - so the reduction over columns is in-lane, plus one
    // exchange between the two lanes of a row, and C is stored 16 bytes at a time.  The NWAVE_N waves that share a row
    // meet in LDS (the operand stages are free once every wave has left the main loop).
    static_assert(FN == 2, "two column blocks per wave");
    __syncthreads();
    float2* part = (float2*)&smem[0][0][0];    // [NWAVE_N][BM]
    constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row_l = wm0 + i * 32 + (lane & 31);
      const int col0 = n0 + wn0 + 4 * (lane >> 5);               // first of the lane's columns; quads at + j * 32 + 8 * q
      if (n0 + BN > N) {                                         // ragged last column tile: columns past N take no part
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (col0 + j * 32 + 8 * q >= N) {
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] = -INFINITY;
            }
      }
      if (m0 + row_l < M) {
        float* crow = Cf + (int64_t)(m0 + row_l) * ldc + col0;
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (col0 + j * 32 + 8 * q < N)
              *(float4*)(crow + j * 32 + 8 * q) = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
      }
      float mx = acc[i][0][0];
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      const float mref = mx == -INFINITY ? 0.0f : mx;            // a wave whose 64 columns all lie past N: sum 0, not NaN
      float se = 0.f;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) se += __builtin_amdgcn_exp2f((acc[i][j][r] - mref) * LOG2E);   // difference first: exact near the maximum
      se += __shfl_xor(se, 32, WAVE);
      if (lane < 32) part[(wave % NWAVE_N) * BM + row_l] = make_float2(mx, se);
    }
    __syncthreads();
    if ((int)threadIdx.x < BM && m0 + (int)threadIdx.x < M) {
      float2 p = part[threadIdx.x];
#pragma unroll
      for (int w = 1; w < NWAVE_N; ++w) {
        const float2 q = part[w * BM + threadIdx.x];
        const float m2 = fmaxf(p.x, q.x);
        if (q.x != -INFINITY)                                    // (a wave past N contributes nothing; wave 0 always holds valid columns)
          p.y = p.y * __builtin_amdgcn_exp2f((p.x - m2) * LOG2E) + q.y * __builtin_amdgcn_exp2f((q.x - m2) * LOG2E);
        p.x = m2;
      }
      stats[(int64_t)(m0 + (int)threadIdx.x) * ((N + BN - 1) / BN) + tn] = p;
    }
    return;
  }
  if constexpr (MODE == 7) {
    // Softmax numerators (Sec. 5 names fused backward operators as the way to cut the per-chunk HBM passes): what the row
    // kernel after the logits GEMM needs of a row is exp(c - lse), and exp(c - max of the 256-column block) differs from it
    // by one factor per block - so the tile stores that, in bf16 (half the bytes of the fp32 logits, and the exponentials
    // are the ones the block's sum needs anyway), next to the block's (max, sum) pair; the sum is taken from the
    // unrounded values.  The logit of each row's target column, which the loss needs exactly, is kept in fp32 on the side.
    // Same accumulator layout as MODE 5 (C^T blocks: a lane owns one row and 32 of its columns).  The four waves that
    // share a row exchange their maxima before the exponentials and their sums after them.
    static_assert(FN == 2, "two column blocks per wave");
    typedef bf16_t bf16x4e __attribute__((ext_vector_type(4)));
    __syncthreads();
    float* pmax = (float*)&smem[0][0][0];      // [NWAVE_N][BM]
    float* psum = pmax + NWAVE_N * BM;         // [NWAVE_N][BM]
    constexpr float LOG2E = 1.4426950408889634f;
    const int wn = wave % NWAVE_N;
    const int col0 = n0 + wn0 + 4 * (lane >> 5);                 // first of the lane's columns; quads at + j * 32 + 8 * q
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row_l = wm0 + i * 32 + (lane & 31);
      if (n0 + BN > N) {                                         // ragged last column tile: columns past N take no part
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (col0 + j * 32 + 8 * q >= N) {
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] = -INFINITY;
            }
      }
      if (m0 + row_l < M) {                                      // the target's logit, if it lies among the lane's columns
        const int r = nf.row_index ? nf.row_index[m0 + row_l] : m0 + row_l;
        const int d = nf.targets[r] - col0;
        if (d >= 0 && d < 64 && (d & 4) == 0) {
          float zt = 0.f;
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (d == j * 32 + 8 * q + e) zt = acc[i][j][4 * q + e];
          if (zt != -INFINITY) nf.target_value[m0 + row_l] = zt;   // (-inf: a masked column past N, i.e. an invalid target)
        }
      }
      float mx = acc[i][0][0];
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      if (lane < 32) pmax[wn * BM + row_l] = mx;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row_l = wm0 + i * 32 + (lane & 31);
      float m = pmax[row_l];
#pragma unroll
      for (int w = 1; w < NWAVE_N; ++w) m = fmaxf(m, pmax[w * BM + row_l]);   // finite: wave 0 always holds valid columns
      bf16_t* crow = Cb + (int64_t)(m0 + row_l) * ldc + col0;
      float se = 0.f;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          bf16x4e o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float ex = __builtin_amdgcn_exp2f((acc[i][j][4 * q + e] - m) * LOG2E);   // difference first: exact near the maximum
            se += ex;
            o[e] = (bf16_t)ex;
          }
          if (m0 + row_l < M && col0 + j * 32 + 8 * q < N) *(bf16x4e*)(crow + j * 32 + 8 * q) = o;
        }
      se += __shfl_xor(se, 32, WAVE);
      if (lane < 32) psum[wn * BM + row_l] = se;
    }
    __syncthreads();
    if ((int)threadIdx.x < BM && m0 + (int)threadIdx.x < M) {
      float m = pmax[threadIdx.x], sum = psum[threadIdx.x];
#pragma unroll
      for (int w = 1; w < NWAVE_N; ++w) { m = fmaxf(m, pmax[w * BM + threadIdx.x]); sum += psum[w * BM + threadIdx.x]; }
      stats[(int64_t)(m0 + (int)threadIdx.x) * ((N + BN - 1) / BN) + tn] = make_float2(m, sum);
    }
    return;
  }
  if constexpr (MODE == 6) {
    // SwiGLU adjoint on the accumulators (Sec. 5 names fused backward operators as the way to cut the per-chunk HBM
    // passes): the products were formed with the operands swapped, so a lane owns one row of the tile and, per column
    // block j and register quad q, four consecutive columns - 8-byte accesses to gate / up / act.  Every element has
    // exactly one owner, so gate and up are rewritten in place.
    typedef bf16_t bf16x4e __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row_l = wm0 + i * 32 + (lane & 31);
      if (m0 + row_l >= M) continue;
      const int64_t base = (int64_t)(m0 + row_l) * ldc + n0 + wn0 + 4 * (lane >> 5);
      bf16x4e gv[FN][4], uv[FN][4];
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bool in = n0 + wn0 + 4 * (lane >> 5) + j * 32 + 8 * q < N;
          gv[j][q] = in ? *(const bf16x4e*)(sw.gate + base + j * 32 + 8 * q) : bf16x4e{};
          uv[j][q] = in ? *(const bf16x4e*)(sw.up + base + j * 32 + 8 * q) : bf16x4e{};
        }
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          bf16x4e a4, dg4, du4;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float z = (float)gv[j][q][e], u = (float)uv[j][q][e], d = acc[i][j][4 * q + e];
            const float sg = 1.0f / (1.0f + __expf(-z));
            a4[e] = (bf16_t)(z * sg * u);
            dg4[e] = (bf16_t)(d * u * sg * (1.0f + z * (1.0f - sg)));
            du4[e] = (bf16_t)(d * z * sg);
          }
          const int64_t idx = base + j * 32 + 8 * q;
          if (n0 + wn0 + 4 * (lane >> 5) + j * 32 + 8 * q >= N) continue;
          if (sw.act) *(bf16x4e*)(sw.act + idx) = a4;
          *(bf16x4e*)(sw.gate + idx) = dg4;
          *(bf16x4e*)(sw.up + idx) = du4;
        }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < M) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int col = n0 + wn0 + j * 32 + (lane & 31);
          if (col >= N) continue;                                // ragged last column tile
          const int64_t idx = (int64_t)row * ldc + col;
          const float v = acc[i][j][r];
          if (MODE == 1) Cb[idx] = (bf16_t)v;
          else if (MODE == 2) unsafeAtomicAdd(&Cf[idx], v);   // one add per element per launch: same rounding as a
                                                               // read-modify-write, but the wave does not wait for C
          else Cf[idx] = v;
        }
      }
    }
}

template <bool TA, bool TB, int MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_k(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                        void* __restrict__ Cv, int M, int N, int K, int64_t lda,
                                                        int64_t ldb, int64_t ldc, int k_per_split,
                                                        const int* __restrict__ rows_dev, int xcds_per_split,
                                                        const bf16_t* __restrict__ A2, const bf16_t* __restrict__ B2,
                                                        float2* __restrict__ row_stats, SwigluFuse sw, NumerFuse nf) {
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE][2][TILE_BYTES];   // [stage][A|B]
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN, n_tiles = tiles_m * tiles_n;
  int tm, tn, split = 0;
  if (MODE == 3 && xcds_per_split > 0) {
    // Split-K with each slice of the reduction pinned to its own group of XCDs (the grid is 1-D: n_tiles x splits
    // workgroups, dealt round-robin to the 8 XCDs by the hardware).  Inside a group every XCD takes a contiguous
    // run of the tile ids, so it touches only its slice of K of the operand panels of that run (measured: 12% less
    // fabric traffic than with every XCD working on all slices of its tiles).
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int run = n_tiles / xcds_per_split;
    split = xcd / xcds_per_split;
    band_coords((xcd % xcds_per_split) * run + q, tiles_m, tiles_n, band_height_for_run(tiles_m, run), tm, tn);
  } else if (MODE == 3) {
    split = blockIdx.x / n_tiles;
    band_coords(xcd_contiguous_id(blockIdx.x % n_tiles, n_tiles), tiles_m, tiles_n, band_height(tiles_m, n_tiles, true), tm, tn);
  } else {
    band_coords(mode_accumulates(MODE) ? (int)blockIdx.x : xcd_contiguous_id(blockIdx.x, n_tiles), tiles_m, tiles_n,
                band_height(tiles_m, n_tiles, !mode_accumulates(MODE)), tm, tn);
  }
  if (MODE == 3) Cv = (float*)Cv + (int64_t)split * M * ldc;   // partial slices are laid out for the host-side M
  if (rows_dev) {                     // run-time row count: rows are M (NT / NN) or the reduction K (dW form)
    const int rows = max(0, *rows_dev);
    if (TA) K = min(K, rows); else M = min(M, rows);
    if (!TA && tm * BM >= M) return;  // no valid row in this tile
  }
  int k_begin = split * k_per_split;
  if (MODE == 3 && A2 != nullptr) {   // two operand pairs instead of two halves of K: slice 1 is A2 B2 over the whole K
    k_begin = 0;
    if (split == 1) { A = A2; B = B2; }
  }
  const int k_end = min(K, k_begin + k_per_split);
  if (k_end <= k_begin && mode_accumulates(MODE)) return;   // nothing to add
  KSegments segs;
  segs.n = 1; segs.A[0] = A; segs.B[0] = B; segs.K[0] = K; segs.k_begin[0] = k_begin; segs.k_end[0] = k_end;
  gemm_tile<TA, TB, MODE>(segs, Cv, M, N, lda, ldb, ldc, tm, tn, smem, row_stats, sw, nf);
}

// Weight-gradient form with a segmented reduction: C += sum_s A_s^T B_s, every segment with its own run-time row
// count.  One pass over C (one atomic add per element) for several chunks' worth of rows.
struct SegLaunch { const bf16_t* A[MAX_SEG]; const bf16_t* B[MAX_SEG]; const int* rows_dev[MAX_SEG]; int K[MAX_SEG]; int n; };
template <bool C_BF16>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_seg_k(const SegLaunch sl, void* __restrict__ C, int M, int N, int64_t lda,
                                                            int64_t ldb, int64_t ldc) {
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE][2][TILE_BYTES];
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tm, tn;
  band_coords((int)blockIdx.x, tiles_m, tiles_n, band_height(tiles_m, tiles_m * tiles_n, false), tm, tn);
  KSegments segs;
  segs.n = sl.n;
  int total = 0;
#pragma unroll
  for (int s = 0; s < MAX_SEG; ++s) {
    int K = 0;
    if (s < sl.n) { K = sl.K[s]; if (sl.rows_dev[s]) K = min(K, max(0, *sl.rows_dev[s])); }
    segs.A[s] = sl.A[s]; segs.B[s] = sl.B[s]; segs.K[s] = K; segs.k_begin[s] = 0; segs.k_end[s] = K;
    total += K;
  }
  if (total == 0) return;   // nothing to add
  gemm_tile<true, false, C_BF16 ? 4 : 2>(segs, C, M, N, lda, ldb, ldc, tm, tn, smem);
}

// Several independent GEMMs of one layout / output mode in a single launch: the tiles of all problems form one
// grid, so small problems fill the tail of large ones instead of each paying its own partial last round.
constexpr int MAX_GROUP = 8;
constexpr int MAX_GSEG = MAX_SEG;   // reduction segments per grouped problem (accumulate form: several chunks' operands)
struct GroupProblem {
  const bf16_t* A[MAX_GSEG]; const bf16_t* B[MAX_GSEG]; void* C;
  int M, N, K[MAX_GSEG], nseg;
  int64_t lda, ldb, ldc;
  int tile_begin, tiles_m, tiles_n;
};
struct GroupArgs { GroupProblem p[MAX_GROUP]; int n; int total_tiles; };

template <bool TA, bool TB, int MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_group_k(const GroupArgs ga) {
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE][2][TILE_BYTES];
  const int id = mode_accumulates(MODE) ? (int)blockIdx.x : xcd_contiguous_id(blockIdx.x, ga.total_tiles);
  int pi = 0;
#pragma unroll
  for (int i = 1; i < MAX_GROUP; ++i)
    if (i < ga.n && id >= ga.p[i].tile_begin) pi = i;
  const GroupProblem& g = ga.p[pi];
  int tm, tn;
  band_coords(id - g.tile_begin, g.tiles_m, g.tiles_n, band_height(g.tiles_m, g.tiles_m * g.tiles_n, !mode_accumulates(MODE)), tm, tn);
  KSegments segs;
  segs.n = g.nseg;
#pragma unroll
  for (int sg = 0; sg < MAX_GSEG; ++sg) {
    segs.A[sg] = g.A[sg]; segs.B[sg] = g.B[sg]; segs.K[sg] = g.K[sg]; segs.k_begin[sg] = 0; segs.k_end[sg] = g.K[sg];
  }
  gemm_tile<TA, TB, MODE>(segs, g.C, g.M, g.N, g.lda, g.ldb, g.ldc, tm, tn, smem);
}

// C (=|+=) sum_z partial[z] in a fixed order; OUT_BF16 rounds once at the end.
template <bool OUT_BF16, bool ACC>
__global__ void splitk_reduce_k(const float* __restrict__ part, void* __restrict__ C, int64_t n, int splits) {
  int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;
  float4 s = *(const float4*)(part + i);
  for (int z = 1; z < splits; ++z) {
    const float4 t = *(const float4*)(part + (int64_t)z * n + i);
    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
  }
  if (OUT_BF16) {
    bf16x4* c = (bf16x4*)((bf16_t*)C + i);
    if (ACC) { const bf16x4 t = *c; s.x += (float)t[0]; s.y += (float)t[1]; s.z += (float)t[2]; s.w += (float)t[3]; }
    bf16x4 o; o[0] = (bf16_t)s.x; o[1] = (bf16_t)s.y; o[2] = (bf16_t)s.z; o[3] = (bf16_t)s.w;
    *c = o;
  } else {
    float4* c = (float4*)((float*)C + i);
    if (ACC) { float4 t = *c; s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w; }
    *c = s;
  }
}

bool gemm_mfma_eligible(const GemmArgs& g) {
  if (g.in_dt != DT_BF16) return false;
  if (g.acc && g.out_dt != DT_F32 && !(g.out_dt == DT_BF16 && g.ta && !g.tb)) return false;   // bf16 C += : dW form only
  // Output widths need not be multiples of the 256-wide tile: a ragged last tile clamps its loads and masks its stores
  // (16-byte granules: multiples of 8 elements), e.g. a 151936-word vocabulary = 593.5 tiles.
  if (g.M < 1 || g.N < 8 || g.K < 1) return false;
  if (g.N % 8 != 0) return false;
  if (g.ta && !g.tb) {                       // TN: both operands reduction-major; ragged K allowed
    if (g.M % 8 != 0) return false;
  } else if (!g.ta) {                        // NT / NN
    if (g.K % BK != 0) return false;
  } else {
    return false;                            // TT is never needed
  }
  if (g.lda % 8 || g.ldb % 8) return false;
  if (g.lda >= (1 << 22) || g.ldb >= (1 << 22)) return false;   // per-lane byte offsets within a tile are 32-bit
  if (((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15) || ((uintptr_t)g.C & 15)) return false;
  if (g.ldc % 4) return false;
  return true;
}

// the operand-pair form needs two partial slices and a dense C
bool gemm_mfma_pair_ok(const GemmArgs& g) {
  return g.A2 && g.B2 && !g.ta && g.scratch && g.ldc == g.N && g.scratch_bytes >= (size_t)2 * g.M * g.ldc * sizeof(float) &&
         !((uintptr_t)g.A2 & 15) && !((uintptr_t)g.B2 & 15);
}

// the fused SwiGLU adjoint exists for the store form C = A B (input-gradient layout), bf16 tensors that share C's layout
bool gemm_mfma_swiglu_ok(const GemmArgs& g) {
  return g.swiglu_gate && g.swiglu_up && !g.ta && !g.tb && !g.acc && !g.A2 && !g.row_stats && g.ldc % 4 == 0 &&
         !((uintptr_t)g.swiglu_gate & 7) && !((uintptr_t)g.swiglu_up & 7) && !((uintptr_t)g.swiglu_act & 7);
}

// the row-statistics epilogue exists for the fp32 store form of C = A B^T
bool gemm_mfma_stats_ok(const GemmArgs& g) {
  return !g.ta && g.tb && g.out_dt == DT_F32 && !g.acc && !g.A2 && !((uintptr_t)g.row_stats & 7) && !g.numer_targets;
}

// ... and its softmax-numerator variant for a bf16 C
bool gemm_mfma_numer_ok(const GemmArgs& g) {
  return !g.ta && g.tb && g.out_dt == DT_BF16 && !g.acc && !g.A2 && g.row_stats && !((uintptr_t)g.row_stats & 7) &&
         g.numer_targets && g.numer_target_value && !g.swiglu_gate;
}

constexpr int MAX_SPLITS = 8;
// Split-K factor (a power of two <= 8) for outputs with too few tiles to fill the chip: the largest split that
// still fits one round of 256 CUs and leaves every slice at least 8 K steps.  Splitting further does not reduce
// the fabric traffic: an XCD runs 32 tiles at a time whatever the split, and those pull (rows + columns) operand
// panels per K step.
int gemm_mfma_splits(const GemmArgs& g) {
  const int64_t tiles = cdiv(g.M, BM) * cdiv(g.N, BN);
  const int k_tiles = (int)cdiv(g.K, BK);
  if (tiles >= 200 || k_tiles < 16 || (g.ta && g.rows_dev)) return 1;
  int s = 1;
  while (s * 2 <= MAX_SPLITS && s * 2 * tiles <= 256 && k_tiles / (s * 2) >= 8) s *= 2;
  return s;
}

size_t gemm_scratch_bytes(int max_m, int max_n, int max_splits) {
  return (size_t)std::min(max_splits, MAX_SPLITS) * max_m * max_n * sizeof(float);
}

hipError_t gemm_mfma(const GemmArgs& g, hipStream_t st) {
  const int tiles_m = (int)cdiv(g.M, BM), tiles_n = (int)cdiv(g.N, BN);
  int splits = gemm_mfma_splits(g);
  if (g.scratch == nullptr || g.ldc != g.N || g.row_stats || g.swiglu_gate) splits = 1;
  while (splits > 1 && g.scratch_bytes < (size_t)splits * g.M * g.ldc * sizeof(float)) splits /= 2;   // what the scratch holds
  int k_per_split = g.K;
  int xcds_per_split = 0;
  if (g.A2) {               // operand-pair form (gemm_mfma_pair_ok has checked the scratch): slice = pair, each over all of K
    splits = 2;
    if ((tiles_m * tiles_n) % 4 == 0) xcds_per_split = 4;
  } else if (splits > 1) {
    k_per_split = (int)(cdiv(cdiv(g.K, BK), splits) * BK);
    if ((int)cdiv(g.K, k_per_split) != splits) splits = (int)cdiv(g.K, k_per_split);
    if (8 % splits == 0 && (tiles_m * tiles_n) % (8 / splits) == 0) xcds_per_split = 8 / splits;
  }
  dim3 grid(tiles_m * tiles_n * splits, 1, 1);
  const bf16_t* A = (const bf16_t*)g.A;
  const bf16_t* B = (const bf16_t*)g.B;
#define LAUNCH(TA, TB, MODE, CPTR) \
  gemm_mfma_k<TA, TB, MODE><<<grid, NTHREADS, 0, st>>>(A, B, CPTR, g.M, g.N, g.K, g.lda, g.ldb, g.ldc, k_per_split, g.rows_dev, \
                                                       xcds_per_split, (const bf16_t*)g.A2, (const bf16_t*)g.B2, g.row_stats, \
                                                       SwigluFuse{(bf16_t*)g.swiglu_gate, (bf16_t*)g.swiglu_up, (bf16_t*)g.swiglu_act}, \
                                                       NumerFuse{g.numer_targets, g.numer_row_index, g.numer_target_value})
#define LAUNCH_LAYOUT(MODE, CPTR)                       \
  do {                                                  \
    if (!g.ta && g.tb) LAUNCH(false, true, MODE, CPTR); \
    else if (!g.ta && !g.tb) LAUNCH(false, false, MODE, CPTR); \
    else LAUNCH(true, false, MODE, CPTR);               \
  } while (0)
  const int layout = g.ta ? 2 : (g.tb ? 0 : 1);
  const int mode = splits > 1 ? 3 : (g.acc ? 2 : (g.out_dt == DT_BF16 ? 1 : 0));   // (both accumulate forms are timed as one kind)
  const int kind = g.numer_targets ? (int)prof::GEMM_NUMER : g.row_stats ? (int)prof::GEMM_STATS : g.swiglu_gate ? (int)prof::GEMM_SWIGLU : prof::GEMM_SINGLE + layout * 4 + mode;
  const double work = 2.0 * g.M * g.N * g.K * (g.A2 ? 2 : 1);
  if (splits > 1) {
    {
      prof::Scope sc(kind, work, g.rows_dev != nullptr, st);   // times the GEMM kernel, not the reduction after it
      LAUNCH_LAYOUT(3, (void*)g.scratch);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t n = (int64_t)g.M * g.N;
    const unsigned blocks = (unsigned)cdiv(n / 4, 256);
    if (g.out_dt == DT_BF16 && g.acc) splitk_reduce_k<true, true><<<blocks, 256, 0, st>>>(g.scratch, g.C, n, splits);
    else if (g.out_dt == DT_BF16) splitk_reduce_k<true, false><<<blocks, 256, 0, st>>>(g.scratch, g.C, n, splits);
    else if (g.acc) splitk_reduce_k<false, true><<<blocks, 256, 0, st>>>(g.scratch, g.C, n, splits);
    else splitk_reduce_k<false, false><<<blocks, 256, 0, st>>>(g.scratch, g.C, n, splits);
    return hipGetLastError();
  }
  prof::Scope sc(kind, work, g.rows_dev != nullptr, st);
  if (g.numer_targets) LAUNCH(false, true, 7, g.C);
  else if (g.row_stats) LAUNCH(false, true, 5, g.C);
  else if (g.swiglu_gate) LAUNCH(false, false, 6, g.C);
  else if (g.out_dt == DT_BF16 && g.acc) LAUNCH(true, false, 4, g.C);
  else if (g.out_dt == DT_BF16) LAUNCH_LAYOUT(1, g.C);
  else if (g.acc) LAUNCH_LAYOUT(2, g.C);
  else LAUNCH_LAYOUT(0, g.C);
#undef LAUNCH_LAYOUT
#undef LAUNCH
  return hipGetLastError();
}


// Grouped launch.  Requires every problem to be eligible, of the same layout / output type / accumulate mode.
// Accumulate-form problems that write the same C (same shape and leading dimensions) are folded into one grouped
// problem with several reduction segments: one pass over that C.
static bool same_output(const GemmArgs& a, const GemmArgs& b) {
  return a.C == b.C && a.M == b.M && a.N == b.N && a.lda == b.lda && a.ldb == b.ldb && a.ldc == b.ldc;
}
static int group_fold(const GemmArgs* gs, int n, int* owner /* [n]: index of the first problem with the same output */) {
  int n_out = 0;
  for (int i = 0; i < n; ++i) {
    owner[i] = i;
    if (gs[i].acc)
      for (int j = 0; j < i; ++j)
        if (owner[j] == j && same_output(gs[j], gs[i])) { owner[i] = j; break; }
    if (owner[i] == i) ++n_out;
  }
  return n_out;
}
constexpr int MAX_BATCH = MAX_GROUP * MAX_GSEG;
bool gemm_mfma_group_eligible(const GemmArgs* gs, int n, bool small_ok) {
  if (n < 2 || n > MAX_BATCH) return false;
  int64_t tiles = 0;
  int owner[MAX_BATCH], nseg[MAX_BATCH] = {0};
  const int n_out = group_fold(gs, n, owner);
  if (n_out > MAX_GROUP) return false;
  for (int i = 0; i < n; ++i) {
    if (!gemm_mfma_eligible(gs[i]) || gs[i].rows_dev || gs[i].A2) return false;
    if (gs[i].ta != gs[0].ta || gs[i].tb != gs[0].tb || gs[i].out_dt != gs[0].out_dt || gs[i].acc != gs[0].acc) return false;
    if (++nseg[owner[i]] > MAX_GSEG) return false;
    if (owner[i] == i) tiles += cdiv(gs[i].M, BM) * cdiv(gs[i].N, BN);
  }
  // few tiles: per-problem launches with split-K fill the chip better - unless problems share an output, where one
  // launch with several reduction segments replaces several passes over it
  // (small_ok: many skinny problems, none of which could fill the chip alone either)
  return (tiles >= 200 || n_out < n || small_ok) && tiles < (1 << 30);
}

hipError_t gemm_mfma_group(const GemmArgs* gs, int n, hipStream_t st) {
  GroupArgs ga{};
  int owner[MAX_BATCH], slot[MAX_BATCH];
  group_fold(gs, n, owner);
  int tiles = 0, np = 0;
  for (int i = 0; i < n; ++i) {
    if (owner[i] == i) {
      slot[i] = np;
      GroupProblem& p = ga.p[np++];
      p.C = gs[i].C; p.M = gs[i].M; p.N = gs[i].N; p.lda = gs[i].lda; p.ldb = gs[i].ldb; p.ldc = gs[i].ldc;
      p.nseg = 0;
      p.tiles_m = (int)cdiv(gs[i].M, BM); p.tiles_n = (int)cdiv(gs[i].N, BN); p.tile_begin = tiles;
      tiles += p.tiles_m * p.tiles_n;
    }
    GroupProblem& p = ga.p[slot[owner[i]]];
    p.A[p.nseg] = (const bf16_t*)gs[i].A; p.B[p.nseg] = (const bf16_t*)gs[i].B; p.K[p.nseg] = gs[i].K;
    ++p.nseg;
  }
  ga.n = np;
  ga.total_tiles = tiles;
  const GemmArgs& g = gs[0];
  double work = 0.0;
  for (int i = 0; i < n; ++i) work += 2.0 * gs[i].M * gs[i].N * gs[i].K;
  const int layout = g.ta ? 2 : (g.tb ? 0 : 1);
  const int mode = g.acc ? 2 : (g.out_dt == DT_BF16 ? 1 : 0);
  prof::Scope sc(prof::GEMM_GROUP + layout * 4 + mode, work, false, st);
#define GLAUNCH(TA, TB, MODE) gemm_mfma_group_k<TA, TB, MODE><<<tiles, NTHREADS, 0, st>>>(ga)
#define GLAUNCH_LAYOUT(MODE)                     \
  do {                                           \
    if (!g.ta && g.tb) GLAUNCH(false, true, MODE); \
    else if (!g.ta && !g.tb) GLAUNCH(false, false, MODE); \
    else GLAUNCH(true, false, MODE);             \
  } while (0)
  if (g.out_dt == DT_BF16 && g.acc) GLAUNCH(true, false, 4);
  else if (g.out_dt == DT_BF16) GLAUNCH_LAYOUT(1);
  else if (g.acc) GLAUNCH_LAYOUT(2);
  else GLAUNCH_LAYOUT(0);
#undef GLAUNCH_LAYOUT
#undef GLAUNCH
  return hipGetLastError();
}

// Segmented weight-gradient launch: gs[0..n) are accumulate-form (TN, fp32 or bf16 C +=) problems that share C, M, N and the
// leading dimensions and differ in A, B, K and rows_dev.
bool gemm_mfma_seg_eligible(const GemmArgs* gs, int n) {
  if (n < 2 || n > MAX_SEG) return false;
  for (int i = 0; i < n; ++i) {
    const GemmArgs& g = gs[i];
    if (!gemm_mfma_eligible(g) || !g.ta || g.tb || !g.acc || g.out_dt != gs[0].out_dt || g.A2) return false;
    if (g.C != gs[0].C || g.M != gs[0].M || g.N != gs[0].N || g.lda != gs[0].lda || g.ldb != gs[0].ldb || g.ldc != gs[0].ldc) return false;
  }
  return true;
}
hipError_t gemm_mfma_seg(const GemmArgs* gs, int n, hipStream_t st) {
  SegLaunch sl{};
  sl.n = n;
  double work = 0.0;
  bool bounded = false;
  for (int i = 0; i < n; ++i) {
    sl.A[i] = (const bf16_t*)gs[i].A; sl.B[i] = (const bf16_t*)gs[i].B; sl.rows_dev[i] = gs[i].rows_dev; sl.K[i] = gs[i].K;
    work += 2.0 * gs[i].M * gs[i].N * gs[i].K;
    bounded = bounded || gs[i].rows_dev != nullptr;
  }
  const GemmArgs& g = gs[0];
  const int tiles = (int)cdiv(g.M, BM) * (int)cdiv(g.N, BN);
  prof::Scope sc(prof::GEMM_SEG, work, bounded, st);
  if (g.out_dt == DT_BF16) gemm_mfma_seg_k<true><<<tiles, NTHREADS, 0, st>>>(sl, g.C, g.M, g.N, g.lda, g.ldb, g.ldc);
  else gemm_mfma_seg_k<false><<<tiles, NTHREADS, 0, st>>>(sl, g.C, g.M, g.N, g.lda, g.ldb, g.ldc);
  return hipGetLastError();
}

// ---- what the matrix pipe sustains on its own -------------------------------------------------------------
// Eight independent 32x32x16 products per round, two waves per SIMD, no global memory traffic.  R of the eight A fragments
// of a round are re-read from LDS (one conflict-free ds_read_b128 = 1 KB per wave each, the way the GEMM and attention
// kernels feed their MFMAs: the GEMM main loop reads 6 fragments per 8 products, the attention backward 8); the others
// and the B fragments never change.  The rate depends on the VALUES of the fragments (power management), which is why
// the caller supplies them.
template <int R>
__global__ __launch_bounds__(NTHREADS) void mfma_rate_probe_k(const bf16x8* __restrict__ operands, float* __restrict__ sink, int iters) {
  __shared__ __attribute__((aligned(1024))) bf16x8 frag[R > 0 ? 2 * NTHREADS * 8 : 1];   // two rounds' worth: 128 KB
  if (R > 0) {
    for (int i = threadIdx.x; i < 2 * NTHREADS * 8; i += NTHREADS) frag[i] = operands[i % 4096];
    __syncthreads();
  }
  const uint32_t base = lds_addr(&frag[0]) + (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 8 * 1024;
  bf16x8 a[8], b[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = operands[(threadIdx.x + i * NTHREADS) % 4096];
#pragma unroll
  for (int j = 0; j < 2; ++j) b[j] = operands[(threadIdx.x + (8 + j) * NTHREADS) % 4096];
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
    const uint32_t off = (uint32_t)(it & 1) * (NTHREADS * 8 * 16);
#pragma unroll
    for (int i = 0; i < R; ++i) a[i] = lds_read_b128(base + off + i * 1024);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i & 1], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[(int64_t)blockIdx.x * NTHREADS + threadIdx.x] = s;
}
hipError_t mfma_rate_probe(const void* operands, float* sink, int workgroups, int iters, int lds_reads, hipStream_t st) {
  if (workgroups <= 0 || iters < 0) return hipErrorInvalidValue;
  if (lds_reads == 0) mfma_rate_probe_k<0><<<workgroups, NTHREADS, 0, st>>>((const bf16x8*)operands, sink, iters);
  else if (lds_reads == 6) mfma_rate_probe_k<6><<<workgroups, NTHREADS, 0, st>>>((const bf16x8*)operands, sink, iters);
  else if (lds_reads == 8) mfma_rate_probe_k<8><<<workgroups, NTHREADS, 0, st>>>((const bf16x8*)operands, sink, iters);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace sbp
