// Device-side helpers of the libstreambp kernels (gfx950 only).
#pragma once
#include "common.h"

namespace sbp {

typedef __bf16 bf16_t;

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return (float)(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = (bf16_t)v; }   // round to nearest even

constexpr int WAVE = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
  return v;
}

// Block-wide reductions for blocks of up to 1024 threads; `red` is LDS scratch of >= 16 floats.
// Every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// 128-bit direct-to-LDS load, SGPR base + per-lane 32-bit byte offset: the wave's 64 x 16 B land contiguously at
// LDS address lds_wave_base.  Inline assembly for two reasons: the compiler must not fold the explicit, counted
// vmcnt waits of a pipeline into vmcnt(0), and this addressing form needs no vector ALU work per load - in an
// MFMA loop every VALU instruction queues behind the MFMAs of the SIMD's other wave, so per-load 64-bit address
// arithmetic (what the flat form needs) stretches the issue of a tile's loads several-fold.
// Every direct-to-LDS load of the library goes through these two functions, each of which sets m0 itself: no kernel
// mixes them with the compiler's builtin form, whose m0 bookkeeping the compiler could otherwise merge or hoist
// across an asm statement it cannot see into (m0 is a reserved register and cannot be named as a clobber).
__device__ __forceinline__ void dma16(const char* base /*uniform*/, uint32_t voff, uint32_t lds_wave_base /*uniform*/) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds_wave_base) : "memory");
}
// 32-bit form: lane l's dword lands at LDS address lds_wave_base + 4 l.
__device__ __forceinline__ void dma4(const char* base /*uniform*/, uint32_t voff, uint32_t lds_wave_base /*uniform*/) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(base), "s"(lds_wave_base) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}
// A pointer the compiler cannot prove wave-uniform (e.g. picked from an array by a loop index), moved to SGPRs.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
// Make a precomputed value opaque so that the compiler keeps it in a register instead of recomputing it in a loop.
__device__ __forceinline__ uint32_t pin(uint32_t v) { asm volatile("" : "+v"(v)); return v; }

}  // namespace sbp
