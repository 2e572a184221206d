// Stand-in for <hip/hip_runtime.h> for the host-only sanitizer build of the library's C-ABI layer (csrc/api.hip):
// just the handful of types and calls that layer uses, so that it compiles with a plain host compiler under
// -fsanitize=address,undefined.  No GPU, no HIP runtime: the "device" is host memory handed in by the test driver.
#pragma once
#include <stddef.h>
#include <stdint.h>

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
typedef struct ihipStream_t* hipStream_t;
typedef struct ihipEvent_t* hipEvent_t;
struct float2 { float x, y; };

#define __device__
#define __host__
#define __global__
#define __forceinline__ inline
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))

inline const char* hipGetErrorString(hipError_t) { return "stub"; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
template <typename T> inline hipError_t hipGetSymbolAddress(void** p, T* sym) { *p = (void*)sym; return hipSuccess; }
