// Host-safe helpers shared by the launchers and the C-ABI layer of libstreambp: nothing in here needs a device
// compiler (the host layer is also compiled with a plain host compiler under sanitizers by the tests).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sbp {

enum DType : int { DT_F32 = 0, DT_BF16 = 1 };

inline size_t dtype_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace sbp
