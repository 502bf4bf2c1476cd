// Internal helpers shared by the warmkv HIP sources (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "warmkv.h"

namespace warmkv {

constexpr int kWave = 64;                       // CDNA wavefront width
constexpr uint32_t kMaxBlocks = 1u << 24;       // planner's supported pool size (blocks)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int hip_rc(hipError_t e) { return e == hipSuccess ? KV_OK : KV_E_HIP; }

// Launch status without clearing an earlier sticky error of the caller's.
inline int launch_rc() { return hip_rc(hipGetLastError()); }

}  // namespace warmkv
