// Internal helpers shared by the warmkv HIP sources (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <new>

#include "warmkv.h"

namespace warmkv {

constexpr int kWave = 64;                       // CDNA wavefront width
constexpr uint32_t kMaxBlocks = 1u << 24;       // planner's supported pool size (blocks)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int hip_rc(hipError_t e) { return e == hipSuccess ? KV_OK : KV_E_HIP; }

// True if every byte offset inside the described pool can be formed without
// overflow: the whole extent stays below 2^48 bytes.
inline bool pool_extent_ok(const kv_pool_desc& p) {
  constexpr uint64_t kMax = 1ull << 48;
  if (p.tile_bytes == 0 || p.num_layers == 0) return false;
  if (p.tile_bytes > kMax / p.num_layers) return false;
  const uint64_t per_block = p.tile_bytes * p.num_layers;
  if (p.num_blocks != 0 && per_block > kMax / p.num_blocks) return false;
  if (p.layer_stride_bytes > kMax / p.num_layers) return false;
  return true;
}

// No exception may cross the C ABI: entry points that allocate host memory (std::vector) run
// their body through this.
template <class Body>
inline auto guarded(Body&& body) noexcept -> decltype(body()) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return KV_E_NOMEM;
  } catch (...) {
    return KV_E_HIP;
  }
}

// The block copy numbers its work units with 32 bits.  True if a plan of `capacity` moves on this
// pool stays below that whatever unit size the copy picks (its units are never below 32 KiB unless
// the caller tunes them), so that a call that chains planner and copy can refuse before the planner
// is launched what the copy would refuse after it.
inline bool copy_units_fit(const kv_pool_desc& p, uint32_t capacity) {
  const bool layer_major = p.layer_stride_bytes != 0;
  const uint64_t segs = layer_major ? p.num_layers : 1u;
  const uint64_t seg_bytes = layer_major ? p.tile_bytes : (uint64_t)p.num_layers * p.tile_bytes;
  const uint64_t chunks = (seg_bytes + 32767u) / 32768u;
  return segs * chunks * (uint64_t)capacity < (1ull << 31);
}

// Launch status without clearing an earlier sticky error of the caller's.
inline int launch_rc() { return hip_rc(hipGetLastError()); }

}  // namespace warmkv
