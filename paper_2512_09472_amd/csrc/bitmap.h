// Bitmap arithmetic shared by the planner kernels: which bits of a live/free word are movers
// (live, id >= boundary), free ids below the boundary, or survivors; packed counts for a single
// scan over both; wavefront scans; selection of the lowest set bits of a word.
#pragma once

#include "common.h"

namespace warmkv {

struct WordBits {
  uint64_t mover;  // live, id >= b
  uint64_t avail;  // free, id < b
  uint64_t keep;   // live, id < b
  uint64_t live;   // live, id < NB
};

__device__ __forceinline__ uint64_t low_mask(uint32_t base, uint32_t limit) {
  // bits j of a word starting at id `base` with base + j < limit
  if (base + 64u <= limit) return ~0ull;
  if (base >= limit) return 0ull;
  return (1ull << (limit - base)) - 1ull;
}

__device__ __forceinline__ WordBits classify(uint64_t word, uint32_t wi, uint32_t num_blocks,
                                             uint32_t boundary) {
  const uint32_t base = wi * 64u;
  const uint64_t valid = low_mask(base, num_blocks);
  const uint64_t lo = low_mask(base, boundary);
  WordBits r;
  r.live = word & valid;
  r.mover = r.live & ~lo;
  r.avail = ~word & lo;
  r.keep = r.live & lo;
  return r;
}

// movers in the high half, free ids in the low half: one scan ranks both
__device__ __forceinline__ uint64_t pack_counts(const WordBits& wb) {
  return ((uint64_t)__popcll(wb.mover) << 32) | (uint64_t)__popcll(wb.avail);
}

__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint64_t up = __shfl_up(v, off, kWave);
    if (lane >= off) v += up;
  }
  return v;
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// The `count` lowest set bits of m (0 < count < popcount(m)).
__device__ __forceinline__ uint64_t lowest_set_bits(uint64_t m, uint32_t count) {
  uint64_t rest = m;
  uint32_t pos = 0;  // becomes the position of the count-th (0-based) set bit
#pragma unroll
  for (uint32_t width = 32; width != 0; width >>= 1) {
    const uint32_t c = (uint32_t)__popcll(rest & ((1ull << width) - 1ull));
    if (count >= c) {
      count -= c;
      rest >>= width;
      pos += width;
    }
  }
  return m & ((1ull << pos) - 1ull);
}

// Position of the r-th (0-based) set bit of m; r < popcount(m).
__device__ __forceinline__ uint32_t nth_set_bit(uint64_t m, uint32_t r) {
  uint32_t pos = 0;
#pragma unroll
  for (uint32_t width = 32; width != 0; width >>= 1) {
    const uint32_t c = (uint32_t)__popcll(m & ((1ull << width) - 1ull));
    if (r >= c) {
      r -= c;
      m >>= width;
      pos += width;
    }
  }
  return pos;
}

}  // namespace warmkv
