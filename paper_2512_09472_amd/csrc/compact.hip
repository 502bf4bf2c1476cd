// Block copy of the KV reclaim: for k < n_moves, block dst[k] <- block src[k].
// This is the bandwidth-bound step (2 * n_moves * block_bytes of HBM traffic);
// the rest of the path is microseconds.  It stands in for the paper's
// "map the physical pages of unused KV blocks to the new model's slot"
// (App. C, Fig. 4b step 2): here the unused space is made contiguous instead.
//
// Shape: a persistent grid (a fixed multiple of the 256 CUs) walks the work
// list of (move, chunk) units in grid-stride order, so neighbouring workgroups
// stream neighbouring chunks of the same block and the launch does not depend
// on n_moves, which lives in device memory (no host sync after the planner).
// Each lane issues UNROLL independent 128-bit loads before the first store;
// a wavefront covers 1 KiB per instruction, fully coalesced.  Accesses are
// non-temporal: 9+ GiB streams through once and must not evict anything.
// Sources lie at or above the boundary and destinations below it, so no two
// moves overlap and any order is correct; the kernel checks that property per
// move instead of staging through LDS.
#include "common.h"

namespace warmkv {
namespace {

constexpr uint32_t kCopyThreads = 256;
constexpr uint32_t kVecBytes = 16;
constexpr uint32_t kRowBytes = kCopyThreads * kVecBytes;  // 4 KiB per workgroup per instruction

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void store16(u32x4* p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <int UNROLL, bool NT>
__global__ __launch_bounds__(kCopyThreads) void compact_kernel(
    uint8_t* __restrict__ base, uint64_t block_bytes, const int32_t* __restrict__ src,
    const int32_t* __restrict__ dst, kv_plan_state* __restrict__ state, uint32_t num_blocks,
    uint32_t boundary, uint32_t chunk_bytes, uint32_t chunks_per_block) {
  if (state->status != KV_OK) return;
  const uint32_t n_moves = state->n_moves;
  const uint64_t n_units = (uint64_t)n_moves * chunks_per_block;
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t kStep = kRowBytes * UNROLL;  // bytes per workgroup per inner iteration

  for (uint64_t u = blockIdx.x; u < n_units; u += gridDim.x) {
    const uint32_t k = (uint32_t)(u / chunks_per_block);
    const uint32_t c = (uint32_t)(u - (uint64_t)k * chunks_per_block);
    const uint32_t s = (uint32_t)src[k], d = (uint32_t)dst[k];
    if (s < boundary || s >= num_blocks || d >= boundary) {  // never true for a planner-made plan
      if (tid == 0) atomicExch(&state->status, KV_E_BADPLAN);
      continue;
    }
    const uint64_t off = (uint64_t)c * chunk_bytes;
    const uint64_t left = block_bytes - off;
    const uint32_t len = left < chunk_bytes ? (uint32_t)left : chunk_bytes;
    const u32x4* __restrict__ sp = (const u32x4*)(base + (uint64_t)s * block_bytes + off);
    u32x4* __restrict__ dp = (u32x4*)(base + (uint64_t)d * block_bytes + off);

    uint32_t done = 0;
    for (; done + kStep <= len; done += kStep) {  // full rows, no bounds checks
      u32x4 v[UNROLL];
      const uint32_t i = done / kVecBytes + tid;
#pragma unroll
      for (int j = 0; j < UNROLL; ++j) v[j] = load16<NT>(sp + i + j * kCopyThreads);
#pragma unroll
      for (int j = 0; j < UNROLL; ++j) store16<NT>(dp + i + j * kCopyThreads, v[j]);
    }
    const uint32_t n_vec = len / kVecBytes;  // ragged tail of the chunk
    for (uint32_t i = done / kVecBytes + tid; i < n_vec; i += kCopyThreads) store16<NT>(dp + i, load16<NT>(sp + i));
  }
}

template <int UNROLL, bool NT>
int launch(const kv_pool_desc* pool, const kv_plan* plan, uint32_t workgroups, uint32_t chunk_bytes,
           hipStream_t s) {
  const uint64_t block_bytes = (uint64_t)pool->num_layers * pool->tile_bytes;
  const uint32_t chunks_per_block = (uint32_t)((block_bytes + chunk_bytes - 1) / chunk_bytes);
  hipLaunchKernelGGL((compact_kernel<UNROLL, NT>), dim3(workgroups), dim3(kCopyThreads), 0, s,
                     (uint8_t*)pool->base, block_bytes, plan->src, plan->dst, plan->state,
                     plan->num_blocks, plan->boundary, chunk_bytes, chunks_per_block);
  return launch_rc();
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int kv_compact_launch(const kv_pool_desc* pool, const kv_plan* plan,
                                 const kv_compact_tuning* tuning, void* stream) {
  if (pool == nullptr || plan == nullptr || plan->state == nullptr) return KV_E_NULL;
  if (pool->num_blocks != plan->num_blocks || plan->boundary > plan->num_blocks) return KV_E_RANGE;
  if (pool->num_layers == 0 || pool->tile_bytes == 0) return KV_E_RANGE;
  if ((pool->tile_bytes % kVecBytes) != 0) return KV_E_ALIGN;
  if (plan->capacity == 0 || pool->num_blocks == 0) return KV_OK;  // nothing can move
  if (pool->base == nullptr || plan->src == nullptr || plan->dst == nullptr) return KV_E_NULL;
  if (((uintptr_t)pool->base % 256u) != 0) return KV_E_ALIGN;
  const uint64_t block_bytes = (uint64_t)pool->num_layers * pool->tile_bytes;
  if (block_bytes / kRowBytes > 0xFFFFFFFFull / 2) return KV_E_RANGE;

  uint32_t workgroups = 256u * 8u, chunk = 16384u, flags = 0u;
  if (tuning != nullptr) {
    if (tuning->workgroups) workgroups = tuning->workgroups;
    if (tuning->chunk_bytes) chunk = tuning->chunk_bytes;
    flags = tuning->flags;
  }
  if ((chunk % kRowBytes) != 0 || workgroups > (1u << 20)) return KV_E_RANGE;
  const bool nt = (flags & 1u) == 0;
  const uint32_t unroll_sel = (flags >> 4) & 0xFu;  // 0 = pick from the chunk size
  hipStream_t s = (hipStream_t)stream;
  int unroll = unroll_sel ? (int)unroll_sel : (chunk >= 8 * kRowBytes ? 8 : (chunk >= 4 * kRowBytes ? 4 : (chunk >= 2 * kRowBytes ? 2 : 1)));
  switch (unroll) {
    case 1: return nt ? launch<1, true>(pool, plan, workgroups, chunk, s) : launch<1, false>(pool, plan, workgroups, chunk, s);
    case 2: return nt ? launch<2, true>(pool, plan, workgroups, chunk, s) : launch<2, false>(pool, plan, workgroups, chunk, s);
    case 4: return nt ? launch<4, true>(pool, plan, workgroups, chunk, s) : launch<4, false>(pool, plan, workgroups, chunk, s);
    case 8: return nt ? launch<8, true>(pool, plan, workgroups, chunk, s) : launch<8, false>(pool, plan, workgroups, chunk, s);
    default: return KV_E_RANGE;
  }
}

extern "C" int kv_compact(const kv_pool_desc* pool, const kv_plan* plan, void* stream) {
  return kv_compact_launch(pool, plan, nullptr, stream);
}
