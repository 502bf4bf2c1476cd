// Weight materialisation: stream a prewarmed model's tensors from pinned host
// memory into the reclaimed byte range of the KV pool (paper App. C, Fig. 4b
// step 3; weights wait in host memory and cross the host link, Sec. 4.1).
//
// The copies go to the DMA engines through hipMemcpyAsync on a stream of
// their own, so they take no CU away from the block copy they overlap with.
// The reclaimed range still holds moving blocks until kv_compact has read
// them; the copy stream therefore waits on the caller's compaction event
// before the first chunk (the paper's rule "copy as soon as the destination is
// ready", at the granularity of the whole region).
#include <algorithm>
#include <vector>

#include "common.h"

namespace warmkv {
namespace {
constexpr uint64_t kChunkBytes = 256ull << 20;  // bound on one DMA request
}
}  // namespace warmkv

using namespace warmkv;

extern "C" int weights_materialize(const kv_pool_desc* pool, uint32_t boundary, const wm_tensor* tensors,
                                   uint32_t n_tensors, void* copy_stream, void* compaction_done) {
  if (pool == nullptr || (n_tensors != 0 && tensors == nullptr)) return KV_E_NULL;
  if (boundary > pool->num_blocks) return KV_E_RANGE;
  const uint64_t block_bytes = (uint64_t)pool->num_layers * pool->tile_bytes;
  const uint64_t region_offset = (uint64_t)boundary * block_bytes;
  const uint64_t region_bytes = (uint64_t)(pool->num_blocks - boundary) * block_bytes;

  // Validate everything before the first byte moves.
  std::vector<uint32_t> order;
  order.reserve(n_tensors);
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const wm_tensor& t = tensors[i];
    if (t.dst_offset > region_bytes || t.bytes > region_bytes - t.dst_offset) return KV_E_TOOBIG;
    if (t.bytes == 0) continue;
    if (t.host_ptr == nullptr) return KV_E_NULL;
    order.push_back(i);
  }
  if (!order.empty() && pool->base == nullptr) return KV_E_NULL;
  std::sort(order.begin(), order.end(),
            [&](uint32_t a, uint32_t b) { return tensors[a].dst_offset < tensors[b].dst_offset; });
  for (size_t j = 1; j < order.size(); ++j) {
    const wm_tensor& prev = tensors[order[j - 1]];
    if (prev.dst_offset + prev.bytes > tensors[order[j]].dst_offset) return KV_E_OVERLAP;
  }

  hipStream_t s = (hipStream_t)copy_stream;
  if (compaction_done != nullptr) {
    const int rc = hip_rc(hipStreamWaitEvent(s, (hipEvent_t)compaction_done, 0));
    if (rc != KV_OK) return rc;
  }
  uint8_t* region = (uint8_t*)pool->base + region_offset;
  for (uint32_t i = 0; i < n_tensors; ++i) {  // caller's order
    const wm_tensor& t = tensors[i];
    for (uint64_t done = 0; done < t.bytes; done += kChunkBytes) {
      const uint64_t len = std::min(kChunkBytes, t.bytes - done);
      const int rc = hip_rc(hipMemcpyAsync(region + t.dst_offset + done, (const uint8_t*)t.host_ptr + done,
                                           len, hipMemcpyHostToDevice, s));
      if (rc != KV_OK) return rc;
    }
  }
  return KV_OK;
}
