// Host-side pieces of the C ABI that launch nothing: workspace layout, plan
// binding, result fetch, the reservation formula and the version string.
#include "common.h"

namespace warmkv {
namespace {

struct Layout {
  size_t state, live_out, src, dst, new_id, total;
};

// state | live_out | src | dst | new_id, each segment 256-byte aligned
Layout layout(uint32_t num_blocks, uint32_t boundary) {
  const size_t n_words = ((size_t)num_blocks + 63) / 64;
  const size_t cap = num_blocks - boundary < boundary ? num_blocks - boundary : boundary;
  Layout l;
  l.state = 0;
  l.live_out = 256;
  l.src = l.live_out + align_up(n_words * 8, 256);
  l.dst = l.src + align_up(cap * 4, 256);
  l.new_id = l.dst + align_up(cap * 4, 256);
  l.total = l.new_id + align_up((size_t)num_blocks * 4, 256);
  return l;
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" size_t kv_plan_workspace_bytes(uint32_t num_blocks, uint32_t boundary) {
  if (boundary > num_blocks || num_blocks > kMaxBlocks) return 0;
  return layout(num_blocks, boundary).total;
}

extern "C" int kv_plan_bind(kv_plan* plan, void* workspace, size_t workspace_bytes, uint32_t num_blocks,
                            uint32_t boundary) {
  if (plan == nullptr || workspace == nullptr) return KV_E_NULL;
  if (boundary > num_blocks || num_blocks > kMaxBlocks) return KV_E_RANGE;
  if (((uintptr_t)workspace % 256u) != 0) return KV_E_ALIGN;
  const Layout l = layout(num_blocks, boundary);
  if (workspace_bytes < l.total) return KV_E_TOOBIG;
  uint8_t* w = (uint8_t*)workspace;
  plan->state = (kv_plan_state*)(w + l.state);
  plan->live_out = (uint64_t*)(w + l.live_out);
  plan->src = (int32_t*)(w + l.src);
  plan->dst = (int32_t*)(w + l.dst);
  plan->new_id = (int32_t*)(w + l.new_id);
  plan->num_blocks = num_blocks;
  plan->boundary = boundary;
  plan->capacity = num_blocks - boundary < boundary ? num_blocks - boundary : boundary;
  plan->reserved = 0;
  return KV_OK;
}

extern "C" int kv_plan_fetch(const kv_plan* plan, void* stream, kv_plan_state* out) {
  if (plan == nullptr || plan->state == nullptr || out == nullptr) return KV_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  int rc = hip_rc(hipMemcpyAsync(out, plan->state, sizeof(kv_plan_state), hipMemcpyDeviceToHost, s));
  if (rc != KV_OK) return rc;
  rc = hip_rc(hipStreamSynchronize(s));
  if (rc == KV_OK && out->status == KV_OK && out->bad_plan != 0u) out->status = KV_E_BADPLAN;
  return rc;
}

// Sec. 3.3, Eq. 4: R = max(C*Q/B, T + C/B).  The ceiling of a maximum is the
// maximum of the ceilings and T is whole, so integer arithmetic is exact.
extern "C" int64_t kv_reserve_blocks(uint64_t capacity_blocks, uint64_t used_blocks, uint32_t running,
                                     uint32_t max_batch) {
  if (max_batch == 0 || used_blocks > capacity_blocks || capacity_blocks > 0xFFFFFFFFull) return KV_E_RANGE;
  const uint64_t expected = (capacity_blocks * running + max_batch - 1) / max_batch;
  const uint64_t headroom = used_blocks + (capacity_blocks + max_batch - 1) / max_batch;
  const uint64_t r = expected > headroom ? expected : headroom;
  return (int64_t)(r > capacity_blocks ? capacity_blocks : r);
}

// Sec. 3.3, last sentence: weights are evicted when the reserve runs short.
// Region offsets count through the reclaimed space: one byte range in a
// block-major pool (one "strip"), L strips taken in layer order in a
// layer-major pool.  Raising the boundary takes the first returned_per_strip
// bytes of every strip away.
extern "C" int64_t kv_grow(const kv_pool_desc* pool, uint32_t old_boundary, uint32_t new_boundary,
                           const wm_tensor* tensors, uint32_t n_tensors, uint8_t* evicted,
                           uint64_t* new_offset) {
  if (pool == nullptr) return KV_E_NULL;
  if (n_tensors != 0 && (tensors == nullptr || evicted == nullptr || new_offset == nullptr)) return KV_E_NULL;
  if (old_boundary > new_boundary || new_boundary > pool->num_blocks) return KV_E_RANGE;
  if ((pool->tile_bytes != 0 && pool->num_layers != 0) && !pool_extent_ok(*pool)) return KV_E_RANGE;
  const bool layer_major = pool->layer_stride_bytes != 0;
  const uint64_t per_block = layer_major ? pool->tile_bytes : (uint64_t)pool->num_layers * pool->tile_bytes;
  const uint64_t strips = layer_major ? pool->num_layers : 1u;
  const uint64_t old_strip = (uint64_t)(pool->num_blocks - old_boundary) * per_block;
  const uint64_t new_strip = (uint64_t)(pool->num_blocks - new_boundary) * per_block;
  const uint64_t returned = (uint64_t)(new_boundary - old_boundary) * per_block;  // per strip, at its start
  const uint64_t old_region = old_strip * strips;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const wm_tensor& t = tensors[i];
    if (t.dst_offset > old_region || t.bytes > old_region - t.dst_offset) return KV_E_TOOBIG;
    if (t.bytes != 0 && t.dst_offset % old_strip + t.bytes > old_strip) return KV_E_TOOBIG;  // straddles two strips
  }
  int64_t lost = 0;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const wm_tensor& t = tensors[i];
    uint64_t strip = old_strip ? t.dst_offset / old_strip : 0;
    uint64_t within = old_strip ? t.dst_offset % old_strip : 0;
    if (strip == strips && strip != 0) {  // an empty extent at the very end of the region
      strip = strips - 1;
      within = old_strip;
    }
    const bool hit = t.bytes != 0 && within < returned;
    evicted[i] = hit ? 1 : 0;
    new_offset[i] = (!hit && within >= returned) ? strip * new_strip + (within - returned) : 0;
    lost += hit;
  }
  return lost;
}

extern "C" const char* warmkv_version(void) { return "0.2"; }

// Hash of the sources this library was compiled from, passed in by the build.
#ifndef WARMKV_BUILD_ID
#define WARMKV_BUILD_ID "unknown"
#endif
// The tag in front lets a loader find the identifier in the file without loading it.
static const char kBuildTag[] = "WARMKV_BUILD_ID=" WARMKV_BUILD_ID;
extern "C" const char* warmkv_build_id(void) { return kBuildTag + 16; }
