// No-move variant of the reclaim, for comparison with compaction: the paper's
// own mechanism (Sec. 3.4, App. C) written against HIP's virtual-memory API.
// Physical memory is created once, one allocation per KV block, and mapped
// into a contiguous KV range; to prewarm, the pages under unused blocks are
// unmapped there and mapped back to back into a second range (the "prewarm
// slot").  No byte is copied and no block table changes; the cost is one
// unmap and one map call per block plus one access grant.
#include <algorithm>
#include <new>
#include <vector>

#include "common.h"

struct kv_vmm_pool {
  int device = 0;
  uint32_t num_blocks = 0;
  uint64_t block_bytes = 0;
  uint8_t* kv_base = nullptr;
  uint8_t* slot_base = nullptr;
  std::vector<hipMemGenericAllocationHandle_t> handles;
  std::vector<uint8_t> have_handle;
  std::vector<uint8_t> in_kv;      // block's pages are mapped in the KV range
  std::vector<int32_t> lent;       // ids whose pages sit in the slot, in slot order
};

namespace warmkv {
namespace {

hipMemAllocationProp device_prop(int device) {
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = device;
  return prop;
}

int grant(void* ptr, size_t bytes, int device) {
  hipMemAccessDesc desc = {};
  desc.location.type = hipMemLocationTypeDevice;
  desc.location.id = device;
  desc.flags = hipMemAccessFlagsProtReadWrite;
  return hip_rc(hipMemSetAccess(ptr, bytes, &desc, 1));
}

// Put the pages of the last lent blocks back under their ids until `keep` are left in the slot.
// Access is granted once, over the span of ids that came back (everything in it is mapped again
// or was never unmapped), instead of block by block.
int give_back(kv_vmm_pool* pool, size_t keep) {
  const uint64_t bb = pool->block_bytes;
  uint32_t lo = ~0u, hi = 0u;
  while (pool->lent.size() > keep) {
    const size_t k = pool->lent.size() - 1;
    const uint32_t id = (uint32_t)pool->lent[k];
    if (hipMemUnmap(pool->slot_base + (uint64_t)k * bb, bb) != hipSuccess) return KV_E_HIP;
    pool->lent.pop_back();
    if (hipMemMap(pool->kv_base + (uint64_t)id * bb, bb, 0, pool->handles[id], 0) != hipSuccess) return KV_E_HIP;
    pool->in_kv[id] = 1;
    lo = std::min(lo, id);
    hi = std::max(hi, id);
  }
  if (lo > hi) return KV_OK;  // nothing came back
  // A span may hold ids that are still lent (keep != 0): grant run by run of mapped ids.
  for (uint32_t i = lo; i <= hi;) {
    if (!pool->in_kv[i]) { ++i; continue; }
    uint32_t j = i;
    while (j <= hi && pool->in_kv[j]) ++j;
    const int rc = grant(pool->kv_base + (uint64_t)i * bb, (size_t)(j - i) * bb, pool->device);
    if (rc != KV_OK) return rc;
    i = j;
  }
  return KV_OK;
}

// The `want` highest unused ids, highest first (empty if there are fewer).
std::vector<int32_t> highest_free(const kv_vmm_pool* pool, const uint64_t* live_host, uint32_t want) {
  std::vector<int32_t> ids;
  ids.reserve(want);
  for (uint32_t i = pool->num_blocks; i-- > 0 && ids.size() < want;)
    if (!((live_host[i >> 6] >> (i & 63)) & 1ull)) ids.push_back((int32_t)i);
  if (ids.size() < want) ids.clear();
  return ids;
}

// Move the pages of ids[first, end) into the slot at their slot positions and make them
// accessible.  On failure the caller rolls back with give_back().
int lend(kv_vmm_pool* pool, const std::vector<int32_t>& ids, uint32_t first, uint32_t end) {
  const uint64_t bb = pool->block_bytes;
  for (uint32_t k = first; k < end; ++k) {
    const uint32_t id = (uint32_t)ids[k];
    if (hipMemUnmap(pool->kv_base + (uint64_t)id * bb, bb) != hipSuccess) return KV_E_HIP;
    pool->in_kv[id] = 0;
    if (hipMemMap(pool->slot_base + (uint64_t)k * bb, bb, 0, pool->handles[id], 0) != hipSuccess) {
      // put the page back where it was so that the pool stays consistent
      if (hipMemMap(pool->kv_base + (uint64_t)id * bb, bb, 0, pool->handles[id], 0) == hipSuccess &&
          grant(pool->kv_base + (uint64_t)id * bb, bb, pool->device) == KV_OK)
        pool->in_kv[id] = 1;
      return KV_E_HIP;
    }
    pool->lent.push_back((int32_t)id);
  }
  if (end == first) return KV_OK;
  return grant(pool->slot_base + (uint64_t)first * bb, (size_t)(end - first) * bb, pool->device);
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

static int create_pool(uint32_t num_blocks, uint64_t block_bytes, kv_vmm_pool** out);

extern "C" int kv_vmm_pool_destroy(kv_vmm_pool* pool) {
  if (pool == nullptr) return KV_E_NULL;
  int rc = hip_rc(hipDeviceSynchronize());
  for (size_t k = 0; k < pool->lent.size(); ++k)
    if (hipMemUnmap(pool->slot_base + k * pool->block_bytes, pool->block_bytes) != hipSuccess) rc = KV_E_HIP;
  for (uint32_t i = 0; i < pool->num_blocks; ++i) {
    if (pool->in_kv[i] && hipMemUnmap(pool->kv_base + (uint64_t)i * pool->block_bytes, pool->block_bytes) != hipSuccess)
      rc = KV_E_HIP;
    if (pool->have_handle[i] && hipMemRelease(pool->handles[i]) != hipSuccess) rc = KV_E_HIP;
  }
  const size_t range = (size_t)pool->num_blocks * pool->block_bytes;
  if (pool->kv_base && hipMemAddressFree(pool->kv_base, range) != hipSuccess) rc = KV_E_HIP;
  if (pool->slot_base && hipMemAddressFree(pool->slot_base, range) != hipSuccess) rc = KV_E_HIP;
  delete pool;
  return rc;
}

extern "C" int kv_vmm_pool_create(uint32_t num_blocks, uint64_t block_bytes, kv_vmm_pool** out) {
  return guarded([&]() -> int { return create_pool(num_blocks, block_bytes, out); });
}

static int create_pool(uint32_t num_blocks, uint64_t block_bytes, kv_vmm_pool** out) {
  if (out == nullptr) return KV_E_NULL;
  *out = nullptr;
  if (num_blocks == 0 || num_blocks > kMaxBlocks || block_bytes == 0) return KV_E_RANGE;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return KV_E_HIP;
  const hipMemAllocationProp prop = device_prop(device);
  size_t gran = 0;
  if (hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum) != hipSuccess || gran == 0)
    return KV_E_HIP;
  if (block_bytes % gran != 0) return KV_E_ALIGN;

  kv_vmm_pool* p = new (std::nothrow) kv_vmm_pool;
  if (p == nullptr) return KV_E_HIP;
  p->device = device;
  p->num_blocks = num_blocks;
  p->block_bytes = block_bytes;
  try {
    p->handles.resize(num_blocks);
    p->have_handle.assign(num_blocks, 0);
    p->in_kv.assign(num_blocks, 0);
    p->lent.reserve(num_blocks);  // so that lending never allocates
  } catch (...) {
    delete p;
    throw;
  }
  const size_t range = (size_t)num_blocks * block_bytes;
  void* a = nullptr;
  void* b = nullptr;
  if (hipMemAddressReserve(&a, range, 0, nullptr, 0) != hipSuccess) { delete p; return KV_E_HIP; }
  p->kv_base = (uint8_t*)a;
  if (hipMemAddressReserve(&b, range, 0, nullptr, 0) != hipSuccess) { kv_vmm_pool_destroy(p); return KV_E_HIP; }
  p->slot_base = (uint8_t*)b;
  for (uint32_t i = 0; i < num_blocks; ++i) {
    if (hipMemCreate(&p->handles[i], block_bytes, &prop, 0) != hipSuccess) { kv_vmm_pool_destroy(p); return KV_E_HIP; }
    p->have_handle[i] = 1;
    if (hipMemMap(p->kv_base + (uint64_t)i * block_bytes, block_bytes, 0, p->handles[i], 0) != hipSuccess) {
      kv_vmm_pool_destroy(p);
      return KV_E_HIP;
    }
    p->in_kv[i] = 1;
  }
  if (grant(p->kv_base, range, device) != KV_OK) { kv_vmm_pool_destroy(p); return KV_E_HIP; }
  *out = p;
  return KV_OK;
}

extern "C" void* kv_vmm_kv_base(const kv_vmm_pool* pool) { return pool ? pool->kv_base : nullptr; }
extern "C" void* kv_vmm_slot_base(const kv_vmm_pool* pool) { return pool ? pool->slot_base : nullptr; }

extern "C" int kv_vmm_reclaim(kv_vmm_pool* pool, const uint64_t* live_host, uint32_t want, int32_t* ids_out) {
  return kv_vmm_reclaim_load(pool, live_host, want, want, nullptr, 0, nullptr, ids_out);
}

extern "C" int kv_vmm_reclaim_load(kv_vmm_pool* pool, const uint64_t* live_host, uint32_t want, uint32_t chunk_blocks,
                                   const wm_tensor* tensors, uint32_t n_tensors, void* copy_stream, int32_t* ids_out) {
  return guarded([&]() -> int {
    if (pool == nullptr || live_host == nullptr || (n_tensors != 0 && tensors == nullptr)) return KV_E_NULL;
    if (!pool->lent.empty()) return KV_E_RANGE;
    const uint64_t bb = pool->block_bytes;
    const uint64_t slot_bytes = (uint64_t)want * bb;
    // weight extents: inside the slot prefix, pairwise disjoint, before anything changes
    std::vector<uint32_t> order;
    for (uint32_t i = 0; i < n_tensors; ++i) {
      if (tensors[i].dst_offset > slot_bytes || tensors[i].bytes > slot_bytes - tensors[i].dst_offset) return KV_E_TOOBIG;
      if (tensors[i].bytes == 0) continue;
      if (tensors[i].host_ptr == nullptr) return KV_E_NULL;
      order.push_back(i);
    }
    std::sort(order.begin(), order.end(),
              [&](uint32_t a, uint32_t b) { return tensors[a].dst_offset < tensors[b].dst_offset; });
    for (size_t j = 1; j < order.size(); ++j)
      if (tensors[order[j - 1]].dst_offset + tensors[order[j - 1]].bytes > tensors[order[j]].dst_offset)
        return KV_E_OVERLAP;
    if (want == 0) return KV_OK;
    const std::vector<int32_t> ids = highest_free(pool, live_host, want);
    if (ids.empty()) return KV_E_NOSPACE;
    int rc = hip_rc(hipDeviceSynchronize());  // nothing may be in flight on pages that change address
    if (rc != KV_OK) return rc;
    if (chunk_blocks == 0) chunk_blocks = 64;
    size_t next = 0;  // first extent (in offset order) that still has bytes to send
    uint64_t sent_to = 0;  // slot offset up to which extent order[next] has been sent
    for (uint32_t first = 0; first < want; first += chunk_blocks) {
      const uint32_t end = want - first < chunk_blocks ? want : first + chunk_blocks;
      rc = lend(pool, ids, first, end);
      if (rc != KV_OK) {
        // Copies already enqueued target pages that are about to leave the slot: let them land first.
        if (n_tensors != 0) (void)hipStreamSynchronize((hipStream_t)copy_stream);
        (void)give_back(pool, 0);
        return rc;
      }
      // every weight byte below the mapped mark goes out now, in offset order
      const uint64_t mark = (uint64_t)end * bb;
      while (next < order.size()) {
        const wm_tensor& t = tensors[order[next]];
        const uint64_t from = std::max(sent_to, t.dst_offset), to = std::min(mark, t.dst_offset + t.bytes);
        if (from < to) {
          rc = hip_rc(hipMemcpyAsync(pool->slot_base + from, (const uint8_t*)t.host_ptr + (from - t.dst_offset),
                                     to - from, hipMemcpyHostToDevice, (hipStream_t)copy_stream));
          if (rc != KV_OK) return rc;  // the pages stay lent; kv_vmm_restore puts them back
        }
        if (t.dst_offset + t.bytes > mark) { sent_to = mark; break; }
        sent_to = 0;
        ++next;
      }
    }
    if (ids_out != nullptr) std::copy(ids.begin(), ids.end(), ids_out);
    return KV_OK;
  });
}

extern "C" uint32_t kv_vmm_lent(const kv_vmm_pool* pool) { return pool ? (uint32_t)pool->lent.size() : 0u; }

extern "C" int kv_vmm_restore(kv_vmm_pool* pool) {
  if (pool == nullptr) return KV_E_NULL;
  const int rc = hip_rc(hipDeviceSynchronize());
  if (rc != KV_OK) return rc;
  return give_back(pool, 0);
}
