// kv_reclaim_static: the reclaim step (plan, block copy, table rewrite) for callers that cannot
// allocate device memory - code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc.  The other entry points take the plan's workspace from the caller
// (kv_plan_bind); here it lives in a file-scope device array, one copy per GPU, which the library
// holds until the process ends.  Nothing in this file allocates or frees.
#include <atomic>
#include <mutex>

#include "common.h"

namespace warmkv {
namespace {

// Room for the plan of the largest supported pool: header, bitmap, two move lists of at most
// num_blocks / 2 entries, and the id map.  About 2 MiB.
constexpr size_t kScratchBytes = 256 + KV_STATIC_MAX_BLOCKS / 8 + 2 * (KV_STATIC_MAX_BLOCKS / 2) * 4 +
                                 (size_t)KV_STATIC_MAX_BLOCKS * 4;

static __device__ __align__(256) uint8_t scratch[kScratchBytes];

// In host code `scratch` is only a handle for the symbol, not a device address: each GPU has its
// own copy of the array at its own address, looked up once per device and kept here.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_of_device[kMaxDevices];
std::mutex g_lookup_mutex;

int scratch_on_current_device(void** out) {
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return KV_E_HIP;
  if (device < 0 || device >= kMaxDevices) return KV_E_RANGE;
  void* ptr = g_scratch_of_device[device].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    std::lock_guard<std::mutex> lock(g_lookup_mutex);
    ptr = g_scratch_of_device[device].load(std::memory_order_relaxed);
    if (ptr == nullptr) {
      if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return KV_E_HIP;
      g_scratch_of_device[device].store(ptr, std::memory_order_release);
    }
  }
  *out = ptr;
  return KV_OK;
}

// The plan's header, as kv_plan_fetch would report it, into the caller's device memory.
__global__ void publish_state_kernel(const kv_plan_state* __restrict__ state, kv_plan_state* __restrict__ out) {
  kv_plan_state st = *state;
  if (st.status == KV_OK && st.bad_plan != 0u) st.status = KV_E_BADPLAN;
  *out = st;
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int kv_reclaim_static(const kv_pool_desc* pool, uint32_t boundary, const uint64_t* live_in,
                                 uint64_t* live_out, int32_t* tables, uint32_t num_seqs,
                                 uint32_t max_blocks_per_seq, kv_plan_state* state_out, void* stream) {
  if (pool == nullptr || live_out == nullptr || state_out == nullptr) return KV_E_NULL;
  const uint32_t nb = pool->num_blocks;
  if (boundary > nb) return KV_E_RANGE;
  if (nb > KV_STATIC_MAX_BLOCKS) return KV_E_TOOBIG;  // the plan would not fit the static workspace
  const size_t need = kv_plan_workspace_bytes(nb, boundary);
  if (need == 0 || need > kScratchBytes) return KV_E_TOOBIG;
  // everything the three steps would refuse is refused before the first launch
  if (!pool_extent_ok(*pool)) return KV_E_RANGE;
  if (!copy_units_fit(*pool, nb - boundary < boundary ? nb - boundary : boundary)) return KV_E_RANGE;
  if ((pool->tile_bytes % 16u) != 0 || ((uintptr_t)pool->base % 256u) != 0) return KV_E_ALIGN;
  if (pool->layer_stride_bytes != 0 && (pool->layer_stride_bytes % 256u != 0 ||
                                        pool->layer_stride_bytes < (uint64_t)nb * pool->tile_bytes))
    return KV_E_RANGE;
  if (nb != 0 && (pool->base == nullptr || live_in == nullptr)) return KV_E_NULL;
  const uint64_t n_entries = (uint64_t)num_seqs * max_blocks_per_seq;
  if (n_entries != 0 && tables == nullptr) return KV_E_NULL;
  if (((uintptr_t)tables % 16u) != 0) return KV_E_ALIGN;

  void* ws = nullptr;
  int rc = scratch_on_current_device(&ws);
  if (rc != KV_OK) return rc;
  kv_plan plan;
  rc = kv_plan_bind(&plan, ws, kScratchBytes, nb, boundary);
  if (rc != KV_OK) return rc;
  plan.live_out = live_out;  // the bitmap after the move is an output: straight into the caller's buffer
  // The planner rewrites the whole header (counters included) and every entry the later steps
  // read, so nothing of a previous call's plan has to be cleared first.
  rc = kv_plan_reclaim(live_in, &plan, stream);
  if (rc != KV_OK) return rc;
  rc = kv_compact(pool, &plan, stream);
  if (rc != KV_OK) return rc;
  rc = kv_remap_tables(tables, num_seqs, max_blocks_per_seq, &plan, stream);
  if (rc != KV_OK) return rc;
  hipLaunchKernelGGL(publish_state_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, plan.state, state_out);
  return launch_rc();
}
