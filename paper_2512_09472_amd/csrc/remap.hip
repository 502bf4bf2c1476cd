// Block-table rewrite: every entry e >= 0 becomes new_id[e].  Runs on the
// stream right behind the block copy, so the engine's next step sees moved
// blocks and rewritten tables together and never learns anything moved (the
// engine keeps one address space: paper App. C).
//
// A few MiB at most: four entries per lane as one 128-bit access, new_id
// (<= 256 KiB for the benchmark pools) served from L2.  Entries that name an id
// outside the pool or a block that was not live are left alone and counted,
// one atomic per wavefront that saw any.
#include "common.h"

namespace warmkv {
namespace {

__device__ __forceinline__ int32_t remap_one(int32_t e, const int32_t* __restrict__ new_id,
                                             uint32_t num_blocks, uint32_t& bad) {
  if (e < 0) return e;
  if ((uint32_t)e >= num_blocks) { ++bad; return e; }
  const int32_t t = new_id[e];
  if (t < 0) { ++bad; return e; }
  return t;
}

__global__ __launch_bounds__(256) void remap_kernel(int32_t* tables, uint64_t n_entries,
                                                    const int32_t* __restrict__ new_id,
                                                    uint32_t num_blocks,
                                                    kv_plan_state* __restrict__ state) {
  if (state->status != KV_OK || state->bad_plan != 0u) return;
  const uint64_t n_vec = n_entries / 4;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  const uint64_t gid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t bad = 0;
  i32x4* tv = (i32x4*)tables;
  for (uint64_t i = gid; i < n_vec; i += stride) {
    const i32x4 e = tv[i];
    i32x4 r;
    r.x = remap_one(e.x, new_id, num_blocks, bad);
    r.y = remap_one(e.y, new_id, num_blocks, bad);
    r.z = remap_one(e.z, new_id, num_blocks, bad);
    r.w = remap_one(e.w, new_id, num_blocks, bad);
    if (r.x != e.x || r.y != e.y || r.z != e.z || r.w != e.w) tv[i] = r;
  }
  for (uint64_t i = n_vec * 4 + gid; i < n_entries; i += stride) {  // up to three tail entries
    const int32_t e = tables[i];
    const int32_t r = remap_one(e, new_id, num_blocks, bad);
    if (r != e) tables[i] = r;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) bad += __shfl_xor(bad, off, kWave);
  if ((threadIdx.x & (kWave - 1)) == 0 && bad != 0) atomicAdd(&state->n_bad_entries, bad);
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int kv_remap_tables(int32_t* tables, uint32_t num_seqs, uint32_t max_blocks_per_seq,
                               const kv_plan* plan, void* stream) {
  if (plan == nullptr || plan->state == nullptr || plan->new_id == nullptr) return KV_E_NULL;
  if (plan->boundary > plan->num_blocks) return KV_E_RANGE;
  const uint64_t n_entries = (uint64_t)num_seqs * max_blocks_per_seq;
  if (n_entries == 0) return KV_OK;
  if (tables == nullptr) return KV_E_NULL;
  if (((uintptr_t)tables % 16u) != 0) return KV_E_ALIGN;
  uint64_t groups = (n_entries / 4 + 255) / 256;
  if (groups == 0) groups = 1;
  if (groups > 256 * 8) groups = 256 * 8;
  hipLaunchKernelGGL(remap_kernel, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream, tables,
                     n_entries, plan->new_id, plan->num_blocks, plan->state);
  return launch_rc();
}
