// Block copy of the KV reclaim: for k < n_moves, block dst[k] <- block src[k].
// This is the bandwidth-bound step (2 * n_moves * block_bytes of HBM traffic);
// the rest of the path is microseconds.  It stands in for the paper's step of
// mapping the pages under unused KV blocks into the new model's slot (App. C,
// Fig. 4b step 2): here the unused space is made contiguous instead.
//
// Shape.  The work list is (move, chunk) units of 64 KiB in list order (in a
// layer-major pool a move is one tile per layer slab: (move, layer, chunk)).  One
// workgroup per compute unit stays resident and draws units from a single
// device-wide ticket counter, so at any moment the 256 workgroups stream one
// narrow, advancing window (about 16 MiB of sources and as much of
// destinations).  Measured on MI355X this ordering is what matters: a static
// grid-stride assignment lets workgroups drift apart, the window smears over
// hundreds of MiB, and the same loads and stores run about 25 % slower.  The
// ticket for the next unit is drawn before the current unit is copied, which
// hides the atomic's latency; 64 KiB per ticket keeps the counter well below
// the rate one address sustains.  The grid never depends on n_moves, which
// lives in device memory (no host sync after the planner).
//
// Each lane issues UNROLL independent 128-bit loads before its first store; a
// wavefront covers 1 KiB per instruction, fully coalesced.  Accesses are
// non-temporal: gigabytes stream through once and should not evict anything.
// Sources lie at or above the boundary and destinations below it, so no two
// moves overlap and any order is correct; the kernel checks that property per
// move instead of staging through LDS.
#include "common.h"

namespace warmkv {
namespace {

constexpr uint32_t kCopyThreads = 256;
constexpr uint32_t kVecBytes = 16;
constexpr uint32_t kRowBytes = kCopyThreads * kVecBytes;  // 4 KiB per workgroup per instruction
constexpr uint32_t kDefaultChunk = 65536;

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void store16(u32x4* p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// A move copies `segs` contiguous segments of seg_bytes each: the whole block
// in a block-major pool (segs = 1), one tile per layer slab in a layer-major
// pool (segs = L).  Segment g of block i starts at i*block_stride + g*seg_stride.
struct CopyArgs {
  uint8_t* base;
  uint64_t block_stride;
  uint64_t seg_stride;
  uint64_t seg_bytes;
  const int32_t* src;
  const int32_t* dst;
  kv_plan_state* state;
  uint32_t num_blocks;
  uint32_t boundary;
  uint32_t chunk_bytes;
  uint32_t chunks_per_seg;
  uint32_t units_per_move;  // segs * chunks_per_seg
  uint32_t seg_outer;       // unit order: 1 = segment-major (layer by layer), 0 = move-major
};

// Copy unit u = (move k, segment g, chunk c).  u is wavefront-uniform.
template <int UNROLL, bool NT>
__device__ __forceinline__ void copy_unit(const CopyArgs& a, uint32_t n_moves, uint32_t u, uint32_t tid) {
  constexpr uint32_t kStep = kRowBytes * UNROLL;  // bytes per workgroup per inner iteration
  uint32_t k, g, c;
  if (a.seg_outer) {  // all moves of segment (layer) 0, then of segment 1, ...
    const uint32_t per_seg = n_moves * a.chunks_per_seg;
    g = u / per_seg;
    const uint32_t r = u - g * per_seg;
    k = r / a.chunks_per_seg;
    c = r - k * a.chunks_per_seg;
  } else {            // all segments of move 0, then of move 1, ...
    k = u / a.units_per_move;
    const uint32_t r = u - k * a.units_per_move;
    g = r / a.chunks_per_seg;
    c = r - g * a.chunks_per_seg;
  }
  const uint32_t s = (uint32_t)a.src[k], d = (uint32_t)a.dst[k];
  if (s < a.boundary || s >= a.num_blocks || d >= a.boundary) {  // never true for a planner-made plan
    if (tid == 0) atomicExch(&a.state->status, KV_E_BADPLAN);
    return;
  }
  const uint64_t off = (uint64_t)g * a.seg_stride + (uint64_t)c * a.chunk_bytes;
  const uint64_t left = a.seg_bytes - (uint64_t)c * a.chunk_bytes;
  const uint32_t len = left < a.chunk_bytes ? (uint32_t)left : a.chunk_bytes;
  const u32x4* __restrict__ sp = (const u32x4*)(a.base + (uint64_t)s * a.block_stride + off);
  u32x4* __restrict__ dp = (u32x4*)(a.base + (uint64_t)d * a.block_stride + off);

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

// Units in ticket order: one device-wide counter, next ticket drawn ahead.
template <int UNROLL, bool NT>
__global__ __launch_bounds__(kCopyThreads) void compact_ticket_kernel(CopyArgs a) {
  // No early return: every workgroup must draw its one out-of-range ticket and
  // sign out below, or the counters would not return to zero.
  const uint32_t n_moves = a.state->status == KV_OK ? a.state->n_moves : 0u;
  const uint32_t n_units = n_moves * a.units_per_move;  // host checked: fits 31 bits
  const uint32_t tid = threadIdx.x;
  __shared__ uint32_t s_ticket[2];
  if (tid == 0) s_ticket[0] = atomicAdd(&a.state->ticket, 1u);
  __syncthreads();
  uint32_t slot = 0;
  for (;;) {
    const uint32_t u = __builtin_amdgcn_readfirstlane(s_ticket[slot]);
    if (u >= n_units) break;
    // The other slot was last read before the previous barrier: free to refill.
    if (tid == 0) s_ticket[slot ^ 1u] = atomicAdd(&a.state->ticket, 1u);
    copy_unit<UNROLL, NT>(a, n_moves, u, tid);
    __syncthreads();
    slot ^= 1u;
  }
  // Every workgroup draws exactly one ticket >= n_units.  The last one out
  // puts both counters back to zero for the next call on this plan.
  if (tid == 0) {
    const uint32_t out = atomicAdd(&a.state->finished, 1u);
    if (out == gridDim.x - 1u) {
      atomicExch(&a.state->ticket, 0u);
      atomicExch(&a.state->finished, 0u);
    }
  }
}

// Units in static grid-stride order (kept for comparison; slower on MI355X).
template <int UNROLL, bool NT>
__global__ __launch_bounds__(kCopyThreads) void compact_static_kernel(CopyArgs a) {
  if (a.state->status != KV_OK) return;
  const uint32_t n_moves = a.state->n_moves;
  const uint32_t n_units = n_moves * a.units_per_move;
  for (uint32_t u = blockIdx.x; u < n_units; u += gridDim.x) copy_unit<UNROLL, NT>(a, n_moves, u, threadIdx.x);
}

template <int UNROLL, bool NT>
int launch(const CopyArgs& a, uint32_t workgroups, bool tickets, hipStream_t s) {
  if (tickets)
    hipLaunchKernelGGL((compact_ticket_kernel<UNROLL, NT>), dim3(workgroups), dim3(kCopyThreads), 0, s, a);
  else
    hipLaunchKernelGGL((compact_static_kernel<UNROLL, NT>), dim3(workgroups), dim3(kCopyThreads), 0, s, a);
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

  uint32_t workgroups = 0, chunk = kDefaultChunk, flags = 0u;
  if (tuning != nullptr) {
    workgroups = tuning->workgroups;
    if (tuning->chunk_bytes) chunk = tuning->chunk_bytes;
    flags = tuning->flags;
  }
  if ((chunk % kRowBytes) != 0 || workgroups > (1u << 20)) return KV_E_RANGE;
  const uint32_t unroll_sel = (flags >> 4) & 0xFu;  // 0 = pick from the chunk size
  const uint32_t unroll = unroll_sel ? unroll_sel
                                     : (chunk >= 8 * kRowBytes ? 8u : (chunk >= 4 * kRowBytes ? 4u : (chunk >= 2 * kRowBytes ? 2u : 1u)));
  if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return KV_E_RANGE;

  const bool layer_major = pool->layer_stride_bytes != 0;
  if (layer_major && (pool->layer_stride_bytes % 256u != 0 ||
                      pool->layer_stride_bytes < (uint64_t)pool->num_blocks * pool->tile_bytes))
    return KV_E_RANGE;
  if (plan->capacity == 0 || pool->num_blocks == 0) return KV_OK;  // nothing can move
  if (pool->base == nullptr || plan->src == nullptr || plan->dst == nullptr) return KV_E_NULL;
  if (((uintptr_t)pool->base % 256u) != 0) return KV_E_ALIGN;

  CopyArgs a;
  a.base = (uint8_t*)pool->base;
  if (layer_major) {
    a.block_stride = pool->tile_bytes;
    a.seg_stride = pool->layer_stride_bytes;
    a.seg_bytes = pool->tile_bytes;
  } else {
    a.block_stride = (uint64_t)pool->num_layers * pool->tile_bytes;
    a.seg_stride = 0;
    a.seg_bytes = a.block_stride;
  }
  const uint64_t segs = layer_major ? pool->num_layers : 1u;
  const uint64_t chunks_per_seg = (a.seg_bytes + chunk - 1) / chunk;
  if (segs * chunks_per_seg * plan->capacity >= (1ull << 31)) return KV_E_RANGE;  // unit ids are 32-bit
  a.src = plan->src;
  a.dst = plan->dst;
  a.state = plan->state;
  a.num_blocks = plan->num_blocks;
  a.boundary = plan->boundary;
  a.chunk_bytes = chunk;
  a.chunks_per_seg = (uint32_t)chunks_per_seg;
  a.units_per_move = (uint32_t)(segs * chunks_per_seg);
  a.seg_outer = (layer_major && (flags & 4u) == 0) ? 1u : 0u;

  if (workgroups == 0) {  // one resident workgroup per compute unit
    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
      return KV_E_HIP;
    workgroups = (uint32_t)cus;
  }

  const bool nt = (flags & 1u) == 0;
  const bool tickets = (flags & 2u) == 0;
  hipStream_t s = (hipStream_t)stream;
  switch (unroll) {
    case 1: return nt ? launch<1, true>(a, workgroups, tickets, s) : launch<1, false>(a, workgroups, tickets, s);
    case 2: return nt ? launch<2, true>(a, workgroups, tickets, s) : launch<2, false>(a, workgroups, tickets, s);
    case 4: return nt ? launch<4, true>(a, workgroups, tickets, s) : launch<4, false>(a, workgroups, tickets, s);
    default: return nt ? launch<8, true>(a, workgroups, tickets, s) : launch<8, false>(a, workgroups, tickets, s);
  }
}

extern "C" int kv_compact(const kv_pool_desc* pool, const kv_plan* plan, void* stream) {
  return kv_compact_launch(pool, plan, nullptr, stream);
}
