// kv_reclaim: the reclaim step (plan, block copy, table rewrite) as one call, and for small pools as
// one kernel launch.  (What the step computes: paper App. C, Fig. 4b steps 1-2, as in plan.hip,
// compact.hip and remap.hip.)
//
// A pool of a few hundred or thousand blocks is reclaimed in microseconds, and then the three
// launches and the waits between them cost more than the work.  Here no workgroup waits for another:
// every workgroup reads the whole bitmap (at most 4 KiB), ranks it in LDS for itself, and from then
// on answers "which id is the k-th mover" and "which is the k-th free id below the boundary" by a
// binary search over the per-word ranks plus a select inside one word.  With that, each workgroup
// writes its share of the plan's arrays, copies its share of the blocks and nothing has to be
// handed from one workgroup to another.  The table rewrite and the count of bad entries are left to
// workgroup 0 (a count needs one owner; tables here are small), which takes no blocks to copy when
// there are other workgroups.
#include "bitmap.h"
#include "common.h"

namespace warmkv {
namespace {

constexpr uint32_t kThreads = 256;
constexpr uint32_t kMaxWords = 2 * kThreads;            // two bitmap words per lane: 32 768 blocks
constexpr uint64_t kMaxRegionBytes = 128ull << 20;      // above this the three-launch path is faster
constexpr uint64_t kMaxEntries = 1u << 14;              // table entries one workgroup rewrites in a few us
constexpr uint32_t kChunk = 65536;
constexpr uint32_t kVec = 16;

struct SmallArgs {
  const uint64_t* live_in;
  uint32_t n_words, num_blocks, boundary;
  int32_t* src;
  int32_t* dst;
  int32_t* new_id;
  uint64_t* live_out;
  kv_plan_state* state;
  uint8_t* base;
  uint64_t block_stride, seg_stride, seg_bytes;
  uint32_t segs, chunks_per_seg;
  int32_t* tables;
  uint32_t n_entries;
};

// len bytes (multiple of 16), all 256 lanes: sixteen 128-bit loads in flight per lane (a whole
// 64 KiB chunk in one round trip), then eight, then a tail.
__device__ __forceinline__ void copy_span(const u32x4* __restrict__ sp, u32x4* __restrict__ dp, uint32_t len,
                                          uint32_t tid) {
  const uint32_t n = len / kVec;
  uint32_t i = tid;
  for (; i + 15u * kThreads < n; i += 16u * kThreads) {
    u32x4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = __builtin_nontemporal_load(sp + i + j * kThreads);
#pragma unroll
    for (int j = 0; j < 16; ++j) __builtin_nontemporal_store(v[j], dp + i + j * kThreads);
  }
  for (; i + 7u * kThreads < n; i += 8u * kThreads) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(sp + i + j * kThreads);
#pragma unroll
    for (int j = 0; j < 8; ++j) __builtin_nontemporal_store(v[j], dp + i + j * kThreads);
  }
  for (; i < n; i += kThreads) __builtin_nontemporal_store(__builtin_nontemporal_load(sp + i), dp + i);
}

__global__ __launch_bounds__(kThreads) void reclaim_small_kernel(SmallArgs a) {
  __shared__ uint64_t s_live[kMaxWords];  // word & valid
  __shared__ uint64_t s_rank[kMaxWords];  // movers before the word (high half), free ids below b before it (low half)
  __shared__ uint64_t s_wave[kThreads / kWave];
  __shared__ uint32_t s_bad[kThreads / kWave];

  const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const uint32_t nb = a.num_blocks, b = a.boundary;

  // ---- ranks of the whole bitmap, in every workgroup: lane t owns words 2t and 2t+1
  const uint32_t w0 = 2u * tid, w1 = w0 + 1u;
  const WordBits b0 = classify(w0 < a.n_words ? a.live_in[w0] : 0ull, w0, nb, b);
  const WordBits b1 = classify(w1 < a.n_words ? a.live_in[w1] : 0ull, w1, nb, b);
  const uint64_t c0 = pack_counts(b0), c1 = pack_counts(b1);
  const uint64_t incl = wave_inclusive_scan(c0 + c1);
  if (lane == kWave - 1) s_wave[wave] = incl;
  __syncthreads();
  uint64_t wave_base = 0, total = 0;
#pragma unroll
  for (uint32_t w = 0; w < kThreads / kWave; ++w) {
    const uint64_t t = s_wave[w];
    if (w < wave) wave_base += t;
    total += t;
  }
  const uint64_t excl = wave_base + incl - (c0 + c1);
  s_live[w0] = b0.live;
  s_live[w1] = b1.live;
  s_rank[w0] = excl;
  s_rank[w1] = excl + c0;
  const uint32_t n_moves = (uint32_t)(total >> 32), n_avail = (uint32_t)total;
  if (n_moves > n_avail) {  // uniform over the grid: nothing else is written
    if (blockIdx.x == 0 && tid == 0) {
      kv_plan_state st = {};
      st.status = KV_E_NOSPACE;
      st.n_free_below = n_avail;
      *a.state = st;
    }
    return;
  }
  __syncthreads();

  const uint32_t n_words = a.n_words;
  // Word that holds the k-th mover (hi = true) or the k-th free id below the boundary: the last
  // word whose rank is <= k.  The next word's rank is > k, so the k-th one lies inside.
  auto word_of = [&](uint32_t k, bool hi) -> uint32_t {
    uint32_t lo_w = 0, hi_w = n_words;
    while (hi_w - lo_w > 1u) {
      const uint32_t mid = (lo_w + hi_w) >> 1;
      const uint64_t r = s_rank[mid];
      if ((hi ? (uint32_t)(r >> 32) : (uint32_t)r) <= k) lo_w = mid;
      else hi_w = mid;
    }
    return lo_w;
  };
  auto kth_mover = [&](uint32_t k) -> uint32_t {
    const uint32_t w = word_of(k, true);
    const uint64_t movers = s_live[w] & ~low_mask(w * 64u, b);
    return w * 64u + nth_set_bit(movers, k - (uint32_t)(s_rank[w] >> 32));
  };
  auto kth_free = [&](uint32_t k) -> uint32_t {
    const uint32_t w = word_of(k, false);
    const uint64_t avail = ~s_live[w] & low_mask(w * 64u, b);
    return w * 64u + nth_set_bit(avail, k - (uint32_t)s_rank[w]);
  };

  // ---- the plan's arrays, one id per lane per pass over the whole grid
  const uint32_t gid = blockIdx.x * kThreads + tid, stride = gridDim.x * kThreads;
  for (uint32_t id = gid; id < nb; id += stride) {
    const uint32_t w = id >> 6, bit = id & 63u;
    const uint64_t live = s_live[w], lo = low_mask(w * 64u, b);
    const uint64_t movers = live & ~lo, avail = ~live & lo, below = (1ull << bit) - 1ull;
    int32_t to = -1;
    if ((movers >> bit) & 1ull) {
      const uint32_t k = (uint32_t)(s_rank[w] >> 32) + (uint32_t)__popcll(movers & below);
      to = (int32_t)kth_free(k);
      a.src[k] = (int32_t)id;
    } else if ((live >> bit) & 1ull) {
      to = (int32_t)id;
    } else if ((avail >> bit) & 1ull) {
      const uint32_t r = (uint32_t)s_rank[w] + (uint32_t)__popcll(avail & below);
      if (r < n_moves) a.dst[r] = (int32_t)id;
    }
    a.new_id[id] = to;
  }
  for (uint32_t w = gid; w < n_words; w += stride) {  // bitmap after the move
    const uint64_t live = s_live[w], lo = low_mask(w * 64u, b), avail = ~live & lo;
    const uint32_t r = (uint32_t)s_rank[w];
    uint64_t taken = 0;
    if (r < n_moves) {
      const uint32_t want = n_moves - r;
      taken = want >= (uint32_t)__popcll(avail) ? avail : lowest_set_bits(avail, want);
    }
    a.live_out[w] = (live & lo) | taken;
  }

  // ---- block copy: unit u = (move, segment, chunk), dealt out round robin; workgroup 0 keeps out
  // of it when it is not alone, it has the tables to do
  const uint32_t units_per_move = a.segs * a.chunks_per_seg;
  const uint32_t n_units = n_moves * units_per_move;
  const uint32_t copiers = gridDim.x > 1u ? gridDim.x - 1u : 1u;
  const uint32_t me = gridDim.x > 1u ? blockIdx.x - 1u : 0u;  // workgroup 0 of a larger grid: 0xFFFFFFFF, no units
  if (gridDim.x == 1u || blockIdx.x != 0u) {
    for (uint32_t u = me; u < n_units; u += copiers) {
      const uint32_t k = u / units_per_move, r = u - k * units_per_move;
      const uint32_t g = r / a.chunks_per_seg, c = r - g * a.chunks_per_seg;
      const uint64_t s_id = kth_mover(k), d_id = kth_free(k);  // same in every lane: LDS broadcasts
      const uint64_t off = (uint64_t)g * a.seg_stride + (uint64_t)c * kChunk;
      const uint64_t left = a.seg_bytes - (uint64_t)c * kChunk;
      const uint32_t len = left < kChunk ? (uint32_t)left : kChunk;
      copy_span((const u32x4*)(a.base + s_id * a.block_stride + off), (u32x4*)(a.base + d_id * a.block_stride + off),
                len, tid);
    }
  }
  if (blockIdx.x != 0u) return;

  // ---- workgroup 0: table rewrite, count of the entries left alone, and the plan's header
  uint32_t bad = 0;
  auto remap_one = [&](int32_t e) -> int32_t {
    if (e < 0) return e;
    if ((uint32_t)e >= nb) { ++bad; return e; }
    const uint32_t w = (uint32_t)e >> 6, bit = (uint32_t)e & 63u;
    const uint64_t live = s_live[w];
    if (!((live >> bit) & 1ull)) { ++bad; return e; }
    if ((uint32_t)e < b) return e;  // stays where it is
    const uint64_t movers = live & ~low_mask(w * 64u, b);
    const uint32_t k = (uint32_t)(s_rank[w] >> 32) + (uint32_t)__popcll(movers & ((1ull << bit) - 1ull));
    return (int32_t)kth_free(k);
  };
  // Four 128-bit loads per lane are in flight before the first entry is looked at: one workgroup
  // has the whole table, so the loads' latency must not add up entry by entry.
  const uint32_t n_vec = a.n_entries / 4u;
  i32x4* tv = (i32x4*)a.tables;
  for (uint32_t i0 = tid; i0 < n_vec; i0 += 4u * kThreads) {
    i32x4 e[4];
#pragma unroll
    for (uint32_t j = 0; j < 4u; ++j)
      if (i0 + j * kThreads < n_vec) e[j] = tv[i0 + j * kThreads];
#pragma unroll
    for (uint32_t j = 0; j < 4u; ++j) {
      if (i0 + j * kThreads >= n_vec) break;
      i32x4 r;
      r.x = remap_one(e[j].x);
      r.y = remap_one(e[j].y);
      r.z = remap_one(e[j].z);
      r.w = remap_one(e[j].w);
      if (r.x != e[j].x || r.y != e[j].y || r.z != e[j].z || r.w != e[j].w) tv[i0 + j * kThreads] = r;
    }
  }
  for (uint32_t i = n_vec * 4u + tid; i < a.n_entries; i += kThreads) {  // up to three tail entries
    const int32_t e = a.tables[i], r = remap_one(e);
    if (r != e) a.tables[i] = r;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) bad += __shfl_xor(bad, off, kWave);
  if (lane == 0) s_bad[wave] = bad;
  __syncthreads();
  if (tid == 0) {
    kv_plan_state st = {};
    st.status = KV_OK;
    st.n_moves = n_moves;
    st.n_free_below = n_avail;
    for (uint32_t w = 0; w < kThreads / kWave; ++w) st.n_bad_entries += s_bad[w];
    *a.state = st;
  }
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int kv_reclaim(const kv_pool_desc* pool, const kv_plan* plan, const uint64_t* live_in, int32_t* tables,
                          uint32_t num_seqs, uint32_t max_blocks_per_seq, void* stream) {
  // Everything the three steps would refuse is refused before the first launch.
  if (pool == nullptr || plan == nullptr || plan->state == nullptr || plan->new_id == nullptr ||
      plan->live_out == nullptr)
    return KV_E_NULL;
  const uint32_t nb = plan->num_blocks, b = plan->boundary;
  if (pool->num_blocks != nb || b > nb || nb > kMaxBlocks) return KV_E_RANGE;
  if (plan->capacity != (nb - b < b ? nb - b : b)) return KV_E_RANGE;
  if (plan->capacity != 0 && (plan->src == nullptr || plan->dst == nullptr)) return KV_E_NULL;
  if (!pool_extent_ok(*pool) || !copy_units_fit(*pool, plan->capacity)) return KV_E_RANGE;
  if ((pool->tile_bytes % kVec) != 0) return KV_E_ALIGN;
  const bool layer_major = pool->layer_stride_bytes != 0;
  if (layer_major && (pool->layer_stride_bytes % 256u != 0 ||
                      pool->layer_stride_bytes < (uint64_t)nb * pool->tile_bytes))
    return KV_E_RANGE;
  const uint32_t n_words = (nb + 63u) / 64u;
  if (n_words != 0 && live_in == nullptr) return KV_E_NULL;
  const uintptr_t a0 = (uintptr_t)live_in, a1 = a0 + (uintptr_t)n_words * 8u;
  const uintptr_t o0 = (uintptr_t)plan->live_out, o1 = o0 + (uintptr_t)n_words * 8u;
  if (n_words != 0 && a0 < o1 && o0 < a1) return KV_E_OVERLAP;
  if (plan->capacity != 0 && (pool->base == nullptr || ((uintptr_t)pool->base % 256u) != 0))
    return pool->base == nullptr ? KV_E_NULL : KV_E_ALIGN;
  const uint64_t n_entries = (uint64_t)num_seqs * max_blocks_per_seq;
  if (n_entries != 0 && tables == nullptr) return KV_E_NULL;
  if (((uintptr_t)tables % 16u) != 0) return KV_E_ALIGN;

  const uint64_t block_bytes = (uint64_t)pool->num_layers * pool->tile_bytes;
  const bool small = n_words <= kMaxWords && n_entries <= kMaxEntries &&
                     (uint64_t)plan->capacity * block_bytes <= kMaxRegionBytes;
  if (!small) {
    int rc = kv_plan_reclaim(live_in, plan, stream);
    if (rc == KV_OK) rc = kv_compact(pool, plan, stream);
    if (rc == KV_OK) rc = kv_remap_tables(tables, num_seqs, max_blocks_per_seq, plan, stream);
    return rc;
  }

  SmallArgs a;
  a.live_in = live_in;
  a.n_words = n_words;
  a.num_blocks = nb;
  a.boundary = b;
  a.src = plan->src;
  a.dst = plan->dst;
  a.new_id = plan->new_id;
  a.live_out = plan->live_out;
  a.state = plan->state;
  a.base = (uint8_t*)pool->base;
  if (layer_major) {
    a.block_stride = pool->tile_bytes;
    a.seg_stride = pool->layer_stride_bytes;
    a.seg_bytes = pool->tile_bytes;
    a.segs = pool->num_layers;
  } else {
    a.block_stride = block_bytes;
    a.seg_stride = 0;
    a.seg_bytes = block_bytes;
    a.segs = 1;
  }
  a.chunks_per_seg = (uint32_t)((a.seg_bytes + kChunk - 1) / kChunk);
  a.tables = tables;
  a.n_entries = (uint32_t)n_entries;
  // One workgroup per compute unit at most, and no more than there can be units to copy (plus
  // workgroup 0 for the tables).
  int device = 0, cus = 0;
  if (hipGetDevice(&device) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
    return KV_E_HIP;
  const uint64_t max_units = (uint64_t)plan->capacity * a.segs * a.chunks_per_seg;
  uint32_t groups = (uint32_t)(max_units + 1 < (uint64_t)cus ? max_units + 1 : (uint64_t)cus);
  const uint32_t id_groups = (nb + kThreads - 1) / kThreads;  // enough lanes to write the id map in one pass
  if (groups < id_groups && id_groups <= (uint32_t)cus) groups = id_groups;
  if (groups == 0) groups = 1;
  hipLaunchKernelGGL(reclaim_small_kernel, dim3(groups), dim3(kThreads), 0, (hipStream_t)stream, a);
  return launch_rc();
}
