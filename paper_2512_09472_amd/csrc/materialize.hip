// Weight materialisation: stream a prewarmed model's tensors from pinned host
// memory into the reclaimed byte range of the KV pool (paper App. C, Fig. 4b
// step 3; weights wait in host memory and cross the host link, Sec. 4.1).
//
// The copies go to the DMA engines through hipMemcpyAsync on a stream of
// their own, so they take no CU away from the block copy they overlap with.
// The reclaimed range still holds moving blocks until kv_compact has read
// them.  The plain entry point therefore waits on the caller's compaction
// event before the first request.  The pipelined one follows the paper's rule
// (a copy starts once its destination is ready, App. C) at block granularity:
// bytes that land in blocks that were free when the plan was made go out
// before the wait.
#include <algorithm>
#include <vector>

#include "common.h"

namespace warmkv {
namespace {

constexpr uint64_t kChunkBytes = 4ull << 30;     // bound on one DMA request (each boundary idles the link ~30 us)
constexpr uint64_t kDefaultEarly = 128ull << 20;  // early bytes when the caller passes 0: about what the link
                                                 // carries during a few ms of block copy; every piece
                                                 // costs ~10 us of request overhead, so more loses
constexpr uint64_t kMinEarlyPiece = 2ull << 20;   // with the default budget, a free run shorter than this stays
                                                  // late: an early piece adds two request boundaries, each of
                                                  // which idles the link for 10-45 us (0.6-2.6 MB of link time).
                                                  // Measured on the 8B-shaped pool kept layer-major (64 KiB
                                                  // tiles): every free tile early 284 ms, runs >= 512 KiB 271 ms,
                                                  // gated 269 ms in the same runs

struct Region {
  bool layer_major;
  uint64_t block_bytes;   // block-major: bytes per block
  uint64_t offset;        // block-major: first byte of the region; layer-major: first byte of a strip in its slab
  uint64_t bytes;         // size of the region (all strips together)
  uint64_t strip_bytes;   // layer-major: bytes per strip
  uint64_t layer_stride;
  uint64_t tile_bytes;
};

// Device address of region offset `at` (validated to lie inside the region).
uint8_t* region_address(const kv_pool_desc* pool, const Region& r, uint64_t at) {
  uint8_t* base = (uint8_t*)pool->base;
  if (!r.layer_major) return base + r.offset + at;
  const uint64_t strip = r.strip_bytes ? at / r.strip_bytes : 0;
  return base + strip * r.layer_stride + r.offset + (at - strip * r.strip_bytes);
}

// Every extent inside the region, contiguous in memory and pairwise disjoint,
// before any byte moves.
int validate(const kv_pool_desc* pool, uint32_t boundary, const wm_tensor* tensors, uint32_t n_tensors,
             Region* region) {
  if (pool == nullptr || (n_tensors != 0 && tensors == nullptr)) return KV_E_NULL;
  if (boundary > pool->num_blocks) return KV_E_RANGE;
  if ((pool->tile_bytes != 0 && pool->num_layers != 0) && !pool_extent_ok(*pool)) return KV_E_RANGE;
  region->layer_major = pool->layer_stride_bytes != 0;
  region->layer_stride = pool->layer_stride_bytes;
  region->block_bytes = (uint64_t)pool->num_layers * pool->tile_bytes;
  region->tile_bytes = pool->tile_bytes;
  if (region->layer_major) {
    if (pool->layer_stride_bytes < (uint64_t)pool->num_blocks * pool->tile_bytes) return KV_E_RANGE;
    region->offset = (uint64_t)boundary * pool->tile_bytes;
    region->strip_bytes = (uint64_t)(pool->num_blocks - boundary) * pool->tile_bytes;
    region->bytes = region->strip_bytes * pool->num_layers;
  } else {
    region->offset = (uint64_t)boundary * region->block_bytes;
    region->strip_bytes = 0;
    region->bytes = (uint64_t)(pool->num_blocks - boundary) * region->block_bytes;
  }
  std::vector<uint32_t> order;
  order.reserve(n_tensors);
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const wm_tensor& t = tensors[i];
    if (t.dst_offset > region->bytes || t.bytes > region->bytes - t.dst_offset) return KV_E_TOOBIG;
    if (t.bytes == 0) continue;
    if (region->layer_major && t.dst_offset % region->strip_bytes + t.bytes > region->strip_bytes)
      return KV_E_TOOBIG;  // would straddle two strips
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
  return KV_OK;
}

// The copy streams of one weight stream.  With more than one, consecutive requests go to different
// streams, i.e. to different DMA engines: the next request is already set up when the previous one
// ends, so the 10-45 us for which the link idles at a request boundary disappear (15 GB in 1000
// requests: 270.7 ms on one stream, 261.4 ms on two, 260.4 ms as four requests).
constexpr uint32_t kMaxLanes = 4;
struct Lanes {
  hipStream_t s[kMaxLanes];
  uint32_t n;
};

inline Lanes one_lane(void* stream) {
  Lanes l;
  l.s[0] = (hipStream_t)stream;
  l.n = 1;
  return l;
}

// Every stream of the set waits for `event` (NULL: no wait).
int wait_all(const Lanes& lanes, void* event) {
  if (event == nullptr) return KV_OK;
  for (uint32_t i = 0; i < lanes.n; ++i) {
    const int rc = hip_rc(hipStreamWaitEvent(lanes.s[i], (hipEvent_t)event, 0));
    if (rc != KV_OK) return rc;
  }
  return KV_OK;
}

// Requests are issued in the caller's order, but neighbours that continue each
// other both in host memory and in the pool (a checkpoint parked in one pinned
// buffer and packed densely) go out as one request: each request costs about
// 10 us of set-up during which the link idles.
class Requests {
 public:
  explicit Requests(const Lanes& lanes) : lanes_(lanes) {}
  int add(uint8_t* dst, const uint8_t* src, uint64_t bytes) {
    if (bytes == 0) return KV_OK;
    if (bytes_ != 0 && dst == dst_ + bytes_ && src == src_ + bytes_) {
      bytes_ += bytes;
      return KV_OK;
    }
    const int rc = flush();
    dst_ = dst;
    src_ = src;
    bytes_ = bytes;
    return rc;
  }
  int flush() {
    int rc = KV_OK;
    for (uint64_t done = 0; done < bytes_ && rc == KV_OK; done += kChunkBytes) {
      const uint64_t len = std::min(kChunkBytes, bytes_ - done);
      rc = hip_rc(hipMemcpyAsync(dst_ + done, src_ + done, len, hipMemcpyHostToDevice, lanes_.s[next_ % lanes_.n]));
      ++next_;
    }
    bytes_ = 0;
    return rc;
  }

 private:
  Lanes lanes_;
  uint32_t next_ = 0;
  uint8_t* dst_ = nullptr;
  const uint8_t* src_ = nullptr;
  uint64_t bytes_ = 0;
};

inline bool was_live(const uint64_t* live, uint64_t block) { return (live[block >> 6] >> (block & 63)) & 1ull; }

// Cut the tensors at block boundaries into early pieces (runs of blocks that
// were free before the move, while the early budget lasts) and late pieces.
// In a layer-major pool the unit is a block's tile in one strip: region offset
// `at` lies in strip at / strip_bytes, in the tile of block boundary +
// (at % strip_bytes) / tile_bytes (strips are whole tiles, and a tensor never
// leaves its strip).
void schedule(const Region& r, uint32_t boundary, const uint64_t* live, const wm_tensor* tensors,
              uint32_t n_tensors, uint64_t early_budget, uint64_t min_early_piece, std::vector<wm_piece>* early,
              std::vector<wm_piece>* late) {
  const uint64_t unit = r.layer_major ? r.tile_bytes : r.block_bytes;
  auto block_of = [&](uint64_t at) -> uint64_t {
    return boundary + (r.layer_major ? (at % r.strip_bytes) / unit : at / unit);
  };
  uint64_t early_total = 0;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const wm_tensor& t = tensors[i];
    uint64_t pos = 0;  // bytes of this tensor already assigned
    while (pos < t.bytes) {
      const uint64_t at = t.dst_offset + pos;
      const bool ready = early_total < early_budget && !was_live(live, block_of(at));
      // extend over following blocks of the same kind
      uint64_t end = std::min(t.bytes, pos + (unit - at % unit));
      uint64_t collected = early_total + (ready ? end - pos : 0);
      while (end < t.bytes) {
        const bool next_ready = collected < early_budget && !was_live(live, block_of(t.dst_offset + end));
        if (next_ready != ready) break;
        const uint64_t next_end = std::min(t.bytes, end + unit);
        if (ready) collected += next_end - end;
        end = next_end;
      }
      const bool take_early = ready && end - pos >= min_early_piece;
      if (!take_early && !late->empty() && late->back().tensor == i &&
          late->back().src_offset + late->back().bytes == pos) {
        late->back().bytes += end - pos;  // continues the late piece in front of it
      } else {
        wm_piece p;
        p.tensor = i;
        p.early = take_early ? 1u : 0u;
        p.src_offset = pos;
        p.dst_offset = at;
        p.bytes = end - pos;
        (take_early ? early : late)->push_back(p);
      }
      if (take_early) early_total += end - pos;
      pos = end;
    }
  }
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

namespace {

// Front-first weight stream over a set of copy streams.  The block copy takes its moves in
// ascending source order, so the reclaimed region becomes ready from its start: once the movers of
// the first front_bytes have been read (front_done), every byte below that mark may be written,
// while the rest of the block copy is still running.  Each tensor is cut at most once.
// front_bytes = 0 with front_done = NULL is the plain gated stream.
int stream_front(const kv_pool_desc* pool, const Region& r, uint64_t front_bytes, const wm_tensor* tensors,
                 uint32_t n_tensors, const Lanes& lanes, void* front_done, void* compaction_done) {
  auto front_part = [&](const wm_tensor& t) -> uint64_t {  // leading bytes of t that lie below the mark
    return t.dst_offset >= front_bytes ? 0 : std::min(t.bytes, front_bytes - t.dst_offset);
  };
  int rc = wait_all(lanes, front_done);
  if (rc != KV_OK) return rc;
  Requests requests(lanes);
  if (front_bytes != 0) {
    for (uint32_t i = 0; i < n_tensors; ++i) {
      if (tensors[i].bytes == 0) continue;
      rc = requests.add(region_address(pool, r, tensors[i].dst_offset), (const uint8_t*)tensors[i].host_ptr,
                        front_part(tensors[i]));
      if (rc != KV_OK) return rc;
    }
    rc = requests.flush();
    if (rc != KV_OK) return rc;
  }
  rc = wait_all(lanes, compaction_done);
  if (rc != KV_OK) return rc;
  for (uint32_t i = 0; i < n_tensors; ++i) {  // caller's order
    const uint64_t head = front_bytes != 0 ? front_part(tensors[i]) : 0;
    if (head == tensors[i].bytes) continue;
    rc = requests.add(region_address(pool, r, tensors[i].dst_offset + head), (const uint8_t*)tensors[i].host_ptr + head,
                      tensors[i].bytes - head);
    if (rc != KV_OK) return rc;
  }
  return requests.flush();
}

// Block-granular pipelining: early pieces before the wait on the compaction event, late ones after.
int stream_pipelined(const kv_pool_desc* pool, const Region& r, uint32_t boundary, const uint64_t* live_host,
                     const wm_tensor* tensors, uint32_t n_tensors, uint64_t early_bytes, const Lanes& lanes,
                     void* compaction_done) {
  if (live_host == nullptr && pool->num_blocks != 0) return KV_E_NULL;
  if (r.block_bytes == 0) return KV_E_RANGE;
  std::vector<wm_piece> early, late;
  schedule(r, boundary, live_host, tensors, n_tensors, early_bytes ? early_bytes : kDefaultEarly,
           early_bytes ? 0 : kMinEarlyPiece, &early, &late);
  Requests requests(lanes);
  int rc = KV_OK;
  for (const wm_piece& p : early) {
    rc = requests.add(region_address(pool, r, p.dst_offset), (const uint8_t*)tensors[p.tensor].host_ptr + p.src_offset,
                      p.bytes);
    if (rc != KV_OK) return rc;
  }
  rc = requests.flush();
  if (rc != KV_OK) return rc;
  rc = wait_all(lanes, compaction_done);
  if (rc != KV_OK) return rc;
  for (const wm_piece& p : late) {
    rc = requests.add(region_address(pool, r, p.dst_offset), (const uint8_t*)tensors[p.tensor].host_ptr + p.src_offset,
                      p.bytes);
    if (rc != KV_OK) return rc;
  }
  return requests.flush();
}

}  // namespace

extern "C" int weights_materialize(const kv_pool_desc* pool, uint32_t boundary, const wm_tensor* tensors,
                                   uint32_t n_tensors, void* copy_stream, void* compaction_done) {
  return guarded([&]() -> int {
    Region r;
    const int rc = validate(pool, boundary, tensors, n_tensors, &r);
    if (rc != KV_OK) return rc;
    return stream_front(pool, r, 0, tensors, n_tensors, one_lane(copy_stream), nullptr, compaction_done);
  });
}

extern "C" int weights_materialize_streams(const kv_pool_desc* pool, uint32_t boundary, uint64_t front_bytes,
                                           const wm_tensor* tensors, uint32_t n_tensors, void* const* copy_streams,
                                           uint32_t n_streams, void* front_done, void* compaction_done) {
  return guarded([&]() -> int {
    Region r;
    const int rc = validate(pool, boundary, tensors, n_tensors, &r);
    if (rc != KV_OK) return rc;
    if (copy_streams == nullptr) return KV_E_NULL;
    if (n_streams == 0 || n_streams > kMaxLanes) return KV_E_RANGE;
    Lanes lanes;
    lanes.n = n_streams;
    for (uint32_t i = 0; i < n_streams; ++i) lanes.s[i] = (hipStream_t)copy_streams[i];
    return stream_front(pool, r, front_bytes, tensors, n_tensors, lanes, front_done, compaction_done);
  });
}

extern "C" int weights_materialize_schedule(const kv_pool_desc* pool, uint32_t boundary,
                                            const uint64_t* live_host, const wm_tensor* tensors,
                                            uint32_t n_tensors, uint64_t early_bytes, wm_piece* out,
                                            uint32_t capacity, uint32_t* n_out) {
  return guarded([&]() -> int {
    Region r;
    const int rc = validate(pool, boundary, tensors, n_tensors, &r);
    if (rc != KV_OK) return rc;
    if (n_out == nullptr || (capacity != 0 && out == nullptr)) return KV_E_NULL;
    if (live_host == nullptr && pool->num_blocks != 0) return KV_E_NULL;
    if (r.block_bytes == 0) return KV_E_RANGE;
    std::vector<wm_piece> early, late;
    schedule(r, boundary, live_host, tensors, n_tensors, early_bytes ? early_bytes : kDefaultEarly,
             early_bytes ? 0 : kMinEarlyPiece, &early, &late);
    const size_t total = early.size() + late.size();
    if (total > 0xFFFFFFFFull) return KV_E_RANGE;
    *n_out = (uint32_t)total;
    if (total > capacity) return KV_E_TOOBIG;
    std::copy(early.begin(), early.end(), out);
    std::copy(late.begin(), late.end(), out + early.size());
    return KV_OK;
  });
}

extern "C" int weights_materialize_pipelined(const kv_pool_desc* pool, uint32_t boundary,
                                             const uint64_t* live_host, const wm_tensor* tensors,
                                             uint32_t n_tensors, uint64_t early_bytes, void* copy_stream,
                                             void* compaction_done) {
  return guarded([&]() -> int {
    Region r;
    const int rc = validate(pool, boundary, tensors, n_tensors, &r);
    if (rc != KV_OK) return rc;
    return stream_pipelined(pool, r, boundary, live_host, tensors, n_tensors, early_bytes, one_lane(copy_stream),
                            compaction_done);
  });
}

extern "C" uint32_t kv_movers_in_front(const uint64_t* live_host, uint32_t num_blocks, uint32_t boundary,
                                       uint32_t front_blocks) {
  if (live_host == nullptr || boundary >= num_blocks) return 0u;
  const uint64_t end = std::min<uint64_t>(num_blocks, (uint64_t)boundary + front_blocks);
  uint32_t n = 0;
  for (uint64_t i = boundary; i < end; ++i) n += was_live(live_host, i) ? 1u : 0u;
  return n;
}

extern "C" int weights_materialize_front(const kv_pool_desc* pool, uint32_t boundary, uint64_t front_bytes,
                                         const wm_tensor* tensors, uint32_t n_tensors, void* copy_stream,
                                         void* front_done, void* compaction_done) {
  return guarded([&]() -> int {
    Region r;
    const int rc = validate(pool, boundary, tensors, n_tensors, &r);
    if (rc != KV_OK) return rc;
    return stream_front(pool, r, front_bytes, tensors, n_tensors, one_lane(copy_stream), front_done, compaction_done);
  });
}

// The whole hand-over in one call.  The separate entry points leave one gap
// to the caller: an infeasible plan turns kv_compact and kv_remap_tables into
// no-ops, but a weight stream enqueued behind them would still overwrite the
// live blocks that could not move.  Here the plan's verdict is fetched (one
// host synchronisation, microseconds against a weight stream of hundreds of
// milliseconds) before anything that writes the pool is enqueued.
extern "C" int kv_switch(const kv_switch_request* rq, kv_plan_state* result) {
  return guarded([&]() -> int {
    if (rq == nullptr || rq->pool == nullptr || rq->plan == nullptr || rq->compaction_done == nullptr) return KV_E_NULL;
    const kv_pool_desc* pool = rq->pool;
    const kv_plan* plan = rq->plan;
    if (pool->num_blocks != plan->num_blocks || plan->boundary > plan->num_blocks) return KV_E_RANGE;
    if (!pool_extent_ok(*pool) || !copy_units_fit(*pool, plan->capacity)) return KV_E_RANGE;
    if ((pool->tile_bytes % 16u) != 0 || ((uintptr_t)pool->base % 256u) != 0) return KV_E_ALIGN;
    const uint64_t n_entries = (uint64_t)rq->num_seqs * rq->max_blocks_per_seq;
    if (n_entries != 0 && rq->tables == nullptr) return KV_E_NULL;
    if (((uintptr_t)rq->tables % 16u) != 0) return KV_E_ALIGN;
    Region r;
    int rc = validate(pool, plan->boundary, rq->tensors, rq->n_tensors, &r);
    if (rc != KV_OK) return rc;
  
    rc = kv_plan_reclaim(rq->live_in, plan, rq->compute_stream);
    if (rc != KV_OK) return rc;
    kv_plan_state st;
    rc = kv_plan_fetch(plan, rq->compute_stream, &st);
    if (rc != KV_OK) return rc;
    if (result != nullptr) *result = st;
    if (st.status != KV_OK) return st.status;  // running requests keep their blocks; no weight byte is sent
  
    const bool can_pipeline = rq->live_host != nullptr && r.block_bytes != 0 && r.bytes != 0;
    const bool front_first = can_pipeline && rq->front_done != nullptr && rq->n_tensors != 0;
    uint64_t front_bytes = 0;
    if (front_first) {
      // Enough weight bytes below the mark to keep the link busy until the block copy has ended:
      // the link carries roughly 1/120 of what the block copy moves in the same time; twice that.
      const uint64_t moved = 2ull * st.n_moves * r.block_bytes;
      front_bytes = rq->early_bytes ? rq->early_bytes : std::max<uint64_t>(64ull << 20, moved / 64);
      if (r.layer_major) {
        // The block copy walks the slabs in layer order, so the region (strip 0, strip 1, ...) is
        // ready strip by strip: the front is a whole number of strips.
        const uint64_t front_strips = std::min<uint64_t>((front_bytes + r.strip_bytes - 1) / r.strip_bytes, pool->num_layers);
        front_bytes = front_strips * r.strip_bytes;
        rc = kv_compact_layers(pool, plan, 0u, (uint32_t)front_strips, rq->compute_stream);
        if (rc != KV_OK) return rc;
        rc = hip_rc(hipEventRecord((hipEvent_t)rq->front_done, (hipStream_t)rq->compute_stream));
        if (rc != KV_OK) return rc;
        rc = kv_compact_layers(pool, plan, (uint32_t)front_strips, ~0u, rq->compute_stream);
      } else {
        const uint64_t front_blocks =
            std::min<uint64_t>((front_bytes + r.block_bytes - 1) / r.block_bytes, pool->num_blocks - plan->boundary);
        front_bytes = front_blocks * r.block_bytes;
        const uint32_t head = kv_movers_in_front(rq->live_host, pool->num_blocks, plan->boundary, (uint32_t)front_blocks);
        rc = kv_compact_moves(pool, plan, 0u, head, rq->compute_stream);
        if (rc != KV_OK) return rc;
        rc = hip_rc(hipEventRecord((hipEvent_t)rq->front_done, (hipStream_t)rq->compute_stream));
        if (rc != KV_OK) return rc;
        rc = kv_compact_moves(pool, plan, head, ~0u, rq->compute_stream);
      }
    } else {
      rc = kv_compact(pool, plan, rq->compute_stream);
    }
    if (rc != KV_OK) return rc;
    rc = hip_rc(hipEventRecord((hipEvent_t)rq->compaction_done, (hipStream_t)rq->compute_stream));
    if (rc != KV_OK) return rc;
    rc = kv_remap_tables(rq->tables, rq->num_seqs, rq->max_blocks_per_seq, plan, rq->compute_stream);
    if (rc != KV_OK) return rc;
    Lanes lanes = one_lane(rq->copy_stream);
    if (rq->copy_stream2 != nullptr) lanes.s[lanes.n++] = (hipStream_t)rq->copy_stream2;
    if (front_first)
      return stream_front(pool, r, front_bytes, rq->tensors, rq->n_tensors, lanes, rq->front_done, rq->compaction_done);
    if (can_pipeline)
      return stream_pipelined(pool, r, plan->boundary, rq->live_host, rq->tensors, rq->n_tensors, rq->early_bytes, lanes,
                              rq->compaction_done);
    return stream_front(pool, r, 0, rq->tensors, rq->n_tensors, lanes, nullptr, rq->compaction_done);
  });
}
