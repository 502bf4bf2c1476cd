// TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.
//
// Plain, slow, single-threaded CPU statement of what the KV-reclaim path
// computes, written from the problem definition and sharing no code, header,
// table or helper with the HIP library.  Only the tests, the smoke check and
// the benchmark's CPU-baseline leg may load it.
//
// The operation, after the paper's proactive prewarming (Sec. 3.3; App. C,
// Fig. 4b steps 1-3): a serving instance in its grace period keeps only the KV
// space it reserved (Eq. 4) and hands the rest to a new model's weights; only
// unused KV blocks may receive weights, and the running engine must still see
// every sequence's KV unchanged.  Here the hand-over is done by compaction:
// every live block whose id is at or above a reclaim boundary b moves into a
// free id below b, the k-th smallest moving id taking the k-th smallest free
// id; block tables are rewritten; weights are then copied into the byte range
// that starts at block b.
//
// Every function below is the definition written out: two ascending loops, a
// zip, memcpy per block, one table pass, memcpy per tensor.  There is no
// floating point anywhere on the path, so results are exact.
//
// Pins (tests/test_oracle_pins.py): exhaustive enumeration of all bitmaps up to
// 12 blocks against property checks that determine the result uniquely; an
// independently written rank/select formulation; closed-form special cases
// (nothing to move; full upper half onto empty lower half == one memmove; the
// exact feasibility threshold); idempotence; hand-worked fixtures under
// tests/golden/; mutation checks showing each pin set rejects planted errors.
#include <cstdint>
#include <cstring>

namespace {

enum : int {
  ORACLE_OK = 0,
  ORACLE_E_NULL = -1,
  ORACLE_E_RANGE = -2,
  ORACLE_E_TOOBIG = -4,
  ORACLE_E_OVERLAP = -5,
  ORACLE_E_NOSPACE = -7,
};

inline bool is_live(const uint64_t* live, uint32_t i) { return (live[i >> 6] >> (i & 63)) & 1u; }

}  // namespace

extern "C" {

// One weight tensor: `bytes` bytes at `host_ptr` go to region offset `dst_offset`.
struct oracle_tensor {
  const void* host_ptr;
  uint64_t bytes;
  uint64_t dst_offset;
};

// Relocation plan.  live: bit (i%64) of word (i/64) set <=> block i holds KV.
// Outputs: src/dst (capacity >= min(num_blocks-boundary, boundary)), new_id
// [num_blocks], live_out [ceil(num_blocks/64)], *n_moves.  On ORACLE_E_NOSPACE
// no output is written.
int oracle_plan(const uint64_t* live, uint32_t num_blocks, uint32_t boundary, int32_t* src,
                int32_t* dst, int32_t* new_id, uint64_t* live_out, uint32_t* n_moves) {
  if (!live || !src || !dst || !new_id || !live_out || !n_moves) return ORACLE_E_NULL;
  if (boundary > num_blocks) return ORACLE_E_RANGE;

  // Count first so that an infeasible request leaves every output untouched.
  uint32_t n_movers = 0, n_free = 0;
  for (uint32_t i = boundary; i < num_blocks; ++i) n_movers += is_live(live, i);
  for (uint32_t j = 0; j < boundary; ++j) n_free += !is_live(live, j);
  if (n_movers > n_free) return ORACLE_E_NOSPACE;

  // M: ascending live ids >= b.  F: ascending free ids < b (first |M| of them).
  uint32_t k = 0;
  for (uint32_t i = boundary; i < num_blocks; ++i)
    if (is_live(live, i)) src[k++] = (int32_t)i;
  k = 0;
  for (uint32_t j = 0; j < boundary && k < n_movers; ++j)
    if (!is_live(live, j)) dst[k++] = (int32_t)j;

  for (uint32_t i = 0; i < num_blocks; ++i)
    new_id[i] = (i < boundary && is_live(live, i)) ? (int32_t)i : -1;
  for (uint32_t m = 0; m < n_movers; ++m) new_id[src[m]] = dst[m];

  const uint32_t n_words = (num_blocks + 63) / 64;
  for (uint32_t w = 0; w < n_words; ++w) live_out[w] = 0;
  for (uint32_t j = 0; j < boundary; ++j)
    if (is_live(live, j)) live_out[j >> 6] |= 1ull << (j & 63);
  for (uint32_t m = 0; m < n_movers; ++m) live_out[dst[m] >> 6] |= 1ull << (dst[m] & 63);

  *n_moves = n_movers;
  return ORACLE_OK;
}

// Block copy: block dst[k] <- block src[k].  Source blocks keep their bytes.
int oracle_compact(uint8_t* pool, uint64_t block_bytes, const int32_t* src, const int32_t* dst,
                   uint32_t n_moves) {
  if (!pool || (n_moves && (!src || !dst))) return ORACLE_E_NULL;
  for (uint32_t k = 0; k < n_moves; ++k)
    std::memcpy(pool + (uint64_t)dst[k] * block_bytes, pool + (uint64_t)src[k] * block_bytes,
                block_bytes);
  return ORACLE_OK;
}

// Table pass: every entry e >= 0 becomes new_id[e].  An entry that names an
// id outside the pool or a block that was not live is an input error: it is
// left as it is and counted.  Returns the count (>= 0) or a negative error.
int64_t oracle_remap(int32_t* tables, uint64_t n_entries, const int32_t* new_id,
                     uint32_t num_blocks) {
  if ((n_entries && !tables) || !new_id) return ORACLE_E_NULL;
  int64_t bad = 0;
  for (uint64_t t = 0; t < n_entries; ++t) {
    const int32_t e = tables[t];
    if (e < 0) continue;
    if ((uint32_t)e >= num_blocks || new_id[e] < 0) { ++bad; continue; }
    tables[t] = new_id[e];
  }
  return bad;
}

// Weight copy into the reclaimed byte range [region_offset, pool_bytes).
// Every extent is checked (inside the region, pairwise disjoint) before the
// first byte is written.
int oracle_materialize(uint8_t* pool, uint64_t pool_bytes, uint64_t region_offset,
                       const oracle_tensor* tensors, uint32_t n_tensors) {
  if (!pool || (n_tensors && !tensors)) return ORACLE_E_NULL;
  if (region_offset > pool_bytes) return ORACLE_E_RANGE;
  const uint64_t region_bytes = pool_bytes - region_offset;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    if (tensors[i].bytes && !tensors[i].host_ptr) return ORACLE_E_NULL;
    if (tensors[i].dst_offset > region_bytes || tensors[i].bytes > region_bytes - tensors[i].dst_offset)
      return ORACLE_E_TOOBIG;
  }
  for (uint32_t i = 0; i < n_tensors; ++i)
    for (uint32_t j = i + 1; j < n_tensors; ++j) {
      const uint64_t a0 = tensors[i].dst_offset, a1 = a0 + tensors[i].bytes;
      const uint64_t b0 = tensors[j].dst_offset, b1 = b0 + tensors[j].bytes;
      if (a0 < a1 && b0 < b1 && a0 < b1 && b0 < a1) return ORACLE_E_OVERLAP;  // an empty extent holds no byte
    }
  for (uint32_t i = 0; i < n_tensors; ++i)
    std::memcpy(pool + region_offset + tensors[i].dst_offset, tensors[i].host_ptr, tensors[i].bytes);
  return ORACLE_OK;
}

// Reserved KV space of a draining instance (Sec. 3.3, Eq. 4), in blocks:
// R = max(C*Q/B, T + C/B) with C total blocks, T blocks in use, Q running
// requests and B the maximum batch; fractional blocks round up and R is
// capped at C.  Returns R, or a negative error for B == 0 or T > C.
int64_t oracle_reserve_blocks(uint64_t capacity_blocks, uint64_t used_blocks, uint32_t running,
                              uint32_t max_batch) {
  if (max_batch == 0 || used_blocks > capacity_blocks) return ORACLE_E_RANGE;
  // Both targets over the common denominator B, maximum first, ceiling last.
  const unsigned __int128 C = capacity_blocks, B = max_batch;
  const unsigned __int128 by_requests = C * running;                       // (C*Q/B) * B
  const unsigned __int128 by_usage = (unsigned __int128)used_blocks * B + C;  // (T + C/B) * B
  const unsigned __int128 numerator = by_requests > by_usage ? by_requests : by_usage;
  unsigned __int128 R = numerator / B;
  if (R * B < numerator) ++R;
  if (R > C) R = C;
  return (int64_t)R;
}

// Block copy in a layer-major pool: layer l's tile of block i is tile_bytes
// bytes at l*layer_stride + i*tile_bytes.  A block move is one tile copy per layer.
int oracle_compact_layer_major(uint8_t* pool, uint64_t tile_bytes, uint32_t num_layers,
                               uint64_t layer_stride, const int32_t* src, const int32_t* dst,
                               uint32_t n_moves) {
  if (!pool || (n_moves && (!src || !dst))) return ORACLE_E_NULL;
  for (uint32_t k = 0; k < n_moves; ++k)
    for (uint32_t l = 0; l < num_layers; ++l) {
      uint8_t* slab = pool + (uint64_t)l * layer_stride;
      std::memcpy(slab + (uint64_t)dst[k] * tile_bytes, slab + (uint64_t)src[k] * tile_bytes, tile_bytes);
    }
  return ORACLE_OK;
}

// Weight copy into a layer-major pool.  The reclaimed space is one strip per
// layer slab, bytes [boundary*tile_bytes, num_blocks*tile_bytes) of the slab;
// region offsets count through strip 0, then strip 1, ...  A tensor must lie
// inside one strip (it has to be contiguous in memory).
int oracle_materialize_strips(uint8_t* pool, uint64_t tile_bytes, uint32_t num_layers,
                              uint32_t num_blocks, uint32_t boundary, uint64_t layer_stride,
                              const oracle_tensor* tensors, uint32_t n_tensors) {
  if (!pool || (n_tensors && !tensors)) return ORACLE_E_NULL;
  if (boundary > num_blocks) return ORACLE_E_RANGE;
  const uint64_t strip = (uint64_t)(num_blocks - boundary) * tile_bytes;
  const uint64_t region_bytes = strip * num_layers;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const oracle_tensor& t = tensors[i];
    if (t.bytes && !t.host_ptr) return ORACLE_E_NULL;
    if (t.dst_offset > region_bytes || t.bytes > region_bytes - t.dst_offset) return ORACLE_E_TOOBIG;
    if (t.bytes && (t.dst_offset / strip != (t.dst_offset + t.bytes - 1) / strip)) return ORACLE_E_TOOBIG;
  }
  for (uint32_t i = 0; i < n_tensors; ++i)
    for (uint32_t j = i + 1; j < n_tensors; ++j) {
      const uint64_t a0 = tensors[i].dst_offset, a1 = a0 + tensors[i].bytes;
      const uint64_t b0 = tensors[j].dst_offset, b1 = b0 + tensors[j].bytes;
      if (a0 < a1 && b0 < b1 && a0 < b1 && b0 < a1) return ORACLE_E_OVERLAP;  // an empty extent holds no byte
    }
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const oracle_tensor& t = tensors[i];
    if (!t.bytes) continue;
    const uint64_t layer = t.dst_offset / strip, within = t.dst_offset % strip;
    std::memcpy(pool + layer * layer_stride + (uint64_t)boundary * tile_bytes + within, t.host_ptr, t.bytes);
  }
  return ORACLE_OK;
}

// Reverse switch (Sec. 3.3: weights are evicted when the reserve runs short).
// The boundary rises from old_boundary to new_boundary; a tensor is lost if any
// of its bytes lies in a block that goes back to the KV cache.  Checked byte
// range by byte range: the tensor occupies absolute pool bytes [lo, hi), the
// returned blocks occupy [old_boundary, new_boundary) * block_bytes.
// Returns the number of lost tensors or a negative error.
int64_t oracle_grow(uint64_t block_bytes, uint32_t num_blocks, uint32_t old_boundary,
                    uint32_t new_boundary, const oracle_tensor* tensors, uint32_t n_tensors,
                    uint8_t* evicted, uint64_t* new_offset) {
  if (n_tensors && (!tensors || !evicted || !new_offset)) return ORACLE_E_NULL;
  if (old_boundary > new_boundary || new_boundary > num_blocks) return ORACLE_E_RANGE;
  const uint64_t pool_bytes = (uint64_t)num_blocks * block_bytes;
  const uint64_t given_back_lo = (uint64_t)old_boundary * block_bytes;
  const uint64_t given_back_hi = (uint64_t)new_boundary * block_bytes;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const uint64_t lo = given_back_lo + tensors[i].dst_offset;
    if (lo > pool_bytes || tensors[i].bytes > pool_bytes - lo) return ORACLE_E_TOOBIG;
  }
  int64_t lost = 0;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const uint64_t lo = given_back_lo + tensors[i].dst_offset, hi = lo + tensors[i].bytes;
    const bool overlaps = lo < hi && lo < given_back_hi && given_back_lo < hi;
    evicted[i] = overlaps;
    new_offset[i] = (!overlaps && lo >= given_back_hi) ? lo - given_back_hi : 0;
    lost += overlaps;
  }
  return lost;
}

// Reverse switch in a layer-major pool.  The reclaimed space is one strip per layer slab, slab
// bytes [boundary*tile_bytes, num_blocks*tile_bytes); region offsets count through strip 0, strip
// 1, ...  Each tensor is placed at its absolute pool byte range under the old boundary; it is lost
// if that range meets a returned tile range [old_boundary*tile_bytes, new_boundary*tile_bytes) of
// its slab; a survivor's new offset is the region offset of the same absolute byte under the new
// boundary.  (An empty extent at the very end of the region counts as the end of the last strip.)
int64_t oracle_grow_strips(uint64_t tile_bytes, uint32_t num_layers, uint32_t num_blocks,
                           uint64_t layer_stride, uint32_t old_boundary, uint32_t new_boundary,
                           const oracle_tensor* tensors, uint32_t n_tensors, uint8_t* evicted,
                           uint64_t* new_offset) {
  if (n_tensors && (!tensors || !evicted || !new_offset)) return ORACLE_E_NULL;
  if (old_boundary > new_boundary || new_boundary > num_blocks) return ORACLE_E_RANGE;
  const uint64_t old_strip = (uint64_t)(num_blocks - old_boundary) * tile_bytes;
  const uint64_t new_strip = (uint64_t)(num_blocks - new_boundary) * tile_bytes;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const oracle_tensor& t = tensors[i];
    if (t.dst_offset > old_strip * num_layers || t.bytes > old_strip * num_layers - t.dst_offset)
      return ORACLE_E_TOOBIG;
    if (t.bytes && t.dst_offset / old_strip != (t.dst_offset + t.bytes - 1) / old_strip) return ORACLE_E_TOOBIG;
  }
  int64_t lost = 0;
  for (uint32_t i = 0; i < n_tensors; ++i) {
    const oracle_tensor& t = tensors[i];
    uint64_t layer = old_strip ? t.dst_offset / old_strip : 0;
    if (layer == num_layers && layer > 0) layer = num_layers - 1;
    const uint64_t slab = layer * layer_stride;
    // absolute pool bytes [lo, hi) of the tensor; returned bytes [back_lo, back_hi) of its slab
    const uint64_t lo = slab + (uint64_t)old_boundary * tile_bytes + (t.dst_offset - layer * old_strip);
    const uint64_t hi = lo + t.bytes;
    const uint64_t back_lo = slab + (uint64_t)old_boundary * tile_bytes;
    const uint64_t back_hi = slab + (uint64_t)new_boundary * tile_bytes;
    const bool overlaps = lo < hi && lo < back_hi && back_lo < hi;
    evicted[i] = overlaps;
    new_offset[i] = (!overlaps && lo >= back_hi) ? layer * new_strip + (lo - back_hi) : 0;
    lost += overlaps;
  }
  return lost;
}

// No-move variant (Sec. 3.4; App. C, Fig. 4b steps 1-2): which unused blocks lend their physical
// pages to the new model's slot.  Any `want` unused blocks would do for the paper; the reading
// taken is "the `want` highest free ids, highest first", which keeps the low ids for the running
// engine.  ids[k] is the block whose pages back slot offset k*block_bytes.
// Returns ORACLE_E_NOSPACE (nothing written) if fewer than `want` blocks are free.
int oracle_vmm_select(const uint64_t* live, uint32_t num_blocks, uint32_t want, int32_t* ids) {
  if (!live || (want && !ids)) return ORACLE_E_NULL;
  uint32_t n_free = 0;
  for (uint32_t i = 0; i < num_blocks; ++i) n_free += !is_live(live, i);
  if (want > n_free) return ORACLE_E_NOSPACE;
  uint32_t k = 0;
  for (uint32_t i = num_blocks; i > 0 && k < want; --i)
    if (!is_live(live, i - 1)) ids[k++] = (int32_t)(i - 1);
  return ORACLE_OK;
}

}  // extern "C"
