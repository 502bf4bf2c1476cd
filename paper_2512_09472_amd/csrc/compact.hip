// Block copy of the KV reclaim: for k < n_moves, block dst[k] <- block src[k].
// This is the bandwidth-bound step (2 * n_moves * block_bytes of HBM traffic);
// the rest of the path is microseconds.  It stands in for the paper's step of
// mapping the pages under unused KV blocks into the new model's slot (App. C,
// Fig. 4b step 2): here the unused space is made contiguous instead.
//
// Shape.  The work list is (move, chunk) units of 64 KiB in list order (in a
// layer-major pool a move is one tile per layer slab: (move, layer, chunk)).  One
// 256-lane workgroup per compute unit stays resident and takes units in list
// order (its own index first, then draws from a single device-wide ticket
// counter), so at any moment the 256 workgroups stream
// one narrow, advancing window (about 16 MiB of sources and as much of
// destinations).  Measured on MI355X this ordering is what matters: a static
// grid-stride assignment lets workgroups drift apart, the window smears over
// hundreds of MiB, and the same loads and stores run about 25 % slower.  More
// workgroups or bigger units widen the window and lose; 32 KiB units hit the
// rate one counter address sustains.  The grid never depends on n_moves, which
// lives in device memory (no host sync after the planner).
//
// Inside a unit every lane issues all 16 of its 128-bit loads (the whole
// 64 KiB, 1 KiB per wavefront instruction, fully coalesced) before its first
// store: long read bursts followed by long write bursts measured 5 % faster
// than interleaving 32 KiB at a time.  Lane 0 draws the ticket and resolves it
// to addresses between two units; the other lanes take them from LDS.
// Accesses are non-temporal: gigabytes stream through once and should not
// evict anything.
// Sources lie at or above the boundary and destinations below it, so no two
// moves overlap and any order is correct; the kernel checks that property per
// move instead of staging through LDS (a refused move is flagged in
// state.bad_plan; state.status stays as the planner left it for the whole launch).
#include "common.h"

namespace warmkv {
namespace {

constexpr uint32_t kCopyThreads = 256;
constexpr uint32_t kVecBytes = 16;
constexpr uint32_t kRowBytes = kCopyThreads * kVecBytes;  // 4 KiB per workgroup per instruction
constexpr uint32_t kDefaultChunk = 65536;
constexpr uint32_t kDefaultUnroll = 16;                   // 16 rows = one whole 64 KiB unit per step
constexpr uint32_t kMaxBurstRows = 21;                    // most rows one burst may have (register budget)

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
  uint32_t move_first;      // this launch copies moves [move_first, move_first + move_count) of the plan;
  uint32_t move_count;      // src and dst already point at entry move_first
};

// Moves of the plan that fall to a launch over [first, first + count).
__device__ __forceinline__ uint32_t moves_of_launch(const kv_plan_state* state, uint32_t first, uint32_t count) {
  if (state->status != KV_OK) return 0u;
  const uint32_t n = state->n_moves;
  if (n <= first) return 0u;
  return n - first < count ? n - first : count;
}

// One unit of work, resolved: where to read, where to write, how much.
struct Unit {
  uint32_t ticket;
  uint32_t len;  // 0: nothing to copy (a move that failed the src >= boundary > dst check)
  uint64_t src_off;
  uint64_t dst_off;
};

// Tickets.  Workgroup i starts with ticket i, which costs nothing; every later
// ticket is gridDim.x plus a draw from the device-wide counter.  When all units
// fit the first round (n_units <= gridDim.x: small pools) nobody draws, the
// counters are never touched and no workgroup has to sign out: 256 workgroups
// hitting one address take about 3 us per round, as much as the copy itself
// on a pool of a few hundred blocks.
__device__ __forceinline__ uint32_t next_ticket(kv_plan_state* state, uint32_t n_units) {
  return n_units > gridDim.x ? gridDim.x + atomicAdd(&state->ticket, 1u) : n_units;
}

// Sign out after a failed draw; the last workgroup out puts both counters back
// to zero for the next call on this plan.  Nothing to do if nobody drew.
__device__ __forceinline__ void sign_out(kv_plan_state* state, uint32_t n_units) {
  if (n_units <= gridDim.x) return;
  const uint32_t out = atomicAdd(&state->finished, 1u);
  if (out == gridDim.x - 1u) {
    atomicExch(&state->ticket, 0u);
    atomicExch(&state->finished, 0u);
  }
}

// Lane 0 only: resolve a ticket to (move k, segment g, chunk c) and on to byte
// offsets.
__device__ __forceinline__ Unit resolve_unit(const CopyArgs& a, uint32_t ticket, uint32_t n_moves, uint32_t n_units) {
  Unit unit;
  unit.ticket = ticket;
  unit.len = 0;
  unit.src_off = unit.dst_off = 0;
  if (unit.ticket >= n_units) return unit;
  const uint32_t u = unit.ticket;
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
    // Flagged in a word of its own: `status` must not change while the launch runs, or workgroups
    // that start later would see a different plan (no moves) and leave the counters dirty.
    atomicExch(&a.state->bad_plan, 1u);
    return unit;
  }
  const uint64_t off = (uint64_t)g * a.seg_stride + (uint64_t)c * a.chunk_bytes;
  const uint64_t left = a.seg_bytes - (uint64_t)c * a.chunk_bytes;
  unit.len = left < a.chunk_bytes ? (uint32_t)left : a.chunk_bytes;
  unit.src_off = (uint64_t)s * a.block_stride + off;
  unit.dst_off = (uint64_t)d * a.block_stride + off;
  return unit;
}

// readfirstlane returns a signed int: go through uint32_t so that a low half
// with bit 31 set is not sign-extended into the high half.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  const uint32_t hi = uniform32((uint32_t)(v >> 32)), lo = uniform32((uint32_t)v);
  return ((uint64_t)hi << 32) | (uint64_t)lo;
}

// One step: ROWS rows of 4 KiB, every load issued before the first store.
template <int ROWS, bool NT>
__device__ __forceinline__ void copy_rows(const u32x4* __restrict__ sp, u32x4* __restrict__ dp, uint32_t i) {
  u32x4 v[ROWS];
#pragma unroll
  for (int j = 0; j < ROWS; ++j) v[j] = load16<NT>(sp + i + j * kCopyThreads);
  // A read burst, then a write burst: all loads are issued back to back and have all
  // returned before the first store goes out (measured 1-3 % faster than letting the
  // compiler interleave stores with the tail of the loads).
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < ROWS; ++j) store16<NT>(dp + i + j * kCopyThreads, v[j]);
}

// copy_rows<rows> for a run-time (uniform) row count in 1..MAX.
template <int MAX, bool NT>
__device__ __forceinline__ void copy_rows_of(const u32x4* __restrict__ sp, u32x4* __restrict__ dp, uint32_t i,
                                             uint32_t rows) {
  if (rows == (uint32_t)MAX) copy_rows<MAX, NT>(sp, dp, i);
  else if constexpr (MAX > 1) copy_rows_of<MAX - 1, NT>(sp, dp, i, rows);
}

// Copy len bytes (multiple of 16) in steps of UNROLL rows; with the default
// shape one step is the whole unit.  A shorter rest (the ragged end of a block
// or tile that is not a whole number of units) goes out as one more burst of
// exactly its row count, and a last partial row after that.
template <int UNROLL, bool NT>
__device__ __forceinline__ void copy_bytes(const u32x4* __restrict__ sp, u32x4* __restrict__ dp, uint32_t len,
                                           uint32_t tid) {
  uint32_t i = tid;                          // this lane's vector index
  uint32_t rows = len / kRowBytes;           // whole rows left
  // A unit of 17 to 21 rows (a 68-84 KiB tile kept in one unit) goes out as one burst too:
  // two segments of 36 KiB in one 18-row burst measured 2.5 % faster than 16 rows and 2.
  if (UNROLL == 16 && rows > 16u && rows <= kMaxBurstRows) {
    copy_rows_of<kMaxBurstRows, NT>(sp, dp, i, rows);
    i += rows * kCopyThreads;
    rows = 0;
  }
  // The first step is kept out of the loop: in the default shape it is the whole unit, and
  // the straight-line form measured 3 % faster than the same step as a loop body.
  if (rows >= (uint32_t)UNROLL) { copy_rows<UNROLL, NT>(sp, dp, i); rows -= UNROLL; i += UNROLL * kCopyThreads; }
  for (; rows >= (uint32_t)UNROLL; rows -= UNROLL, i += UNROLL * kCopyThreads) copy_rows<UNROLL, NT>(sp, dp, i);
  if (UNROLL > 16 && rows >= 16u) { copy_rows<16, NT>(sp, dp, i); rows -= 16u; i += 16u * kCopyThreads; }
  if (rows != 0) copy_rows_of<15, NT>(sp, dp, i, rows);  // one read burst and one write burst whatever the count
  i += rows * kCopyThreads;
  if (i < len / kVecBytes) store16<NT>(dp + i, load16<NT>(sp + i));  // partial last row
}

// Persistent workgroups; units are handed out in list order, the first round by
// workgroup index and the rest by one ticket counter.  Lane 0 draws and resolves the next unit after the current one is
// copied (default) or while it is copied (PREFETCH); the others pick it up from
// LDS.  Drawing ahead hides the atomic and the two id loads, yet measured 4 %
// slower on every workload: the short pause between units keeps fewer bytes in
// flight per compute unit, and the memory system is saturated either way.
// WHOLE: every unit is exactly one step of UNROLL rows (segments that are a
// whole number of units: the benchmark pools); the copy is then that one step
// and nothing else, with no code for ragged ends anywhere near it.
template <int UNROLL, bool NT, bool PREFETCH, bool WHOLE>
__global__ __launch_bounds__(kCopyThreads) void compact_ticket_kernel(CopyArgs a) {
  // No early return once tickets are drawn: every workgroup must draw its one
  // out-of-range ticket and sign out below, or the counters would not return to zero.
  const uint32_t n_moves = moves_of_launch(a.state, a.move_first, a.move_count);
  const uint32_t n_units = n_moves * a.units_per_move;  // host checked: fits 31 bits
  const uint32_t tid = threadIdx.x;
  __shared__ Unit s_unit[2];
  if (tid == 0) s_unit[0] = resolve_unit(a, blockIdx.x, n_moves, n_units);
  __syncthreads();
  uint32_t slot = 0;
  for (;;) {
    const uint32_t ticket = uniform32(s_unit[slot].ticket);
    if (ticket >= n_units) break;
    const uint32_t len = uniform32(s_unit[slot].len);
    const uint64_t src_off = uniform64(s_unit[slot].src_off);
    const uint64_t dst_off = uniform64(s_unit[slot].dst_off);
    // The other slot was last read before the previous barrier: free to refill.
    if (PREFETCH && tid == 0) s_unit[slot ^ 1u] = resolve_unit(a, next_ticket(a.state, n_units), n_moves, n_units);
    if (WHOLE) {
      if (len != 0) copy_rows<UNROLL, NT>((const u32x4*)(a.base + src_off), (u32x4*)(a.base + dst_off), tid);
    } else {
      copy_bytes<UNROLL, NT>((const u32x4*)(a.base + src_off), (u32x4*)(a.base + dst_off), len, tid);
    }
    if (!PREFETCH) {
      __syncthreads();
      if (tid == 0) s_unit[slot ^ 1u] = resolve_unit(a, next_ticket(a.state, n_units), n_moves, n_units);
    }
    __syncthreads();
    slot ^= 1u;
  }
  // Every workgroup ends on exactly one ticket >= n_units.
  if (tid == 0) sign_out(a.state, n_units);
}

// Small segments (half a ticket or less: tiles of a layer-major pool with few
// heads, blocks of a one-layer pool).  One ticket per segment would be drawn
// faster than one counter address can hand them out (16 KiB units ran at 40 %
// of the 64 KiB rate, 4 KiB units at 10 %), so a ticket here covers `pack`
// consecutive moves of one segment: up to 64 KiB again, the same burst per
// lane, and consecutive moves have ascending sources and destinations, so the
// window still advances in order.  The first wavefront draws the ticket and
// resolves its moves into LDS (lane i: move i); every lane knows from the start
// which move of a ticket each of its vectors belongs to (tickets begin at a move
// boundary), found once by a multiply-high with a host-made reciprocal.
//
// The copy of a whole ticket is straight-line code with no predicate: a
// conditional load or store costs a branch, and the wait the compiler puts at
// each join serialises the burst (measured 10 % slower).  ROWS is the number of
// 4 KiB rows a whole ticket takes; where the last row is only part filled, its
// idle lanes repeat a vector of the same ticket (same bytes to the same place,
// harmless) instead of being masked off.
constexpr uint32_t kMaxPack = 256;   // moves per ticket: what one LDS table holds
constexpr uint32_t kPackRows = 16;   // 128-bit accesses per lane per ticket (64 KiB per workgroup) ...
                                     // ... but two segments of 32-42 KiB share a ticket of up to kMaxBurstRows rows:
                                     // one such segment per ticket is drawn faster than the counter hands tickets out
constexpr uint64_t kSkip = ~0ull;    // LDS marker of a move that failed the src >= boundary > dst check

struct PackArgs {
  uint8_t* base;
  uint64_t block_stride;
  uint64_t seg_stride;
  const int32_t* src;
  const int32_t* dst;
  kv_plan_state* state;
  uint32_t num_blocks;
  uint32_t boundary;
  uint32_t segs;         // segments per move (layers of a layer-major pool, else 1)
  uint32_t seg_vecs;     // 128-bit vectors per segment
  uint32_t recip;        // ceil(2^32 / seg_vecs); v / seg_vecs == mulhi(v, recip) for v < 2^16 (unused if seg_vecs == 1)
  uint32_t pack;         // moves per ticket, 2..kMaxPack
  uint32_t ticket_vecs;  // pack * seg_vecs, in (ROWS-1)*256 .. ROWS*256
  uint32_t move_first;   // as in CopyArgs
  uint32_t move_count;
};

template <bool NT, int ROWS>
__global__ __launch_bounds__(kCopyThreads) void compact_packed_kernel(PackArgs a) {
  const uint32_t n_moves = moves_of_launch(a.state, a.move_first, a.move_count);
  const uint32_t groups = (n_moves + a.pack - 1u) / a.pack;  // tickets per segment
  const uint32_t n_units = groups * a.segs;                  // host checked: fits 31 bits
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t kWholeTicket = ~0u;  // a.pack moves, none refused
  __shared__ uint32_t s_ticket, s_count;  // s_count: moves of the ticket, or kWholeTicket
  __shared__ uint64_t s_src[kMaxPack], s_dst[kMaxPack];

  uint32_t move_of[ROWS], within[ROWS];  // per vector of this lane: move of the ticket, byte offset in the segment
#pragma unroll
  for (int j = 0; j < ROWS; ++j) {
    uint32_t idx = tid + (uint32_t)j * kCopyThreads;
    if (idx >= a.ticket_vecs) idx %= a.ticket_vecs;  // idle lane of the last row: repeat another vector
    const uint32_t m = a.seg_vecs == 1u ? idx : __umulhi(idx, a.recip);
    move_of[j] = m;
    within[j] = (idx - m * a.seg_vecs) * kVecBytes;
  }

  bool first = true;  // the first ticket is the workgroup's index, later ones are drawn
  for (;;) {
    if (tid < (uint32_t)kWave) {
      uint32_t ticket = blockIdx.x;
      if (!first && tid == 0) ticket = next_ticket(a.state, n_units);
      first = false;
      ticket = uniform32(ticket);
      uint32_t cnt = 0;
      bool refused = false;
      if (ticket < n_units) {
        // All tickets of segment (layer) 0, then of segment 1, ...
        const uint32_t g = ticket / groups;
        const uint32_t k0 = (ticket - g * groups) * a.pack;
        cnt = n_moves - k0 < a.pack ? n_moves - k0 : a.pack;
        const uint64_t seg_off = (uint64_t)g * a.seg_stride;
        for (uint32_t i = tid; i < cnt; i += kWave) {
          const uint32_t s = (uint32_t)a.src[k0 + i], d = (uint32_t)a.dst[k0 + i];
          const bool ok = s >= a.boundary && s < a.num_blocks && d < a.boundary;  // always true for a planner-made plan
          if (!ok) {
            atomicExch(&a.state->bad_plan, 1u);  // not `status`: see resolve_unit
            refused = true;
          }
          s_src[i] = ok ? (uint64_t)s * a.block_stride + seg_off : kSkip;
          s_dst[i] = (uint64_t)d * a.block_stride + seg_off;
        }
      }
      const bool whole = cnt == a.pack && __ballot(refused) == 0ull;
      if (tid == 0) {
        s_ticket = ticket;
        s_count = whole ? kWholeTicket : cnt;
      }
    }
    __syncthreads();
    if (uniform32(s_ticket) >= n_units) break;
    const uint32_t cnt = uniform32(s_count);
    u32x4 v[ROWS];
    uint64_t to[ROWS];
    if (cnt == kWholeTicket) {
      uint64_t from[ROWS];
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        from[j] = s_src[move_of[j]] + within[j];
        to[j] = s_dst[move_of[j]] + within[j];
      }
#pragma unroll
      for (int j = 0; j < ROWS; ++j) v[j] = load16<NT>((const u32x4*)(a.base + from[j]));
      // Read burst, then write burst, as in copy_rows.
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < ROWS; ++j) store16<NT>((u32x4*)(a.base + to[j]), v[j]);
    } else {  // the short last ticket of a segment, or a ticket with a refused move
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        to[j] = kSkip;
        if (move_of[j] < cnt) {
          const uint64_t from = s_src[move_of[j]];
          if (from != kSkip) {
            v[j] = load16<NT>((const u32x4*)(a.base + from + within[j]));
            to[j] = s_dst[move_of[j]] + within[j];
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < ROWS; ++j)
        if (to[j] != kSkip) store16<NT>((u32x4*)(a.base + to[j]), v[j]);
    }
    __syncthreads();  // the LDS words are rewritten by the next round
  }
  if (tid == 0) sign_out(a.state, n_units);
}

// Launch compact_packed_kernel<NT, rows> for a run-time row count in 1..MAX.
template <int MAX>
int launch_packed(const PackArgs& p, uint32_t rows, uint32_t workgroups, bool nt, hipStream_t s) {
  if (rows == (uint32_t)MAX || MAX == 1) {
    const dim3 grid(workgroups), block(kCopyThreads);
    if (nt) hipLaunchKernelGGL((compact_packed_kernel<true, MAX>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((compact_packed_kernel<false, MAX>), grid, block, 0, s, p);
    return launch_rc();
  }
  if constexpr (MAX > 1) return launch_packed<MAX - 1>(p, rows, workgroups, nt, s);
  return KV_E_RANGE;
}

template <int UNROLL, bool WHOLE>
int launch_shape(const CopyArgs& a, uint32_t workgroups, bool nt, bool prefetch, hipStream_t s) {
  const dim3 grid(workgroups), block(kCopyThreads);
  if (nt && prefetch) hipLaunchKernelGGL((compact_ticket_kernel<UNROLL, true, true, WHOLE>), grid, block, 0, s, a);
  else if (nt) hipLaunchKernelGGL((compact_ticket_kernel<UNROLL, true, false, WHOLE>), grid, block, 0, s, a);
  else if (prefetch) hipLaunchKernelGGL((compact_ticket_kernel<UNROLL, false, true, WHOLE>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((compact_ticket_kernel<UNROLL, false, false, WHOLE>), grid, block, 0, s, a);
  return launch_rc();
}

template <int UNROLL>
int launch(const CopyArgs& a, uint32_t workgroups, bool nt, bool prefetch, hipStream_t s) {
  const bool whole = a.chunk_bytes == (uint32_t)UNROLL * kRowBytes && a.seg_bytes % a.chunk_bytes == 0;
  return whole ? launch_shape<UNROLL, true>(a, workgroups, nt, prefetch, s)
               : launch_shape<UNROLL, false>(a, workgroups, nt, prefetch, s);
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

namespace {

// Copies the tiles of layers [layer_first, layer_first + layer_count) (clipped to the pool's layers)
// of moves [move_first, move_first + move_count) (clipped to the plan's moves on the device).
int launch_copy(const kv_pool_desc* pool, const kv_plan* plan, const kv_compact_tuning* tuning,
                uint32_t move_first, uint32_t move_count, uint32_t layer_first, uint32_t layer_count, void* stream) {
  if (pool == nullptr || plan == nullptr || plan->state == nullptr) return KV_E_NULL;
  if (pool->num_blocks != plan->num_blocks || plan->boundary > plan->num_blocks) return KV_E_RANGE;
  if (!pool_extent_ok(*pool)) return KV_E_RANGE;  // zero or absurd sizes
  if ((pool->tile_bytes % kVecBytes) != 0) return KV_E_ALIGN;

  uint32_t workgroups = 0, chunk = kDefaultChunk, flags = 0u;
  if (tuning != nullptr) {
    workgroups = tuning->workgroups;
    if (tuning->chunk_bytes) chunk = tuning->chunk_bytes;
    flags = tuning->flags;
  }
  if ((chunk % kRowBytes) != 0 || workgroups > (1u << 20)) return KV_E_RANGE;
  const uint32_t unroll = (flags >> 4) & 0x3Fu ? (flags >> 4) & 0x3Fu : kDefaultUnroll;
  if (unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16 && unroll != 32) return KV_E_RANGE;

  const bool layer_major = pool->layer_stride_bytes != 0;
  if (layer_major && (pool->layer_stride_bytes % 256u != 0 ||
                      pool->layer_stride_bytes < (uint64_t)pool->num_blocks * pool->tile_bytes))
    return KV_E_RANGE;
  if (plan->capacity == 0 || pool->num_blocks == 0) return KV_OK;  // nothing can move
  if (move_first >= plan->capacity || move_count == 0) return KV_OK;   // no such moves
  if (layer_first >= pool->num_layers || layer_count == 0) return KV_OK;  // no such layers
  if (layer_count > pool->num_layers - layer_first) layer_count = pool->num_layers - layer_first;
  if (pool->base == nullptr || plan->src == nullptr || plan->dst == nullptr) return KV_E_NULL;
  if (((uintptr_t)pool->base % 256u) != 0) return KV_E_ALIGN;

  CopyArgs a;
  if (layer_major) {  // one segment (tile) per chosen layer slab
    a.base = (uint8_t*)pool->base + (uint64_t)layer_first * pool->layer_stride_bytes;
    a.block_stride = pool->tile_bytes;
    a.seg_stride = pool->layer_stride_bytes;
    a.seg_bytes = pool->tile_bytes;
  } else {            // the chosen layers' tiles are one contiguous run inside the block
    a.base = (uint8_t*)pool->base + (uint64_t)layer_first * pool->tile_bytes;
    a.block_stride = (uint64_t)pool->num_layers * pool->tile_bytes;
    a.seg_stride = 0;
    a.seg_bytes = (uint64_t)layer_count * pool->tile_bytes;
  }
  const uint64_t segs = layer_major ? layer_count : 1u;
  // Default units are 64 KiB, the last one of a segment shorter.  A short unit costs a whole
  // ticket, and tickets of 40 KiB or less on average are drawn faster than one counter address
  // can hand them out, so small ragged segments (up to four units) are cut differently where
  // that measured faster: a tail of at most 20 KiB behind a single unit stays in that unit (one
  // burst of 17 to 21 rows; 72 KiB tiles: 5.7 -> 6.7 TB/s), and where equal units come out at
  // 48 KiB or more the segment is cut into equal units (96 KiB: two of 48, 6.5 -> 6.6;
  // 160 KiB: three of 56, 6.6 -> 6.7).
  if ((tuning == nullptr || tuning->chunk_bytes == 0) && a.seg_bytes > kDefaultChunk &&
      a.seg_bytes <= 4ull * kDefaultChunk && a.seg_bytes % kDefaultChunk != 0) {
    const uint64_t whole = a.seg_bytes / kDefaultChunk, tail = a.seg_bytes % kDefaultChunk;
    uint64_t units = 0;  // 0: keep the default
    if (whole == 1 && tail <= 20u * 1024u) units = 1;
    else if (a.seg_bytes >= 48ull * 1024ull * (whole + 1)) units = whole + 1;
    if (units != 0) {
      const uint64_t each = (a.seg_bytes + units - 1) / units;
      chunk = (uint32_t)((each + kRowBytes - 1) / kRowBytes * kRowBytes);
    }
  }
  const uint64_t chunks_per_seg = (a.seg_bytes + chunk - 1) / chunk;
  if (segs * chunks_per_seg * plan->capacity >= (1ull << 31)) return KV_E_RANGE;  // unit ids are 32-bit
  a.src = plan->src + move_first;
  a.dst = plan->dst + move_first;
  a.move_first = move_first;
  a.move_count = move_count;
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
  const bool prefetch = (flags & 2u) != 0;
  hipStream_t s = (hipStream_t)stream;

  // Segments of half a ticket or less: several moves per ticket.
  uint32_t ticket_bytes = chunk < kPackRows * kRowBytes ? chunk : kPackRows * kRowBytes;
  if ((tuning == nullptr || tuning->chunk_bytes == 0) && a.seg_bytes * 2u > ticket_bytes &&
      a.seg_bytes * 2u <= kMaxBurstRows * kRowBytes)
    ticket_bytes = kMaxBurstRows * kRowBytes;  // 40 KiB blocks: 6.05 -> 6.3 TB/s
  if ((flags & 8u) == 0 && a.seg_bytes * 2u <= ticket_bytes) {
    PackArgs p;
    p.base = a.base;
    p.block_stride = a.block_stride;
    p.seg_stride = a.seg_stride;
    p.src = a.src;
    p.dst = a.dst;
    p.state = a.state;
    p.num_blocks = a.num_blocks;
    p.boundary = a.boundary;
    p.segs = (uint32_t)segs;
    p.seg_vecs = (uint32_t)(a.seg_bytes / kVecBytes);
    p.recip = p.seg_vecs > 1u ? (uint32_t)(0xFFFFFFFFull / p.seg_vecs) + 1u : 0u;
    const uint32_t fit = ticket_bytes / (uint32_t)a.seg_bytes;
    p.pack = fit < kMaxPack ? fit : kMaxPack;
    p.ticket_vecs = p.pack * p.seg_vecs;
    p.move_first = move_first;
    p.move_count = move_count;
    return launch_packed<kMaxBurstRows>(p, (p.ticket_vecs + kCopyThreads - 1u) / kCopyThreads, workgroups, nt, s);
  }

  switch (unroll) {
    case 2: return launch<2>(a, workgroups, nt, prefetch, s);
    case 4: return launch<4>(a, workgroups, nt, prefetch, s);
    case 8: return launch<8>(a, workgroups, nt, prefetch, s);
    case 16: return launch<16>(a, workgroups, nt, prefetch, s);
    default: return launch<32>(a, workgroups, nt, prefetch, s);
  }
}

}  // namespace

extern "C" int kv_compact_launch(const kv_pool_desc* pool, const kv_plan* plan,
                                 const kv_compact_tuning* tuning, void* stream) {
  return launch_copy(pool, plan, tuning, 0u, ~0u, 0u, ~0u, stream);
}

extern "C" int kv_compact(const kv_pool_desc* pool, const kv_plan* plan, void* stream) {
  return launch_copy(pool, plan, nullptr, 0u, ~0u, 0u, ~0u, stream);
}

extern "C" int kv_compact_moves(const kv_pool_desc* pool, const kv_plan* plan, uint32_t first_move,
                                uint32_t max_moves, void* stream) {
  return launch_copy(pool, plan, nullptr, first_move, max_moves, 0u, ~0u, stream);
}

extern "C" int kv_compact_layers(const kv_pool_desc* pool, const kv_plan* plan, uint32_t first_layer,
                                 uint32_t max_layers, void* stream) {
  return launch_copy(pool, plan, nullptr, 0u, ~0u, first_layer, max_layers, stream);
}
