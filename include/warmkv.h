/* warmkv - MI355X (gfx950) KV-cache reclaim and weight materialisation.
 *
 * The scenario is the paper's proactive prewarming (arXiv 2512.09472, Sec. 3.3
 * and App. C, Fig. 4b steps 1-3): a serving instance that is about to be shut
 * down keeps only the KV space it reserved (Eq. 4) and gives the rest to the
 * weights of a model being prewarmed, while its running requests carry on.
 * Only unused KV blocks may receive weights, and the engine must keep seeing
 * every sequence's KV unchanged.  The paper gets there by re-pointing page
 * tables; this library gets there by compacting the paged KV pool:
 *
 *   every live block whose physical id is at or above a reclaim boundary b is
 *   moved into a free id below b - the k-th smallest moving id takes the k-th
 *   smallest free id - the per-sequence block tables are rewritten, and the
 *   new model's weights are streamed from pinned host memory into the byte
 *   range that starts at block b.
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is marked [device] or [host].  The library
 *     allocates and frees nothing (except where a function says otherwise) and
 *     owns nothing that outlives a call; the caller owns pool, tables, bitmap,
 *     workspace, pinned host tensors, streams and events.
 *   - `stream` / `event` arguments are hipStream_t / hipEvent_t passed as
 *     void*; NULL stream = the default stream.
 *   - Calls that take a stream are asynchronous on it and return after
 *     enqueueing.  Return value: KV_OK or a negative KV_E_* for errors the host
 *     can see (bad argument, failed launch).  Nothing is enqueued and no byte
 *     is written when a call returns an error.
 *   - The one data-dependent failure - more moving blocks than free ids below
 *     the boundary - is recorded on the device in kv_plan_state.status.
 *     kv_compact and kv_remap_tables read it and do nothing unless it is KV_OK,
 *     so an infeasible request modifies no pool byte and no table entry
 *     (existing requests take precedence over prewarmed weights, Sec. 3.3).
 *   - Pool layout: one allocation, block-major by default: block i occupies
 *     bytes [i*block_bytes, (i+1)*block_bytes), block_bytes = num_layers *
 *     tile_bytes, layer l's K and V tile at + l*tile_bytes.  A layer-major pool
 *     is described by kv_pool_desc.layer_stride_bytes.  Bytes are never
 *     interpreted (bf16 or fp8 alike).
 *   - Re-entrant; no global state.  Two calls that touch the same plan or pool
 *     must be ordered by the caller (same stream, or events).
 */
#ifndef WARMKV_H
#define WARMKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KV_OK          0
#define KV_E_NULL     (-1)  /* a required pointer is NULL                                  */
#define KV_E_RANGE    (-2)  /* boundary > num_blocks, sizes that do not match the plan, ... */
#define KV_E_ALIGN    (-3)  /* pool base not 256-byte aligned, tile_bytes not a multiple of 16 */
#define KV_E_TOOBIG   (-4)  /* a weight extent leaves the reclaimed region; workspace too small */
#define KV_E_OVERLAP  (-5)  /* two weight extents overlap; live_out aliases live_in          */
#define KV_E_HIP      (-6)  /* a HIP call failed                                             */
#define KV_E_NOSPACE  (-7)  /* device status: more movers than free ids below the boundary   */
#define KV_E_BADPLAN  (-8)  /* device status: a move violates src >= boundary > dst          */
#define KV_E_NOMEM    (-9)  /* host memory for the call's own bookkeeping could not be had   */

/* Describes the caller-owned paged KV pool (one allocation).
 * layer_stride_bytes == 0: block-major.  Block i is block_bytes = L*tile_bytes
 *   contiguous bytes at i*block_bytes; layer l's tile sits at + l*tile_bytes.
 * layer_stride_bytes != 0: layer-major (one slab per layer, the layout paged
 *   attention engines usually keep).  Layer l's tile of block i sits at
 *   l*layer_stride_bytes + i*tile_bytes; layer_stride_bytes >= NB*tile_bytes
 *   and a multiple of 256.  A block is then L separate tiles and the reclaimed
 *   space is L strips, one per slab: bytes [b*tile_bytes, NB*tile_bytes) of
 *   each.  An engine that keeps K and V of a layer in two slabs of their own
 *   describes 2L slabs of half-tiles (num_layers = 2L, tile_bytes = one K or
 *   V tile) if the 2L slabs are equally spaced, else one pool per slab set. */
typedef struct kv_pool_desc {
  void*    base;                /* [device] 256-byte aligned                           */
  uint32_t num_blocks;          /* NB, at most 2^24                                    */
  uint32_t num_layers;          /* L >= 1                                              */
  uint64_t tile_bytes;          /* one block in one layer (K and V); multiple of 16    */
  uint64_t layer_stride_bytes;  /* 0 = block-major, else bytes between layer slabs     */
} kv_pool_desc;

/* Device-resident result header of a plan (32 bytes). */
typedef struct kv_plan_state {
  int32_t  status;         /* the planner's verdict: KV_OK or KV_E_NOSPACE; as returned by
                              kv_plan_fetch also KV_E_BADPLAN (see bad_plan)             */
  uint32_t n_moves;        /* number of blocks to move (0 unless status == KV_OK)        */
  uint32_t n_free_below;   /* free ids below the boundary before the move                */
  uint32_t n_bad_entries;  /* table entries kv_remap_tables left alone (see there)       */
  uint32_t ticket;         /* kv_compact's work counter; zero between calls              */
  uint32_t finished;       /* kv_compact's exit counter; zero between calls              */
  uint32_t bad_plan;       /* set to 1 by kv_compact when it skipped a move (see there);
                              never changes `status` on the device, so that every
                              workgroup of a launch sees the same plan                   */
  uint32_t reserved;
} kv_plan_state;

/* A relocation plan.  All pointers are [device] and point into the workspace
 * the caller passed to kv_plan_bind. */
typedef struct kv_plan {
  int32_t*       src;        /* [capacity] moving ids, ascending; first n_moves valid    */
  int32_t*       dst;        /* [capacity] destination ids, ascending, all < boundary    */
  int32_t*       new_id;     /* [num_blocks] i -> id after the move, -1 for free ids     */
  uint64_t*      live_out;   /* [ceil(num_blocks/64)] live bitmap after the move         */
  kv_plan_state* state;
  uint32_t       num_blocks;
  uint32_t       boundary;   /* first reclaimed block id b                               */
  uint32_t       capacity;   /* min(num_blocks - boundary, boundary)                     */
  uint32_t       reserved;
} kv_plan;

/* Bytes of device workspace a plan for (num_blocks, boundary) needs; 0 if
 * boundary > num_blocks. */
size_t kv_plan_workspace_bytes(uint32_t num_blocks, uint32_t boundary);

/* Carve `workspace` [device, 256-byte aligned, >= kv_plan_workspace_bytes()]
 * into the arrays of `plan` [host].  Touches no device memory. */
int kv_plan_bind(kv_plan* plan, void* workspace, size_t workspace_bytes,
                 uint32_t num_blocks, uint32_t boundary);

/* Relocation planner: which physical blocks are unused, and where each block
 * that is in the way goes (App. C, Fig. 4b step 1; how much to reclaim is
 * Eq. 4's business and arrives as `boundary`).
 * live_in [device]: uint64[ceil(NB/64)], bit (i%64) of word (i/64) set <=> block
 * i holds live KV; bits at or beyond NB in the last word are ignored.  Must
 * not overlap plan->live_out.
 * Writes plan->state always; if feasible also src/dst[0..n_moves), new_id[NB]
 * (identity for live ids < b, dst[k] for src[k], -1 for free ids) and live_out
 * (bits >= b cleared, bits dst[0..n) set).  If infeasible: state.status =
 * KV_E_NOSPACE, n_moves = 0, and the other outputs are unspecified. */
int kv_plan_reclaim(const uint64_t* live_in, const kv_plan* plan, void* stream);

/* Block copy: for k < n_moves, block dst[k] <- block src[k] (block_bytes each;
 * in a layer-major pool, tile by tile in every layer slab).  This is what makes
 * the unused space one byte range for the new model (it stands where the paper
 * maps the pages of unused blocks into the prewarm slot: App. C, Fig. 4b step 2).
 * Source blocks keep their bytes; no byte at or above block `boundary` and no
 * byte of a non-destination block is written.  Does nothing unless
 * state.status == KV_OK.  A move with src < boundary, src >= NB or dst >=
 * boundary (possible only in a hand-built plan) is skipped and sets
 * state.bad_plan = 1; every other move is still copied.  kv_plan_fetch then
 * reports KV_E_BADPLAN and kv_remap_tables does nothing.
 * pool->num_blocks must equal plan->num_blocks.
 * Uses state.ticket / state.finished as scratch counters (zeroed by the
 * planner, left at zero on exit): two kv_compact calls on one plan must not
 * overlap in time. */
int kv_compact(const kv_pool_desc* pool, const kv_plan* plan, void* stream);

/* Launch shape of kv_compact, for tuning.  Zero fields select the defaults. */
typedef struct kv_compact_tuning {
  uint32_t workgroups;     /* persistent grid size (default: one per compute unit)       */
  uint32_t chunk_bytes;    /* bytes per work ticket; multiple of 4096 (default 65536)    */
  uint32_t flags;          /* bit 0: plain (cached) instead of non-temporal accesses;
                              bit 1: draw the next ticket during the copy, not after it;
                              bit 2: layer-major pools: move by move instead of slab by slab
                                     (tiles above half a ticket only);
                              bit 3: one ticket per tile or block even when it is half a ticket
                                     or less (default: such small units are packed, several
                                     consecutive moves to a ticket of at most 64 KiB);
                              bits 4-9: 128-bit loads in flight per lane: 2, 4, 8, 16 (default)
                                        or 32                                              */
  uint32_t reserved;
} kv_compact_tuning;

/* kv_compact with an explicit launch shape (same results, same rules). */
int kv_compact_launch(const kv_pool_desc* pool, const kv_plan* plan,
                      const kv_compact_tuning* tuning, void* stream);

/* Block-table rewrite, run right after kv_compact on the same stream: every
 * entry e >= 0 of tables [device, int32, num_seqs x max_blocks_per_seq,
 * row-major, -1 = empty] becomes new_id[e].  Entries that name an id >= NB or
 * a block that was not live are left as they are and counted in
 * state.n_bad_entries (added to what is there).  Does nothing unless
 * state.status == KV_OK and state.bad_plan == 0.  (The engine goes on seeing
 * one address space and never learns that blocks moved: App. C.) */
int kv_remap_tables(int32_t* tables, uint32_t num_seqs, uint32_t max_blocks_per_seq,
                    const kv_plan* plan, void* stream);

/* The reclaim step as one call (App. C, Fig. 4b steps 1-2, as the three calls
 * above): kv_plan_reclaim, kv_compact and kv_remap_tables
 * on `stream`, with the same arguments, rules and results (all of the plan's
 * arrays and its header are written as the three calls write them).  A small
 * pool - at most 32 768 blocks, at most 16 384 table entries, at most 128 MiB
 * of blocks that could move - takes a single kernel launch, in which every
 * workgroup ranks the bitmap for itself so that none waits for another; on a
 * pool of a thousand blocks the three launches and the gaps between them cost
 * more than the work.  Larger pools take the three launches. */
int kv_reclaim(const kv_pool_desc* pool, const kv_plan* plan, const uint64_t* live_in,
               int32_t* tables, uint32_t num_seqs, uint32_t max_blocks_per_seq, void* stream);

/* Synchronise `stream` and copy the plan's header to `out` [host];
 * out->status is KV_E_BADPLAN if the planner said KV_OK and kv_compact has
 * since skipped a move (state.bad_plan). */
int kv_plan_fetch(const kv_plan* plan, void* stream, kv_plan_state* out);

/* One weight tensor: `bytes` bytes at host_ptr [host, pinned] go to byte
 * offset dst_offset of the reclaimed region. */
typedef struct wm_tensor {
  const void* host_ptr;
  uint64_t    bytes;
  uint64_t    dst_offset;
} wm_tensor;

/* Weight materialisation: the new model's weights go into the space that
 * unused KV blocks gave up (App. C, Fig. 4b step 3), from host memory over the
 * host link (Sec. 4.1), each copy issued once its destination is ready (App. C).
 * The reclaimed region is bytes [boundary*block_bytes, num_blocks*block_bytes)
 * of the pool.  In a layer-major pool it is the L strips taken one after the
 * other in layer order (strip l = region offsets [l*S, (l+1)*S), S =
 * (num_blocks-boundary)*tile_bytes); an extent that would straddle two strips
 * is not contiguous in memory and is refused with KV_E_TOOBIG.
 * All extents are validated first (inside the region: else
 * KV_E_TOOBIG; pairwise disjoint: else KV_E_OVERLAP).  Then, on copy_stream:
 * wait for `compaction_done` (hipEvent_t recorded after kv_compact; NULL = no
 * wait, the caller has ordered the streams) and enqueue the host-to-device
 * copies in chunks.  The region still holds moving blocks until kv_compact has
 * read them, hence the event.  tensors [host] may be freed on return; the
 * host_ptr buffers must stay valid until copy_stream has drained.
 * WARNING: this call knows nothing of the plan.  If the plan was infeasible
 * (KV_E_NOSPACE), kv_compact and kv_remap_tables did nothing and the region
 * still holds the live blocks that could not move: a weight stream enqueued
 * behind them overwrites running requests' KV.  Read the verdict first
 * (kv_plan_fetch) or use kv_switch, which does and sends nothing then. */
int weights_materialize(const kv_pool_desc* pool, uint32_t boundary,
                        const wm_tensor* tensors, uint32_t n_tensors,
                        void* copy_stream, void* compaction_done);

/* One host-to-device request of the pipelined schedule below. */
typedef struct wm_piece {
  uint32_t tensor;      /* index into the caller's tensor array                        */
  uint32_t early;       /* 1: enqueued before the wait on the compaction event         */
  uint64_t src_offset;  /* bytes from tensors[tensor].host_ptr                          */
  uint64_t dst_offset;  /* bytes from the start of the reclaimed region                */
  uint64_t bytes;
} wm_piece;

/* Block-granular pipelining of the weight stream (the paper pipelines page
 * mapping and weight copying page by page, App. C).  A block of the reclaimed region that was free when the plan was
 * made is ready at once; one that holds a moving block is ready only after
 * kv_compact has read it.  live_host [host] is the bitmap kv_plan_reclaim was
 * given (before the move).  Tensors are walked in the caller's order and cut
 * at block boundaries; runs that lie wholly in free blocks become early pieces
 * until early_bytes have been collected (0 = the library's own policy: 128 MiB,
 * and only runs of at least 2 MiB, below which a request costs more than it
 * hides); all other bytes become late pieces, one per tensor remainder run.
 * Host arithmetic only.
 * In a layer-major pool the unit is a block's tile in one strip: region offset
 * x lies in the tile of block boundary + (x mod strip bytes) / tile_bytes.
 * Writes at most `capacity` pieces to out [host] (early pieces first) and the
 * full count to *n_out; returns KV_E_TOOBIG if capacity is too small, and the
 * validation errors of weights_materialize. */
int weights_materialize_schedule(const kv_pool_desc* pool, uint32_t boundary,
                                 const uint64_t* live_host,
                                 const wm_tensor* tensors, uint32_t n_tensors,
                                 uint64_t early_bytes, wm_piece* out,
                                 uint32_t capacity, uint32_t* n_out);

/* weights_materialize with that schedule: same bytes in the pool, but the
 * early pieces are enqueued on copy_stream before the wait on compaction_done
 * and so overlap the block copy; the late pieces follow the event. */
int weights_materialize_pipelined(const kv_pool_desc* pool, uint32_t boundary,
                                  const uint64_t* live_host,
                                  const wm_tensor* tensors, uint32_t n_tensors,
                                  uint64_t early_bytes,
                                  void* copy_stream, void* compaction_done);

/* Block copy of a part of the plan: moves [first_move, first_move + max_moves)
 * that exist (k < n_moves); otherwise as kv_compact.  Moves are listed in
 * ascending source order, so "the first h moves" are the movers of the first
 * blocks of the reclaimed region. */
int kv_compact_moves(const kv_pool_desc* pool, const kv_plan* plan, uint32_t first_move,
                     uint32_t max_moves, void* stream);

/* Block copy of a part of every move: only the tiles of layers [first_layer,
 * first_layer + max_layers) that exist; otherwise as kv_compact.  In a
 * layer-major pool that is the slabs of those layers, so "the first f layers"
 * evacuate the first f strips of the reclaimed space, which is the order region
 * offsets count in. */
int kv_compact_layers(const kv_pool_desc* pool, const kv_plan* plan, uint32_t first_layer,
                      uint32_t max_layers, void* stream);

/* Number of live blocks among the first front_blocks blocks at and above
 * `boundary` in live_host [host bitmap, as given to kv_plan_reclaim]: how many
 * moves of a feasible plan evacuate that front.  Host arithmetic only. */
uint32_t kv_movers_in_front(const uint64_t* live_host, uint32_t num_blocks, uint32_t boundary,
                            uint32_t front_blocks);

/* Front-first weight stream (a copy starts once its destination is ready,
 * App. C): the block copy frees the reclaimed region from its start, so the
 * bytes of every tensor that lie below region offset front_bytes are enqueued
 * behind front_done (hipEvent_t recorded after kv_compact_moves(0, h), h =
 * kv_movers_in_front(.., ceil(front_bytes / block_bytes))) and the remaining
 * bytes behind compaction_done (recorded after the rest of the block copy).
 * Either event may be NULL (no wait).  Same validation, same bytes in the pool
 * as weights_materialize; each tensor is cut at most once.
 * In a layer-major pool region offsets count strip by strip, and the region
 * becomes ready strip by strip when the block copy takes the slabs in layer
 * order: front_done is then recorded after kv_compact_layers(0, f) with
 * f = ceil(front_bytes / strip bytes), compaction_done after
 * kv_compact_layers(f, all the rest). */
int weights_materialize_front(const kv_pool_desc* pool, uint32_t boundary, uint64_t front_bytes,
                              const wm_tensor* tensors, uint32_t n_tensors,
                              void* copy_stream, void* front_done, void* compaction_done);

/* The weight stream over several copy streams.  As weights_materialize_front
 * (front_bytes = 0 and front_done = NULL: as weights_materialize), but the
 * host-to-device requests are dealt out in turn to copy_streams[0..n_streams)
 * [host array of hipStream_t, 1 to 4 streams], each of which waits for the
 * events as the single stream would.  Streams are served by different DMA
 * engines, so the next request is set up while the previous one still runs and
 * the link does not idle at request boundaries: what a checkpoint of many
 * tensors that do not continue each other in host memory loses on one stream
 * (10-45 us per tensor).  The same bytes arrive; the caller synchronises every
 * stream it passed. */
int weights_materialize_streams(const kv_pool_desc* pool, uint32_t boundary, uint64_t front_bytes,
                                const wm_tensor* tensors, uint32_t n_tensors,
                                void* const* copy_streams, uint32_t n_streams,
                                void* front_done, void* compaction_done);

/* One request for the whole hand-over (App. C, Fig. 4b steps 1-3). */
typedef struct kv_switch_request {
  const kv_pool_desc* pool;
  const kv_plan*      plan;          /* bound by kv_plan_bind; its boundary is the reclaim boundary   */
  const uint64_t*     live_in;       /* [device] live bitmap, as for kv_plan_reclaim                  */
  const uint64_t*     live_host;     /* [host] the same bitmap, or NULL: weights wait for the whole
                                        block copy instead of being pipelined block by block         */
  int32_t*            tables;        /* [device] as for kv_remap_tables                               */
  uint32_t            num_seqs;
  uint32_t            max_blocks_per_seq;
  const wm_tensor*    tensors;       /* [host] as for weights_materialize                             */
  uint32_t            n_tensors;
  uint32_t            reserved;
  uint64_t            early_bytes;   /* as for weights_materialize_pipelined (0 = default)            */
  void*               compute_stream;
  void*               copy_stream;
  void*               compaction_done;  /* hipEvent_t created by the caller; recorded by this call    */
  void*               front_done;    /* second hipEvent_t of the caller's, or NULL; with live_host it
                                        selects the front-first weight stream (see below)            */
  void*               copy_stream2;  /* a second copy stream, or NULL: weight requests alternate
                                        between the two (see weights_materialize_streams)            */
} kv_switch_request;

/* The hand-over as one call: plan, block copy and table rewrite on
 * compute_stream, the weight stream on copy_stream behind compaction_done.
 * If live_host is given the weight stream is
 * pipelined with the block copy: front first if front_done is given too (the
 * block copy is launched in two parts, the movers under the first early_bytes
 * of the region and the rest, with front_done recorded in between; early_bytes
 * 0 = sized from the plan so that the link stays busy until the block copy has
 * ended; in a layer-major pool the front is a whole number of strips and the
 * two parts are layer ranges), else block by block as in
 * weights_materialize_pipelined.  Existing requests take precedence over prewarmed weights
 * (Sec. 3.3): after the planner has run, compute_stream is synchronised once
 * and its verdict read; if the request is infeasible the call returns
 * KV_E_NOSPACE and nothing else is enqueued - no pool byte, table entry or
 * weight byte moves.  (With the separate calls the caller has to make that
 * check before weights_materialize, which would otherwise overwrite the blocks
 * that could not move.)  All arguments, weight extents included, are validated
 * before the planner is launched.  *result [host, may be NULL] receives the
 * plan's header.  On KV_OK everything is enqueued and the call returns without
 * waiting for it. */
int kv_switch(const kv_switch_request* request, kv_plan_state* result);

/* For callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  kv_plan_reclaim +
 * kv_compact + kv_remap_tables on `stream`, with the plan's workspace (the
 * move lists, the id map, the work counters) in a static device array inside
 * the library instead of a caller's buffer; the call allocates and frees
 * nothing, on the host or on the device.  Inputs and outputs are the caller's:
 * pool, live_in, tables as for the three calls; live_out [device,
 * uint64[ceil(NB/64)], must not overlap live_in] receives the bitmap after the
 * move and state_out [device, one kv_plan_state] the plan's header as
 * kv_plan_fetch would report it (status KV_E_NOSPACE: nothing was moved or
 * rewritten and live_out is unspecified).
 * Limits: pool->num_blocks <= KV_STATIC_MAX_BLOCKS, else KV_E_TOOBIG and nothing
 * is enqueued.  The array (about 2 MiB) exists once per GPU the library is
 * used on, for the life of the process; its address on the current device is
 * looked up on the first call there (make that call outside stream capture;
 * later calls may be captured).  Every call on a GPU uses that one array:
 * two calls that overlap in time on one GPU (different streams with no
 * ordering between them) race, so order them.  Each call rewrites all of
 * the array it reads, so a smaller request after a larger one is fine. */
#define KV_STATIC_MAX_BLOCKS 262144u
int kv_reclaim_static(const kv_pool_desc* pool, uint32_t boundary, const uint64_t* live_in,
                      uint64_t* live_out, int32_t* tables, uint32_t num_seqs,
                      uint32_t max_blocks_per_seq, kv_plan_state* state_out, void* stream);

/* Reserved KV space of a draining instance, Sec. 3.3 Eq. 4, in blocks:
 * R = max(C*Q/B, T + C/B), fractional blocks rounded up, capped at C.
 * C = capacity_blocks (<= 2^32 - 1), T = used_blocks, Q = running requests,
 * B = max_batch.  The reclaim boundary is R.  Host arithmetic only.
 * Returns R, or KV_E_RANGE if B == 0, T > C or C too large. */
int64_t kv_reserve_blocks(uint64_t capacity_blocks, uint64_t used_blocks,
                          uint32_t running, uint32_t max_batch);

/* Reverse switch: the reserve proved too small, so prewarmed weights are
 * evicted and give their space back to the KV cache (Sec. 3.3, end).  The boundary
 * rises from old_boundary to new_boundary (old <= new <= num_blocks); blocks
 * [old, new) return to the KV allocator as free ids (no block is live there,
 * so no bitmap bit changes and no byte moves).  For every tensor placed by
 * weights_materialize relative to the old region: evicted[i] = 1 if it has a
 * byte inside the returned blocks (it is lost), else 0 and new_offset[i] is its
 * offset relative to the new region's start.  Host arithmetic only; evicted,
 * new_offset [host] have n_tensors entries.  In a layer-major pool every
 * strip loses its first (new - old) tiles: a tensor is lost if it has a byte
 * in them, and a survivor's new offset counts through the shorter strips.
 * Returns the number of evicted
 * tensors, or KV_E_RANGE / KV_E_NULL / KV_E_TOOBIG (an extent outside the
 * old region). */
int64_t kv_grow(const kv_pool_desc* pool, uint32_t old_boundary, uint32_t new_boundary,
                const wm_tensor* tensors, uint32_t n_tensors,
                uint8_t* evicted, uint64_t* new_offset);

/* ------------------------------------------------------------------------
 * No-move variant: the paper's own mechanism on HIP's virtual-memory API
 * (Sec. 3.4 and App. C: physical pages are pre-allocated once, a "prewarm
 * slot" is a second virtual range, and the pages under unused KV blocks are
 * mapped into it; nothing is copied and no block table changes).  Kept for
 * comparison with compaction.  Unlike the rest of this library these calls
 * own memory (physical handles and address ranges) and synchronise the device.
 * ------------------------------------------------------------------------ */
typedef struct kv_vmm_pool kv_vmm_pool;   /* opaque, host object */

/* Create a pool of num_blocks physical allocations of block_bytes each
 * (block_bytes must be a multiple of the device's allocation granularity:
 * else KV_E_ALIGN), all mapped read-write into one contiguous KV range, and
 * reserve an equally large, still unmapped slot range.  Current device. */
int kv_vmm_pool_create(uint32_t num_blocks, uint64_t block_bytes, kv_vmm_pool** out);

/* [device] base of the KV range (block i at + i*block_bytes while it is mapped
 * there) and of the slot range. */
void* kv_vmm_kv_base(const kv_vmm_pool* pool);
void* kv_vmm_slot_base(const kv_vmm_pool* pool);

/* Hand the pages of `want` unused blocks to the slot: the highest free ids of
 * live_host [host bitmap, as for kv_plan_reclaim] are unmapped from the KV
 * range and mapped, in descending id order, at slot offsets 0, block_bytes,
 * ...; the slot prefix [0, want*block_bytes) is then readable and writable.
 * Those ids must not be touched through the KV range until kv_vmm_restore.
 * Fails with KV_E_NOSPACE (nothing changed) if fewer than `want` blocks are
 * free, KV_E_RANGE if pages are already lent.  If a driver call fails half way
 * (KV_E_HIP) the pages lent so far are put back before the call returns; only
 * if that fails too do pages stay in the slot, and kv_vmm_lent() says how many.
 * ids_out [host, may be NULL] receives the `want` ids.  Synchronises the
 * device first. */
int kv_vmm_reclaim(kv_vmm_pool* pool, const uint64_t* live_host, uint32_t want, int32_t* ids_out);

/* kv_vmm_reclaim with the weight stream pipelined behind the mapping, the way
 * the paper hides its mapping cost (App. C: a copy is triggered as soon as its
 * page is mapped).  Pages are handed over `chunk_blocks` blocks at a time
 * (0 = 64); after each chunk the slot bytes it added are made accessible and
 * every byte of `tensors` [host; dst_offset counts from the slot's start]
 * that lies in them is enqueued on copy_stream from its pinned host_ptr, while
 * this thread goes on mapping the next chunk.  Extents must lie inside
 * [0, want*block_bytes) and be pairwise disjoint (KV_E_TOOBIG / KV_E_OVERLAP,
 * checked before anything changes).  Returns after the last copy is enqueued;
 * the host buffers must stay valid until copy_stream has drained. */
int kv_vmm_reclaim_load(kv_vmm_pool* pool, const uint64_t* live_host, uint32_t want, uint32_t chunk_blocks,
                        const wm_tensor* tensors, uint32_t n_tensors, void* copy_stream, int32_t* ids_out);

/* Number of blocks whose pages are in the slot right now. */
uint32_t kv_vmm_lent(const kv_vmm_pool* pool);

/* Give every lent page back to its block's place in the KV range. */
int kv_vmm_restore(kv_vmm_pool* pool);

/* Unmap everything, release the physical memory and both ranges. */
int kv_vmm_pool_destroy(kv_vmm_pool* pool);

/* ------------------------------------------------------------------------
 * Control-plane formulas of the paper (host arithmetic in double precision;
 * no device work).  They decide what the path above is asked to do: which
 * model to prewarm where.
 * ------------------------------------------------------------------------ */

/* Corrective seasonal predictor, Sec. 3.1, Eq. 1-3.  history [host] is
 * loads[n_days][n_windows], row-major, day 0 the oldest; the call predicts the
 * load of window `window` on day `day` from the D previous days (all windows)
 * and the windows of day `day` before `window`:
 *   P(k,i)     = (1/D) * sum_{d=1..D} L(k-d, i)
 *   Delta(k,i) = sum_{w=1..m} (L(k,i-w) - P(k,i-w)) * 2^(w-1) / (2^m - 1),  m = min(i, N)
 *   prediction = P(k,i) + Delta(k,i);   Delta = 0 when i = 0.
 * Requires D >= 1, day >= D, day < n_days, window < n_windows, N <= 62
 * (else KV_E_RANGE).  The paper's settings are D = 7, N = 10. */
int ws_predict_load(const double* history, uint32_t n_days, uint32_t n_windows,
                    uint32_t day, uint32_t window, uint32_t D, uint32_t N, double* prediction);

/* One served model, inputs of the prewarming score and of the placement. */
typedef struct ws_model {
  double   size_bytes;     /* S: bytes of weights of one replica                         */
  double   load_avg;       /* L_A: predicted average load of the next window            */
  double   load_peak;      /* L_P: predicted peak load                                   */
  double   cold_latency;   /* T_c: time to load the whole model from scratch            */
  uint32_t degree;         /* D: GPUs per replica, >= 1                                  */
  uint32_t batch;          /* B: maximum batch size, >= 1                                */
  uint32_t active;         /* K: instances serving now                                   */
  uint32_t reserved;
} ws_model;

/* Replicas to prewarm for one model and their scores, App. B.1:
 *   N_basic = max(ceil(L_A/B) - K, 0),  N_burst = max(ceil(L_P/B) - N_basic - K, 0)
 *   S_basic(i) = exp(-i/(N_basic+N_burst)) * T_c
 *   S_burst(i) = exp(-(N_basic+i)/(N_basic+N_burst)) * T_c * (L_P - L_A)/L_A
 * scores [host, capacity entries] receives the basic scores, then the burst
 * scores (a burst score is +infinity when L_A == 0).  Returns KV_E_TOOBIG if
 * capacity < N_basic + N_burst (the counts are still written), KV_E_RANGE for
 * negative loads, B == 0, degree == 0 or more than 10^6 replicas. */
int ws_replica_scores(const ws_model* model, uint32_t* n_basic, uint32_t* n_burst,
                      double* scores, uint32_t capacity);

/* One placement decision: replica `replica` (0-based; basic ones first) of
 * model `model` goes to GPUs [first_gpu, first_gpu + degree). */
typedef struct ws_placement {
  uint32_t model;
  uint32_t replica;
  uint32_t first_gpu;
  uint32_t is_burst;
  double   score;
} ws_placement;

/* Prewarming model placement, Sec. 3.2 Alg. 1 and App. B.2.  Replicas of all
 * models are ordered basic before burst, then by score descending (ties: lower
 * model index, then lower replica index).  Candidate groups for a replica of
 * degree D are the aligned runs of D GPUs inside one server
 * (gpus_per_server % D == 0 required), every GPU with at least ceil(S/D) free
 * bytes; aligned runs make any two placements disjoint or nested, never
 * partially overlapping.  For each group, H and R are the highest and the sum
 * of the scores of replicas already placed on any of its GPUs (H = -infinity,
 * R = 0 for an untouched group).  If some group has H < score, the one with
 * the least R among those is taken, else the one with the least R overall
 * (ties: lowest first_gpu); its GPUs lose ceil(S/D) free bytes.  A replica with
 * no candidate group is skipped.
 * out [host, capacity] receives the decisions in placement order and *n_out
 * their number; gpu_free_bytes [host, n_gpus] is updated only on KV_OK. */
int ws_place_replicas(const ws_model* models, uint32_t n_models,
                      double* gpu_free_bytes, uint32_t n_gpus, uint32_t gpus_per_server,
                      ws_placement* out, uint32_t capacity, uint32_t* n_out);

/* Library version, "major.minor". */
const char* warmkv_version(void);

/* Identifier of the source text this binary was compiled from (a hash over the
 * HIP sources and headers, baked in by the build).  A loader that has the
 * sources can tell a stale binary from a current one. */
const char* warmkv_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* WARMKV_H */
