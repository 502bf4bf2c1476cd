// Relocation planner: from the live/free bitmap and the reclaim boundary b,
// build the ascending list of moving ids (live, >= b), the ascending list of
// the smallest free ids below b, their pairing, the dense id map and the bitmap
// after the move.  (Which blocks are unused and where the ones in the way go:
// paper App. C, Fig. 4b step 1; b itself comes from Sec. 3.3, Eq. 4.)
//
// Shape: one bitmap word per thread, 1024 threads (16 wavefronts) per
// workgroup.  Ranks come from a popcount per word, a 64-lane shuffle scan, and
// a cross-wave prefix in LDS; movers and free ids are ranked in one pass by
// packing both counts into one 64-bit scan value.  Small pools (up to 32 768
// blocks) are done by one workgroup, fused in one launch.  Larger ones use
// several workgroups (256 or 1024 words each); each gets its carry by reducing
// the words in front of it (a few KiB from L2) instead of talking to its
// neighbours, and a tiny second kernel joins the two lists into new_id.
// All outputs are produced in id order (ranks are monotone in ids), so even
// the two lists are written nearly coalesced: a one-workgroup kernel lives on
// one compute unit, and per-lane bit walks with strided stores cost it 3x.
#include "bitmap.h"
#include "common.h"

namespace warmkv {
namespace {

template <int THREADS, bool FUSED>
__global__ __launch_bounds__(THREADS) void plan_kernel(
    const uint64_t* __restrict__ live_in, uint32_t n_words, uint32_t num_blocks, uint32_t boundary,
    int32_t* __restrict__ src, int32_t* __restrict__ dst, int32_t* __restrict__ new_id,
    uint64_t* __restrict__ live_out, kv_plan_state* __restrict__ state) {
  constexpr int kWaves = THREADS / kWave;
  __shared__ uint64_t s_wave[kWaves];
  __shared__ uint64_t s_carry[2][kWaves];
  __shared__ uint64_t s_live[THREADS];
  __shared__ uint64_t s_rank[THREADS];

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & (kWave - 1);
  const uint32_t wave = tid / kWave;
  const uint32_t first_word = blockIdx.x * THREADS;
  const uint32_t wi = first_word + tid;

  const uint64_t word = wi < n_words ? live_in[wi] : 0ull;
  const WordBits wb = classify(word, wi, num_blocks, boundary);
  const uint64_t mine = pack_counts(wb);

  // exclusive prefix of `mine` inside the workgroup
  const uint64_t incl = wave_inclusive_scan(mine);
  if (lane == kWave - 1) s_wave[wave] = incl;

  // carry-in (words before this workgroup) and grand total (all words)
  uint64_t before = 0, total = 0;
  if (!FUSED) {
    uint64_t acc_before = 0, acc_all = 0;
    for (uint32_t i = tid; i < n_words; i += THREADS) {
      const uint64_t c = pack_counts(classify(live_in[i], i, num_blocks, boundary));
      acc_all += c;
      if (i < first_word) acc_before += c;
    }
    acc_before = wave_sum(acc_before);
    acc_all = wave_sum(acc_all);
    if (lane == 0) {
      s_carry[0][wave] = acc_before;
      s_carry[1][wave] = acc_all;
    }
  }
  __syncthreads();
  uint64_t wave_base = 0, group_total = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint64_t t = s_wave[w];
    if ((uint32_t)w < wave) wave_base += t;
    group_total += t;
    if (!FUSED) {
      before += s_carry[0][w];
      total += s_carry[1][w];
    }
  }
  if (FUSED) total = group_total;

  const uint64_t excl = before + wave_base + incl - mine;
  const uint32_t n_moves = (uint32_t)(total >> 32);
  const uint32_t n_avail = (uint32_t)total;
  const bool feasible = n_moves <= n_avail;

  if (blockIdx.x == 0 && tid == 0) {
    kv_plan_state st;
    st.status = feasible ? KV_OK : KV_E_NOSPACE;
    st.n_moves = feasible ? n_moves : 0u;
    st.n_free_below = n_avail;
    st.n_bad_entries = 0u;
    st.ticket = 0u;
    st.finished = 0u;
    st.bad_plan = 0u;
    st.reserved = 0u;
    *state = st;
  }
  if (!feasible) return;  // uniform over the whole grid: nothing else is written

  // Everything below is written in id order, four consecutive ids (same bitmap
  // word) per lane per pass.  Ranks grow with ids, so neighbouring lanes write
  // neighbouring list entries: the src/dst lists come out (nearly) coalesced,
  // which matters because this whole kernel runs on one compute unit.
  s_live[tid] = wb.live;
  s_rank[tid] = excl;  // movers before this word (high half), free ids before it (low half)
  if (wi < n_words) {
    // bitmap after the move: survivors below the boundary plus the free ids that get taken
    const uint32_t a_rank = (uint32_t)excl;
    uint64_t taken = 0;
    if (a_rank < n_moves) {
      const uint32_t want = n_moves - a_rank;
      taken = want >= (uint32_t)__popcll(wb.avail) ? wb.avail : lowest_set_bits(wb.avail, want);
    }
    live_out[wi] = wb.keep | taken;
  }
  __syncthreads();

  const uint32_t group_first_id = first_word * 64u;
  const uint32_t first_pass_at_boundary = boundary > group_first_id ? (boundary - group_first_id) / (THREADS * 4u) : 0u;
  for (uint32_t it = 0; it < 16u; ++it) {
    const uint32_t local = (it * THREADS + tid) * 4u;
    const uint32_t id0 = group_first_id + local;
    if (id0 >= num_blocks) break;
    const uint32_t wl = local >> 6, bit0 = local & 63u;
    const uint64_t live = s_live[wl];
    const uint64_t lo = low_mask(id0 - bit0, boundary);
    const uint64_t valid = low_mask(id0 - bit0, num_blocks);
    const uint64_t movers = live & ~lo, avail = ~live & lo & valid;
    const uint64_t below = (1ull << bit0) - 1ull;
    const uint64_t rank = s_rank[wl];
    uint32_t m_rank = (uint32_t)(rank >> 32) + (uint32_t)__popcll(movers & below);
    uint32_t a_rank = (uint32_t)rank + (uint32_t)__popcll(avail & below);
    int32_t out[4];
#pragma unroll
    for (uint32_t e = 0; e < 4u; ++e) {
      const uint32_t bit = bit0 + e;
      const int32_t id = (int32_t)(id0 + e);
      out[e] = -1;
      if ((movers >> bit) & 1ull) {
        src[m_rank++] = id;      // its new_id entry follows below (fused) or in join_kernel
      } else if ((live >> bit) & 1ull) {
        out[e] = id;             // live below the boundary: stays
      } else if ((avail >> bit) & 1ull) {
        if (a_rank < n_moves) dst[a_rank] = id;
        ++a_rank;
      }
    }
    if (id0 + 3u < num_blocks) {
      const i32x4 v = {out[0], out[1], out[2], out[3]};
      *(i32x4*)(new_id + id0) = v;
    } else {
      for (uint32_t e = 0; e < 4u && id0 + e < num_blocks; ++e) new_id[id0 + e] = out[e];
    }
  }
  if (!FUSED) return;

  // Fused shape: the whole dst list was written by this workgroup; after the
  // barrier every mover reads its destination by rank (neighbouring lanes read
  // neighbouring entries) and the groups that hold movers are stored again.
  __syncthreads();
  for (uint32_t it = first_pass_at_boundary; it < 16u; ++it) {
    const uint32_t local = (it * THREADS + tid) * 4u;
    const uint32_t id0 = group_first_id + local;
    if (id0 >= num_blocks) break;
    const uint32_t wl = local >> 6, bit0 = local & 63u;
    const uint64_t movers = s_live[wl] & ~low_mask(id0 - bit0, boundary);
    if (((movers >> bit0) & 0xFull) == 0) continue;
    uint32_t m_rank = (uint32_t)(s_rank[wl] >> 32) + (uint32_t)__popcll(movers & ((1ull << bit0) - 1ull));
#pragma unroll
    for (uint32_t e = 0; e < 4u; ++e)
      if ((movers >> (bit0 + e)) & 1ull) new_id[id0 + e] = dst[m_rank++];
  }
}

// new_id[src[k]] = dst[k]; second launch of the multi-workgroup shape.
__global__ __launch_bounds__(256) void join_kernel(const int32_t* __restrict__ src,
                                                   const int32_t* __restrict__ dst,
                                                   int32_t* __restrict__ new_id,
                                                   const kv_plan_state* __restrict__ state) {
  if (state->status != KV_OK) return;
  const uint32_t n = state->n_moves;
  for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x)
    new_id[src[k]] = dst[k];
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int kv_plan_reclaim(const uint64_t* live_in, const kv_plan* plan, void* stream) {
  if (plan == nullptr || plan->state == nullptr || plan->new_id == nullptr || plan->live_out == nullptr)
    return KV_E_NULL;
  const uint32_t nb = plan->num_blocks, b = plan->boundary;
  if (b > nb || nb > kMaxBlocks) return KV_E_RANGE;
  if (plan->capacity != (nb - b < b ? nb - b : b)) return KV_E_RANGE;
  if (plan->capacity != 0 && (plan->src == nullptr || plan->dst == nullptr)) return KV_E_NULL;
  const uint32_t n_words = (nb + 63u) / 64u;
  if (n_words != 0 && live_in == nullptr) return KV_E_NULL;
  const uintptr_t a0 = (uintptr_t)live_in, a1 = a0 + (uintptr_t)n_words * 8u;
  const uintptr_t o0 = (uintptr_t)plan->live_out, o1 = o0 + (uintptr_t)n_words * 8u;
  if (n_words != 0 && a0 < o1 && o0 < a1) return KV_E_OVERLAP;

  hipStream_t s = (hipStream_t)stream;
  // Shape, from measurement: up to 32 768 blocks one 1024-lane workgroup does everything in one
  // launch (12 us at 20 480 blocks).  Above that the bitmap is split into groups that run on
  // different compute units, 256 words each up to 2^20 blocks (18 us at 65 536 blocks, against
  // 27 us fused) and 1024 words beyond (fewer groups, each of which reduces all words in front of
  // it), followed by the join kernel.
  if (n_words <= 512) {
    hipLaunchKernelGGL((plan_kernel<1024, true>), dim3(1), dim3(1024), 0, s, live_in, n_words, nb, b, plan->src,
                       plan->dst, plan->new_id, plan->live_out, plan->state);
    return launch_rc();
  }
  if (nb <= (1u << 20)) {
    const uint32_t groups = (n_words + 255u) / 256u;
    hipLaunchKernelGGL((plan_kernel<256, false>), dim3(groups), dim3(256), 0, s, live_in, n_words, nb, b, plan->src,
                       plan->dst, plan->new_id, plan->live_out, plan->state);
  } else {
    const uint32_t groups = (n_words + 1023u) / 1024u;
    hipLaunchKernelGGL((plan_kernel<1024, false>), dim3(groups), dim3(1024), 0, s, live_in, n_words, nb, b,
                       plan->src, plan->dst, plan->new_id, plan->live_out, plan->state);
  }
  int rc = launch_rc();
  if (rc != KV_OK) return rc;
  uint32_t join_groups = (plan->capacity + 255u) / 256u;
  if (join_groups > 1024u) join_groups = 1024u;
  if (join_groups == 0u) join_groups = 1u;
  hipLaunchKernelGGL(join_kernel, dim3(join_groups), dim3(256), 0, s, plan->src, plan->dst, plan->new_id,
                     plan->state);
  return launch_rc();
}
