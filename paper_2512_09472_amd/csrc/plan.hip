// Relocation planner: from the live/free bitmap and the reclaim boundary b,
// build the ascending list of moving ids (live, >= b), the ascending list of
// the smallest free ids below b, their pairing, the dense id map and the bitmap
// after the move.  (Which blocks are unused and where the ones in the way go:
// paper App. C, Fig. 4b step 1; b itself comes from Sec. 3.3, Eq. 4.)
//
// Shape: one bitmap word per thread, 1024 threads (16 wavefronts) per
// workgroup, so one workgroup covers 65 536 blocks.  Ranks come from a popcount
// per word, a 64-lane shuffle scan, and a 16-entry cross-wave prefix in LDS;
// movers and free ids are ranked in one pass by packing both counts into one
// 64-bit scan value.  Pools above 65 536 blocks use several workgroups; each
// gets its carry by reducing the words in front of it (a few KiB from L2)
// instead of talking to its neighbours, and a tiny second kernel joins the two
// lists into new_id.  With one workgroup everything is fused in one launch.
#include "common.h"

namespace warmkv {
namespace {

struct WordBits {
  uint64_t mover;  // live, id >= b
  uint64_t avail;  // free, id < b
  uint64_t keep;   // live, id < b
  uint64_t live;   // live, id < NB
};

__device__ __forceinline__ uint64_t low_mask(uint32_t base, uint32_t limit) {
  // bits j of a word starting at id `base` with base + j < limit
  if (base + 64u <= limit) return ~0ull;
  if (base >= limit) return 0ull;
  return (1ull << (limit - base)) - 1ull;
}

__device__ __forceinline__ WordBits classify(uint64_t word, uint32_t wi, uint32_t num_blocks,
                                             uint32_t boundary) {
  const uint32_t base = wi * 64u;
  const uint64_t valid = low_mask(base, num_blocks);
  const uint64_t lo = low_mask(base, boundary);
  WordBits r;
  r.live = word & valid;
  r.mover = r.live & ~lo;
  r.avail = ~word & lo;
  r.keep = r.live & lo;
  return r;
}

// movers in the high half, free ids in the low half: one scan ranks both
__device__ __forceinline__ uint64_t pack_counts(const WordBits& wb) {
  return ((uint64_t)__popcll(wb.mover) << 32) | (uint64_t)__popcll(wb.avail);
}

__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint64_t up = __shfl_up(v, off, kWave);
    if (lane >= off) v += up;
  }
  return v;
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

template <bool FUSED>
__global__ __launch_bounds__(kPlanThreads) void plan_kernel(
    const uint64_t* __restrict__ live_in, uint32_t n_words, uint32_t num_blocks, uint32_t boundary,
    int32_t* __restrict__ src, int32_t* __restrict__ dst, int32_t* __restrict__ new_id,
    uint64_t* __restrict__ live_out, kv_plan_state* __restrict__ state) {
  constexpr int kWaves = kPlanThreads / kWave;
  __shared__ uint64_t s_wave[kWaves];
  __shared__ uint64_t s_carry[2][kWaves];
  __shared__ uint64_t s_live[kPlanThreads];
  __shared__ uint32_t s_mrank[kPlanThreads];

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & (kWave - 1);
  const uint32_t wave = tid / kWave;
  const uint32_t first_word = blockIdx.x * kPlanThreads;
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
    for (uint32_t i = tid; i < n_words; i += kPlanThreads) {
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
    st.reserved[0] = st.reserved[1] = 0u;
    *state = st;
  }
  if (!feasible) return;  // uniform over the whole grid: nothing else is written

  // movers and free ids, each written at its rank
  const uint32_t base_id = wi * 64u;
  uint32_t m_rank = (uint32_t)(excl >> 32);
  uint32_t a_rank = (uint32_t)excl;
  s_live[tid] = wb.live;
  s_mrank[tid] = m_rank;
  for (uint64_t bits = wb.mover; bits; bits &= bits - 1)
    src[m_rank++] = (int32_t)(base_id + (uint32_t)__builtin_ctzll(bits));
  uint64_t taken = 0;
  for (uint64_t bits = wb.avail; bits && a_rank < n_moves; bits &= bits - 1) {
    const uint32_t j = (uint32_t)__builtin_ctzll(bits);
    dst[a_rank++] = (int32_t)(base_id + j);
    taken |= 1ull << j;
  }
  if (wi < n_words) live_out[wi] = wb.keep | taken;

  // Makes s_live/s_mrank visible and, in the fused shape, the whole dst list
  // (all of it written by this workgroup).
  __syncthreads();

  // dense id map, coalesced over this workgroup's 65 536 ids
  const uint32_t group_first_id = first_word * 64u;
  for (uint32_t it = 0; it < 64u; ++it) {
    const uint32_t local = it * kPlanThreads + tid;
    const uint32_t id = group_first_id + local;
    if (id >= num_blocks) break;
    const uint32_t wl = local >> 6, bit = local & 63u;
    const uint64_t w = s_live[wl];
    int32_t out = -1;
    if ((w >> bit) & 1ull) {
      if (id < boundary) {
        out = (int32_t)id;
      } else if (FUSED) {
        const uint64_t movers_before = w & ~low_mask((first_word + wl) * 64u, boundary) & ((1ull << bit) - 1ull);
        out = dst[s_mrank[wl] + (uint32_t)__popcll(movers_before)];
      }
      // not fused: join_kernel fills the movers' entries
    }
    new_id[id] = out;
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
  const uint32_t groups = n_words == 0 ? 1u : (n_words + kPlanThreads - 1) / kPlanThreads;
  if (groups == 1) {
    hipLaunchKernelGGL(plan_kernel<true>, dim3(1), dim3(kPlanThreads), 0, s, live_in, n_words, nb, b,
                       plan->src, plan->dst, plan->new_id, plan->live_out, plan->state);
    return launch_rc();
  }
  hipLaunchKernelGGL(plan_kernel<false>, dim3(groups), dim3(kPlanThreads), 0, s, live_in, n_words, nb, b,
                     plan->src, plan->dst, plan->new_id, plan->live_out, plan->state);
  int rc = launch_rc();
  if (rc != KV_OK) return rc;
  uint32_t join_groups = (plan->capacity + 255u) / 256u;
  if (join_groups > 1024u) join_groups = 1024u;
  if (join_groups == 0u) join_groups = 1u;
  hipLaunchKernelGGL(join_kernel, dim3(join_groups), dim3(256), 0, s, plan->src, plan->dst, plan->new_id,
                     plan->state);
  return launch_rc();
}
