/* Plain C99 client of the warmkv C ABI: no Python, no C++.  Builds a small
 * pool with hipMalloc, marks every third block live, reclaims the upper half,
 * and checks on the host that every sequence still reads the same bytes
 * through its rewritten table, that all ids are below the boundary, and that
 * weights streamed into the reclaimed region arrived.  Exit code 0 = all good.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "warmkv.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_KV(x) do { int r_ = (x); if (r_ != KV_OK) { printf("warmkv error %d at line %d\n", r_, __LINE__); return 3; } } while (0)

int main(void) {
  enum { NB = 300, B = 150, LAYERS = 3, TILE = 4096, SEQS = 10, WIDTH = 10 };
  const size_t block_bytes = (size_t)LAYERS * TILE, pool_bytes = (size_t)NB * block_bytes;
  unsigned char* host_pool = (unsigned char*)malloc(pool_bytes);
  unsigned char* after = (unsigned char*)malloc(pool_bytes);
  uint64_t live[(NB + 63) / 64];
  int32_t tables[SEQS][WIDTH], before_tables[SEQS][WIDTH];
  memset(live, 0, sizeof live);
  for (size_t i = 0; i < pool_bytes; ++i) host_pool[i] = (unsigned char)((i * 2654435761u) >> 13);
  int next = 0;
  for (int s = 0; s < SEQS; ++s)
    for (int j = 0; j < WIDTH; ++j) {
      if (next < NB && j < 9) {                      /* blocks 0, 3, 6, ... are live */
        tables[s][j] = next;
        live[next / 64] |= (uint64_t)1 << (next % 64);
        next += 3;
      } else {
        tables[s][j] = -1;
      }
    }
  memcpy(before_tables, tables, sizeof tables);

  void *pool_d, *ws_d, *live_d, *tables_d, *weights_h;
  CHECK_HIP(hipMalloc(&pool_d, pool_bytes));
  CHECK_HIP(hipMalloc(&live_d, sizeof live));
  CHECK_HIP(hipMalloc(&tables_d, sizeof tables));
  const size_t ws_bytes = kv_plan_workspace_bytes(NB, B);
  if (ws_bytes == 0) return 4;
  CHECK_HIP(hipMalloc(&ws_d, ws_bytes));
  CHECK_HIP(hipMemcpy(pool_d, host_pool, pool_bytes, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(live_d, live, sizeof live, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(tables_d, tables, sizeof tables, hipMemcpyHostToDevice));
  const size_t weight_bytes = 5 * block_bytes + 128;
  CHECK_HIP(hipHostMalloc(&weights_h, weight_bytes, 0));
  memset(weights_h, 0xC3, weight_bytes);

  kv_plan plan;
  kv_pool_desc pool = {pool_d, NB, LAYERS, TILE, 0};
  hipStream_t compute, copy;
  hipEvent_t done;
  CHECK_HIP(hipStreamCreate(&compute));
  CHECK_HIP(hipStreamCreate(&copy));
  CHECK_HIP(hipEventCreateWithFlags(&done, hipEventDisableTiming));
  CHECK_KV(kv_plan_bind(&plan, ws_d, ws_bytes, NB, B));
  CHECK_KV(kv_plan_reclaim((const uint64_t*)live_d, &plan, compute));
  CHECK_KV(kv_compact(&pool, &plan, compute));
  CHECK_HIP(hipEventRecord(done, compute));
  wm_tensor w = {weights_h, weight_bytes, 256};
  CHECK_KV(weights_materialize(&pool, B, &w, 1, copy, done));
  CHECK_KV(kv_remap_tables((int32_t*)tables_d, SEQS, WIDTH, &plan, compute));
  kv_plan_state st;
  CHECK_KV(kv_plan_fetch(&plan, compute, &st));
  CHECK_HIP(hipStreamSynchronize(copy));
  if (st.status != KV_OK || st.n_bad_entries != 0) { printf("status %d bad %u\n", st.status, st.n_bad_entries); return 5; }

  CHECK_HIP(hipMemcpy(after, pool_d, pool_bytes, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(tables, tables_d, sizeof tables, hipMemcpyDeviceToHost));
  unsigned moved = 0;
  for (int s = 0; s < SEQS; ++s)
    for (int j = 0; j < WIDTH; ++j) {
      const int32_t old_id = before_tables[s][j], new_id = tables[s][j];
      if ((old_id < 0) != (new_id < 0)) return 6;
      if (old_id < 0) continue;
      if (new_id >= B) return 7;                                   /* everything below the boundary */
      if (old_id < B && new_id != old_id) return 8;                /* ids below the boundary stay   */
      moved += old_id >= B;
      if (memcmp(after + (size_t)new_id * block_bytes, host_pool + (size_t)old_id * block_bytes, block_bytes) != 0)
        return 9;                                                  /* same KV through the new table */
    }
  if (moved != st.n_moves) return 10;
  for (size_t i = 0; i < weight_bytes; ++i)
    if (after[(size_t)B * block_bytes + 256 + i] != 0xC3) return 11;
  if (kv_reserve_blocks(20480, 5120, 8, 32) != 5760) return 12;    /* Eq. 4 hand case */

  /* The same reclaim once more from the original state, through the one-call entry points: kv_reclaim on
   * the caller's workspace and kv_reclaim_static on the library's own.  Pool and tables must come out as
   * they did above (below the boundary; above it the first run also placed weights). */
  {
    void *live_out_d, *state_d;
    unsigned char* again = (unsigned char*)malloc(pool_bytes);
    int32_t tables2[SEQS][WIDTH];
    CHECK_HIP(hipMalloc(&live_out_d, sizeof live));
    CHECK_HIP(hipMalloc(&state_d, sizeof(kv_plan_state)));
    for (int variant = 0; variant < 2; ++variant) {
      CHECK_HIP(hipMemcpy(pool_d, host_pool, pool_bytes, hipMemcpyHostToDevice));
      CHECK_HIP(hipMemcpy(tables_d, before_tables, sizeof tables, hipMemcpyHostToDevice));
      kv_plan_state st2;
      if (variant == 0) {
        CHECK_KV(kv_reclaim(&pool, &plan, (const uint64_t*)live_d, (int32_t*)tables_d, SEQS, WIDTH, compute));
        CHECK_KV(kv_plan_fetch(&plan, compute, &st2));
      } else {
        CHECK_KV(kv_reclaim_static(&pool, B, (const uint64_t*)live_d, (uint64_t*)live_out_d, (int32_t*)tables_d, SEQS,
                                   WIDTH, (kv_plan_state*)state_d, compute));
        CHECK_HIP(hipStreamSynchronize(compute));
        CHECK_HIP(hipMemcpy(&st2, state_d, sizeof st2, hipMemcpyDeviceToHost));
      }
      if (st2.status != KV_OK || st2.n_moves != st.n_moves || st2.n_bad_entries != 0) return 13;
      CHECK_HIP(hipMemcpy(again, pool_d, pool_bytes, hipMemcpyDeviceToHost));
      CHECK_HIP(hipMemcpy(tables2, tables_d, sizeof tables2, hipMemcpyDeviceToHost));
      if (memcmp(tables2, tables, sizeof tables) != 0) return 14;
      if (memcmp(again, after, (size_t)B * block_bytes) != 0) return 15;
      if (memcmp(again + (size_t)B * block_bytes, host_pool + (size_t)B * block_bytes, pool_bytes - (size_t)B * block_bytes) != 0)
        return 16;                                                 /* sources keep their bytes */
    }
    free(again);
  }
  printf("c_abi_demo ok: %u blocks moved, version %s\n", st.n_moves, warmkv_version());
  return 0;
}
