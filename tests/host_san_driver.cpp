// Host-only driver for the library's host arithmetic (schedules, validation,
// the reserve formula, the reverse switch, the control-plane formulas), meant
// to be linked with the library sources built with -fsanitize=address,undefined
// on the host side.  Every buffer has its exact size, so an out-of-bounds
// access or an overflowing shift in host code aborts the run.  Nothing here
// reaches a HIP call: every call either is host arithmetic by contract or is
// given arguments that are refused before the first launch.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "warmkv.h"

static uint64_t state = 2512'09472;
static uint64_t next() {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
static uint64_t below(uint64_t n) { return n ? next() % n : 0; }

#define REQUIRE(cond)                                                  \
  do {                                                                 \
    if (!(cond)) {                                                     \
      std::printf("line %d: %s\n", __LINE__, #cond);                   \
      return 1;                                                        \
    }                                                                  \
  } while (0)

static bool bit(const std::vector<uint64_t>& w, uint64_t i) { return (w[i >> 6] >> (i & 63)) & 1ull; }

int main() {
  uint8_t* const fake_dev = (uint8_t*)0x7F0000000000ull;  // never dereferenced
  std::vector<uint8_t> host_bytes(1 << 16, 7);

  // ---- workspace layout and binding
  for (uint32_t nb : {0u, 1u, 63u, 64u, 65u, 4097u, 1u << 20, 1u << 24}) {
    for (uint32_t b : {0u, nb / 3, nb}) {
      const size_t need = kv_plan_workspace_bytes(nb, b);
      REQUIRE(need % 256 == 0 && need >= 256);
      kv_plan plan;
      REQUIRE(kv_plan_bind(&plan, fake_dev, need, nb, b) == KV_OK);
      REQUIRE(kv_plan_bind(&plan, fake_dev, need - 1, nb, b) == KV_E_TOOBIG);
      REQUIRE((uint8_t*)plan.new_id + 4ull * nb <= fake_dev + need);
    }
  }
  REQUIRE(kv_plan_workspace_bytes((1u << 24) + 1, 0) == 0);

  // ---- Eq. 4 at the edges of its range
  REQUIRE(kv_reserve_blocks(0xFFFFFFFFull, 0xFFFFFFFFull, 0xFFFFFFFFu, 1) == 0xFFFFFFFFll);
  REQUIRE(kv_reserve_blocks(0xFFFFFFFFull, 0, 0xFFFFFFFFu, 0xFFFFFFFFu) == 0xFFFFFFFFll);
  REQUIRE(kv_reserve_blocks(100, 40, 3, 32) == 44);
  REQUIRE(kv_reserve_blocks(100, 101, 3, 32) == KV_E_RANGE);
  REQUIRE(kv_reserve_blocks(1ull << 32, 0, 1, 1) == KV_E_RANGE);

  // ---- schedules, front counts and the reverse switch on random pools
  for (int trial = 0; trial < 300; ++trial) {
    const uint32_t nb = 1 + (uint32_t)below(700);
    const uint32_t b = (uint32_t)below(nb + 1);
    const uint32_t layers = 1 + (uint32_t)below(4);
    const uint64_t tile = 16 * (1 + below(64));
    const uint64_t bb = layers * tile;
    const uint64_t region = (uint64_t)(nb - b) * bb;
    std::vector<uint64_t> live((nb + 63) / 64, 0);
    for (uint32_t i = 0; i < nb; ++i)
      if (below(100) < 45) live[i >> 6] |= 1ull << (i & 63);
    kv_pool_desc pool = {fake_dev, nb, layers, tile, 0};

    // disjoint extents in random order
    std::vector<wm_tensor> tensors;
    uint64_t at = below(40);
    while (at < region && tensors.size() < 12) {
      const uint64_t len = 1 + below(region - at < 5 * bb ? region - at : 5 * bb);
      tensors.push_back({host_bytes.data(), len > host_bytes.size() ? host_bytes.size() : len, at});
      at += len + below(3 * bb);
    }
    for (size_t i = tensors.size(); i > 1; --i) std::swap(tensors[i - 1], tensors[below(i)]);
    const uint32_t n = (uint32_t)tensors.size();

    uint32_t count = 0;
    std::vector<wm_piece> none;
    const uint64_t early_budget = below(8 * bb);  // 0 selects the default
    int rc = weights_materialize_schedule(&pool, b, live.data(), tensors.data(), n, early_budget, none.data(), 0, &count);
    REQUIRE(rc == (count ? KV_E_TOOBIG : KV_OK));
    std::vector<wm_piece> pieces(count);
    rc = weights_materialize_schedule(&pool, b, live.data(), tensors.data(), n, early_budget, pieces.data(), count, &count);
    REQUIRE(rc == KV_OK && count <= pieces.size());
    std::vector<uint64_t> covered(n, 0);
    bool late_seen = false;
    for (uint32_t k = 0; k < count; ++k) {
      const wm_piece& p = pieces[k];
      REQUIRE(p.tensor < n && p.bytes > 0);
      REQUIRE(p.src_offset + p.bytes <= tensors[p.tensor].bytes);
      REQUIRE(p.dst_offset == tensors[p.tensor].dst_offset + p.src_offset);
      covered[p.tensor] += p.bytes;
      if (p.early) {
        REQUIRE(!late_seen);  // early pieces come first
        for (uint64_t blk = p.dst_offset / bb; blk <= (p.dst_offset + p.bytes - 1) / bb; ++blk)
          REQUIRE(!bit(live, b + blk));  // an early piece touches only blocks that were free
      } else {
        late_seen = true;
      }
    }
    for (uint32_t i = 0; i < n; ++i) REQUIRE(covered[i] == tensors[i].bytes);

    const uint32_t front = (uint32_t)below(nb + 5);
    uint32_t want = 0;
    for (uint64_t i = b; i < nb && i < (uint64_t)b + front; ++i) want += bit(live, i);
    REQUIRE(kv_movers_in_front(live.data(), nb, b, front) == want);

    const uint32_t nb2 = b + (uint32_t)below(nb - b + 1);
    std::vector<uint8_t> evicted(n);
    std::vector<uint64_t> new_off(n);
    const int64_t lost = kv_grow(&pool, b, nb2, tensors.data(), n, evicted.data(), new_off.data());
    REQUIRE(lost >= 0);
    int64_t seen = 0;
    for (uint32_t i = 0; i < n; ++i) {
      const bool hit = tensors[i].dst_offset < (uint64_t)(nb2 - b) * bb;
      REQUIRE((evicted[i] != 0) == hit);
      if (!hit) REQUIRE(new_off[i] == tensors[i].dst_offset - (uint64_t)(nb2 - b) * bb);
      seen += hit;
    }
    REQUIRE(seen == lost);

    // the same through a layer-major description of the pool: extents inside strips
    if (nb > b) {
      const uint64_t strip = (uint64_t)(nb - b) * tile;
      kv_pool_desc lm = {fake_dev, nb, layers, tile, ((uint64_t)nb * tile + 255) / 256 * 256 + 256 * below(3)};
      std::vector<wm_tensor> ext;
      for (uint32_t l = 0; l < layers; ++l) {
        uint64_t pos = below(40);
        while (pos < strip && ext.size() < 16) {
          const uint64_t len = 1 + below(strip - pos < 5 * tile ? strip - pos : 5 * tile);
          ext.push_back({host_bytes.data(), len > host_bytes.size() ? host_bytes.size() : len, l * strip + pos});
          pos += len + below(3 * tile);
        }
      }
      for (size_t i = ext.size(); i > 1; --i) std::swap(ext[i - 1], ext[below(i)]);
      const uint32_t m = (uint32_t)ext.size();
      uint32_t cnt = 0;
      rc = weights_materialize_schedule(&lm, b, live.data(), ext.data(), m, early_budget, none.data(), 0, &cnt);
      REQUIRE(rc == (cnt ? KV_E_TOOBIG : KV_OK));
      std::vector<wm_piece> ps(cnt);
      rc = weights_materialize_schedule(&lm, b, live.data(), ext.data(), m, early_budget, ps.data(), cnt, &cnt);
      REQUIRE(rc == KV_OK);
      std::vector<uint64_t> cov(m, 0);
      for (uint32_t k = 0; k < cnt; ++k) {
        const wm_piece& p = ps[k];
        REQUIRE(p.tensor < m && p.bytes > 0 && p.dst_offset == ext[p.tensor].dst_offset + p.src_offset);
        cov[p.tensor] += p.bytes;
        if (p.early)
          for (uint64_t t = (p.dst_offset % strip) / tile; t <= ((p.dst_offset + p.bytes - 1) % strip) / tile; ++t)
            REQUIRE(!bit(live, b + t));  // only tiles of blocks that were free
      }
      for (uint32_t i = 0; i < m; ++i) REQUIRE(cov[i] == ext[i].bytes);
      std::vector<uint8_t> ev(m);
      std::vector<uint64_t> no(m);
      const int64_t gone = kv_grow(&lm, b, nb2, ext.data(), m, ev.data(), no.data());
      REQUIRE(gone >= 0);
      const uint64_t back = (uint64_t)(nb2 - b) * tile, new_strip = (uint64_t)(nb - nb2) * tile;
      for (uint32_t i = 0; i < m; ++i) {
        const uint64_t l = ext[i].dst_offset / strip, within = ext[i].dst_offset % strip;
        REQUIRE((ev[i] != 0) == (within < back));
        if (within >= back) REQUIRE(no[i] == l * new_strip + within - back);
      }
      wm_tensor across = {host_bytes.data(), 2, strip - 1};
      if (layers > 1) REQUIRE(weights_materialize(&lm, b, &across, 1, nullptr, nullptr) == KV_E_TOOBIG);
    }

    // refused before any launch: an extent one byte too long, two that overlap
    if (n >= 1) {
      std::vector<wm_tensor> bad = tensors;
      bad[0].dst_offset = region;
      bad[0].bytes = 1;
      REQUIRE(weights_materialize(&pool, b, bad.data(), n, nullptr, nullptr) == KV_E_TOOBIG);
      REQUIRE(weights_materialize_front(&pool, b, bb, bad.data(), n, nullptr, nullptr, nullptr) == KV_E_TOOBIG);
      kv_plan plan;
      REQUIRE(kv_plan_bind(&plan, fake_dev + (1ull << 30), kv_plan_workspace_bytes(nb, b), nb, b) == KV_OK);
      kv_switch_request rq = {};
      rq.pool = &pool;
      rq.plan = &plan;
      rq.live_in = (const uint64_t*)(fake_dev + (2ull << 30));
      rq.tensors = bad.data();
      rq.n_tensors = n;
      rq.compaction_done = fake_dev;
      REQUIRE(kv_switch(&rq, nullptr) == KV_E_TOOBIG);
    }
    if (n >= 2) {
      std::vector<wm_tensor> bad = tensors;
      bad[1].dst_offset = bad[0].dst_offset + bad[0].bytes - 1;
      bad[1].bytes = 1;
      REQUIRE(weights_materialize(&pool, b, bad.data(), n, nullptr, nullptr) == KV_E_OVERLAP);
    }
  }

  // ---- control-plane formulas on exact-size arrays
  for (int trial = 0; trial < 50; ++trial) {
    const uint32_t D = 1 + (uint32_t)below(7), N = (uint32_t)below(12);
    const uint32_t n_windows = 1 + (uint32_t)below(30), n_days = D + 1 + (uint32_t)below(3);
    std::vector<double> hist((size_t)n_days * n_windows);
    for (double& h : hist) h = (double)below(1000) / 7.0;
    double pred = 0;
    REQUIRE(ws_predict_load(hist.data(), n_days, n_windows, n_days - 1, (uint32_t)below(n_windows), D, N, &pred) == KV_OK);
    REQUIRE(pred == pred);  // not NaN
    REQUIRE(ws_predict_load(hist.data(), n_days, n_windows, D - 1, 0, D, N, &pred) == KV_E_RANGE);

    ws_model m = {};
    m.size_bytes = 1e9 * (1 + below(60));
    m.load_avg = (double)below(200);
    m.load_peak = m.load_avg + (double)below(200);
    m.cold_latency = 1.0 + (double)below(30);
    m.degree = 1u << below(4);
    m.batch = 1 + (uint32_t)below(64);
    m.active = (uint32_t)below(4);
    uint32_t nbasic = 0, nburst = 0;
    int rc = ws_replica_scores(&m, &nbasic, &nburst, nullptr, 0);
    REQUIRE(rc == KV_OK || rc == KV_E_TOOBIG);
    std::vector<double> scores(nbasic + nburst);
    REQUIRE(ws_replica_scores(&m, &nbasic, &nburst, scores.data(), (uint32_t)scores.size()) == KV_OK);

    const uint32_t gpus_per_server = 8, n_gpus = 8 * (1 + (uint32_t)below(3));
    std::vector<double> free_bytes(n_gpus, 192e9);
    std::vector<ws_model> models(1 + below(4), m);
    for (ws_model& x : models) x.load_peak = x.load_avg + (double)below(300);
    uint32_t placed = 0;
    std::vector<ws_placement> out(4096);
    rc = ws_place_replicas(models.data(), (uint32_t)models.size(), free_bytes.data(), n_gpus, gpus_per_server, out.data(),
                           (uint32_t)out.size(), &placed);
    REQUIRE(rc == KV_OK && placed <= out.size());
    for (uint32_t i = 0; i < placed; ++i) REQUIRE(out[i].first_gpu + models[out[i].model].degree <= n_gpus);
  }
  std::printf("ok\n");
  return 0;
}
