// Host-only driver for the CPU oracle, meant to be built with
// -fsanitize=address,undefined: exact-size heap buffers, so any out-of-bounds
// access or undefined shift in the oracle aborts the run.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
struct oracle_tensor { const void* host_ptr; uint64_t bytes; uint64_t dst_offset; };
int oracle_plan(const uint64_t*, uint32_t, uint32_t, int32_t*, int32_t*, int32_t*, uint64_t*, uint32_t*);
int oracle_compact(uint8_t*, uint64_t, const int32_t*, const int32_t*, uint32_t);
int64_t oracle_remap(int32_t*, uint64_t, const int32_t*, uint32_t);
int oracle_materialize(uint8_t*, uint64_t, uint64_t, const oracle_tensor*, uint32_t);
int oracle_compact_layer_major(uint8_t*, uint64_t, uint32_t, uint64_t, const int32_t*, const int32_t*, uint32_t);
int oracle_materialize_strips(uint8_t*, uint64_t, uint32_t, uint32_t, uint32_t, uint64_t, const oracle_tensor*, uint32_t);
int64_t oracle_grow(uint64_t, uint32_t, uint32_t, uint32_t, const oracle_tensor*, uint32_t, uint8_t*, uint64_t*);
int64_t oracle_grow_strips(uint64_t, uint32_t, uint32_t, uint64_t, uint32_t, uint32_t, const oracle_tensor*, uint32_t,
                           uint8_t*, uint64_t*);
int oracle_vmm_select(const uint64_t*, uint32_t, uint32_t, int32_t*);
}

static uint64_t state = 12345;
static uint64_t next() {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

int main() {
  const uint32_t sizes[][2] = {{1, 0}, {1, 1}, {2, 1}, {63, 31}, {64, 64}, {65, 64}, {300, 170}, {4096, 2048}, {4097, 1}};
  for (auto& s : sizes) {
    const uint32_t nb = s[0], b = s[1];
    const uint32_t words = (nb + 63) / 64;
    for (int pct : {0, 20, 45, 100}) {
      std::vector<uint64_t> live(words, 0), live_out(words, 0);
      for (uint32_t i = 0; i < nb; ++i)
        if ((int)(next() % 100) < pct) live[i >> 6] |= 1ull << (i & 63);
      const uint32_t cap = (nb - b < b) ? nb - b : b;
      std::vector<int32_t> src(cap ? cap : 1), dst(cap ? cap : 1), new_id(nb);
      uint32_t n = 0;
      const int rc = oracle_plan(live.data(), nb, b, src.data(), dst.data(), new_id.data(), live_out.data(), &n);
      if (rc != 0 && rc != -7) { std::printf("plan rc %d\n", rc); return 1; }
      if (rc != 0) continue;
      const uint64_t bb = 48;
      std::vector<uint8_t> pool((uint64_t)nb * bb);
      for (auto& x : pool) x = (uint8_t)next();
      if (oracle_compact(pool.data(), bb, src.data(), dst.data(), n) != 0) return 2;
      std::vector<int32_t> table;
      for (uint32_t i = 0; i < nb; ++i)
        if ((live[i >> 6] >> (i & 63)) & 1) table.push_back((int32_t)i);
      table.push_back(-1);
      if (oracle_remap(table.data(), table.size(), new_id.data(), nb) != 0) return 3;
      const uint64_t region = (uint64_t)b * bb, room = pool.size() - region;
      if (room >= 32) {
        std::vector<uint8_t> w0(16, 7), w1(room - 16, 9);
        oracle_tensor t[2] = {{w0.data(), 16, 0}, {w1.data(), room - 16, 16}};
        if (oracle_materialize(pool.data(), pool.size(), region, t, 2) != 0) return 4;
      }
      // the same plan on a layer-major pool of exact size (3 slabs, the last one unpadded), weights
      // at the start of the first strip and up to the last byte of the last one, and the reverse switch
      const uint64_t tile = 16, layers = 3, stride = (uint64_t)nb * tile + 32;
      std::vector<uint8_t> lm((layers - 1) * stride + (uint64_t)nb * tile);
      for (auto& x : lm) x = (uint8_t)next();
      if (oracle_compact_layer_major(lm.data(), tile, layers, stride, src.data(), dst.data(), n) != 0) return 5;
      const uint64_t strip = (uint64_t)(nb - b) * tile;
      if (strip >= 32) {
        std::vector<uint8_t> w0(16, 7), w1(strip - 16, 9);
        oracle_tensor t[2] = {{w0.data(), 16, 0}, {w1.data(), strip - 16, (layers - 1) * strip + 16}};
        if (oracle_materialize_strips(lm.data(), tile, layers, nb, b, stride, t, 2) != 0) return 6;
        std::vector<uint8_t> ev(2);
        std::vector<uint64_t> no(2);
        if (oracle_grow_strips(tile, layers, nb, stride, b, b + (nb - b) / 2, t, 2, ev.data(), no.data()) < 0) return 7;
        oracle_tensor flat[2] = {{nullptr, 16, 0}, {nullptr, strip - 16, 16}};
        if (oracle_grow(tile, nb, b, nb, flat, 2, ev.data(), no.data()) < 0) return 8;
      }
      // page choice of the no-move variant: every free block, and one more than there are
      uint32_t n_free = 0;
      for (uint32_t i = 0; i < nb; ++i) n_free += !((live[i >> 6] >> (i & 63)) & 1);
      std::vector<int32_t> ids(n_free ? n_free : 1);
      if (oracle_vmm_select(live.data(), nb, n_free, ids.data()) != 0) return 9;
      if (oracle_vmm_select(live.data(), nb, n_free + 1, ids.data()) != -7) return 10;
    }
  }
  std::puts("ok");
  return 0;
}
