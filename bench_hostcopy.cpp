// Bench-only host baseline: the same move list copied by several threads
// (static split of the list).  Not the oracle and not part of the library: it
// only answers "what can this box's host memory do on the same job".
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

extern "C" void hostcopy_moves(uint8_t* pool, uint64_t block_bytes, const int32_t* src, const int32_t* dst,
                               uint32_t n_moves, uint32_t n_threads) {
  if (n_threads == 0) n_threads = 1;
  std::vector<std::thread> workers;
  for (uint32_t t = 0; t < n_threads; ++t) {
    const uint32_t k0 = (uint32_t)((uint64_t)n_moves * t / n_threads);
    const uint32_t k1 = (uint32_t)((uint64_t)n_moves * (t + 1) / n_threads);
    workers.emplace_back([=] {
      for (uint32_t k = k0; k < k1; ++k)
        std::memcpy(pool + (uint64_t)dst[k] * block_bytes, pool + (uint64_t)src[k] * block_bytes, block_bytes);
    });
  }
  for (auto& w : workers) w.join();
}
