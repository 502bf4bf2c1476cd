// Device-side seeded content generator for synthetic KV pools and weights.
// Same arithmetic as content.py: word w of item cid is output w+1 of a
// SplitMix64 stream seeded with mix64(seed + (cid+1)*GOLDEN); rendered either as
// 8 raw bytes or as four bf16 table look-ups.  Input generation only.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ __forceinline__ uint64_t render(uint64_t x, const uint16_t* __restrict__ table) {
  if (table == nullptr) return x;
  uint64_t r = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) r |= (uint64_t)table[(x >> (16 * i)) & 0xFFFF] << (16 * i);
  return r;
}

typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(256) void fill_kernel(u64x2* __restrict__ dst, uint64_t n_items,
                                                   uint64_t units_per_item, uint64_t seed,
                                                   const int32_t* __restrict__ cids, int64_t cid0,
                                                   const uint16_t* __restrict__ table, uint64_t word0) {
  const uint64_t total = n_items * units_per_item;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += stride) {
    const uint64_t item = u / units_per_item;
    const uint64_t w = word0 + (u - item * units_per_item) * 2;
    const int64_t cid = cids ? (int64_t)cids[item] : cid0 + (int64_t)item;
    const uint64_t base = mix64(seed + (uint64_t)(cid + 1) * kGolden);
    u64x2 v;
    v.x = render(mix64(base + (w + 1) * kGolden), table);
    v.y = render(mix64(base + (w + 2) * kGolden), table);
    dst[u] = v;
  }
}

}  // namespace

// dst, cids, table: device pointers.  item_bytes must be a multiple of 16 and
// dst 16-byte aligned.  Each item receives item_bytes of its content starting
// at 64-bit word `word0` (so a slice of a larger item can be generated alone).
// Returns 0, or a non-zero code on a bad argument or a failed launch.
extern "C" int synth_fill(void* dst, uint64_t n_items, uint64_t item_bytes, uint64_t seed,
                          const int32_t* cids, int64_t cid0, const uint16_t* table, uint64_t word0,
                          void* stream) {
  if (dst == nullptr || (item_bytes & 15) != 0 || ((uintptr_t)dst & 15) != 0) return 1;
  if (n_items == 0 || item_bytes == 0) return 0;
  const uint64_t units = item_bytes / 16;
  const uint64_t total = n_items * units;
  uint64_t blocks = (total + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (u64x2*)dst, n_items, units, seed, cids, cid0, table, word0);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Pinned host memory of an exact size for the harness (a host copy of a whole pool), and plain
// synchronous copies to and from it.  Returns nullptr / non-zero on failure.
extern "C" void* synth_host_alloc(uint64_t bytes) {
  void* p = nullptr;
  if (hipHostMalloc(&p, bytes, hipHostMallocDefault) == hipSuccess) return p;
  (void)hipGetLastError();  // a refused allocation must not be reported by the caller's next call
  return nullptr;
}

extern "C" int synth_host_free(void* p) { return hipHostFree(p) == hipSuccess ? 0 : 2; }

extern "C" int synth_copy(void* dst, const void* src, uint64_t bytes) {
  return hipMemcpy(dst, src, bytes, hipMemcpyDefault) == hipSuccess ? 0 : 2;
}

// Identifier of the source text this file was compiled from, passed in by the build.
#ifndef SYNTH_BUILD_ID
#define SYNTH_BUILD_ID "unknown"
#endif
static const char kSynthTag[] = "SYNTH_BUILD_ID=" SYNTH_BUILD_ID;
extern "C" const char* synth_build_id(void) { return kSynthTag + 15; }
