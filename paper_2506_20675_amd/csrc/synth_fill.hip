// Device-side twin of synth.normal_bf16: fills HBM with seeded bf16 "normal" weights.
//
// Test/bench infrastructure only (input generation) — built into its own small
// library, separate from the MoE library, and containing none of the method's
// arithmetic.  Integer-only: element i = table[ 16-bit field (i % 4) of
// splitmix64_out(key + (i/4 + 1) * GOLDEN) ], so the values equal the host
// generator's bit for bit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <thread>
#include <vector>

namespace {

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// One thread produces blocks of 4 elements (one hash each); dst + 4*b is 8-byte
// aligned because dst is required to be 8-byte aligned and start % 4 == 0.
__global__ __launch_bounds__(256) void fill_kernel(uint16_t* __restrict__ dst, uint64_t key, uint64_t first_block,
                                                   uint64_t n_full_blocks, uint64_t tail,
                                                   const uint16_t* __restrict__ table) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t b = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; b < n_full_blocks; b += stride) {
    const uint64_t h = mix64(key + (first_block + b + 1) * 0x9E3779B97F4A7C15ull);
    const uint32_t v0 = table[h & 0xFFFF], v1 = table[(h >> 16) & 0xFFFF];
    const uint32_t v2 = table[(h >> 32) & 0xFFFF], v3 = table[(h >> 48) & 0xFFFF];
    uint2 o;
    o.x = v0 | (v1 << 16);
    o.y = v2 | (v3 << 16);
    *reinterpret_cast<uint2*>(dst + 4 * b) = o;
  }
  if (tail && blockIdx.x == 0 && threadIdx.x == 0) {
    const uint64_t h = mix64(key + (first_block + n_full_blocks + 1) * 0x9E3779B97F4A7C15ull);
    for (uint64_t j = 0; j < tail; ++j) dst[4 * n_full_blocks + j] = table[(h >> (16 * j)) & 0xFFFF];
  }
}

// 8-bit twin: same walk (4 elements per hash, 16-bit table index each), table of 65536 bytes.
__global__ __launch_bounds__(256) void fill_kernel_u8(uint8_t* __restrict__ dst, uint64_t key, uint64_t first_block,
                                                      uint64_t n_full_blocks, uint64_t tail,
                                                      const uint8_t* __restrict__ table) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t b = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; b < n_full_blocks; b += stride) {
    const uint64_t h = mix64(key + (first_block + b + 1) * 0x9E3779B97F4A7C15ull);
    const uint32_t v0 = table[h & 0xFFFF], v1 = table[(h >> 16) & 0xFFFF];
    const uint32_t v2 = table[(h >> 32) & 0xFFFF], v3 = table[(h >> 48) & 0xFFFF];
    *reinterpret_cast<uint32_t*>(dst + 4 * b) = v0 | (v1 << 8) | (v2 << 16) | (v3 << 24);
  }
  if (tail && blockIdx.x == 0 && threadIdx.x == 0) {
    const uint64_t h = mix64(key + (first_block + n_full_blocks + 1) * 0x9E3779B97F4A7C15ull);
    for (uint64_t j = 0; j < tail; ++j) dst[4 * n_full_blocks + j] = table[(h >> (16 * j)) & 0xFFFF];
  }
}

}  // namespace

// dst: device pointer, 8-byte aligned, `count` uint16 elements; start must be a multiple of 4.
// table: device pointer to 65536 uint16.  Returns 0 or a hipError_t value.  Asynchronous on `stream`.
extern "C" int synth_fill_bf16(void* dst, uint64_t key, uint64_t start, uint64_t count, const void* table,
                               void* stream) {
  if (!dst || !table || (start & 3) || (reinterpret_cast<uintptr_t>(dst) & 7)) return (int)hipErrorInvalidValue;
  if (count == 0) return 0;
  const uint64_t n_full = count / 4, tail = count % 4;
  uint64_t blocks = (n_full + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     static_cast<uint16_t*>(dst), key, start / 4, n_full, tail, static_cast<const uint16_t*>(table));
  return (int)hipGetLastError();
}

// Host twin (same integers, plain loops split over a few threads) for building oracle inputs quickly.
// dst, table: HOST pointers; start % 4 == 0.  Returns 0, or -1 on bad arguments.
extern "C" int synth_fill_bf16_host(uint16_t* dst, uint64_t key, uint64_t start, uint64_t count,
                                    const uint16_t* table, int n_threads) {
  if (!dst || !table || (start & 3)) return -1;
  const uint64_t first_block = start / 4, n_blocks = (count + 3) / 4;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  auto work = [=](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      const uint64_t h = mix64(key + (first_block + b + 1) * 0x9E3779B97F4A7C15ull);
      for (uint64_t j = 0; j < 4; ++j) {
        const uint64_t i = 4 * b + j;
        if (i < count) dst[i] = table[(h >> (16 * j)) & 0xFFFF];
      }
    }
  };
  std::vector<std::thread> pool;
  const uint64_t per = (n_blocks + n_threads - 1) / n_threads;
  for (int t = 0; t < n_threads; ++t) {
    const uint64_t b0 = (uint64_t)t * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    if (b0 < b1) pool.emplace_back(work, b0, b1);
  }
  for (auto& th : pool) th.join();
  return 0;
}


// 8-bit variants (FP8 code streams).  dst: device pointer, 4-byte aligned, `count` bytes; start % 4 == 0;
// table: device pointer to 65536 bytes.
extern "C" int synth_fill_u8(void* dst, uint64_t key, uint64_t start, uint64_t count, const void* table,
                             void* stream) {
  if (!dst || !table || (start & 3) || (reinterpret_cast<uintptr_t>(dst) & 3)) return (int)hipErrorInvalidValue;
  if (count == 0) return 0;
  const uint64_t n_full = count / 4, tail = count % 4;
  uint64_t blocks = (n_full + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_kernel_u8, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     static_cast<uint8_t*>(dst), key, start / 4, n_full, tail, static_cast<const uint8_t*>(table));
  return (int)hipGetLastError();
}

extern "C" int synth_fill_u8_host(uint8_t* dst, uint64_t key, uint64_t start, uint64_t count, const uint8_t* table,
                                  int n_threads) {
  if (!dst || !table || (start & 3)) return -1;
  const uint64_t first_block = start / 4, n_blocks = (count + 3) / 4;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  auto work = [=](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      const uint64_t h = mix64(key + (first_block + b + 1) * 0x9E3779B97F4A7C15ull);
      for (uint64_t j = 0; j < 4; ++j) {
        const uint64_t i = 4 * b + j;
        if (i < count) dst[i] = table[(h >> (16 * j)) & 0xFFFF];
      }
    }
  };
  std::vector<std::thread> pool;
  const uint64_t per = (n_blocks + n_threads - 1) / n_threads;
  for (int t = 0; t < n_threads; ++t) {
    const uint64_t b0 = (uint64_t)t * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    if (b0 < b1) pool.emplace_back(work, b0, b1);
  }
  for (auto& th : pool) th.join();
  return 0;
}
