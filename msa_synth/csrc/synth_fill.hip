// Device twin of msa_synth.normal_bf16_bits: fills a bf16 buffer in place with the seeded
// standard-normal stream, bit-identical to the host generator.  Input generation only -- no
// arithmetic of the method lives here.
//   word(e)  = splitmix64_finalize(seed * 0x9E3779B97F4A7C15 + (e >> 2))
//   value(e) = table[(word(e) >> (16 * (e & 3))) & 0xFFFF]
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

// One thread per group of four consecutive elements; start must be a multiple of 4.
__global__ __launch_bounds__(256) void synth_fill_kernel(const uint16_t* __restrict__ table,
                                                         uint16_t* __restrict__ out, uint64_t seed_mul,
                                                         uint64_t start, uint64_t count) {
  const uint64_t n_words = (count + 3) >> 2;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t w = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; w < n_words; w += stride) {
    const uint64_t word = mix64(seed_mul + (start >> 2) + w);
    const uint16_t v0 = table[word & 0xFFFF];
    const uint16_t v1 = table[(word >> 16) & 0xFFFF];
    const uint16_t v2 = table[(word >> 32) & 0xFFFF];
    const uint16_t v3 = table[(word >> 48) & 0xFFFF];
    const uint64_t e = w << 2;
    if (e + 4 <= count) {
      uint2 pk;
      pk.x = (uint32_t)v0 | ((uint32_t)v1 << 16);
      pk.y = (uint32_t)v2 | ((uint32_t)v3 << 16);
      *reinterpret_cast<uint2*>(out + e) = pk;
    } else {
      if (e + 0 < count) out[e + 0] = v0;
      if (e + 1 < count) out[e + 1] = v1;
      if (e + 2 < count) out[e + 2] = v2;
    }
  }
}

extern "C" int msa_synth_fill_bf16(const void* table_dev, void* out_dev, uint64_t seed, uint64_t start,
                                   uint64_t count, void* stream) {
  if (table_dev == nullptr || out_dev == nullptr) return -1;
  if ((start & 3) != 0 || (reinterpret_cast<uintptr_t>(out_dev) & 7) != 0) return -1;
  if (count == 0) return 0;
  const uint64_t n_words = (count + 3) >> 2;
  uint64_t blocks = (n_words + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (const uint16_t*)table_dev, (uint16_t*)out_dev, seed * 0x9E3779B97F4A7C15ull,
                     start, count);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
