// Device twin of the counter-based input generator (see include/duo_synth.h).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "duo_synth.h"

namespace {

__device__ inline uint64_t mix64(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__global__ __launch_bounds__(256) void fill_kernel(uint16_t* dst, const uint16_t* __restrict__ table, uint64_t key,
                                                   uint64_t first_counter, int64_t count) {
  // 8 consecutive values (one 16-byte store) per thread.
  const int64_t i8 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i8 >= count) return;
  uint16_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint64_t c = first_counter + (uint64_t)(i8 + j);
    v[j] = table[mix64(key ^ (c * 0x9E3779B97F4A7C15ull)) >> 48];
  }
  uint4 w;
  w.x = v[0] | ((uint32_t)v[1] << 16); w.y = v[2] | ((uint32_t)v[3] << 16);
  w.z = v[4] | ((uint32_t)v[5] << 16); w.w = v[6] | ((uint32_t)v[7] << 16);
  *(uint4*)(dst + i8) = w;
}

}  // namespace

extern "C" int duo_synth_fill_bf16(void* dst, const uint16_t* table, uint64_t key, int64_t pos_start, int64_t n_pos,
                                   int32_t n_heads, int32_t head_dim, void* stream) {
  if (!dst || !table || n_pos < 0 || pos_start < 0 || n_heads < 1 || head_dim < 8 || head_dim % 8 != 0) return -1;
  const int64_t per_pos = (int64_t)n_heads * head_dim;
  const int64_t count = n_pos * per_pos;
  if (count == 0) return 0;
  const int64_t blocks = (count / 8 + 255) / 256;
  if (blocks > 0x7FFFFFFF) return -1;
  fill_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
      (uint16_t*)dst, table, key, (uint64_t)pos_start * (uint64_t)per_pos, count);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
