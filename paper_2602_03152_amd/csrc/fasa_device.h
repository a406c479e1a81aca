// Device-side helpers shared by the kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace fasa {

constexpr int kWave = 64;

// bf16 pair packed in one 32-bit word: element 0 in the low half, element 1 in the high half
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Order-preserving map float32 -> uint32 (larger score <=> larger key); -0 is folded onto +0 so
// that the two compare equal, as they do as floats.
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __float_as_uint(s);
  u = (u == 0x80000000u) ? 0u : u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Inclusive suffix sum over the 64 lanes of a wave: result(lane) = sum of v over lanes >= lane.
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v) {
  const int lane = lane_id();
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t x = __shfl_down(v, o, kWave);
    if (lane + o < kWave) v += x;
  }
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t v) {
  const int lane = lane_id();
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t x = __shfl_up(v, o, kWave);
    if (lane >= o) v += x;
  }
  return v;
}

// Inclusive suffix sum over a 256-thread block (thread t gets the sum over threads >= t).
// `wtot` is a 4-entry LDS scratch.  Contains two block barriers.
__device__ __forceinline__ uint32_t block256_suffix_sum(uint32_t v, uint32_t* wtot) {
  const int wave = (int)(threadIdx.x >> 6);
  uint32_t s = wave_suffix_sum(v);
  __syncthreads();  // protects wtot against a previous use
  if (lane_id() == 0) wtot[wave] = s;
  __syncthreads();
  uint32_t add = 0;
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (w > wave) add += wtot[w];
  return s + add;
}

}  // namespace fasa
