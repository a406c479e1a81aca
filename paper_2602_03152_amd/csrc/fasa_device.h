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

// ---------------------------------------------------------------------------------------------
// Adaptive histogram bins of the fused step.  The scoring kernel predicts where a row's B-th largest
// score will lie - mu = location + z(B/N) * scale, from a robust location and scale of a small fixed
// sample of the row's scores and the normal quantile z - and counts every score in one of kLinBins
// bins whose resolution is highest around that prediction; the selection reads (mu, inv = 1 / scale)
// back and classifies with the same function, so both sides agree bit for bit.  The map is monotone
// in s whatever mu and inv are: a poor prediction costs resolution (more candidates to resolve
// exactly), never correctness.  With u = (s - mu) * inv, in units of the scale:
//   |u| <= 0.75        128 bins per unit          (the threshold bin then holds N * pdf / 128 tokens)
//   0.75 < |u| <= 2     32 bins per unit
//   2 < |u| <= 8         4 bins per unit
//   |u| > 8              8 bins per octave of |u|, at most 200 more
// Few scores fall where the bins are fine, so a workgroup's 1024 scores touch only ~100 distinct bins
// (every distinct bin is one global atomic when the workgroup's histogram is flushed).
// ---------------------------------------------------------------------------------------------
constexpr int kLinBins = 1024;
__device__ __forceinline__ uint32_t lin_bin(float s, float mu, float inv) {
#pragma clang fp contract(off)
  const float u = (s - mu) * inv;
  const float a = fabsf(u);
  // every term is non-decreasing in a, and so is their rounded sum
  const float tail = (float)min((__float_as_uint(fmaxf(a, 8.0f)) - 0x41000000u) >> 20, 200u);
  const float g = 128.0f * fminf(a, 0.75f) + 32.0f * (fminf(fmaxf(a, 0.75f), 2.0f) - 0.75f) +
                  4.0f * (fminf(fmaxf(a, 2.0f), 8.0f) - 2.0f) + tail;          // 0 .. 360
  return (uint32_t)(512 + (int)floorf(copysignf(g, u)));
}
// z with P(Z > z) = p for a standard normal Z (rational approximation, |error| < 5e-3: it only has to
// place the fine bins)
__device__ __forceinline__ float normal_upper_quantile(float p) {
  const bool flip = p > 0.5f;
  const float pp = fmaxf(flip ? 1.0f - p : p, 1e-30f);
  const float t = sqrtf(-2.0f * __logf(pp));
  const float z = t - (2.30753f + 0.27061f * t) / (1.0f + t * (0.99229f + 0.04481f * t));
  return flip ? -z : z;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// DPP move of a 32-bit value; lanes without a source keep 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes of a wave, entirely on the vector ALU: Hillis-Steele
// inside each row of 16 lanes (row_shr 1, 2, 4, 8), then the last lane of row 0/2 is added to row
// 1/3 (row_bcast15) and the last lane of the lower half to the upper half (row_bcast31).
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t v) {
  v += dpp_u32<0x111, 0xF>(v);
  v += dpp_u32<0x112, 0xF>(v);
  v += dpp_u32<0x114, 0xF>(v);
  v += dpp_u32<0x118, 0xF>(v);
  v += dpp_u32<0x142, 0xA>(v);
  v += dpp_u32<0x143, 0xC>(v);
  return v;
}

// Inclusive suffix sum over the 64 lanes of a wave: result(lane) = sum of v over lanes >= lane.
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v) {
  const uint32_t incl = wave_prefix_sum(v);
  const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
  return total - incl + v;
}

// Inclusive suffix sum over a block of NT threads (thread t gets the sum over threads >= t).
// `wtot` is an LDS scratch of NT / 64 entries.  Contains two block barriers.
template <int NT>
__device__ __forceinline__ uint32_t block_suffix_sum(uint32_t v, uint32_t* wtot) {
  constexpr int NW = NT / kWave;
  const int wave = (int)(threadIdx.x >> 6);
  uint32_t s = wave_suffix_sum(v);
  __syncthreads();  // protects wtot against a previous use
  if (lane_id() == 0) wtot[wave] = s;
  __syncthreads();
  uint32_t add = 0;
#pragma unroll
  for (int w = 1; w < NW; ++w)
    if (w > wave) add += wtot[w];
  return s + add;
}
__device__ __forceinline__ uint32_t block256_suffix_sum(uint32_t v, uint32_t* wtot) {
  return block_suffix_sum<256>(v, wtot);
}

// Exclusive prefix sum over a block of NT threads; `total` gets the block sum.
// `wtot` is an LDS scratch of NT / 64 entries.  Contains two block barriers.
template <int NT>
__device__ __forceinline__ uint32_t block_prefix_sum(uint32_t v, uint32_t* wtot, uint32_t& total) {
  constexpr int NW = NT / kWave;
  const int wave = (int)(threadIdx.x >> 6);
  const uint32_t incl = wave_prefix_sum(v);
  __syncthreads();
  if (lane_id() == kWave - 1) wtot[wave] = incl;
  __syncthreads();
  uint32_t before = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wave) before += wtot[w];
    total += wtot[w];
  }
  return before + incl - v;
}

// Exclusive prefix over a 256-thread block of two counters at once; also returns the block totals.
// `ws` is an 8-entry LDS scratch.  Contains two block barriers.
__device__ __forceinline__ void block256_prefix2(uint32_t a, uint32_t b, uint32_t* ws, uint32_t& pa,
                                                 uint32_t& pb, uint32_t& ta, uint32_t& tb) {
  const int wave = (int)(threadIdx.x >> 6);
  const uint32_t ia = wave_prefix_sum(a), ib = wave_prefix_sum(b);
  __syncthreads();
  if (lane_id() == kWave - 1) { ws[wave] = ia; ws[4 + wave] = ib; }
  __syncthreads();
  uint32_t oa = 0, ob = 0;
  ta = 0; tb = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w < wave) { oa += ws[w]; ob += ws[4 + w]; }
    ta += ws[w]; tb += ws[4 + w];
  }
  pa = oa + ia - a;
  pb = ob + ib - b;
}

// Maps the linear workgroup id of a 1-D grid of rows * nslices workgroups to (row, slice).
// Workgroups are handed to the 8 XCDs round-robin, so when the row count is a multiple of 8 the
// mapping keeps every workgroup of a row on one XCD: the row's counters, histogram and score
// slice then live in that XCD's L2 and its atomics do not bounce between dies.
__device__ __forceinline__ void row_slice_of_block(int rows, int nslices, int& row, int& slice) {
  const unsigned id = blockIdx.x;
  if ((rows & 7) == 0) {
    const unsigned xcd = id & 7u, k = id >> 3;
    slice = (int)(k % (unsigned)nslices);
    row = (int)(k / (unsigned)nslices) * 8 + (int)xcd;
  } else {
    row = (int)(id / (unsigned)nslices);
    slice = (int)(id % (unsigned)nslices);
  }
}

// ---------------------------------------------------------------------------------------------
// Publishing small results to another workgroup of the same kernel without a device-scope fence.
// A release fence at agent scope writes back the whole L2 of the XCD (hundreds of ns, serialised
// per die), far too much for kernels of a few microseconds.  Instead the producer writes the
// shared words with agent-scope (write-through) stores, waits until they are acknowledged, and
// only then bumps a ticket; the consumer reads the words with agent-scope loads, which are served
// from the coherence point and never from a stale line.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int32_t* p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint2* p, uint2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                     ((unsigned long long)v.y << 32) | v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint2 ld_agent(const uint2* p) {
  const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void st_agent(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                     ((unsigned long long)__float_as_uint(v.y) << 32) | __float_as_uint(v.x),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent(const float2* p) {
  const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}
// All of this workgroup's earlier stores are acknowledged; then a block barrier.  After it one
// thread may bump the ticket that tells another workgroup the data is there.
__device__ __forceinline__ void publish_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);   // vmcnt = expcnt = lgkmcnt = 0
  __syncthreads();
}

// per-sequence length and budget (see RaggedLens): clamped into [1, upper bound]
__device__ __forceinline__ int seq_n_ctx(const int32_t* n_ctx, int b, int upper) {
  return n_ctx ? min(max(n_ctx[b], 1), upper) : upper;
}
__device__ __forceinline__ int seq_bsel(const int32_t* budget, int b, int n, int upper_budget) {
  const int bud = budget ? min(max(budget[b], 1), upper_budget) : upper_budget;
  return min(bud, n);
}

// DPP lane exchanges inside a row of 16 lanes (no LDS traffic)
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a DPP row; every lane of the row gets the same bits
__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_mov<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);  // row_half_mirror
  x += dpp_mov<0x140>(x);  // row_mirror
  return x;
}

// max over the 16 lanes of a DPP row
__device__ __forceinline__ float row16_max(float x) {
  x = fmaxf(x, dpp_mov<0xB1>(x));
  x = fmaxf(x, dpp_mov<0x4E>(x));
  x = fmaxf(x, dpp_mov<0x141>(x));
  x = fmaxf(x, dpp_mov<0x140>(x));
  return x;
}

// Lane exchanges between the four rows of a wave with the gfx950 permlane swaps (vector ALU, no
// LDS): both results of a swap of x with itself are the two partners of a butterfly step.
//   v_permlane16_swap: odd rows of the first operand <-> even rows of the second
//   v_permlane32_swap: upper half of the first operand <-> lower half of the second
__device__ __forceinline__ float xor16_sum(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor32_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor16_max(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// reductions over all 64 lanes; every lane gets the result
__device__ __forceinline__ float wave_sum(float x) { return xor32_sum(xor16_sum(row16_sum(x))); }
__device__ __forceinline__ float wave_max(float x) { return xor32_max(xor16_max(row16_max(x))); }

}  // namespace fasa
