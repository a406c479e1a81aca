// Offline calibration (paper Sec. 3.3 eq. ca_k and Alg. 1): contextual agreement of every single
// frequency chunk with the full head, computed on the device with the same scoring and selection
// kernels as the decode step.  Trick: the FC-major packed copy of ALL d/2 FCs,
// Kp_all[b][h][i][n][2], is bit for bit the packed copy of a "virtual" cache with Hkv * d/2 KV
// heads and one FC each, so single-FC scoring of all FCs is ONE call of the ordinary scoring
// kernel on that virtual shape (with the group's queries replicated per virtual head), and the d/2
// top-K problems per head are one call of the ordinary selection kernel.
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

constexpr int kCalibMaxCtx = 262144;   // bitmap of the full-head top-K set lives in LDS (32 KB)

// grid = batch * Hkv * half workgroups of 128 threads: virtual KV head (h, i) gets the G query heads
// of real KV head h; plus the two index lists.
template <typename ET>
__global__ __launch_bounds__(128) void calib_prepare_kernel(const ET* __restrict__ q,
                                                            ET* __restrict__ q_v,
                                                            int32_t* __restrict__ fc_all,
                                                            int32_t* __restrict__ fc_v, int Hq,
                                                            int Hkv, int half) {
  constexpr int D = kHeadDim;
  const int G = Hq / Hkv;
  const int vb = blockIdx.x;                     // b * Hkv * half + h * half + i
  const int i = vb % half, h = (vb / half) % Hkv, b = vb / (half * Hkv);
  const int t = threadIdx.x;
  for (int g = 0; g < G; ++g)
    q_v[(((size_t)b * Hkv * half + (size_t)h * half + i) * G + g) * D + t] =
        q[((size_t)b * Hq + (size_t)h * G + g) * D + t];
  if (b == 0 && t == 0) {
    fc_all[h * half + i] = i;
    fc_v[h * half + i] = i;
  }
}

constexpr int kCalibFcPerWg = 4;   // FCs counted by one workgroup (each workgroup rebuilds the row's bitmap)

// grid = rows * ceil(half / kCalibFcPerWg) workgroups of 256 threads.
// CA_sum[row][i] += |T_full[row] & T_v[row][i]| / kk for the workgroup's FCs i.  The index lists are
// read 8 entries per thread at a time, all 8 loads issued before the first is used.
__global__ __launch_bounds__(256) void calib_intersect_kernel(const int32_t* __restrict__ T_full,
                                                              const int32_t* __restrict__ T_v,
                                                              float* __restrict__ CA_sum, int half,
                                                              int groups, int kk, int n_ctx) {
  __shared__ uint32_t bits[kCalibMaxCtx / 32];
  __shared__ uint32_t cnt[kCalibFcPerWg];
  const int row = blockIdx.x / groups;
  const int i0 = (blockIdx.x % groups) * kCalibFcPerWg;
  const int t = threadIdx.x;
  const int words = (n_ctx + 31) / 32;
  for (int w = t; w < words; w += 256) bits[w] = 0;
  if (t < kCalibFcPerWg) cnt[t] = 0;
  __syncthreads();
  const int32_t* tf = T_full + (size_t)row * kk;
  for (int j0 = 0; j0 < kk; j0 += 8 * 256) {
    int tok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) tok[u] = tf[min(j0 + u * 256 + t, kk - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (j0 + u * 256 + t < kk && tok[u] >= 0 && tok[u] < n_ctx) atomicOr(&bits[tok[u] >> 5], 1u << (tok[u] & 31));
  }
  __syncthreads();
  for (int f = 0; f < kCalibFcPerWg; ++f) {
    const int i = i0 + f;
    if (i >= half) break;
    const int32_t* tv = T_v + ((size_t)row * half + i) * kk;
    uint32_t mine = 0;
    for (int j0 = 0; j0 < kk; j0 += 8 * 256) {
      int tok[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) tok[u] = tv[min(j0 + u * 256 + t, kk - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = min(max(tok[u], 0), n_ctx - 1);
        const uint32_t bit = (bits[c >> 5] >> (c & 31)) & 1u;
        mine += (j0 + u * 256 + t < kk && tok[u] == c) ? bit : 0u;
      }
    }
    mine = wave_prefix_sum(mine);
    if (lane_id() == kWave - 1) atomicAdd(&cnt[f], mine);
  }
  __syncthreads();
  if (t < kCalibFcPerWg && i0 + t < half) CA_sum[(size_t)row * half + i0 + t] += (float)cnt[t] / (float)kk;
}

hipError_t launch_calib_prepare(const fasa_shape& s, const void* q, void* q_v, int32_t* fc_all,
                                int32_t* fc_v, hipStream_t st) {
  const int half = s.head_dim / 2;
  dim3 grid(s.batch * s.n_kv_heads * half), block(128);
  if (s.dtype == FASA_BF16)
    return launch("fasa_calib_prepare", calib_prepare_kernel<uint16_t>, grid, block, st,
                  (const uint16_t*)q, (uint16_t*)q_v, fc_all, fc_v, s.n_q_heads, s.n_kv_heads, half);
  return launch("fasa_calib_prepare", calib_prepare_kernel<float>, grid, block, st, (const float*)q,
                (float*)q_v, fc_all, fc_v, s.n_q_heads, s.n_kv_heads, half);
}

hipError_t launch_calib_intersect(const fasa_shape& s, const int32_t* T_full, const int32_t* T_v,
                                  float* CA_sum, int kk, hipStream_t st) {
  const int half = s.head_dim / 2;
  const int groups = (half + kCalibFcPerWg - 1) / kCalibFcPerWg;
  return launch("fasa_calib_intersect", calib_intersect_kernel, dim3(s.batch * s.n_kv_heads * groups),
                dim3(256), st, T_full, T_v, CA_sum, half, groups, kk, s.n_ctx);
}

int calib_max_ctx() { return kCalibMaxCtx; }

}  // namespace fasa
