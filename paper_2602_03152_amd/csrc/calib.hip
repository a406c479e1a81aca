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

// grid = rows (real KV heads), 256 threads.  CA_sum[row][i] += |T_full[row] & T_v[row][i]| / kk.
__global__ __launch_bounds__(256) void calib_intersect_kernel(const int32_t* __restrict__ T_full,
                                                              const int32_t* __restrict__ T_v,
                                                              float* __restrict__ CA_sum, int half,
                                                              int kk, int n_ctx) {
  __shared__ uint32_t bits[kCalibMaxCtx / 32];
  __shared__ uint32_t cnt;
  const int row = blockIdx.x;
  const int t = threadIdx.x;
  const int words = (n_ctx + 31) / 32;
  for (int w = t; w < words; w += 256) bits[w] = 0;
  __syncthreads();
  for (int j = t; j < kk; j += 256) {
    const int tok = T_full[(size_t)row * kk + j];
    if (tok >= 0 && tok < n_ctx) atomicOr(&bits[tok >> 5], 1u << (tok & 31));
  }
  __syncthreads();
  for (int i = 0; i < half; ++i) {
    if (t == 0) cnt = 0;
    __syncthreads();
    uint32_t mine = 0;
    const int32_t* tv = T_v + ((size_t)row * half + i) * kk;
    for (int j = t; j < kk; j += 256) {
      const int tok = tv[j];
      if (tok >= 0 && tok < n_ctx) mine += (bits[tok >> 5] >> (tok & 31)) & 1u;
    }
    mine = wave_prefix_sum(mine);
    if (lane_id() == kWave - 1) atomicAdd(&cnt, mine);
    __syncthreads();
    if (t == 0) CA_sum[(size_t)row * half + i] += (float)cnt / (float)kk;
    __syncthreads();
  }
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
  return launch("fasa_calib_intersect", calib_intersect_kernel, dim3(s.batch * s.n_kv_heads), dim3(256),
                st, T_full, T_v, CA_sum, s.head_dim / 2, kk, s.n_ctx);
}

int calib_max_ctx() { return kCalibMaxCtx; }

}  // namespace fasa
