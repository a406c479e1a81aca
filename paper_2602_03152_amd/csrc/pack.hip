// Dominant-key cache maintenance: the FC-major packed copy Kp of the dominant K dims
// (paper Alg. 2, Split + UpdateCache of k^dom) for a range of cached tokens.  The per-step append
// of one freshly decoded row happens inside the scoring kernel.
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

constexpr int kPackTile = 64;  // tokens per workgroup

// One workgroup copies the dominant columns of kPackTile cached key rows.
// Rows are read whole and coalesced into LDS (the dominant dims are scattered over the row, so
// every 128-byte line of the row is touched anyway); the F planes are then written with one
// (lo, hi) pair per token, contiguous along the token axis.
template <typename ET>
__global__ __launch_bounds__(256) void pack_kernel(const ET* __restrict__ K,
                                                   const int32_t* __restrict__ fc_idx,
                                                   ET* __restrict__ Kp, int Hkv, int F, int n_cap,
                                                   int n_begin, int n_end, long long sb,
                                                   long long sh, long long sn, PageMap pm,
                                                   int pairing) {
  constexpr int D = kHeadDim;
  constexpr int PITCH = D + 16 / sizeof(ET);  // keeps 16-byte alignment, staggers LDS banks
  __shared__ __align__(16) ET tile[kPackTile][PITCH];
  __shared__ int fcs[D / 2];

  const int row = blockIdx.y;
  const int b = row / Hkv, h = row % Hkv;
  const int n0 = n_begin + blockIdx.x * kPackTile;
  const int nt = min(kPackTile, n_end - n0);
  const int t = threadIdx.x;

  if (t < F)
    fcs[t] = pair_dims(pairing, fc_idx[list_word(pairing, F, h, t, 0)], fc_idx[list_word(pairing, F, h, t, 1)]);

  constexpr int VEC = 16 / sizeof(ET);    // elements per 16-byte load
  constexpr int LPR = D / VEC;            // lanes per row
  const ET* src = K + h * sh;
  for (int i = t; i < nt * LPR; i += 256) {
    const int r = i / LPR, c = i % LPR;
    const uint4 v = *reinterpret_cast<const uint4*>(src + kv_row_offset(pm, b, n0 + r, sb, sn) + c * VEC);
    *reinterpret_cast<uint4*>(&tile[r][c * VEC]) = v;
  }
  __syncthreads();

  ET* dst = Kp + ((long long)row * F) * n_cap * 2;
  for (int i = t; i < F * kPackTile; i += 256) {
    const int f = i / kPackTile, r = i % kPackTile;
    if (r < nt) {
      const int pr = fcs[f];
      ET* o = dst + ((long long)f * n_cap + (n0 + r)) * 2;
      o[0] = tile[r][pr & 255];
      o[1] = tile[r][pr >> 8];
    }
  }
}

hipError_t launch_pack(const fasa_shape& s, const void* K, const int32_t* fc_idx, void* Kp,
                       int n_begin, int n_end, hipStream_t st, PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid((n_end - n_begin + kPackTile - 1) / kPackTile, rows), block(256);
  if (s.dtype == FASA_BF16)
    return launch("fasa_pack", pack_kernel<uint16_t>, grid, block, st, (const uint16_t*)K, fc_idx,
                  (uint16_t*)Kp, s.n_kv_heads, s.n_fc, s.n_cap, n_begin, n_end,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, pm, s.pairing);
  return launch("fasa_pack", pack_kernel<float>, grid, block, st, (const float*)K, fc_idx,
                (float*)Kp, s.n_kv_heads, s.n_fc, s.n_cap, n_begin, n_end,
                (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, pm, s.pairing);
}

}  // namespace fasa
