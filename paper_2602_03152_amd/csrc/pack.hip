// Dominant-key cache maintenance: the FC-major packed copy Kp of the dominant K dims
// (paper Alg. 2, Split + UpdateCache of k^dom), and the per-step append of a freshly decoded
// K/V row.
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
                                                   long long sh, long long sn, PageMap pm) {
  constexpr int D = kHeadDim;
  constexpr int PITCH = D + 16 / sizeof(ET);  // keeps 16-byte alignment, staggers LDS banks
  __shared__ __align__(16) ET tile[kPackTile][PITCH];
  __shared__ int fcs[D / 2];

  const int row = blockIdx.y;
  const int b = row / Hkv, h = row % Hkv;
  const int n0 = n_begin + blockIdx.x * kPackTile;
  const int nt = min(kPackTile, n_end - n0);
  const int t = threadIdx.x;

  if (t < F) fcs[t] = fc_idx[h * F + t];

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
      const int d0 = fcs[f];
      ET* o = dst + ((long long)f * n_cap + (n0 + r)) * 2;
      o[0] = tile[r][d0];
      o[1] = tile[r][d0 + D / 2];
    }
  }
}

// grid = rows, 256 threads: writes the freshly decoded token (position n_ctx - 1) into K, V and
// the packed planes (paper Alg. 2: the new key joins the dominant cache before scoring).
template <typename ET>
__global__ __launch_bounds__(256) void append_kernel(ET* __restrict__ K, ET* __restrict__ V,
                                                     ET* __restrict__ Kp,
                                                     const int32_t* __restrict__ fc_idx,
                                                     const ET* __restrict__ k_new,
                                                     const ET* __restrict__ v_new, int Hkv, int F,
                                                     int n_cap, int n_ctx, long long sb,
                                                     long long sh, long long sn,
                                                     const int32_t* __restrict__ n_ctx_seq,
                                                     PageMap pm) {
  constexpr int D = kHeadDim;
  const int row = blockIdx.x;
  const int t = threadIdx.x;
  const int b = row / Hkv, h = row % Hkv;
  const int n = seq_n_ctx(n_ctx_seq, b, n_ctx) - 1;
  const ET* ks = k_new + (size_t)row * D;
  const ET* vs = v_new + (size_t)row * D;
  const long long ro = kv_row_offset(pm, b, n, sb, sn) + h * sh;
  if (t < D) {
    K[ro + t] = ks[t];
  } else {
    V[ro + (t - D)] = vs[t - D];
  }
  if (t < F) {
    const int d0 = fc_idx[h * F + t];
    ET* o = Kp + (((long long)row * F + t) * n_cap + n) * 2;
    o[0] = ks[d0];
    o[1] = ks[d0 + D / 2];
  }
}

hipError_t launch_pack(const fasa_shape& s, const void* K, const int32_t* fc_idx, void* Kp,
                       int n_begin, int n_end, hipStream_t st, PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid((n_end - n_begin + kPackTile - 1) / kPackTile, rows), block(256);
  if (s.dtype == FASA_BF16)
    return launch("fasa_pack", pack_kernel<uint16_t>, grid, block, st, (const uint16_t*)K, fc_idx,
                  (uint16_t*)Kp, s.n_kv_heads, s.n_fc, s.n_cap, n_begin, n_end,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, pm);
  return launch("fasa_pack", pack_kernel<float>, grid, block, st, (const float*)K, fc_idx,
                (float*)Kp, s.n_kv_heads, s.n_fc, s.n_cap, n_begin, n_end,
                (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, pm);
}

hipError_t launch_append(const fasa_shape& s, void* K, void* V, void* Kp, const int32_t* fc_idx,
                         const void* k_new, const void* v_new, hipStream_t st, RaggedLens rl,
                         PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid(rows), block(256);
  if (s.dtype == FASA_BF16)
    return launch("fasa_append", append_kernel<uint16_t>, grid, block, st, (uint16_t*)K,
                  (uint16_t*)V, (uint16_t*)Kp, fc_idx, (const uint16_t*)k_new,
                  (const uint16_t*)v_new, s.n_kv_heads, s.n_fc, s.n_cap, s.n_ctx,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n,
                  rl.n_ctx, pm);
  return launch("fasa_append", append_kernel<float>, grid, block, st, (float*)K, (float*)V,
                (float*)Kp, fc_idx, (const float*)k_new, (const float*)v_new, s.n_kv_heads, s.n_fc,
                s.n_cap, s.n_ctx, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                (long long)s.kv_stride_n, rl.n_ctx, pm);
}

}  // namespace fasa
