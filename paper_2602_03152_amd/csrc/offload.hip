// Memory-optimised variant (paper Sec. 4.3 and Alg. 2, "FASA-M"): only the dominant key dims (the
// FC-major copy Kp) stay in HBM; the non-dominant key dims and all values live in pinned host
// memory that the GPU can address.  Per step the B selected rows are fetched over PCIe by the GPU
// itself (zero-copy reads, no host-side gather), the full key rows are rebuilt from the two parts
// (Alg. 2: SelectTokens + TransferToGPU + Combine) into a compact staging buffer, and the usual
// attention kernel runs over that buffer.
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

constexpr int kOffTile = 64;   // tokens per workgroup of the split kernel

// Where output dim j of a rebuilt key row comes from: bit 15 set -> dominant pair entry
// (f * 2 + which), else index into the row's non-dominant part.
__device__ __forceinline__ void build_dim_map(const int32_t* __restrict__ fc_idx_h, int F, int pairing,
                                              uint16_t* src /*[D]*/, uint8_t* is_dom /*[D]*/) {
  constexpr int D = kHeadDim;
  const int t = threadIdx.x;
  if (t < D) is_dom[t] = 0;
  __syncthreads();
  if (t < F) {
    const int pr = pair_dims(pairing, fc_idx_h[t], 0);   // FC numbers only (rotate-half or interleaved)
    const int lo = pr & 255, hi = pr >> 8;
    is_dom[lo] = 1;
    is_dom[hi] = 1;
    src[lo] = (uint16_t)(0x8000u | (uint32_t)(2 * t));
    src[hi] = (uint16_t)(0x8000u | (uint32_t)(2 * t + 1));
  }
  __syncthreads();
  if (t < D && !is_dom[t]) {
    int pos = 0;
    for (int j = 0; j < t; ++j) pos += is_dom[j] ? 0 : 1;
    src[t] = (uint16_t)pos;
  }
  __syncthreads();
}

// grid = (ceil(tokens / kOffTile), rows): dominant dims -> Kp planes (HBM), the rest -> host rows
template <typename ET>
__global__ __launch_bounds__(256) void offload_split_kernel(const ET* __restrict__ K,
                                                            const int32_t* __restrict__ fc_idx,
                                                            ET* __restrict__ Kp,
                                                            ET* __restrict__ Knd, int Hkv, int F,
                                                            int n_cap, int n_begin, int n_end,
                                                            long long sb, long long sh, long long sn,
                                                            int pairing) {
  constexpr int D = kHeadDim;
  constexpr int PITCH = D + 16 / sizeof(ET);
  __shared__ __align__(16) ET tile[kOffTile][PITCH];
  __shared__ uint16_t src[D];
  __shared__ uint8_t is_dom[D];
  const int row = blockIdx.y;
  const int b = row / Hkv, h = row % Hkv;
  const int n0 = n_begin + blockIdx.x * kOffTile;
  const int nt = min(kOffTile, n_end - n0);
  const int t = threadIdx.x;
  build_dim_map(fc_idx + h * F, F, pairing, src, is_dom);

  constexpr int VEC = 16 / sizeof(ET);
  constexpr int LPR = D / VEC;
  const ET* ksrc = K + b * sb + h * sh;
  for (int i = t; i < nt * LPR; i += 256) {
    const int r = i / LPR, c = i % LPR;
    *reinterpret_cast<uint4*>(&tile[r][c * VEC]) =
        *reinterpret_cast<const uint4*>(ksrc + (long long)(n0 + r) * sn + c * VEC);
  }
  __syncthreads();
  const int nd = D - 2 * F;
  ET* kp = Kp + ((long long)row * F) * n_cap * 2;
  ET* knd = Knd + (long long)row * n_cap * nd;
  // every dim of every token goes to exactly one of the two destinations
  for (int i = t; i < nt * D; i += 256) {
    const int r = i / D, dim = i % D;
    const uint32_t s = src[dim];
    const ET v = tile[r][dim];
    if (s & 0x8000u) {
      const int f = (int)(s & 0x7FFFu) >> 1, which = (int)(s & 1u);
      kp[((long long)f * n_cap + (n0 + r)) * 2 + which] = v;
    } else {
      knd[(long long)(n0 + r) * nd + s] = v;
    }
  }
}

// grid = rows: the freshly decoded token (position n_ctx - 1) is split the same way; its value row
// goes to the host value cache.
template <typename ET>
__global__ __launch_bounds__(256) void offload_append_kernel(ET* __restrict__ Kp, ET* __restrict__ Knd,
                                                             ET* __restrict__ Vh,
                                                             const int32_t* __restrict__ fc_idx,
                                                             const ET* __restrict__ k_new,
                                                             const ET* __restrict__ v_new, int Hkv,
                                                             int F, int n_cap, int n_ctx, long long sb,
                                                             long long sh, long long sn, int pairing) {
  constexpr int D = kHeadDim;
  __shared__ uint16_t src[D];
  __shared__ uint8_t is_dom[D];
  const int row = blockIdx.x;
  const int b = row / Hkv, h = row % Hkv;
  const int t = threadIdx.x;
  const int n = n_ctx - 1;
  build_dim_map(fc_idx + h * F, F, pairing, src, is_dom);
  const int nd = D - 2 * F;
  if (t < D) {
    const ET v = k_new[(size_t)row * D + t];
    const uint32_t s = src[t];
    if (s & 0x8000u) {
      const int f = (int)(s & 0x7FFFu) >> 1, which = (int)(s & 1u);
      Kp[(((long long)row * F + f) * n_cap + n) * 2 + which] = v;
    } else {
      Knd[((long long)row * n_cap + n) * nd + s] = v;
    }
  } else {
    Vh[b * sb + h * sh + (long long)n * sn + (t - D)] = v_new[(size_t)row * D + (t - D)];
  }
}

// grid = (ceil(count / TOK), rows), TOK = 256 / (D / VEC) tokens per workgroup.
// Reads the selected tokens' non-dominant key part and value row from host memory, their dominant
// pairs from Kp, and writes full rows KT[row][j][:], VT[row][j][:] (j = position in the index list).
template <typename ET>
__global__ __launch_bounds__(256) void offload_gather_kernel(const ET* __restrict__ Kp,
                                                             const ET* __restrict__ Knd,
                                                             const ET* __restrict__ Vh,
                                                             const int32_t* __restrict__ fc_idx,
                                                             const int32_t* __restrict__ T,
                                                             ET* __restrict__ KT, ET* __restrict__ VT,
                                                             int Hkv, int F, int n_cap, int n_ctx,
                                                             int count, long long sb, long long sh,
                                                             long long sn, int pairing) {
  constexpr int D = kHeadDim;
  constexpr int VEC = 16 / sizeof(ET);
  constexpr int LPR = D / VEC;
  constexpr int TOK = 256 / LPR;
  __shared__ uint16_t src[D];
  __shared__ uint8_t is_dom[D];
  __shared__ int toks[TOK];
  __shared__ ET l_nd[TOK][D];
  __shared__ ET l_dom[TOK][D];
  const int row = blockIdx.y;
  const int b = row / Hkv, h = row % Hkv;
  const int j0 = blockIdx.x * TOK;
  const int nt = min(TOK, count - j0);
  const int t = threadIdx.x;
  if (t < nt) toks[t] = min(max(T[(size_t)row * count + j0 + t], 0), n_ctx - 1);
  build_dim_map(fc_idx + h * F, F, pairing, src, is_dom);   // contains barriers: toks is visible after it

  const int nd = D - 2 * F;
  const ET* knd = Knd + (long long)row * n_cap * nd;
  for (int i = t; i < nt * nd; i += 256) {
    const int s = i / nd, j = i % nd;
    l_nd[s][j] = knd[(long long)toks[s] * nd + j];                       // host memory, coalesced per row
  }
  const ET* kp = Kp + ((long long)row * F) * n_cap * 2;
  for (int i = t; i < nt * 2 * F; i += 256) {
    const int s = i / (2 * F), e = i % (2 * F);
    l_dom[s][e] = kp[((long long)(e >> 1) * n_cap + toks[s]) * 2 + (e & 1)];
  }
  const int s = t / LPR, c = t % LPR;
  uint4 vrow = make_uint4(0, 0, 0, 0);
  if (s < nt) vrow = *reinterpret_cast<const uint4*>(Vh + b * sb + h * sh + (long long)toks[s] * sn + c * VEC);
  __syncthreads();
  if (s < nt) {
    ET out[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      const uint32_t m = src[c * VEC + k];
      out[k] = (m & 0x8000u) ? l_dom[s][m & 0x7FFFu] : l_nd[s][m];
    }
    const size_t o = ((size_t)row * count + j0 + s) * D + c * VEC;
    *reinterpret_cast<uint4*>(KT + o) = *reinterpret_cast<const uint4*>(out);
    *reinterpret_cast<uint4*>(VT + o) = vrow;
  }
}

hipError_t launch_offload_split(const fasa_shape& s, const void* K, const int32_t* fc_idx, void* Kp,
                                void* Knd, int n_begin, int n_end, hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid((n_end - n_begin + kOffTile - 1) / kOffTile, rows), block(256);
  if (s.dtype == FASA_BF16)
    return launch("fasa_offload_split", offload_split_kernel<uint16_t>, grid, block, st,
                  (const uint16_t*)K, fc_idx, (uint16_t*)Kp, (uint16_t*)Knd, s.n_kv_heads, s.n_fc,
                  s.n_cap, n_begin, n_end, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                  (long long)s.kv_stride_n, s.pairing);
  return launch("fasa_offload_split", offload_split_kernel<float>, grid, block, st, (const float*)K,
                fc_idx, (float*)Kp, (float*)Knd, s.n_kv_heads, s.n_fc, s.n_cap, n_begin, n_end,
                (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, s.pairing);
}

hipError_t launch_offload_append(const fasa_shape& s, void* Kp, void* Knd, void* Vh,
                                 const int32_t* fc_idx, const void* k_new, const void* v_new,
                                 hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  if (s.dtype == FASA_BF16)
    return launch("fasa_offload_append", offload_append_kernel<uint16_t>, dim3(rows), dim3(256), st,
                  (uint16_t*)Kp, (uint16_t*)Knd, (uint16_t*)Vh, fc_idx, (const uint16_t*)k_new,
                  (const uint16_t*)v_new, s.n_kv_heads, s.n_fc, s.n_cap, s.n_ctx,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, s.pairing);
  return launch("fasa_offload_append", offload_append_kernel<float>, dim3(rows), dim3(256), st,
                (float*)Kp, (float*)Knd, (float*)Vh, fc_idx, (const float*)k_new, (const float*)v_new,
                s.n_kv_heads, s.n_fc, s.n_cap, s.n_ctx, (long long)s.kv_stride_b,
                (long long)s.kv_stride_h, (long long)s.kv_stride_n, s.pairing);
}

hipError_t launch_offload_gather(const fasa_shape& s, const void* Kp, const void* Knd, const void* Vh,
                                 const int32_t* fc_idx, const int32_t* T, void* KT, void* VT,
                                 hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  const int count = s.budget < s.n_ctx ? s.budget : s.n_ctx;
  if (s.dtype == FASA_BF16) {
    dim3 grid((count + 15) / 16, rows), block(256);
    return launch("fasa_offload_gather", offload_gather_kernel<uint16_t>, grid, block, st,
                  (const uint16_t*)Kp, (const uint16_t*)Knd, (const uint16_t*)Vh, fc_idx, T,
                  (uint16_t*)KT, (uint16_t*)VT, s.n_kv_heads, s.n_fc, s.n_cap, s.n_ctx, count,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, s.pairing);
  }
  dim3 grid((count + 7) / 8, rows), block(256);
  return launch("fasa_offload_gather", offload_gather_kernel<float>, grid, block, st, (const float*)Kp,
                (const float*)Knd, (const float*)Vh, fc_idx, T, (float*)KT, (float*)VT, s.n_kv_heads,
                s.n_fc, s.n_cap, s.n_ctx, count, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                (long long)s.kv_stride_n, s.pairing);
}

}  // namespace fasa
