// FAC (paper Sec. 4.2, eq. fac_output): exact softmax attention over the selected rows of K and V,
// as split-K flash decoding: every workgroup owns a chunk of the row's index list, gathers the
// K/V rows it names, keeps a running (max, sum, weighted V) per query head of the GQA group, and
// a second small kernel merges the chunks.  The same kernel with the index list replaced by the
// identity is the full-KV baseline (paper Sec. 4.4).
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

constexpr int kAttU = 4;                  // rows in flight per 16-lane group and batch
constexpr int kAttBatch = 4 * kAttU;      // rows per wave and batch
constexpr float kNegBig = -1.0e30f;       // finite stand-in for -inf (keeps exp2 arguments finite)

// 8 consecutive head dims of one cached row, widened to float32
template <typename ET> struct Row8;
template <> struct Row8<uint16_t> {
  uint4 w;
  __device__ __forceinline__ void load(const uint16_t* p) { w = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void unpack(float* f) const {
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x); f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z); f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
  }
};
template <> struct Row8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p);
    b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void unpack(float* f) const {
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
};

__device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ float to_f32(float v) { return v; }

// grid = (n_splits, rows), 256 threads.  A wave is 4 groups of 16 lanes; a group reads one cached
// row per load instruction (16 lanes x 16 bytes = one 256-byte bf16 row), lane c owning head dims
// [8c, 8c+8) of K (for the logit) and of V (for the output).
template <typename ET, int G, bool DENSE>
__global__ __launch_bounds__(256) void attend_kernel(const ET* __restrict__ q,
                                                     const ET* __restrict__ K,
                                                     const ET* __restrict__ V,
                                                     const int32_t* __restrict__ T,
                                                     float* __restrict__ part_acc,
                                                     float* __restrict__ part_ml, int Hq, int Hkv,
                                                     int count, int n_ctx, int tok_per_split,
                                                     long long sb, long long sh, long long sn,
                                                     float scale_log2e) {
  constexpr int D = kHeadDim;
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float sm_acc[4][G][D];

  const int row = blockIdx.y;
  const int b = row / Hkv, h = row % Hkv;
  const int split = blockIdx.x;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int r = lane >> 4, c = lane & 15;

  const int s0 = split * tok_per_split;
  const int s1 = min(count, s0 + tok_per_split);

  float qr[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const ET* qp = q + ((size_t)b * Hq + (size_t)h * G + g) * D + 8 * c;
#pragma unroll
    for (int k = 0; k < 8; ++k) qr[g][k] = to_f32(qp[k]) * scale_log2e;
  }
  float acc[G][8], m[G], l[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[g][k] = 0.f;
  }

  const ET* Kb = K + b * sb + h * sh + 8 * c;
  const ET* Vb = V + b * sb + h * sh + 8 * c;
  const int32_t* Trow = DENSE ? nullptr : T + (size_t)row * count;

  for (int j0 = s0 + wave * kAttBatch; j0 < s1; j0 += 4 * kAttBatch) {
    bool valid[kAttU];
    Row8<ET> kv[kAttU], vv[kAttU];
    long long off[kAttU];
#pragma unroll
    for (int u = 0; u < kAttU; ++u) {
      const int j = j0 + u * 4 + r;
      valid[u] = j < s1;
      const int jj = valid[u] ? j : s0;              // any in-range entry; its weight is zeroed
      // a stray index can never become a stray address: entries are clamped to the cache
      const int tok = DENSE ? jj : min(max(Trow[jj], 0), n_ctx - 1);
      off[u] = (long long)tok * sn;
    }
#pragma unroll
    for (int u = 0; u < kAttU; ++u) kv[u].load(Kb + off[u]);
#pragma unroll
    for (int u = 0; u < kAttU; ++u) vv[u].load(Vb + off[u]);

    float s[kAttU][G];
#pragma unroll
    for (int u = 0; u < kAttU; ++u) {
      float kf[8];
      kv[u].unpack(kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) d = fmaf(qr[g][k], kf[k], d);
        s[u][g] = d;
      }
    }
    // sum the 16 partial dot products of a group (all 16 lanes end up with the logit)
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
#pragma unroll
      for (int u = 0; u < kAttU; ++u)
#pragma unroll
        for (int g = 0; g < G; ++g) s[u][g] += __shfl_xor(s[u][g], o, kWave);
    }
    float p[kAttU][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mx = m[g];
#pragma unroll
      for (int u = 0; u < kAttU; ++u) mx = valid[u] ? fmaxf(mx, s[u][g]) : mx;
      const float sc = exp2f(m[g] - mx);
      m[g] = mx;
      float ls = l[g] * sc;
#pragma unroll
      for (int u = 0; u < kAttU; ++u) {
        p[u][g] = valid[u] ? exp2f(s[u][g] - mx) : 0.f;
        ls += p[u][g];
      }
      l[g] = ls;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[g][k] *= sc;
    }
#pragma unroll
    for (int u = 0; u < kAttU; ++u) {
      float vf[8];
      vv[u].unpack(vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[g][k] = fmaf(p[u][g], vf[k], acc[g][k]);
    }
  }

  // merge the 4 groups of the wave (lanes c, c+16, c+32, c+48 hold the same head dims)
#pragma unroll
  for (int o = 16; o < 64; o <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(m[g], o, kWave);
      const float mn = fmaxf(m[g], mo);
      const float sc = exp2f(m[g] - mn);
      m[g] = mn;
      l[g] *= sc;
      l[g] += __shfl_xor(l[g], o, kWave);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        acc[g][k] *= sc;
        acc[g][k] += __shfl_xor(acc[g][k], o, kWave);
      }
    }
  }
  if (r == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (c == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
#pragma unroll
      for (int k = 0; k < 8; ++k) sm_acc[wave][g][8 * c + k] = acc[g][k];
    }
  }
  __syncthreads();

  // merge the 4 waves; one (query head, head dim) per thread and pass
  const size_t pbase = ((size_t)row * gridDim.x + split) * G;
  for (int i = t; i < G * D; i += 256) {
    const int g = i / D, dim = i % D;
    float mn = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < 4; ++w) mn = fmaxf(mn, sm_m[w][g]);
    float ls = 0.f, a = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float sc = exp2f(sm_m[w][g] - mn);
      ls = fmaf(sm_l[w][g], sc, ls);
      a = fmaf(sm_acc[w][g][dim], sc, a);
    }
    part_acc[(pbase + g) * D + dim] = a;
    if (dim == 0) {
      part_ml[(pbase + g) * 2] = mn;
      part_ml[(pbase + g) * 2 + 1] = ls;
    }
  }
}

// grid = batch * Hq, 128 threads (one head dim each): O = sum_s acc_s 2^(m_s - m*) / sum_s l_s 2^(m_s - m*)
__global__ __launch_bounds__(128) void combine_kernel(const float* __restrict__ part_acc,
                                                      const float* __restrict__ part_ml,
                                                      float* __restrict__ O, int Hq, int Hkv,
                                                      int n_splits) {
  constexpr int D = kHeadDim;
  const int bh = blockIdx.x;
  const int b = bh / Hq, hq = bh % Hq;
  const int G = Hq / Hkv;
  const int row = b * Hkv + hq / G, g = hq % G;
  const int dim = threadIdx.x;
  float mn = kNegBig;
  for (int s = 0; s < n_splits; ++s)
    mn = fmaxf(mn, part_ml[(((size_t)row * n_splits + s) * G + g) * 2]);
  float ls = 0.f, a = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const size_t pi = ((size_t)row * n_splits + s) * G + g;
    const float sc = exp2f(part_ml[pi * 2] - mn);
    ls = fmaf(part_ml[pi * 2 + 1], sc, ls);
    a = fmaf(part_acc[pi * D + dim], sc, a);
  }
  O[(size_t)bh * D + dim] = a / ls;
}

template <typename ET, int G>
static hipError_t launch_attend_g(const fasa_shape& s, bool dense, const AttendPlan& p,
                                  const void* q, const void* K, const void* V, const int32_t* T,
                                  float* part_acc, float* part_ml, hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid(p.n_splits, rows), block(256);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)s.head_dim);
  if (dense)
    return launch("fasa_dense_attend", attend_kernel<ET, G, true>, grid, block, st, (const ET*)q,
                  (const ET*)K, (const ET*)V, T, part_acc, part_ml, s.n_q_heads, s.n_kv_heads,
                  p.count, s.n_ctx, p.tok_per_split, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                  (long long)s.kv_stride_n, scale_log2e);
  return launch("fasa_sparse_attend", attend_kernel<ET, G, false>, grid, block, st, (const ET*)q,
                (const ET*)K, (const ET*)V, T, part_acc, part_ml, s.n_q_heads, s.n_kv_heads,
                p.count, s.n_ctx, p.tok_per_split, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                (long long)s.kv_stride_n, scale_log2e);
}

template <typename ET>
static hipError_t launch_attend_t(const fasa_shape& s, bool dense, const AttendPlan& p,
                                  const void* q, const void* K, const void* V, const int32_t* T,
                                  float* part_acc, float* part_ml, hipStream_t st) {
  switch (s.n_q_heads / s.n_kv_heads) {
    case 1: return launch_attend_g<ET, 1>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 2: return launch_attend_g<ET, 2>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 3: return launch_attend_g<ET, 3>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 4: return launch_attend_g<ET, 4>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 5: return launch_attend_g<ET, 5>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 6: return launch_attend_g<ET, 6>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 7: return launch_attend_g<ET, 7>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    case 8: return launch_attend_g<ET, 8>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_attend(const fasa_shape& s, bool dense, const void* q, const void* K,
                         const void* V, const int32_t* T, float* O, float* part_acc, float* part_ml,
                         hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  const int count = dense ? s.n_ctx : (s.budget < s.n_ctx ? s.budget : s.n_ctx);
  const AttendPlan p = plan_attend(rows, count);
  hipError_t e = s.dtype == FASA_BF16
                     ? launch_attend_t<uint16_t>(s, dense, p, q, K, V, T, part_acc, part_ml, st)
                     : launch_attend_t<float>(s, dense, p, q, K, V, T, part_acc, part_ml, st);
  if (e != hipSuccess) return e;
  return launch("fasa_combine", combine_kernel, dim3(s.batch * s.n_q_heads), dim3(128), st,
                (const float*)part_acc, (const float*)part_ml, O, s.n_q_heads, s.n_kv_heads,
                p.n_splits);
}

}  // namespace fasa
