// FAC (paper Sec. 4.2, eq. fac_output): exact softmax attention over the selected rows of K and V,
// as split-K flash decoding: every workgroup owns a chunk of the row's index list, gathers the
// K/V rows it names, keeps a running (max, sum, weighted V) per query head of the GQA group, and
// the workgroup that finishes a row last merges the row's chunks.  The same kernel with the index list replaced by the
// identity is the full-KV baseline (paper Sec. 4.4).
#include "mfma_tile.h"

namespace fasa {

constexpr int kAttU = 4;                  // rows in flight per 16-lane group and batch
constexpr int kAttBatch = 4 * kAttU;      // rows per wave and batch

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

// 1-D grid of rows * n_splits workgroups, 256 threads.  A wave is 4 groups of 16 lanes; a group
// reads one cached row per load instruction (16 lanes x 16 bytes = one 256-byte bf16 row), lane c
// owning head dims [8c, 8c+8) of K (for the logit) and of V (for the output).  The workgroup that
// finishes a row last merges the row's partials into O.
template <typename ET, int G, bool DENSE>
__global__ __launch_bounds__(256) void attend_kernel(const ET* __restrict__ q,
                                                     const ET* __restrict__ K,
                                                     const ET* __restrict__ V,
                                                     const int32_t* __restrict__ T,
                                                     float* __restrict__ O,
                                                     RowCtl* __restrict__ ctl,
                                                     float* __restrict__ part_acc,
                                                     float* __restrict__ part_ml, int rows,
                                                     int n_splits, int Hq, int Hkv, int count_max,
                                                     int n_ctx_max, int tok_per_split, long long sb,
                                                     long long sh, long long sn,
                                                     float scale_log2e,
                                                     const int32_t* __restrict__ n_ctx_seq,
                                                     const int32_t* __restrict__ budget_seq,
                                                     PageMap pm) {
  constexpr int D = kHeadDim;
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float sm_acc[4][G][D];
  __shared__ float wsm[G * kMaxSplitsLds];
  __shared__ float red[G];
  __shared__ uint32_t ticket;

  int row, split;
  row_slice_of_block(rows, n_splits, row, split);
  const int b = row / Hkv, h = row % Hkv;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int r = lane >> 4, c = lane & 15;

  // entries of this row: the shape's values, or this sequence's own (never more than the shape's)
  const int n_ctx = seq_n_ctx(n_ctx_seq, b, n_ctx_max);
  const int count = DENSE ? n_ctx : seq_bsel(budget_seq, b, n_ctx, count_max);
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

  // list entries are token numbers, or pool slots of a paged cache (block << shift | offset)
  const bool paged = pm.table != nullptr;
  const int pshift = paged ? pm.shift : 31, pmask = paged ? (1 << pm.shift) - 1 : 0x7fffffff;
  const long long blk_stride = paged ? sb : 0;
  const int slot_max = paged ? (pm.n_pool << pm.shift) - 1 : n_ctx - 1;
  const ET* Kb = K + (paged ? 0 : b * sb) + h * sh + 8 * c;
  const ET* Vb = V + (paged ? 0 : b * sb) + h * sh + 8 * c;
  const int32_t* Trow = DENSE ? nullptr : T + (size_t)row * count_max;

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
      const int tok = DENSE ? jj : min(max(Trow[jj], 0), slot_max);
      off[u] = (long long)(tok >> pshift) * blk_stride + (long long)(tok & pmask) * sn;
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
        s[u][g] = row16_sum(d);   // all 16 lanes of the group end up with the logit
      }
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
  for (int g = 0; g < G; ++g) {
    const float mn = xor32_max(xor16_max(m[g]));
    const float sc = exp2f(m[g] - mn);
    m[g] = mn;
    l[g] = xor32_sum(xor16_sum(l[g] * sc));
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[g][k] = xor32_sum(xor16_sum(acc[g][k] * sc));
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
  const size_t pbase = ((size_t)row * n_splits + split) * G;
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
    if (n_splits == 1) {
      O[((size_t)b * Hq + (size_t)h * G + g) * D + dim] = a / ls;   // nothing to merge
    } else {
      // read by the row's last workgroup: published with agent-scope stores
      st_agent(&part_acc[(pbase + g) * D + dim], a);
      if (dim == 0) {
        st_agent(&part_ml[(pbase + g) * 2], mn);
        st_agent(&part_ml[(pbase + g) * 2 + 1], ls);
      }
    }
  }
  if (n_splits == 1) return;

  // ---- the row's last workgroup merges the splits ----
  publish_barrier();
  if (t == 0) ticket = atomicAdd(&ctl[row].done_att, 1u);
  __syncthreads();
  if (ticket != (uint32_t)n_splits - 1u) return;
  if (t == 0) ctl[row].done_att = 0;   // clean for the next call
  combine_row<G>(part_acc, part_ml, O, row, b, h, Hq, n_splits, n_splits, wsm, red, &sm_acc[0][0][0]);
}

// ---------------------------------------------------------------------------------------------
// bf16 variant with both products of a 16-row tile on the matrix cores (mfma_tile.h): the logits
// K_tile . Q^T of the GQA group and the weighted sum P . V_tile.  The tile loop is software-pipelined:
// while a tile is computed, the next tile's K/V rows and the list entries of the tile after it are in
// flight.  Loads inside the loop are unconditional (straight-line code keeps the compiler's wait
// counts exact: a test around a load would turn every later wait into a wait for everything);
// entries beyond the range are clamped into it and only fetched, the K/V prefetch is issued for real
// tiles only (the last tile is peeled).
// ---------------------------------------------------------------------------------------------
template <int G, bool DENSE>
__global__ __launch_bounds__(256) void attend_mfma_kernel(const uint16_t* __restrict__ q,
                                                          const uint16_t* __restrict__ K,
                                                          const uint16_t* __restrict__ V,
                                                          const int32_t* __restrict__ T,
                                                          float* __restrict__ O,
                                                          RowCtl* __restrict__ ctl,
                                                          float* __restrict__ part_acc,
                                                          float* __restrict__ part_ml, int rows,
                                                          int n_splits, int Hq, int Hkv, int count_max,
                                                          int n_ctx_max, int tok_per_split, long long sb,
                                                          long long sh, long long sn,
                                                          float scale_log2e,
                                                          const int32_t* __restrict__ n_ctx_seq,
                                                          const int32_t* __restrict__ budget_seq,
                                                          PageMap pm) {
  constexpr int D = kHeadDim;
  // the waves' totals, later the merge's partition scratch (< 8 KB) and, behind it, its split weights
  constexpr int ACC_BYTES = 4 * G * D * 4;
  constexpr int MERGE_BYTES = 8192 + G * kMaxSplitsLds * 4;
  __shared__ __align__(16) unsigned char big[ACC_BYTES > MERGE_BYTES ? ACC_BYTES : MERGE_BYTES];
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float red[G];
  __shared__ uint32_t ticket;
  __shared__ __align__(16) float scs[4][16];      // per wave: rescale factor of each head's running sums
  float (*sm_o)[G][D] = reinterpret_cast<float (*)[G][D]>(big);
  float* wsm = reinterpret_cast<float*>(big + 8192);

  int row, split;
  row_slice_of_block(rows, n_splits, row, split);
  const int b = row / Hkv, h = row % Hkv;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int lo = lane & 15, hi = lane >> 4;

  // entries of this row: the shape's values, or this sequence's own (never more than the shape's)
  const int n_ctx = seq_n_ctx(n_ctx_seq, b, n_ctx_max);
  const int count = DENSE ? n_ctx : seq_bsel(budget_seq, b, n_ctx, count_max);
  const int s0 = split * tok_per_split;
  const int s1 = min(count, s0 + tok_per_split);
  FASA_T_DECL(5);
  FASA_T(0);

  MfmaTile<G> tile;
  tile.load_q(q + ((size_t)b * Hq + (size_t)h * G) * D, lo, hi);
  tile.reset();

  // list entries are token numbers, or pool slots of a paged cache (block << shift | offset)
  const bool paged = pm.table != nullptr;
  const int pshift = paged ? pm.shift : 31, pmask = paged ? (1 << pm.shift) - 1 : 0x7fffffff;
  const long long blk_stride = paged ? sb : 0;
  const int slot_max = paged ? (pm.n_pool << pm.shift) - 1 : n_ctx - 1;
  const uint16_t* Kb = K + (paged ? 0 : b * sb) + h * sh;
  const uint16_t* Vb = V + (paged ? 0 : b * sb) + h * sh + 8 * lo;
  const int32_t* Trow = DENSE ? nullptr : T + (size_t)row * count_max;

  struct TileIdx { int k; int v[4]; };        // list entries of one tile: K row lo, V rows 4hi .. 4hi+3
  auto load_idx = [&](int j0) {
    TileIdx r;
    if constexpr (DENSE) {
      r.k = min(j0 + lo, s1 - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) r.v[i] = min(j0 + 4 * hi + i, s1 - 1);
    } else {
      // a stray index can never become a stray address: entries are clamped to the cache below
      r.k = Trow[min(j0 + lo, s1 - 1)];
#pragma unroll
      for (int i = 0; i < 4; ++i) r.v[i] = Trow[min(j0 + 4 * hi + i, s1 - 1)];
    }
    return r;
  };
  auto load_kv = [&](const TileIdx& ix) {
    TileKV r;
    auto row_off = [&](int e) {
      const int sl = min(max(e, 0), slot_max);
      return (long long)(sl >> pshift) * blk_stride + (long long)(sl & pmask) * sn;
    };
    const long long koff = row_off(ix.k);
#pragma unroll
    for (int i = 0; i < 4; ++i) r.kc[i] = *reinterpret_cast<const uint4*>(Kb + koff + 8 * (hi + 4 * i));
#pragma unroll
    for (int i = 0; i < 4; ++i) r.vr[i] = *reinterpret_cast<const uint4*>(Vb + row_off(ix.v[i]));
    return r;
  };
  auto compute_tile = [&](const TileKV& kv, int j0) {
    float sv[4];
    tile.logits(kv, scale_log2e, sv);
    bool valid[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) valid[e] = j0 + 4 * hi + e < s1;
    tile.accumulate(kv, sv, valid, &scs[wave][0], lo, hi);
  };

  const int jw = s0 + wave * 16;               // this wave's tiles start at jw, jw + 64, ...
  if (jw < s1) {
    const int n_tiles = (s1 - jw + 63) / 64;
    TileIdx ix_next = load_idx(jw + 64);
    TileKV cur = load_kv(load_idx(jw));
    for (int i = 0; i + 1 < n_tiles; ++i) {
      const int j0 = jw + 64 * i;
      const TileKV nxt = load_kv(ix_next);
      ix_next = load_idx(j0 + 128);
      compute_tile(cur, j0);
      cur = nxt;
    }
    compute_tile(cur, jw + 64 * (n_tiles - 1));
  }
  FASA_T(1);
  tile.finish(&sm_m[wave][0], &sm_l[wave][0], &sm_o[wave][0][0], lo, hi);
  __syncthreads();

  // workgroup totals: thread (query head g, 4 head dims)
  const size_t pbase = ((size_t)row * n_splits + split) * G;
  if (t < G * (D / 4)) {
    const int g = t / (D / 4), d4 = t % (D / 4);
    float mn, ls;
    float4 a;
    tile_wg_totals<G>(&sm_m[0][0], &sm_l[0][0], &sm_o[0][0][0], g, d4, mn, ls, a);
    if (n_splits == 1) {
      *reinterpret_cast<float4*>(O + ((size_t)b * Hq + (size_t)h * G + g) * D + 4 * d4) =
          make_float4(a.x / ls, a.y / ls, a.z / ls, a.w / ls);
    } else {
      float2* pa = reinterpret_cast<float2*>(part_acc + (pbase + g) * D + 4 * d4);
      st_agent(pa, make_float2(a.x, a.y));
      st_agent(pa + 1, make_float2(a.z, a.w));
      if (d4 == 0) st_agent(reinterpret_cast<float2*>(part_ml + (pbase + g) * 2), make_float2(mn, ls));
    }
  }
  if (n_splits == 1) return;
  FASA_T(2);
  publish_barrier();
  if (t == 0) ticket = atomicAdd(&ctl[row].done_att, 1u);
  __syncthreads();
  FASA_T(3);
  FASA_T_PRINT(t == 0 && row == 0 && split == 0, "attend blk0: tiles %llu merge %llu publish+ticket %llu (x10ns)\n",
               FASA_T_D(1, 0), FASA_T_D(2, 1), FASA_T_D(3, 2));
  if (ticket != (uint32_t)n_splits - 1u) return;
  if (t == 0) ctl[row].done_att = 0;
  combine_row<G>(part_acc, part_ml, O, row, b, h, Hq, n_splits, n_splits, wsm, red, reinterpret_cast<float*>(big));
  FASA_T(4);
  FASA_T_PRINT(t == 0 && row == 0, "attend last(row0, split %d): tiles %llu merge %llu publish+ticket %llu combine %llu (x10ns)\n",
               split, FASA_T_D(1, 0), FASA_T_D(2, 1), FASA_T_D(3, 2), FASA_T_D(4, 3));
}

template <typename ET, int G>
static hipError_t launch_attend_g(const fasa_shape& s, bool dense, const AttendPlan& p,
                                  const void* q, const void* K, const void* V, const int32_t* T,
                                  float* O, RowCtl* ctl, float* part_acc, float* part_ml,
                                  hipStream_t st, RaggedLens rl, PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  dim3 grid(rows * p.n_splits), block(256);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)s.head_dim);
  if constexpr (sizeof(ET) == 2) {
    if (dense)
      return launch("fasa_dense_attend", attend_mfma_kernel<G, true>, grid, block, st,
                    (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, T, O, ctl, part_acc,
                    part_ml, rows, p.n_splits, s.n_q_heads, s.n_kv_heads, p.count, s.n_ctx,
                    p.tok_per_split, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                    (long long)s.kv_stride_n, scale_log2e, rl.n_ctx, rl.budget, pm);
    return launch("fasa_sparse_attend", attend_mfma_kernel<G, false>, grid, block, st,
                  (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, T, O, ctl, part_acc,
                  part_ml, rows, p.n_splits, s.n_q_heads, s.n_kv_heads, p.count, s.n_ctx,
                  p.tok_per_split, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                  (long long)s.kv_stride_n, scale_log2e, rl.n_ctx, rl.budget, pm);
  }
  if (dense)
    return launch("fasa_dense_attend", attend_kernel<ET, G, true>, grid, block, st, (const ET*)q,
                  (const ET*)K, (const ET*)V, T, O, ctl, part_acc, part_ml, rows, p.n_splits,
                  s.n_q_heads, s.n_kv_heads, p.count, s.n_ctx, p.tok_per_split,
                  (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n,
                  scale_log2e, rl.n_ctx, rl.budget, pm);
  return launch("fasa_sparse_attend", attend_kernel<ET, G, false>, grid, block, st, (const ET*)q,
                (const ET*)K, (const ET*)V, T, O, ctl, part_acc, part_ml, rows, p.n_splits,
                s.n_q_heads, s.n_kv_heads, p.count, s.n_ctx, p.tok_per_split,
                (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n,
                scale_log2e, rl.n_ctx, rl.budget, pm);
}

template <typename ET>
static hipError_t launch_attend_t(const fasa_shape& s, bool dense, const AttendPlan& p,
                                  const void* q, const void* K, const void* V, const int32_t* T,
                                  float* O, RowCtl* ctl, float* part_acc, float* part_ml,
                                  hipStream_t st, RaggedLens rl, PageMap pm) {
  switch (s.n_q_heads / s.n_kv_heads) {
    case 1: return launch_attend_g<ET, 1>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 2: return launch_attend_g<ET, 2>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 3: return launch_attend_g<ET, 3>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 4: return launch_attend_g<ET, 4>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 5: return launch_attend_g<ET, 5>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 6: return launch_attend_g<ET, 6>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 7: return launch_attend_g<ET, 7>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    case 8: return launch_attend_g<ET, 8>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_attend(const fasa_shape& s, bool dense, const void* q, const void* K,
                         const void* V, const int32_t* T, float* O, RowCtl* ctl, float* part_acc,
                         float* part_ml, hipStream_t st, RaggedLens rl, PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  if (dense && pm.table != nullptr) return hipErrorInvalidValue;   // identity lists are token numbers
  const int count = dense ? s.n_ctx : (s.budget < s.n_ctx ? s.budget : s.n_ctx);
  const AttendPlan p = plan_attend(rows, count, s.n_q_heads / s.n_kv_heads);
  return s.dtype == FASA_BF16
             ? launch_attend_t<uint16_t>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm)
             : launch_attend_t<float>(s, dense, p, q, K, V, T, O, ctl, part_acc, part_ml, st, rl, pm);
}

}  // namespace fasa
