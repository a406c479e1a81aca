// TopK-I (paper Sec. 4.1): index set of the B largest scores of each (b,h) row.
//
// Radix select on the order-preserving 32-bit key of the float32 score, ties towards the
// lower token index:
//   level 0  the per-row histogram of the top 12 key bits (built by the scoring kernel or by
//            hist_kernel) fixes the threshold bin: bins above it hold fewer than B tokens, bins
//            from it upwards at least B;
//   filter   many workgroups per row stream S once; tokens above the threshold bin are winners
//            and go straight to T, tokens inside it are appended to a candidate list;
//   final    the last workgroup of the row to finish resolves the candidates exactly: radix
//            select, 8 bits a pass, over the 56-bit composite (low 20 key bits : ~index), which
//            is unique per token, so exactly B - |winners| candidates come out.
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

constexpr int kSelTokPerBlock = 2048;  // slice of a row filtered by one workgroup
constexpr int kCandLds = 4096;         // candidates resolved out of LDS; more spill to global reads

__device__ __forceinline__ unsigned long long cand_composite(uint2 c) {
  return ((unsigned long long)(c.x & ((1u << kKeyLowBits) - 1u)) << 32) | (unsigned long long)(~c.y);
}

// Exact selection of the `need` largest composites among cand[0..n).  Whole block participates.
__device__ void resolve_candidates(const uint2* cand, int n, int need, int32_t* out,
                                   uint32_t* dh /*256*/, uint32_t* wtot /*4*/,
                                   uint32_t* bc /*4: digit, need, count, out counter*/) {
  const int t = threadIdx.x;
  const uint32_t out_cap = (uint32_t)need;  // never write past the row's share of T
  unsigned long long prefix = 0;
  int shift = 56;
  if (need < n) {
    while (shift > 0) {
      shift -= 8;
      dh[t] = 0;
      __syncthreads();
      for (int i = t; i < n; i += 256) {
        const unsigned long long c = cand_composite(cand[i]);
        if ((c >> (shift + 8)) == prefix) atomicAdd(&dh[(uint32_t)(c >> shift) & 0xFFu], 1u);
      }
      __syncthreads();
      const uint32_t cnt = dh[t];
      const uint32_t incl = block256_suffix_sum(cnt, wtot);
      const uint32_t excl = incl - cnt;
      if (excl < (uint32_t)need && (uint32_t)need <= incl) {
        bc[0] = (uint32_t)t;
        bc[1] = (uint32_t)need - excl;
        bc[2] = cnt;
      }
      __syncthreads();
      prefix = (prefix << 8) | bc[0];
      need = (int)bc[1];
      const uint32_t in_digit = bc[2];
      __syncthreads();
      if ((uint32_t)need == in_digit) break;  // everything under this prefix is a winner
    }
  } else {
    shift = 56;  // take all: (c >> 56) == 0 >= 0
  }
  for (int i = t; i < n; i += 256) {
    const uint2 c = cand[i];
    if ((cand_composite(c) >> shift) >= prefix) {
      const uint32_t pos = atomicAdd(&bc[3], 1u);
      if (pos < out_cap) out[pos] = (int32_t)c.y;
    }
  }
}

// grid = (ceil(N / kSelTokPerBlock), rows)
__global__ __launch_bounds__(256) void select_kernel(const float* __restrict__ S,
                                                     const uint32_t* __restrict__ hist,
                                                     RowCtl* __restrict__ ctl,
                                                     uint2* __restrict__ cand,
                                                     int32_t* __restrict__ T, int N, int n_cap,
                                                     int bsel) {
  __shared__ uint32_t wtot[4];
  __shared__ uint32_t bc[4];
  __shared__ uint32_t thr[2];  // threshold bin, tokens above it
  __shared__ uint32_t dh[256];
  __shared__ uint2 lc[kCandLds];

  const int row = blockIdx.y;
  const int t = threadIdx.x;
  const int lane = lane_id();
  const uint32_t* gh = hist + (size_t)row * kHistBins;

  // ---- threshold bin from the coarse histogram (every workgroup of the row redoes this) ----
  if (t == 0) { thr[0] = 0; thr[1] = 0; }
  {
    uint32_t hb[16];
    const uint4* hp = reinterpret_cast<const uint4*>(gh + t * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint4 v = hp[j];
      hb[4 * j] = v.x; hb[4 * j + 1] = v.y; hb[4 * j + 2] = v.z; hb[4 * j + 3] = v.w;
    }
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) mine += hb[j];
    const uint32_t incl = block256_suffix_sum(mine, wtot);
    uint32_t cum = incl - mine;
    if (cum < (uint32_t)bsel && (uint32_t)bsel <= incl) {
#pragma unroll
      for (int j = 15; j >= 0; --j) {
        if (cum < (uint32_t)bsel && cum + hb[j] >= (uint32_t)bsel) {
          thr[0] = (uint32_t)(t * 16 + j);
          thr[1] = cum;
        }
        cum += hb[j];
      }
    }
    __syncthreads();
  }
  const uint32_t tbin = thr[0];
  const uint32_t n_above = thr[1];

  // ---- filter this workgroup's slice ----
  const float* s = S + (size_t)row * n_cap;
  int32_t* trow = T + (size_t)row * bsel;
  uint2* crow = cand + (size_t)row * n_cap;
  const int base = blockIdx.x * kSelTokPerBlock;
#pragma unroll 1
  for (int it = 0; it < kSelTokPerBlock / 1024; ++it) {
    const int n0 = base + (it * 256 + t) * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (n0 + 4 <= N) {
      const float4 x = *reinterpret_cast<const float4*>(s + n0);
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else {
      for (int k = 0; k < 4; ++k)
        if (n0 + k < N) v[k] = s[n0 + k];
    }
    uint32_t key[4];
    uint32_t win = 0, cnd = 0;  // bit k set: token n0 + k is a winner / candidate
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      key[k] = score_key(v[k]);
      const uint32_t bin = key[k] >> kKeyLowBits;
      const bool ok = n0 + k < N;
      win |= (ok && bin > tbin) ? (1u << k) : 0u;
      cnd |= (ok && bin == tbin) ? (1u << k) : 0u;
    }
    const uint32_t nw = __popc(win), nc = __popc(cnd);
    const uint32_t pw = wave_prefix_sum(nw), pc = wave_prefix_sum(nc);
    const uint32_t tw = __shfl(pw, kWave - 1, kWave), tc = __shfl(pc, kWave - 1, kWave);
    uint32_t bw = 0, bcand = 0;
    if (lane == 0) {
      if (tw) bw = atomicAdd(&ctl[row].n_sel, tw);
      if (tc) bcand = atomicAdd(&ctl[row].n_cand, tc);
    }
    bw = __shfl(bw, 0, kWave) + pw - nw;
    bcand = __shfl(bcand, 0, kWave) + pc - nc;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // the bounds hold by construction of the histogram; they are re-checked so that a
      // histogram that does not match S can never turn into an out-of-range store
      if ((win & (1u << k)) && bw < (uint32_t)bsel) trow[bw++] = n0 + k;
      if ((cnd & (1u << k)) && bcand < (uint32_t)n_cap) crow[bcand++] = make_uint2(key[k], (uint32_t)(n0 + k));
    }
  }

  // ---- last workgroup of the row resolves the threshold bin ----
  __threadfence();
  __syncthreads();
  if (t == 0) bc[0] = atomicAdd(&ctl[row].done, 1u);
  __syncthreads();
  const bool last = bc[0] == gridDim.x - 1;
  __syncthreads();
  if (!last) return;
  __threadfence();
  int n_cand = (int)__hip_atomic_load(&ctl[row].n_cand, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  n_cand = min(n_cand, n_cap);
  const int need = max(0, min(bsel - (int)n_above, n_cand));
  if (t == 0) bc[3] = 0;
  const uint2* src = crow;
  if (n_cand <= kCandLds) {
    for (int i = t; i < n_cand; i += 256)
      lc[i] = crow[i];
    src = lc;
  }
  __syncthreads();
  resolve_candidates(src, n_cand, need, trow + n_above, dh, wtot, bc);
}

// budget >= N: every token is selected
__global__ __launch_bounds__(256) void select_all_kernel(int32_t* __restrict__ T, int N) {
  const int row = blockIdx.y;
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n < N) T[(size_t)row * N + n] = n;
}

hipError_t launch_select(const fasa_shape& s, const float* S, const uint32_t* hist, RowCtl* ctl,
                         uint2* cand, int32_t* T, hipStream_t st) {
  const int rows = s.batch * s.n_kv_heads;
  if (s.budget >= s.n_ctx) {
    dim3 grid((s.n_ctx + 255) / 256, rows), block(256);
    return launch("fasa_select_all", select_all_kernel, grid, block, st, T, s.n_ctx);
  }
  dim3 grid((s.n_ctx + kSelTokPerBlock - 1) / kSelTokPerBlock, rows), block(256);
  return launch("fasa_select", select_kernel, grid, block, st, S, hist, ctl, cand, T, s.n_ctx,
                s.n_cap, s.budget);
}

}  // namespace fasa
