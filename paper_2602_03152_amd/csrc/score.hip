// TIP scoring (paper Sec. 4.1): S = (sum over the GQA group of q^dom) . k^dom for every cached
// token, streamed from the FC-major packed copy Kp; optionally also the coarse per-row histogram
// of the order-preserving score keys that the selection stage starts from.
#include <type_traits>

#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

template <typename ET> struct ScoreTraits;
template <> struct ScoreTraits<uint16_t> { static constexpr int TPT = 4; };  // tokens per 16-byte load
template <> struct ScoreTraits<float> { static constexpr int TPT = 2; };

template <typename ET>
__device__ __forceinline__ void fma_pairs(const uint4& w, float qlo, float qhi, float* acc);

template <>
__device__ __forceinline__ void fma_pairs<uint16_t>(const uint4& w, float qlo, float qhi, float* acc) {
  acc[0] = fmaf(qhi, bf16_hi(w.x), fmaf(qlo, bf16_lo(w.x), acc[0]));
  acc[1] = fmaf(qhi, bf16_hi(w.y), fmaf(qlo, bf16_lo(w.y), acc[1]));
  acc[2] = fmaf(qhi, bf16_hi(w.z), fmaf(qlo, bf16_lo(w.z), acc[2]));
  acc[3] = fmaf(qhi, bf16_hi(w.w), fmaf(qlo, bf16_lo(w.w), acc[3]));
}

template <>
__device__ __forceinline__ void fma_pairs<float>(const uint4& w, float qlo, float qhi, float* acc) {
  acc[0] = fmaf(qhi, __uint_as_float(w.y), fmaf(qlo, __uint_as_float(w.x), acc[0]));
  acc[1] = fmaf(qhi, __uint_as_float(w.w), fmaf(qlo, __uint_as_float(w.z), acc[1]));
}

constexpr int kScoreFB = 16;  // FC planes in flight per thread

// 1-D grid of rows * nslices workgroups, nslices = ceil(N / (256 * TPT)).  One 16-byte load per
// thread per FC plane: a wave reads 1 KiB contiguous from each plane.  NB > 0: F == 8 * NB and all
// F plane loads of a thread are in flight at once, issued as straight-line code; NB == 0: any F,
// 16 planes at a time.
//
// Vector loads of a wave return in order, so nothing the K planes do not depend on may queue behind
// them, and a wait for an earlier load is only cheap if the loads after it are unconditional.  Order
// of issue, all of it branch-free and by every lane (so that nothing can be moved into a test):
//   1. this lane's column of the group's query heads (lane t: head dim t mod 128, up to 8 heads)
//      and one entry (one or two words) of the head's dominant list; neither depends on the other;
//   2. the K planes (lanes beyond the row's length re-read its first tokens);
//   3. wait for 1 only: group sum per head dim -> LDS, then lanes < F pick their FC's two
//      components.  This and the LDS clearing run under the latency of 2.
//
// APPEND (paper Alg. 2, Split + UpdateCache before scoring): the step's freshly decoded K/V row of
// every (b, h) joins the caches inside this kernel instead of a kernel of its own.  The row is token
// N - 1.  Every lane fetches one element of (k_new | v_new) with the loads of 1; the new key goes
// through LDS, lanes < F extract their FC's pair from it, the workgroup whose slice holds token
// N - 1 writes the pairs to the Kp planes and the whole row to K and V, and the one thread that owns
// the token replaces, in its registers, what it loaded from the (not yet written) planes.
//
// PAIR (a fasa_pairing): the list holds FC numbers i, stored at dims (i, i + d/2) or (2i, 2i + 1),
// or explicit dim pairs (two words per entry).
//
// HIST: 0 = scores only; 1 = also the per-row histogram of the top 12 bits of the score keys (what the
// stand-alone selection kernel starts from); 2 = the adaptive histogram of the fused step: bins of
// lin_bin(), placed by (mu, inv) from a fixed sample of 64 of the row's tokens and the row's budget - 16
// consecutive tokens at each quarter of the row, one group per wave, the same tokens in every
// workgroup of the row, so that all of them arrive at the same two numbers bit for bit.  The sample
// loads go out with the loads of 1 (they only need the plane addresses); the token an APPEND call is
// about to write is never sampled.  The workgroup of slice 0 leaves (mu, inv) in the row's counters for
// the selection kernel.
constexpr int kHistNone = 0, kHistKeyBits = 1, kHistAdaptive = 2;

template <typename ET, int HIST, int NB, bool APPEND, int PAIR>
__global__ __launch_bounds__(256) void score_kernel(const ET* __restrict__ q, ET* Kp,
                                                    const int32_t* __restrict__ fc_idx,
                                                    float* __restrict__ S,
                                                    uint32_t* __restrict__ hist, int rows,
                                                    int nslices, int Hq, int Hkv, int F, int N_max,
                                                    int n_cap, const int32_t* __restrict__ n_ctx_seq,
                                                    const ET* __restrict__ k_new,
                                                    const ET* __restrict__ v_new, ET* Kc, ET* Vc,
                                                    long long sb, long long sh, long long sn,
                                                    PageMap pm, RowCtl* __restrict__ ctl, int budget_max,
                                                    const int32_t* __restrict__ budget_seq) {
  constexpr int D = kHeadDim;
  constexpr int TPT = ScoreTraits<ET>::TPT;
  constexpr int NBINS = HIST == kHistAdaptive ? kLinBins : kHistBins;
  constexpr int NW = NB ? NB * 8 : kScoreFB;
  constexpr bool PAIRS = PAIR == FASA_PAIR_LIST;
  constexpr int PAIR_SHIFT = PAIR == FASA_PAIR_INTERLEAVED ? 1 : 0;       // FC number -> first dim
  constexpr int PAIR_ADD = PAIR == FASA_PAIR_INTERLEAVED ? 1 : D / 2;     // first dim -> second dim
  __shared__ float qsum[256];      // [t]: sum over the group of q[., t mod 128] (upper half: copies)
  __shared__ int32_t fcl[256];     // [t]: dims of list entry min(t, F - 1): lo (PAIRS: lo | hi << 8)
  __shared__ float2 qs[D / 2];
  __shared__ __align__(8) uint32_t lh[HIST ? NBINS : 2];
  __shared__ float2 sst[4];        // adaptive histogram: per wave, sum and sum of squares of its sample scores
  __shared__ ET knew[APPEND ? D : 1];          // the new key row
  __shared__ uint2 kpair[APPEND ? D / 2 : 1];  // per plane: the new key's (lo, hi) as stored in Kp

  int row, slice;
  row_slice_of_block(rows, nslices, row, slice);
  const int b = row / Hkv, h = row % Hkv;
  const int G = Hq / Hkv;
  const int t = threadIdx.x;
  const int N = seq_n_ctx(n_ctx_seq, b, N_max);
  if (slice * 256 * TPT >= N) return;   // whole workgroup beyond this sequence (ragged batches only)

  // ---- 1 ----
  const ET* qh = q + ((size_t)b * Hq + (size_t)h * G) * D + (t & (D - 1));
  ET qcol[kMaxGroup];
#pragma unroll
  for (int g = 0; g < kMaxGroup; ++g) qcol[g] = qh[(size_t)min(g, G - 1) * D];   // beyond the group: its last head, not added
  const int fe = h * F + min(t, F - 1);
  const int32_t fci = fc_idx[PAIRS ? 2 * fe : fe];
  int32_t fcj = 0;
  if constexpr (PAIRS) fcj = fc_idx[2 * fe + 1];
  ET newkv = ET(0);
  if constexpr (APPEND) newkv = (t < D ? k_new : v_new)[(size_t)row * D + (t & (D - 1))];
  // sample of the adaptive histogram: wave w scores tokens w * Q .. w * Q + 15, Q = a quarter of the
  // row rounded down to whole 64-byte lines.  Lane (token = lane mod 16, part = lane / 16) reads every
  // fourth plane starting at plane `part`: a quarter of the loads per lane, the four parts of a token's
  // score meeting through two lane swaps.
  using SmpT = typename std::conditional<sizeof(ET) == 2, uint32_t, uint2>::type;
  constexpr int NSMP = HIST == kHistAdaptive ? (NB ? NB * 2 : kScoreFB / 4) : 1;
  SmpT smp[NSMP];
  const int spart = (t >> 4) & 3;
  if constexpr (HIST == kHistAdaptive) {
    const int Ns = APPEND ? N - 1 : N;
    const int ps = max(min((t >> 6) * ((Ns >> 2) & ~15) + (t & 15), Ns - 1), 0);
    const ET* sp = Kp + ((size_t)row * F * n_cap + ps) * 2;
    const int nsf = NB ? NB * 8 : min(F, kScoreFB);
#pragma unroll
    for (int u = 0; u < NSMP; ++u)
      smp[u] = *reinterpret_cast<const SmpT*>(sp + (size_t)min(4 * u + spart, nsf - 1) * n_cap * 2);
  }
  // the appended token: which workgroup and thread own it, and which of the thread's tokens it is
  const int n_app = N - 1;
  const bool own_wg = APPEND && n_app / (256 * TPT) == slice;
  const bool own_thread = own_wg && (n_app - slice * 256 * TPT) / TPT == t;
  const int kin = n_app % TPT;

  // ---- 2 ----
  const int n0 = (slice * 256 + t) * TPT;
  const bool active = n0 < N;
  const ET* p = Kp + ((size_t)row * F * n_cap + (active ? n0 : 0)) * 2;
  const size_t plane = (size_t)n_cap * 2;
  uint4 w[NW];
  int nf = NB ? NW : min(F, kScoreFB);
#pragma unroll
  for (int u = 0; u < NW; ++u)
    if (NB || u < nf) w[u] = *reinterpret_cast<const uint4*>(p + (size_t)u * plane);

  // adaptive histogram: where the B-th largest of N normal scores lies, in standard deviations (needs no
  // memory: computed while the first loads are on their way)
  float zq = 0.f;
  if constexpr (HIST == kHistAdaptive)
    zq = normal_upper_quantile((float)seq_bsel(budget_seq, b, N, budget_max) / (float)N);
  // ---- 3 ----  sum_g (q_g . k) = (sum_g q_g) . k, g ascending
  {
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g) {
      float a;
      if constexpr (sizeof(ET) == 2) a = __uint_as_float((uint32_t)qcol[g] << 16);
      else a = qcol[g];
      sum += g < G ? a : 0.f;
    }
    qsum[t] = sum;
    // LDS indices below stay in range whatever the list holds
    if constexpr (PAIRS) fcl[t] = min(max(fci, 0), D - 1) | (min(max(fcj, 0), D - 1) << 8);
    else fcl[t] = min(max(fci, 0), D / 2 - 1) << PAIR_SHIFT;
    if constexpr (APPEND) {
      if (t < D) knew[t] = newkv;
    }
  }
  if constexpr (HIST != 0) {
    for (int i = t; i < NBINS; i += 256) lh[i] = 0;
  }
  __syncthreads();
  if (t < F) {
    const int dl = PAIRS ? fcl[t] & 255 : fcl[t];
    const int dh = PAIRS ? fcl[t] >> 8 : dl + PAIR_ADD;
    qs[t] = make_float2(qsum[dl], qsum[dh]);
    if constexpr (APPEND) {
      const ET lo = knew[dl], hi = knew[dh];
      if constexpr (sizeof(ET) == 2) kpair[t] = make_uint2((uint32_t)lo | ((uint32_t)hi << 16), 0u);
      else kpair[t] = make_uint2(__float_as_uint(lo), __float_as_uint(hi));
      if (own_wg) {
        ET* o = Kp + (((size_t)row * F + t) * n_cap + n_app) * 2;
        o[0] = lo;
        o[1] = hi;
      }
    }
  }
  __syncthreads();
  if constexpr (HIST == kHistAdaptive) {
    const int nsf = NB ? NB * 8 : min(F, kScoreFB);
    float xs = 0.f;
#pragma unroll
    for (int u = 0; u < NSMP; ++u) {
      const float2 qf = qs[min(4 * u + spart, nsf - 1)];
      float lo, hi;
      if constexpr (sizeof(ET) == 2) { lo = bf16_lo(smp[u]); hi = bf16_hi(smp[u]); }
      else { lo = __uint_as_float(smp[u].x); hi = __uint_as_float(smp[u].y); }
      xs = 4 * u + spart < nsf ? fmaf(qf.y, hi, fmaf(qf.x, lo, xs)) : xs;
    }
    xs = xor32_sum(xor16_sum(xs));   // every lane of a token now holds the token's whole sample score
    // per wave: mean of its 16 sample scores and their mean absolute deviation from it
    const float gm = row16_sum(xs) * (1.0f / 16.0f);
    const float gd = row16_sum(fabsf(xs - gm)) * (1.0f / 16.0f);
    if ((t & 63) == 0) sst[t >> 6] = make_float2(gm, gd);
  }
  float bin_mu = 0.f, bin_inv = 0.f;
  if constexpr (HIST == kHistAdaptive) {
    __syncthreads();   // the four waves' sample statistics (the K planes are still in flight)
    // Robust against a group that holds outliers (salient tokens score far above the rest): the
    // location is the median of the four group means, the scale the second smallest of the four group
    // deviations, rescaled to a standard deviation (E|x - mean of 16| = 0.7725 sigma; the second
    // smallest of four such estimates sits another 6 % lower).
    const float2 a0 = sst[0], a1 = sst[1], a2 = sst[2], a3 = sst[3];
    const float mmin = fminf(fminf(a0.x, a1.x), fminf(a2.x, a3.x)), mmax = fmaxf(fmaxf(a0.x, a1.x), fmaxf(a2.x, a3.x));
    const float loc = 0.5f * ((a0.x + a1.x) + (a2.x + a3.x) - mmin - mmax);   // mean of the middle two
    const float d01 = fminf(a0.y, a1.y), D01 = fmaxf(a0.y, a1.y), d23 = fminf(a2.y, a3.y), D23 = fmaxf(a2.y, a3.y);
    const float second = fminf(fmaxf(d01, d23), fminf(D01, D23));             // second smallest of four
    const float sigma = 1.373f * second;
    bin_mu = fmaf(zq, sigma, loc);
    bin_inv = sigma > 1e-30f ? 1.0f / sigma : 0.f;
  }
  // the planes did not hold the appended token yet: its owner takes the pairs from LDS
  auto patch = [&](uint4& wv, int pf) {
    const uint2 kp2 = kpair[pf];
    if constexpr (sizeof(ET) == 2) {
      wv.x = kin == 0 ? kp2.x : wv.x;
      wv.y = kin == 1 ? kp2.x : wv.y;
      wv.z = kin == 2 ? kp2.x : wv.z;
      wv.w = kin == 3 ? kp2.x : wv.w;
    } else {
      wv.x = kin == 0 ? kp2.x : wv.x;
      wv.y = kin == 0 ? kp2.y : wv.y;
      wv.z = kin == 1 ? kp2.x : wv.z;
      wv.w = kin == 1 ? kp2.y : wv.w;
    }
  };

  float acc[TPT];
#pragma unroll
  for (int k = 0; k < TPT; ++k) acc[k] = 0.f;
  if constexpr (NB > 0) {
    if constexpr (APPEND) {
      if (own_thread) {
#pragma unroll
        for (int u = 0; u < NW; ++u) patch(w[u], u);
      }
    }
#pragma unroll
    for (int u = 0; u < NW; ++u) {
      const float2 qf = qs[u];
      fma_pairs<ET>(w[u], qf.x, qf.y, acc);
    }
  } else {
    for (int f0 = 0;;) {
      if constexpr (APPEND) {
        if (own_thread) {
#pragma unroll
          for (int u = 0; u < kScoreFB; ++u)
            if (u < nf) patch(w[u], f0 + u);
        }
      }
#pragma unroll
      for (int u = 0; u < kScoreFB; ++u) {
        if (u < nf) {
          const float2 qf = qs[f0 + u];
          fma_pairs<ET>(w[u], qf.x, qf.y, acc);
        }
      }
      f0 += kScoreFB;
      if (f0 >= F) break;
      nf = min(F - f0, kScoreFB);
#pragma unroll
      for (int u = 0; u < kScoreFB; ++u)
        if (u < nf) w[u] = *reinterpret_cast<const uint4*>(p + (size_t)(f0 + u) * plane);
    }
  }
  if (active) {
    float* out = S + (size_t)row * n_cap + n0;
    if (n0 + TPT <= N) {
      if constexpr (TPT == 4) *reinterpret_cast<float4*>(out) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      else *reinterpret_cast<float2*>(out) = make_float2(acc[0], acc[1]);
    } else {
#pragma unroll
      for (int k = 0; k < TPT; ++k)
        if (n0 + k < N) out[k] = acc[k];
    }
    if constexpr (HIST == kHistKeyBits) {
#pragma unroll
      for (int k = 0; k < TPT; ++k)
        if (n0 + k < N) atomicAdd(&lh[score_key(acc[k]) >> kKeyLowBits], 1u);
    }
    if constexpr (HIST == kHistAdaptive) {
#pragma unroll
      for (int k = 0; k < TPT; ++k)
        if (n0 + k < N) atomicAdd(&lh[lin_bin(acc[k], bin_mu, bin_inv)], 1u);
    }
  }
  if constexpr (APPEND) {
    if (own_wg) {   // the whole new row to K (threads 0..127) and V (threads 128..255)
      ET* dst = (t < D ? Kc : Vc) + kv_row_offset(pm, b, n_app, sb, sn) + h * sh + (t & (D - 1));
      *dst = newkv;
    }
  }
  if constexpr (HIST == kHistAdaptive) {   // for the selection kernel (stored last: no load waits behind it)
    if (slice == 0 && t == 0) { ctl[row].bin_mu = bin_mu; ctl[row].bin_inv = bin_inv; }
  }
  if constexpr (HIST == kHistKeyBits) {
    __syncthreads();
    // all counters of the thread are read before the first is tested: one LDS round trip, not one each
    uint32_t* gh = hist + (size_t)row * kHistBins;
    uint32_t c[NBINS / 256];
#pragma unroll
    for (int k = 0; k < NBINS / 256; ++k) c[k] = lh[t + 256 * k];
#pragma unroll
    for (int k = 0; k < NBINS / 256; ++k)
      if (c[k]) atomicAdd(&gh[t + 256 * k], c[k]);
  }
  if constexpr (HIST == kHistAdaptive) {
    __syncthreads();
    // Neighbouring bins are flushed as ONE 64-bit add (a 32-bit counter never carries into the next):
    // the fine bins around the threshold are populated in runs, so this nearly halves the global
    // atomics, which are what the flush costs.  Thread t: bin pairs t and t + 256 of the row's
    // kLinBins = 1024 bins (a row's histogram region is kHistBins counters whichever binning fills it).
    static_assert(kLinBins == 1024, "two bin pairs per thread");
    unsigned long long* gh = reinterpret_cast<unsigned long long*>(hist + (size_t)row * kHistBins);
    const uint2 c0 = reinterpret_cast<const uint2*>(lh)[t], c1 = reinterpret_cast<const uint2*>(lh)[t + 256];
    if (c0.x | c0.y) atomicAdd(&gh[t], (unsigned long long)c0.x | ((unsigned long long)c0.y << 32));
    if (c1.x | c1.y) atomicAdd(&gh[t + 256], (unsigned long long)c1.x | ((unsigned long long)c1.y << 32));
  }
}

// Histogram of an existing score vector (stand-alone fasa_topk).  grid = (ceil(N / 4096), rows).
__global__ __launch_bounds__(256) void hist_kernel(const float* __restrict__ S,
                                                   uint32_t* __restrict__ hist, int N, int n_cap) {
  __shared__ uint32_t lh[kHistBins];
  const int row = blockIdx.y;
  const int t = threadIdx.x;
  for (int i = t; i < kHistBins; i += 256) lh[i] = 0;
  __syncthreads();
  const float* s = S + (size_t)row * n_cap;
  const int base = blockIdx.x * 4096;
  for (int it = 0; it < 4; ++it) {
    const int n0 = base + (it * 256 + t) * 4;
    if (n0 + 4 <= N) {
      const float4 v = *reinterpret_cast<const float4*>(s + n0);
      atomicAdd(&lh[score_key(v.x) >> kKeyLowBits], 1u);
      atomicAdd(&lh[score_key(v.y) >> kKeyLowBits], 1u);
      atomicAdd(&lh[score_key(v.z) >> kKeyLowBits], 1u);
      atomicAdd(&lh[score_key(v.w) >> kKeyLowBits], 1u);
    } else {
      for (int k = 0; k < 4; ++k)
        if (n0 + k < N) atomicAdd(&lh[score_key(s[n0 + k]) >> kKeyLowBits], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = hist + (size_t)row * kHistBins;
  uint32_t c[kHistBins / 256];
#pragma unroll
  for (int k = 0; k < kHistBins / 256; ++k) c[k] = lh[t + 256 * k];
#pragma unroll
  for (int k = 0; k < kHistBins / 256; ++k)
    if (c[k]) atomicAdd(&gh[t + 256 * k], c[k]);
}

template <typename ET, int HIST, int NB, bool APPEND, int PAIR>
static hipError_t launch_score_v(const fasa_shape& s, const void* q, void* Kp, const int32_t* fc_idx,
                                 float* S, uint32_t* hist, hipStream_t st, RaggedLens rl,
                                 const AppendArgs& ap, RowCtl* ctl) {
  const int rows = s.batch * s.n_kv_heads;
  const int per_block = 256 * ScoreTraits<ET>::TPT;
  const int nslices = (s.n_ctx + per_block - 1) / per_block;
  return launch(HIST ? "fasa_score_hist" : "fasa_score", score_kernel<ET, HIST, NB, APPEND, PAIR>,
                dim3(rows * nslices), dim3(256), st, (const ET*)q, (ET*)Kp, fc_idx, S, hist, rows, nslices,
                s.n_q_heads, s.n_kv_heads, s.n_fc, s.n_ctx, s.n_cap, rl.n_ctx, (const ET*)ap.k_new,
                (const ET*)ap.v_new, (ET*)ap.K, (ET*)ap.V, (long long)s.kv_stride_b, (long long)s.kv_stride_h,
                (long long)s.kv_stride_n, ap.pm, ctl, s.budget, rl.budget);
}

template <typename ET, int HIST, bool APPEND, int PAIR>
static hipError_t launch_score_f(const fasa_shape& s, const void* q, void* Kp, const int32_t* fc_idx,
                                 float* S, uint32_t* hist, hipStream_t st, RaggedLens rl,
                                 const AppendArgs& ap, RowCtl* ctl) {
  switch (s.n_fc) {   // the usual settings (an eighth to a half of the FCs) get straight-line loads
    case 8: return launch_score_v<ET, HIST, 1, APPEND, PAIR>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    case 16: return launch_score_v<ET, HIST, 2, APPEND, PAIR>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    case 24: return launch_score_v<ET, HIST, 3, APPEND, PAIR>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    case 32: return launch_score_v<ET, HIST, 4, APPEND, PAIR>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    default: return launch_score_v<ET, HIST, 0, APPEND, PAIR>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
  }
}

template <typename ET, int HIST, bool APPEND>
static hipError_t launch_score_h(const fasa_shape& s, const void* q, void* Kp, const int32_t* fc_idx,
                                 float* S, uint32_t* hist, hipStream_t st, RaggedLens rl,
                                 const AppendArgs& ap, RowCtl* ctl) {
  switch (s.pairing) {
    case FASA_PAIR_INTERLEAVED:
      return launch_score_f<ET, HIST, APPEND, FASA_PAIR_INTERLEAVED>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    case FASA_PAIR_LIST:
      return launch_score_f<ET, HIST, APPEND, FASA_PAIR_LIST>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
    default:
      return launch_score_f<ET, HIST, APPEND, FASA_PAIR_ROTATE_HALF>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
  }
}

template <typename ET, bool APPEND>
static hipError_t launch_score_a(const fasa_shape& s, const void* q, void* Kp, const int32_t* fc_idx,
                                 float* S, uint32_t* hist, hipStream_t st, RaggedLens rl,
                                 const AppendArgs& ap, RowCtl* ctl) {
  if (!hist) return launch_score_h<ET, kHistNone, APPEND>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
  if (ctl) return launch_score_h<ET, kHistAdaptive, APPEND>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
  return launch_score_h<ET, kHistKeyBits, APPEND>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
}

template <typename ET>
static hipError_t launch_score_t(const fasa_shape& s, const void* q, void* Kp, const int32_t* fc_idx,
                                 float* S, uint32_t* hist, hipStream_t st, RaggedLens rl,
                                 const AppendArgs& ap, RowCtl* ctl) {
  return ap.k_new ? launch_score_a<ET, true>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl)
                  : launch_score_a<ET, false>(s, q, Kp, fc_idx, S, hist, st, rl, ap, ctl);
}

hipError_t launch_score(const fasa_shape& s, const void* q, const void* Kp, const int32_t* fc_idx,
                        float* S, uint32_t* hist, hipStream_t st, RaggedLens rl, AppendArgs ap,
                        RowCtl* adaptive_ctl) {
  // Kp is only written when a row is appended (ap.k_new != nullptr)
  return s.dtype == FASA_BF16
             ? launch_score_t<uint16_t>(s, q, const_cast<void*>(Kp), fc_idx, S, hist, st, rl, ap, adaptive_ctl)
             : launch_score_t<float>(s, q, const_cast<void*>(Kp), fc_idx, S, hist, st, rl, ap, adaptive_ctl);
}

hipError_t launch_hist(const fasa_shape& s, const float* S, uint32_t* hist, hipStream_t st) {
  dim3 grid((s.n_ctx + 4095) / 4096, s.batch * s.n_kv_heads), block(256);
  return launch("fasa_hist", hist_kernel, grid, block, st, S, hist, s.n_ctx, s.n_cap);
}

}  // namespace fasa
