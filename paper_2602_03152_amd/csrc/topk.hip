// TopK-I (paper Sec. 4.1): index set of the B largest scores of each (b,h) row.
//
// Radix select on the order-preserving 32-bit key of the float32 score, ties towards the
// lower token index:
//   level 0  the per-row histogram of the top 12 key bits (built by the scoring kernel or by
//            hist_kernel) fixes the threshold bin: bins above it hold fewer than B tokens, bins
//            from it upwards at least B;
//   filter   several workgroups per row stream S once; tokens above the threshold bin are winners
//            and go straight to T, tokens inside it are appended to a candidate list; positions
//            come from a block-wide prefix sum plus ONE 64-bit atomic per workgroup that reserves
//            both ranges;
//   final    the last workgroup of the row to finish resolves the candidates exactly: radix
//            select (first digit 12 bits, then 8 bits a pass) over the 52-bit composite
//            (low 20 key bits : ~index), which is unique per token, so exactly B - |winners|
//            candidates come out.  It then zeroes the row's histogram and counters, which leaves
//            the workspace clean for the next call.
#include "select_common.h"

namespace fasa {

// Slice of a row filtered by one workgroup: 2048 tokens, or 1024 when that still leaves at most two
// workgroups per CU (small problems are latency-bound: the shorter slice shortens every workgroup;
// large ones are throughput-bound: fewer, longer workgroups publish and queue less).
constexpr int kSelTokLong = 2048, kSelTokShort = 1024;
constexpr int kSelShortMaxBlocks = 2 * kAssumedCUs;
constexpr int kCandLds = 4096;                  // candidates resolved out of LDS; more: global reads

// 1-D grid of rows * nslices workgroups, nslices = ceil(N / TPB), TPB tokens per workgroup
template <int TPB>
__global__ __launch_bounds__(256) void select_kernel(const float* __restrict__ S,
                                                     uint32_t* __restrict__ hist,
                                                     RowCtl* __restrict__ ctl,
                                                     uint2* __restrict__ cand,
                                                     int32_t* __restrict__ T, int rows, int nslices,
                                                     int N_max, int n_cap, int budget_max, int t_pitch,
                                                     int Hkv, const int32_t* __restrict__ n_ctx_seq,
                                                     const int32_t* __restrict__ budget_seq, PageMap pm,
                                                     int32_t* __restrict__ Tslot) {
  constexpr int kSelTokPerBlock = TPB;
  constexpr int kSelPerThread = TPB / 256;
  __shared__ uint32_t wtot[8];
  __shared__ uint32_t bc[4];
  __shared__ uint32_t thr[3];  // threshold bin, tokens above it, tokens inside it
  __shared__ uint32_t dh[256];
  __shared__ uint2 lc[kCandLds];

  int row, slice;
  row_slice_of_block(rows, nslices, row, slice);
  const int t = threadIdx.x;
  const int N = seq_n_ctx(n_ctx_seq, row / Hkv, N_max);
  const int bsel = seq_bsel(budget_seq, row / Hkv, N, budget_max);
  const float* s = S + (size_t)row * n_cap;
  const int base = slice * kSelTokPerBlock;
  FASA_T_DECL(6);
  FASA_T(0);

  // ---- this workgroup's scores: loads go out first, the histogram work hides their latency ----
  float v[kSelPerThread];
#pragma unroll
  for (int it = 0; it < kSelPerThread / 4; ++it) {
    const int n0 = base + (it * 256 + t) * 4;
    if (n0 + 4 <= N) {
      const float4 x = *reinterpret_cast<const float4*>(s + n0);
      v[4 * it] = x.x; v[4 * it + 1] = x.y; v[4 * it + 2] = x.z; v[4 * it + 3] = x.w;
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) v[4 * it + k] = (n0 + k < N) ? s[n0 + k] : 0.f;
    }
  }

  // ---- threshold bin from the coarse histogram (every workgroup of the row redoes this) ----
  uint32_t* gh = hist + (size_t)row * kHistBins;
  if (t == 0) { thr[0] = 0; thr[1] = 0; thr[2] = 0; }
  {
    uint32_t hb[16];
    const uint4* hp = reinterpret_cast<const uint4*>(gh + t * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint4 x = hp[j];
      hb[4 * j] = x.x; hb[4 * j + 1] = x.y; hb[4 * j + 2] = x.z; hb[4 * j + 3] = x.w;
    }
    find_bin_256<16>(hb, (uint32_t)bsel, wtot, thr);   // its first barrier orders the zeroing of thr
  }
  const uint32_t tbin = thr[0];
  const uint32_t n_above = thr[1];
  FASA_T(1);

  // ---- classify, then one position range per workgroup and counter ----
  uint32_t key[kSelPerThread];
  uint32_t win = 0, cnd = 0;  // bit k set: this thread's k-th token is a winner / candidate
#pragma unroll
  for (int k = 0; k < kSelPerThread; ++k) {
    const int n = base + ((k >> 2) * 256 + t) * 4 + (k & 3);
    key[k] = score_key(v[k]);
    const uint32_t bin = key[k] >> kKeyLowBits;
    const bool ok = n < N;
    win |= (ok && bin > tbin) ? (1u << k) : 0u;
    cnd |= (ok && bin == tbin) ? (1u << k) : 0u;
  }
  // paged cache: the pool slots of this thread's tokens are looked up now, all loads together and
  // before any store (a load issued after stores would wait for every one of them to be acknowledged)
  int32_t* srow = Tslot ? Tslot + (size_t)row * t_pitch : nullptr;
  int slot[kSelPerThread];
  if (srow) {
#pragma unroll
    for (int k = 0; k < kSelPerThread; ++k)
      slot[k] = kv_slot(pm, row / Hkv, min(base + ((k >> 2) * 256 + t) * 4 + (k & 3), N - 1));
  }
  uint32_t pw, pc, tw, tc;
  block256_prefix2(__popc(win), __popc(cnd), wtot, pw, pc, tw, tc);
  if (t == 0) {
    // n_sel and n_cand are adjacent: one 64-bit add reserves both ranges in one round trip
    const unsigned long long old = atomicAdd(reinterpret_cast<unsigned long long*>(&ctl[row].n_sel),
                                             (unsigned long long)tw | ((unsigned long long)tc << 32));
    bc[0] = (uint32_t)old;
    bc[1] = (uint32_t)(old >> 32);
  }
  __syncthreads();
  FASA_T(2);
  uint32_t bw = bc[0] + pw, bcand = bc[1] + pc;
  int32_t* trow = T + (size_t)row * t_pitch;
  uint2* crow = cand + (size_t)row * n_cap;
#pragma unroll
  for (int k = 0; k < kSelPerThread; ++k) {
    const int n = base + ((k >> 2) * 256 + t) * 4 + (k & 3);
    // the bounds hold by construction of the histogram; they are re-checked so that a
    // histogram that does not match S can never turn into an out-of-range store
    if ((win & (1u << k)) && bw < (uint32_t)bsel) {
      trow[bw] = n;
      if (srow) srow[bw] = slot[k];
      ++bw;
    }
    // candidates are read by the row's last workgroup: published with agent-scope stores
    if ((cnd & (1u << k)) && bcand < (uint32_t)n_cap) st_agent(&crow[bcand++], make_uint2(key[k], (uint32_t)n));
  }

  // ---- last workgroup of the row resolves the threshold bin ----
  publish_barrier();
  if (t == 0) bc[2] = atomicAdd(&ctl[row].done_sel, 1u);
  __syncthreads();
  const bool last = bc[2] == (uint32_t)nslices - 1u;
  __syncthreads();
  FASA_T(3);
  FASA_T_PRINT(!last && t == 0 && row == 0 && slice == 0, "select blk0: thr %llu pos %llu ticket %llu (x10ns)\n",
               FASA_T_D(1, 0), FASA_T_D(2, 1), FASA_T_D(3, 2));
  if (!last) return;
  // the candidates are exactly the tokens of the threshold bin: their number is in the histogram
  const int n_cand = (int)min(thr[2], (uint32_t)n_cap);
  const int need = max(0, min(bsel - (int)n_above, n_cand));
  if (t == 0) bc[3] = 0;
  const bool in_lds = n_cand <= kCandLds;
  if (in_lds) {
    // four loads per thread in flight: up to 1024 candidates cost one memory round trip
    for (int i0 = 0; i0 < n_cand; i0 += 4 * 256) {
      uint2 c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) c[u] = ld_agent(&crow[min(i0 + u * 256 + t, n_cand - 1)]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i0 + u * 256 + t < n_cand) lc[i0 + u * 256 + t] = c[u];
    }
  }
  __syncthreads();
  FASA_T(4);
  // with <= 2048 candidates the upper half of lc is free: 4096 counters for a 12-bit first digit
  uint32_t* dhw = n_cand <= kCandLds / 2 ? reinterpret_cast<uint32_t*>(lc + kCandLds / 2) : nullptr;
  int32_t* sout = srow ? srow + n_above : nullptr;
  if (in_lds) resolve_candidates<false, 256, 52>(lc, n_cand, need, trow + n_above, dh, wtot, bc, dhw, sout, pm, row / Hkv);
  else resolve_candidates<true, 256, 52>(crow, n_cand, need, trow + n_above, dh, wtot, bc, nullptr, sout, pm, row / Hkv);
  FASA_T(5);
  FASA_T_PRINT(t == 0 && row == 0, "select last(row0,slice %d): thr %llu pos %llu ticket %llu candload %llu resolve %llu ncand %d need %d (x10ns)\n",
               slice, FASA_T_D(1, 0), FASA_T_D(2, 1), FASA_T_D(3, 2), FASA_T_D(4, 3), FASA_T_D(5, 4), n_cand, need);

  // leave the row's histogram and counters zeroed for the next call
  {
    uint4* hp = reinterpret_cast<uint4*>(gh + t * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) hp[j] = make_uint4(0, 0, 0, 0);
    if (t == 0) { ctl[row].n_sel = 0; ctl[row].n_cand = 0; ctl[row].done_sel = 0; }
  }
}

// budget >= N: every token is selected
__global__ __launch_bounds__(256) void select_all_kernel(int32_t* __restrict__ T, int N, int Hkv,
                                                         PageMap pm, int32_t* __restrict__ Tslot) {
  const int row = blockIdx.y;
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n < N) {
    T[(size_t)row * N + n] = n;
    if (Tslot) Tslot[(size_t)row * N + n] = kv_slot(pm, row / Hkv, n);
  }
}

// zeroes the histogram and the row counters: 1-D grid, one uint4 per thread
__global__ __launch_bounds__(256) void ws_clear_kernel(uint4* __restrict__ p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_select(const fasa_shape& s, const float* S, const uint32_t* hist, RowCtl* ctl,
                         uint2* cand, int32_t* T, hipStream_t st, RaggedLens rl, PageMap pm,
                         int32_t* Tslot) {
  const int rows = s.batch * s.n_kv_heads;
  const bool ragged = rl.n_ctx != nullptr || rl.budget != nullptr;
  if (s.budget >= s.n_ctx && !ragged) {
    dim3 grid((s.n_ctx + 255) / 256, rows), block(256);
    return launch("fasa_select_all", select_all_kernel, grid, block, st, T, s.n_ctx, s.n_kv_heads, pm, Tslot);
  }
  const int t_pitch = s.budget < s.n_ctx ? s.budget : s.n_ctx;
  const int n_short = (s.n_ctx + kSelTokShort - 1) / kSelTokShort;
  if ((long long)rows * n_short <= kSelShortMaxBlocks)
    return launch("fasa_select", select_kernel<kSelTokShort>, dim3(rows * n_short), dim3(256), st, S,
                  const_cast<uint32_t*>(hist), ctl, cand, T, rows, n_short, s.n_ctx, s.n_cap, s.budget,
                  t_pitch, s.n_kv_heads, rl.n_ctx, rl.budget, pm, Tslot);
  const int nslices = (s.n_ctx + kSelTokLong - 1) / kSelTokLong;
  return launch("fasa_select", select_kernel<kSelTokLong>, dim3(rows * nslices), dim3(256), st, S,
                const_cast<uint32_t*>(hist), ctl, cand, T, rows, nslices, s.n_ctx, s.n_cap, s.budget,
                t_pitch, s.n_kv_heads, rl.n_ctx, rl.budget, pm, Tslot);
}

hipError_t launch_ws_clear(const fasa_shape& s, uint32_t* hist, RowCtl* ctl, hipStream_t st) {
  // histogram and counters are adjacent in the workspace: [hist | ctl]
  const size_t bytes = (size_t)((char*)(ctl + s.batch * s.n_kv_heads) - (char*)hist);
  const size_t n16 = bytes / 16;
  return launch("fasa_ws_clear", ws_clear_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), st,
                (uint4*)hist, n16);
}

}  // namespace fasa
