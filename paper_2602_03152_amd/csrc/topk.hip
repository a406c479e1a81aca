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
#include "fasa_device.h"
#include "fasa_internal.h"

namespace fasa {

// Slice of a row filtered by one workgroup: 2048 tokens, or 1024 when that still leaves at most two
// workgroups per CU (small problems are latency-bound: the shorter slice shortens every workgroup;
// large ones are throughput-bound: fewer, longer workgroups publish and queue less).
constexpr int kSelTokLong = 2048, kSelTokShort = 1024;
constexpr int kSelShortMaxBlocks = 512;
constexpr int kCandLds = 4096;                  // candidates resolved out of LDS; more: global reads

__device__ __forceinline__ unsigned long long cand_composite(uint2 c) {
  return ((unsigned long long)(c.x & ((1u << kKeyLowBits) - 1u)) << 32) | (unsigned long long)(~c.y);
}

// Block-wide search in a 4096-bin histogram of which thread t holds bins 16t .. 16t+15 in hb[]:
// the bin b with  (entries in bins above b) < need <= (entries in bins >= b).  All 256 threads
// call; out[0..2] = b, entries above it, entries inside it (LDS; zero if need exceeds the total,
// the caller presets them).  Ends with a block barrier.
__device__ __forceinline__ void find_bin_256x16(const uint32_t* hb, uint32_t need, uint32_t* wtot,
                                                uint32_t* out) {
  const int t = threadIdx.x;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) mine += hb[j];
  const uint32_t incl = block256_suffix_sum(mine, wtot);
  uint32_t cum = incl - mine;
  const bool owner = cum < need && need <= incl;   // true for exactly one thread of the block
  // branch-free scan of the 16 bins from the top; the one hit is kept in registers
  uint32_t bj = 0, ba = 0, bn = 0;
#pragma unroll
  for (int j = 15; j >= 0; --j) {
    const bool hit = cum < need && cum + hb[j] >= need;
    bj = hit ? (uint32_t)j : bj;
    ba = hit ? cum : ba;
    bn = hit ? hb[j] : bn;
    cum += hb[j];
  }
  if (owner) {
    out[0] = (uint32_t)(t * 16) + bj;
    out[1] = ba;
    out[2] = bn;
  }
  __syncthreads();
}

// Exact selection of the `need` largest composites among cand[0..n).  Whole block participates.
// SHARED_SRC: the list lives in global memory and was written by other workgroups.
// dhw: LDS scratch of 4096 counters, or null.  With it the first pass takes the top 12 bits of the
// composite at once, which for a few hundred candidates almost always isolates the boundary
// candidate, so that no second pass is needed; without it every pass takes 8 bits.
// out_slot (paged caches, else null): receives the pool slot of every token written to out.
template <bool SHARED_SRC, int NT>
__device__ void resolve_candidates(const uint2* cand, int n, int need, int32_t* out,
                                   uint32_t* dh /*256*/, uint32_t* wtot /*NT/64*/,
                                   uint32_t* bc /*4: digit, need, count, out counter*/,
                                   uint32_t* dhw, int32_t* out_slot, const PageMap& pm, int b) {
  const int t = threadIdx.x;
  const uint32_t out_cap = (uint32_t)need;  // never write past the row's share of T
  unsigned long long prefix = 0;
  int shift = 52;            // the composite has 52 significant bits: digits at 44, 36, ..., 4, 0
  // The list is walked four entries per thread at a time, the four reads issued together (one LDS
  // or memory round trip per chunk instead of one per entry); entry u of chunk i0 is i0 + u*NT + t.
  constexpr int CH = 4;
  auto load_chunk = [&](int i0, uint2 (&c)[CH]) {
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const int i = min(i0 + u * NT + t, n - 1);
      c[u] = SHARED_SRC ? ld_agent(&cand[i]) : cand[i];
    }
  };
#ifdef FASA_TRACE
  unsigned long long rt[5]; for (int i = 0; i < 5; ++i) rt[i] = wall_clock64();
  int npass = 0;
#endif
  if (need < n) {
    bool done = false;
    if (NT == 256 && dhw != nullptr) {
      shift = 40;            // 12-bit digit first, then 8-bit digits at 32, 24, ..., 0
      for (int i = t; i < kHistBins; i += NT) dhw[i] = 0;
      if (t == 0) { bc[0] = 0; bc[1] = 0; bc[2] = 0; }
      __syncthreads();
      for (int i0 = 0; i0 < n; i0 += CH * NT) {
        uint2 c[CH];
        load_chunk(i0, c);
#pragma unroll
        for (int u = 0; u < CH; ++u)
          if (i0 + u * NT + t < n) atomicAdd(&dhw[(uint32_t)(cand_composite(c[u]) >> 40)], 1u);
      }
      __syncthreads();
#ifdef FASA_TRACE
      rt[1] = wall_clock64();
#endif
      uint32_t hb[16];
      const uint4* hp = reinterpret_cast<const uint4*>(dhw + t * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint4 v = hp[j];
        hb[4 * j] = v.x; hb[4 * j + 1] = v.y; hb[4 * j + 2] = v.z; hb[4 * j + 3] = v.w;
      }
      find_bin_256x16(hb, (uint32_t)need, wtot, bc);
      prefix = bc[0];
      const uint32_t in_digit = bc[2];
      need -= (int)bc[1];
      done = (uint32_t)need == in_digit;     // everything under this prefix is a winner
      __syncthreads();                       // bc is rewritten by the passes below
#ifdef FASA_TRACE
      rt[2] = wall_clock64();
#endif
    }
    while (!done && shift > 0) {
      const int width = shift >= 8 ? 8 : shift;   // the last digit is the 4 bits left over
      shift -= width;
#ifdef FASA_TRACE
      ++npass;
#endif
      if (t < 256) dh[t] = 0;
      __syncthreads();
      for (int i0 = 0; i0 < n; i0 += CH * NT) {
        uint2 c[CH];
        load_chunk(i0, c);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
          const unsigned long long cc = cand_composite(c[u]);
          if (i0 + u * NT + t < n && (cc >> (shift + width)) == prefix)
            atomicAdd(&dh[(uint32_t)(cc >> shift) & ((1u << width) - 1u)], 1u);
        }
      }
      __syncthreads();
      const uint32_t cnt = t < 256 ? dh[t] : 0u;
      const uint32_t incl = block_suffix_sum<NT>(cnt, wtot);
      const uint32_t excl = incl - cnt;
      if (t < 256 && excl < (uint32_t)need && (uint32_t)need <= incl) {
        bc[0] = (uint32_t)t;
        bc[1] = (uint32_t)need - excl;
        bc[2] = cnt;
      }
      __syncthreads();
      prefix = (prefix << width) | bc[0];
      need = (int)bc[1];
      const uint32_t in_digit = bc[2];
      // no barrier needed here: bc is next written three barriers into the following pass
      if ((uint32_t)need == in_digit) break;  // everything under this prefix is a winner
    }
  } else {
    shift = 52;  // take all: (c >> 52) == 0 >= 0
  }
#ifdef FASA_TRACE
  rt[3] = wall_clock64();
#endif
  // output: one position atomic per wave and chunk (ballots give every taken entry its offset)
  for (int i0 = 0; i0 < n; i0 += CH * NT) {
    uint2 c[CH];
    load_chunk(i0, c);
    unsigned long long m[CH];
    uint32_t taken = 0;
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      m[u] = __ballot(i0 + u * NT + t < n && (cand_composite(c[u]) >> shift) >= prefix);
      taken += (uint32_t)__popcll(m[u]);
    }
    int sl[CH];
    if (out_slot) {   // paged cache: where the rows live; looked up before the stores below
#pragma unroll
      for (int u = 0; u < CH; ++u) sl[u] = kv_slot(pm, b, (int)(c[u].y & 0x7fffffffu));
    }
    uint32_t pos = 0;
    if (lane_id() == 0 && taken) pos = atomicAdd(&bc[3], taken);
    pos = (uint32_t)__builtin_amdgcn_readfirstlane((int)pos);
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const uint32_t mine = pos + __builtin_amdgcn_mbcnt_hi((uint32_t)(m[u] >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((uint32_t)m[u], 0u));
      if (((m[u] >> lane_id()) & 1ull) && mine < out_cap) {
        out[mine] = (int32_t)c[u].y;
        if (out_slot) out_slot[mine] = sl[u];
      }
      pos += (uint32_t)__popcll(m[u]);
    }
  }
#ifdef FASA_TRACE
  rt[4] = wall_clock64();
  if (t == 0 && blockIdx.x < 64) printf("resolve: widehist %llu findbin %llu passes(%d) %llu output %llu (x10ns)\n", rt[1]-rt[0], rt[2]-rt[1], npass, rt[3]-rt[2], rt[4]-rt[3]);
#endif
}

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
#ifdef FASA_TRACE
  unsigned long long tt[8]; for (int i = 0; i < 8; ++i) tt[i] = 0; tt[0] = wall_clock64();
#endif

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
    find_bin_256x16(hb, (uint32_t)bsel, wtot, thr);   // its first barrier orders the zeroing of thr
  }
  const uint32_t tbin = thr[0];
  const uint32_t n_above = thr[1];
#ifdef FASA_TRACE
  tt[1] = wall_clock64();
#endif

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
#ifdef FASA_TRACE
  tt[2] = wall_clock64();
#endif
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
#ifdef FASA_TRACE
  tt[3] = wall_clock64();
  if (!last && t == 0 && row == 0 && slice == 0) printf("select blk0: thr %llu pos %llu ticket %llu (x10ns)\n", tt[1]-tt[0], tt[2]-tt[1], tt[3]-tt[2]);
#endif
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
#ifdef FASA_TRACE
  tt[4] = wall_clock64();
#endif
  // with <= 2048 candidates the upper half of lc is free: 4096 counters for a 12-bit first digit
  uint32_t* dhw = n_cand <= kCandLds / 2 ? reinterpret_cast<uint32_t*>(lc + kCandLds / 2) : nullptr;
  int32_t* sout = srow ? srow + n_above : nullptr;
  if (in_lds) resolve_candidates<false, 256>(lc, n_cand, need, trow + n_above, dh, wtot, bc, dhw, sout, pm, row / Hkv);
  else resolve_candidates<true, 256>(crow, n_cand, need, trow + n_above, dh, wtot, bc, nullptr, sout, pm, row / Hkv);
#ifdef FASA_TRACE
  tt[5] = wall_clock64();
  if (t == 0 && row == 0) printf("select last(row0,slice %d): thr %llu pos %llu ticket %llu candload %llu resolve %llu ncand %d need %d (x10ns)\n", slice, tt[1]-tt[0], tt[2]-tt[1], tt[3]-tt[2], tt[4]-tt[3], tt[5]-tt[4], n_cand, need);
#endif

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
