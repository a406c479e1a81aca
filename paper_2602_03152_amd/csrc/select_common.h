// Pieces of TopK-I (paper Sec. 4.1) shared by the stand-alone selection kernel and the fused
// selection + attention kernel: the block-wide search of the threshold bin in a histogram and the
// exact resolve of the threshold bin's candidates (ties towards the lower token index).
#pragma once

#include "fasa_device.h"
#include "fasa_internal.h"
#include "fasa_trace.h"

namespace fasa {

// A candidate is (order-preserving score key, token index).  Its composite sorts candidates the way
// the selection ranks tokens: larger key first, equal keys by lower index (the index is inverted).
// CB = significant bits of the composite:
//   52  all candidates share the top 12 key bits (bins of the exponent-based histogram): the low 20
//       key bits and the index decide;
//   64  candidates of an arbitrary score interval (bins of the adaptive histogram): the whole key.
template <int CB>
__device__ __forceinline__ unsigned long long cand_composite(uint2 c) {
  if constexpr (CB == 52)
    return ((unsigned long long)(c.x & ((1u << kKeyLowBits) - 1u)) << 32) | (unsigned long long)(~c.y);
  else
    return ((unsigned long long)c.x << 32) | (unsigned long long)(~c.y);
}

// Block-wide search in a histogram of 256 * PER bins of which thread t holds bins PER t .. PER t + PER - 1
// in hb[]: the bin b with  (entries in bins above b) < need <= (entries in bins >= b).  All 256 threads
// call; out[0..2] = b, entries above it, entries inside it (LDS; left as they are if need exceeds the
// total, the caller presets them).  Ends with a block barrier.
template <int PER>
__device__ __forceinline__ void find_bin_256(const uint32_t* hb, uint32_t need, uint32_t* wtot, uint32_t* out) {
  const int t = threadIdx.x;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) mine += hb[j];
  const uint32_t incl = block256_suffix_sum(mine, wtot);
  uint32_t cum = incl - mine;
  const bool owner = cum < need && need <= incl;   // true for exactly one thread of the block
  // branch-free scan of the thread's bins from the top; the one hit is kept in registers
  uint32_t bj = 0, ba = 0, bn = 0;
#pragma unroll
  for (int j = PER - 1; j >= 0; --j) {
    const bool hit = cum < need && cum + hb[j] >= need;
    bj = hit ? (uint32_t)j : bj;
    ba = hit ? cum : ba;
    bn = hit ? hb[j] : bn;
    cum += hb[j];
  }
  if (owner) {
    out[0] = (uint32_t)(t * PER) + bj;
    out[1] = ba;
    out[2] = bn;
  }
  __syncthreads();
}

// Exact selection of the `need` largest composites among cand[0..n).  Whole block participates.
// SHARED_SRC: the list lives in global memory and was written by other workgroups.
// dhw: LDS scratch of 4096 counters, or null.  With it the first pass takes the top 12 bits of the
// composite at once, which for a few hundred candidates of one exponent-based bin almost always isolates
// the boundary candidate, so that no second pass is needed; without it every pass takes 8 bits.
// out receives the token numbers of the taken candidates (at most `need`), in no particular order.
// out_slot (paged caches, else null): receives the pool slot of every token written to out.
// out_lds (or null): LDS copy of what the attention gathers by (the slot if out_slot is given, else the
// token number), same positions as out.
template <bool SHARED_SRC, int NT, int CB>
__device__ void resolve_candidates(const uint2* cand, int n, int need, int32_t* out,
                                   uint32_t* dh /*256*/, uint32_t* wtot /*NT/64*/,
                                   uint32_t* bc /*4: digit, need, count, out counter*/,
                                   uint32_t* dhw, int32_t* out_slot, const PageMap& pm, int b,
                                   int32_t* out_lds = nullptr) {
  const int t = threadIdx.x;
  const uint32_t out_cap = (uint32_t)need;  // never write past the row's share of T
  unsigned long long prefix = 0;
  int shift = CB;            // bits of the composite not yet decided
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
  FASA_T_DECL(5);
  FASA_T(0);
  if (need < n) {
    bool done = false;
    if (NT == 256 && dhw != nullptr) {
      shift = CB - 12;       // 12-bit digit first, then 8-bit digits
      for (int i = t; i < kHistBins; i += NT) dhw[i] = 0;
      if (t == 0) { bc[0] = 0; bc[1] = 0; bc[2] = 0; }
      __syncthreads();
      for (int i0 = 0; i0 < n; i0 += CH * NT) {
        uint2 c[CH];
        load_chunk(i0, c);
#pragma unroll
        for (int u = 0; u < CH; ++u)
          if (i0 + u * NT + t < n) atomicAdd(&dhw[(uint32_t)(cand_composite<CB>(c[u]) >> (CB - 12))], 1u);
      }
      __syncthreads();
      FASA_T(1);
      uint32_t hb[16];
      const uint4* hp = reinterpret_cast<const uint4*>(dhw + t * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint4 v = hp[j];
        hb[4 * j] = v.x; hb[4 * j + 1] = v.y; hb[4 * j + 2] = v.z; hb[4 * j + 3] = v.w;
      }
      find_bin_256<16>(hb, (uint32_t)need, wtot, bc);
      prefix = bc[0];
      const uint32_t in_digit = bc[2];
      need -= (int)bc[1];
      done = (uint32_t)need == in_digit;     // everything under this prefix is a winner
      __syncthreads();                       // bc is rewritten by the passes below
      FASA_T(2);
    }
    while (!done && shift > 0) {
      const int width = shift >= 8 ? 8 : shift;   // the last digit is whatever is left over
      const bool first = shift == 64;             // nothing decided yet: every candidate is in play
      shift -= width;
      if (t < 256) dh[t] = 0;
      __syncthreads();
      for (int i0 = 0; i0 < n; i0 += CH * NT) {
        uint2 c[CH];
        load_chunk(i0, c);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
          const unsigned long long cc = cand_composite<CB>(c[u]);
          const bool in_play = first || (cc >> ((shift + width) & 63)) == prefix;
          if (i0 + u * NT + t < n && in_play)
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
    shift = 63;   // take all: (c >> 63) >= 0
  }
  FASA_T(3);
  // output: one position atomic per wave and chunk (ballots give every taken entry its offset)
  for (int i0 = 0; i0 < n; i0 += CH * NT) {
    uint2 c[CH];
    load_chunk(i0, c);
    unsigned long long m[CH];
    uint32_t taken = 0;
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      m[u] = __ballot(i0 + u * NT + t < n && (cand_composite<CB>(c[u]) >> shift) >= prefix);
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
        if (out_lds) out_lds[mine] = out_slot ? sl[u] : (int32_t)c[u].y;
      }
      pos += (uint32_t)__popcll(m[u]);
    }
  }
  FASA_T(4);
  FASA_T_PRINT(t == 0 && blockIdx.x < 64, "resolve: widehist %llu findbin %llu passes %llu output %llu (x10ns)\n",
               FASA_T_D(1, 0), FASA_T_D(2, 1), FASA_T_D(3, 2), FASA_T_D(4, 3));
}

}  // namespace fasa
