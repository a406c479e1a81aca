// Shared by the attention kernels (paper Sec. 4.2): the merge of a row's split partials into O.
#pragma once

#include "fasa_device.h"
#include "fasa_internal.h"
#include "fasa_trace.h"

namespace fasa {

constexpr float kNegBig = -1.0e30f;       // finite stand-in for -inf (keeps exp2 arguments finite)
constexpr int kMaxSplitsLds = 256;        // most splits per row the merging workgroup can weight

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load that is coherent at agent scope (served from the coherence point like an agent-scope
// atomic load, which the language only offers up to 8 bytes).  Two forms:
//  - agent_load_u128: a raw buffer load with the sc1 cache-policy bit.  An ordinary load to the
//    compiler, which counts it and places the waits itself.  base + 2 GB must cover every offset.
//  - agent_b128_issue / agent_b128_wait: the same load as inline assembly, for the merge of the split
//    partials, which keeps 32 of them in flight per thread and wants them issued exactly where they
//    are written (measured: the merge is 1.3 us faster per step than with compiler-scheduled buffer
//    loads).  The compiler does not count these: agent_b128_wait() must run before a destination is
//    read, and the build checks in the generated assembly that nothing touches one before
//    (paper_2602_03152_amd/build.py, check_untracked_loads).
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCachePolicySc1 = 16;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t agent_buffer(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ uint4 agent_load_u128(__amdgpu_buffer_rsrc_t rs, uint32_t byte_offset) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_offset, 0, kCachePolicySc1);
  return make_uint4(v.x, v.y, v.z, v.w);
}
typedef float f32x4_ld __attribute__((ext_vector_type(4)));
#ifndef FASA_MERGE_LOADS_TRACKED
__device__ __forceinline__ void agent_b128_issue(f32x4_ld& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
// waits for every outstanding vector memory operation of the wave; the eight destinations are tied
// to the statement so that no use of them can be moved above it
__device__ __forceinline__ void agent_b128_wait(f32x4_ld* x) {
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
               :: "memory");
}
#else
// The fallback for a toolchain on which the build's assembly check of the form above does not hold
// (build.py switches to it by itself): the language's own agent-scope loads, 8 bytes each, which the
// compiler counts.  Twice the requests: the merge is 0.5 - 0.9 us slower per step.
__device__ __forceinline__ void agent_b128_issue(f32x4_ld& dst, const void* p) {
  const float2* p2 = reinterpret_cast<const float2*>(p);
  const float2 a = ld_agent(p2), c = ld_agent(p2 + 1);
  dst = f32x4_ld{a.x, a.y, c.x, c.y};
}
__device__ __forceinline__ void agent_b128_wait(f32x4_ld*) {}
#endif

// One more split that the merging workgroup holds in its own LDS instead of the partial buffers
// (the fused step's threshold-bin tokens, attended by the merging workgroup itself).
struct ExtraSplit {
  const float* m;     // [G]     running maximum (log2 domain) per query head, or null: no extra split
  const float* l;     // [G]     sum of weights at that maximum
  const float* acc;   // [G][D]  weighted V at that maximum
  float* w;           // [G]     scratch: receives the split's merge weight
};

// Merges the split partials of one row into O.  Called by the row's last workgroup (all 256
// threads).  The partials were published by other workgroups with agent-scope stores and are read
// with agent-scope loads, the weighted-V partials 16 bytes at a time (agent_b128_issue): one CU's rate
// of load requests bounds this phase, so the wider the request the better (64 KB of fresh partials:
// 0.8 us with 16-byte loads against 1.4 us with 8-byte ones; an acquire fence followed by ordinary
// loads reads as fast but slows the other workgroups of the die down).  One memory round trip: every
// thread first requests the (max, sum) pairs its wave turns into weights, then ALL the weighted-V
// partials it will sum (they do not depend on the weights) - a split's partial is C = 32 G columns of
// four floats; thread t owns column t mod C of every P-th split, the P partitions meeting in LDS at
// the end.  `stride` is the distance between two rows' partials, in splits (>= n_splits).
// under_loads(): called by all threads once every load of the first round has been requested and
// before any is waited for - work placed there (it may fill the extra split) shares the merge's one
// memory round trip.  It must leave wsm, red and the extra split's arrays consistent behind a block
// barrier of its own if it writes them.
struct NothingUnderLoads { __device__ void operator()() const {} };
template <int G, typename UnderLoads = NothingUnderLoads, int RS = 32 /* splits in flight per thread and round */>
__device__ __forceinline__ void combine_row(const float* __restrict__ part_acc,
                                            const float* __restrict__ part_ml,
                                            float* __restrict__ O, int row, int b, int h, int Hq,
                                            int n_splits, int stride, float* wsm /* [G][kMaxSplitsLds] */,
                                            float* red /* [G] */, float* xbuf /* [P - 1][C][4] */,
                                            const ExtraSplit ex = {nullptr, nullptr, nullptr, nullptr},
                                            UnderLoads&& under_loads = NothingUnderLoads()) {
  constexpr int D = kHeadDim;
  constexpr int C = G * (D / 4);
  constexpr int P = 256 / C >= 4 ? 4 : (256 / C >= 2 ? 2 : 1);
  static_assert(RS % 8 == 0 && RS >= 8, "whole chunks of eight");
  constexpr int NG = (G + 3) / 4;
  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const size_t rbase = (size_t)row * stride * G;
  FASA_T_DECL(8);
  FASA_T(0);
  // (max, sum) pairs: wave w serves query heads w, w + 4; lane = split (+ 64 i).  Indices are
  // clamped, not tested: the duplicates are masked below.
  float2 ml[NG][kMaxSplitsLds / 64];
#pragma unroll
  for (int gi = 0; gi < NG; ++gi) {
    const int g = min(wave + 4 * gi, G - 1);
#pragma unroll
    for (int i = 0; i < kMaxSplitsLds / 64; ++i) {
      const int sp = min(lane + 64 * i, n_splits - 1);
      ml[gi][i] = ld_agent(reinterpret_cast<const float2*>(part_ml) + (rbase + (size_t)sp * G + g));
    }
  }

  const int part = t / C;                               // split partition of this thread
  const int c0 = t % C;
  const bool owner = t < P * C;
  const float4* pa = reinterpret_cast<const float4*>(part_acc + rbase * D);
  const int K = (n_splits + P - 1) / P;                 // splits per partition
  f32x4_ld x[RS];
  auto load_round = [&](int k0) {
#pragma unroll
    for (int u0 = 0; u0 < RS; u0 += 8) {
      if (k0 + u0 < K) {
#pragma unroll
        for (int u = u0; u < u0 + 8; ++u) {
          const int sp = min(part + P * (k0 + u), n_splits - 1);
          agent_b128_issue(x[u], pa + (size_t)sp * C + c0);
        }
      }
    }
  };
  load_round(0);
  FASA_T(4);
  under_loads();
  FASA_T(5);

#pragma unroll
  for (int gi = 0; gi < NG; ++gi) {
    const int g = wave + 4 * gi;
    const int gc = min(g, G - 1);
    float mx = ex.m ? ex.m[gc] : kNegBig;
#pragma unroll
    for (int i = 0; i < kMaxSplitsLds / 64; ++i)
      mx = (lane + 64 * i < n_splits) ? fmaxf(mx, ml[gi][i].x) : mx;
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxSplitsLds / 64; ++i) {
      const int sp = lane + 64 * i;
      const float wgt = sp < n_splits ? exp2f(ml[gi][i].x - mx) : 0.f;
      wsm[gc * kMaxSplitsLds + sp] = wgt;   // waves beyond the group rewrite the last head's own values
      sum = fmaf(ml[gi][i].y, wgt, sum);
    }
    sum = wave_sum(sum);
    if (ex.m) {
      const float wx = exp2f(ex.m[gc] - mx);
      sum = fmaf(ex.l[gc], wx, sum);
      if (lane == 0 && g < G) ex.w[g] = wx;
    }
    if (lane == 0 && g < G) red[g] = 1.0f / sum;
  }
  __syncthreads();
  FASA_T(1);

  const int gcol = min(c0 / (D / 4), G - 1);            // query head of this thread's column
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  int k0 = 0;
  do {   // K >= 1: the first round always runs
    if (k0) load_round(k0);
    // One wait for the whole round, on every path (which chunks were requested is a run-time matter;
    // that nothing touches a destination before this point must hold however the conditions fall).
#pragma unroll
    for (int u0 = 0; u0 < RS; u0 += 8) agent_b128_wait(&x[u0]);
    if (k0 == 0) FASA_T(6);
#pragma unroll
    for (int u0 = 0; u0 < RS; u0 += 8) {
      if (k0 + u0 < K) {
        // straight-line inside a chunk of 8 splits: the weight reads go out together.  A split
        // beyond the row's count has a finite (re-read) partial and weight 0.
        float wgt[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int sp = part + P * (k0 + u0 + u);
          const float w0 = wsm[gcol * kMaxSplitsLds + min(sp, kMaxSplitsLds - 1)];
          wgt[u] = sp < n_splits ? w0 : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          a.x = fmaf(x[u0 + u].x, wgt[u], a.x);
          a.y = fmaf(x[u0 + u].y, wgt[u], a.y);
          a.z = fmaf(x[u0 + u].z, wgt[u], a.z);
          a.w = fmaf(x[u0 + u].w, wgt[u], a.w);
        }
      }
    }
    k0 += RS;
  } while (k0 < K);
  FASA_T(2);
  FASA_T_PRINT(t == 0 && row == 0,
               "combine: requests %llu under-loads work %llu weights %llu partials arrive %llu sum %llu (x10ns) n_splits %d\n",
               FASA_T_D(4, 0), FASA_T_D(5, 4), FASA_T_D(1, 5), FASA_T_D(6, 1), FASA_T_D(2, 6), n_splits);
  if constexpr (P > 1) {
    float4* xb = reinterpret_cast<float4*>(xbuf);
    if (owner && part > 0) xb[(part - 1) * C + c0] = a;
    __syncthreads();
    if (owner && part == 0) {
#pragma unroll
      for (int pp = 1; pp < P; ++pp) {
        const float4 o = xb[(pp - 1) * C + c0];
        a.x += o.x; a.y += o.y; a.z += o.z; a.w += o.w;
      }
    }
  }
  if (owner && part == 0) {
    const int g = c0 / (D / 4), d4 = c0 % (D / 4);
    if (ex.m) {
      const float4 e = *reinterpret_cast<const float4*>(ex.acc + g * D + 4 * d4);
      const float wx = ex.w[g];
      a.x = fmaf(e.x, wx, a.x); a.y = fmaf(e.y, wx, a.y); a.z = fmaf(e.z, wx, a.z); a.w = fmaf(e.w, wx, a.w);
    }
    const float r = red[g];
    *reinterpret_cast<float4*>(O + ((size_t)b * Hq + (size_t)h * G + g) * D + 4 * d4) =
        make_float4(a.x * r, a.y * r, a.z * r, a.w * r);
  }
}

}  // namespace fasa
