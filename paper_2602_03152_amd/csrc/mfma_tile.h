// The attention tile engine shared by the stand-alone attention kernels and the fused selection +
// attention kernel (paper Sec. 4.2, eq. fac_output; bf16 caches): 16 cached rows at a time, both
// products of a tile on the matrix cores, a running softmax per query head of the GQA group.
//
//   logits  C[row][head] = K_tile (16 rows x 128 dims) . Q^T: four v_mfma_f32_16x16x32_bf16; lane
//           (lo = lane mod 16, hi = lane / 16) supplies chunks hi, hi+4, hi+8, hi+12 (16 bytes each) of
//           K row lo and receives the logits of rows 4hi .. 4hi+3 for query head lo;
//   output  O[head][dim] += P (16 heads x 16 rows) . V_tile (16 rows x 128 dims): the lane's four
//           weights are already where the A operand wants them (head lo, rows 4hi .. 4hi+3).  The B
//           operand wants, per lane, the same four rows at ONE head dim: lane (lo, hi) loads 16 bytes
//           (dims 8lo .. 8lo+7) of V rows 4hi .. 4hi+3, and MFMA j of eight takes dim 8lo + j of each:
//           two byte permutes per MFMA.  Its result column lo is head dim 8lo + j, its rows 4hi .. 4hi+3
//           are query heads 4hi .. 4hi+3.
// The weights are float32 numbers in [0, 1]; the matrix cores take bf16.  Each weight goes in as
// hi + lo, hi = its top 16 bits, lo = the top 16 bits of the exact remainder: k-slots 0-3 of the 32-deep
// MFMA carry the hi parts, slots 4-7 the lo parts, against the same four V values twice.  What is
// dropped is below 2^-16 of the weight; V is bf16 already, products are exact, sums float32.
#pragma once

#include "attend_common.h"

namespace fasa {

struct TileKV { uint4 kc[4], vr[4]; };   // one lane's share of a tile: 4 chunks of its K row, 4 V rows x 16 bytes

// G: query heads per KV head (1 .. 8; the tile is padded to 16 heads, lanes lo >= G carry zeros)
template <int G>
struct MfmaTile {
  bf16x8_t qb[4];        // B operands of the logits: Q^T, column lo, k-slots (hi, 0..7) of MFMA i = dims 8(hi+4i)..+7
  f32x4_t oc[8];         // oc[j][e]: weighted V of query head 4hi + e at head dim 8lo + j
  float m_run, l_run;    // of query head lo (log2 domain); l_run over this lane's rows only until finish()

  __device__ __forceinline__ void load_q(const uint16_t* q_group /* [G][128] */, int lo, int hi) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4 x = make_uint4(0, 0, 0, 0);
      if (lo < G) x = *reinterpret_cast<const uint4*>(q_group + (size_t)lo * kHeadDim + 8 * (hi + 4 * i));
      qb[i] = __builtin_bit_cast(bf16x8_t, x);
    }
  }
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int j = 0; j < 8; ++j) oc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    m_run = kNegBig;
    l_run = 0.f;
  }
  // scaled logits (log2 domain) of rows 4hi .. 4hi+3 of the tile for query head lo
  __device__ __forceinline__ void logits(const TileKV& kv, float scale_log2e, float (&sv)[4]) const {
    // The scaled logit is rounded once and that rounded value is what the running maximum and the
    // exponent see: the scaling is never fused into the subtraction of the maximum (the weight of
    // the maximal row must be exactly 1).
#pragma clang fp contract(off)
    f32x4_t c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};   // two chains of two: half the latency
    c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv.kc[0]), qb[0], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv.kc[1]), qb[1], c1, 0, 0, 0);
    c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv.kc[2]), qb[2], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv.kc[3]), qb[3], c1, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 4; ++e) sv[e] = (c0[e] + c1[e]) * scale_log2e;
  }
  // Folds the tile into the running softmax: rows with valid[e] false get weight 0.  scs_wave: 16 floats
  // of LDS owned by this wave.
  __device__ __forceinline__ void accumulate(const TileKV& kv, const float (&sv)[4], const bool (&valid)[4],
                                             float* scs_wave, int lo, int hi) {
#pragma clang fp contract(off)
    float mx = kNegBig;
#pragma unroll
    for (int e = 0; e < 4; ++e) mx = valid[e] ? fmaxf(mx, sv[e]) : mx;
    mx = xor32_max(xor16_max(mx));
    const float m_new = fmaxf(m_run, mx);
    const float sc = exp2f(m_run - m_new);
    m_run = m_new;
    uint32_t ph[4], pl[4];
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float pv = valid[e] ? exp2f(sv[e] - m_new) : 0.f;
      psum += pv;
      ph[e] = __float_as_uint(pv) & 0xffff0000u;
      pl[e] = __float_as_uint(pv - __uint_as_float(ph[e]));      // exact; its own top 16 bits go in
    }
    l_run = fmaf(l_run, sc, psum);
    // A operand: k-slots (hi, 0..3) = hi parts of rows 4hi .. 4hi+3, (hi, 4..7) = lo parts
    const uint4 aw = make_uint4(__builtin_amdgcn_perm(ph[1], ph[0], 0x07060302u), __builtin_amdgcn_perm(ph[3], ph[2], 0x07060302u),
                                __builtin_amdgcn_perm(pl[1], pl[0], 0x07060302u), __builtin_amdgcn_perm(pl[3], pl[2], 0x07060302u));
    const bf16x8_t pa = __builtin_bit_cast(bf16x8_t, aw);
    // The running sums only need rescaling when some head's maximum moved in this tile - after the first
    // few tiles of a list that is rare, and the whole exchange (the factor of head lo has to reach the
    // lanes that hold head lo's sums, through LDS) and 32 multiplies are skipped: a wave-uniform test.
    if (__ballot(sc != 1.0f) != 0ull) {
      if (hi == 0) scs_wave[lo] = sc;
      // same wave writes and reads: LDS operations of a wave complete in order; the fences only keep the
      // compiler from moving the accesses across
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const float4 s4 = *reinterpret_cast<const float4*>(scs_wave + 4 * hi);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();   // read before the next tile overwrites it
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        oc[j][0] *= s4.x; oc[j][1] *= s4.y; oc[j][2] *= s4.z; oc[j][3] *= s4.w;
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;   // which half of word j / 2
      const uint32_t w0 = j < 2 ? kv.vr[0].x : j < 4 ? kv.vr[0].y : j < 6 ? kv.vr[0].z : kv.vr[0].w;
      const uint32_t w1 = j < 2 ? kv.vr[1].x : j < 4 ? kv.vr[1].y : j < 6 ? kv.vr[1].z : kv.vr[1].w;
      const uint32_t w2 = j < 2 ? kv.vr[2].x : j < 4 ? kv.vr[2].y : j < 6 ? kv.vr[2].z : kv.vr[2].w;
      const uint32_t w3 = j < 2 ? kv.vr[3].x : j < 4 ? kv.vr[3].y : j < 6 ? kv.vr[3].z : kv.vr[3].w;
      const uint32_t b01 = __builtin_amdgcn_perm(w1, w0, sel), b23 = __builtin_amdgcn_perm(w3, w2, sel);
      const bf16x8_t vb = __builtin_bit_cast(bf16x8_t, make_uint4(b01, b23, b01, b23));
      oc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vb, oc[j], 0, 0, 0);
    }
  }
  // The wave's totals to LDS: sm_m_wave, sm_l_wave [G]; sm_o_wave [G][128].  (A block barrier must follow
  // before another wave reads them.)
  __device__ __forceinline__ void finish(float* sm_m_wave, float* sm_l_wave, float* sm_o_wave, int lo, int hi) {
    l_run = xor32_sum(xor16_sum(l_run));
    if (hi == 0 && lo < G) { sm_m_wave[lo] = m_run; sm_l_wave[lo] = l_run; }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int g = 4 * hi + e;
      if (g < G) {
        float4* dst = reinterpret_cast<float4*>(sm_o_wave + g * kHeadDim + 8 * lo);
        dst[0] = make_float4(oc[0][e], oc[1][e], oc[2][e], oc[3][e]);
        dst[1] = make_float4(oc[4][e], oc[5][e], oc[6][e], oc[7][e]);
      }
    }
  }
};

// Workgroup totals from the four waves' finish() output, for thread (query head g, 4 head dims d4):
// max, sum of weights at that max, weighted V.  sm_m, sm_l: [4][G]; sm_o: [4][G][128].
template <int G>
__device__ __forceinline__ void tile_wg_totals(const float* sm_m, const float* sm_l, const float* sm_o, int g, int d4,
                                               float& mn, float& ls, float4& a) {
  mn = sm_m[g];
#pragma unroll
  for (int w = 1; w < 4; ++w) mn = fmaxf(mn, sm_m[w * G + g]);
  ls = 0.f;
  a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float sc = exp2f(sm_m[w * G + g] - mn);
    ls = fmaf(sm_l[w * G + g], sc, ls);
    const float4 sw = *reinterpret_cast<const float4*>(sm_o + ((size_t)(w * G + g)) * kHeadDim + 4 * d4);
    a.x = fmaf(sw.x, sc, a.x); a.y = fmaf(sw.y, sc, a.y);
    a.z = fmaf(sw.z, sc, a.z); a.w = fmaf(sw.w, sc, a.w);
  }
}

}  // namespace fasa
