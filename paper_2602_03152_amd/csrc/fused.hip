// TopK-I and FAC in one kernel (paper Sec. 4.1 - 4.2), by token-range ownership: the workgroup that
// classifies a slice of a row's scores attends at once over the winners it found there, so the
// selected set never travels through memory on its way to the attention, one kernel boundary and the
// serial tail of a stand-alone selection disappear, and the index set T is written on the side.
//
//   every workgroup (row, slice of at most TPB tokens):
//     1. loads its scores, the row's adaptive histogram (kLinBins bins of lin_bin, built by the scoring
//        kernel) and the two numbers that define the bins; finds the threshold bin: bins above it hold
//        fewer than B tokens, bins from it upwards at least B;
//     2. classifies its tokens: above the threshold bin = winner, inside it = candidate; winners go
//        to a list in LDS (what the gather needs: token number, or pool slot of a paged cache);
//     3. attends over its winners (16-row tiles, logits on the matrix cores, running softmax);
//        The adaptive bins leave a few dozen candidates per row.  While there are at most kFuseRich of
//        them (and at most kStashRecs in any one workgroup), the workgroup also runs its candidates
//        through the tiles - masked out of its softmax - and leaves each one's logits and V row in a
//        record: whether a candidate is selected is only known at the end, but then everything its
//        contribution needs is one load away;
//     4. writes its winners to T and its candidates to the row's candidate list (positions from one
//        64-bit atomic whose round trip runs under the gather of the first tile), publishes its
//        (max, sum, weighted V) partial and takes the row's ticket;
//   the row's last workgroup:
//     5. requests the candidates with their records and, in the same round trip, all partials; ranks
//        the candidates exactly by counting in LDS, writes the taken ones to T and folds their records
//        into one more partial.  Rows with more candidates (degenerate score distributions) resolve by
//        counting or by the radix resolve and gather the taken rows themselves;
//     6. merges all partials into O and leaves histogram and counters zeroed for the next call.
#include "mfma_tile.h"
#include "select_common.h"

namespace fasa {

constexpr int kFuseCandLds = 1024;    // candidates resolved out of LDS; more: read from global memory
constexpr int kFuseCountMax = 256;    // candidates ranked by counting; more: radix resolve
// kFuseRich (fasa_internal.h): candidates per row that get a record; a record is kRecLogits floats
// (one logit per query head of the group, log2 domain) and the candidate's V row
#ifndef FASA_FUSE_MERGE_IN_FLIGHT
#define FASA_FUSE_MERGE_IN_FLIGHT 32
#endif
constexpr int kFuseMergeInFlight = FASA_FUSE_MERGE_IN_FLIGHT;   // partials per thread in flight in the merge
constexpr int kStashRecs = 8;          // candidates of ONE workgroup that ride along with its winners
constexpr int kRecLogits = kMaxGroup;
constexpr size_t kRecRowBytes = (size_t)kFuseRich * (kRecLogits * 4 + kHeadDim * 2);
static_assert(kRecRowBytes == kFuseRecBytesPerRow, "workspace carve-up and kernel disagree");


// Rank of candidate i among the n candidates of an LDS list: how many of them sort before it (larger
// key, or equal key and lower index).  Composites are distinct, so ranks are a permutation of 0..n-1
// and "rank < need" takes exactly the `need` best.  32-bit compares only; the list is read eight
// entries at a time (one LDS round trip per eight).  Thread t serves candidate t / PARTS and counts
// the entries j = t % PARTS (mod PARTS); the PARTS partial counts of a candidate sit in adjacent lanes
// and are added with DPP moves.  Returns the rank in every one of the candidate's threads.
template <int PARTS>
__device__ __forceinline__ int rank_in_list(const uint2* lc, int n, int i) {
  const int t = threadIdx.x;
  const uint2 me = lc[min(i, n - 1)];
  int rank = 0;
  for (int j0 = t % PARTS; j0 < n; j0 += 8 * PARTS) {
    uint2 c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = lc[min(j0 + u * PARTS, n - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool before = c[u].x > me.x || (c[u].x == me.x && c[u].y < me.y);
      rank += (j0 + u * PARTS < n && before) ? 1 : 0;
    }
  }
  if constexpr (PARTS >= 2) rank += __builtin_amdgcn_update_dpp(0, rank, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
  if constexpr (PARTS >= 4) rank += __builtin_amdgcn_update_dpp(0, rank, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
  return rank;
}

template <int G, int TPB>
__global__ __launch_bounds__(256) void select_attend_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const float* __restrict__ S, uint32_t* __restrict__ hist, RowCtl* __restrict__ ctl,
    uint2* __restrict__ cand, int32_t* __restrict__ T, float* __restrict__ O, float* __restrict__ part_acc,
    float* __restrict__ part_ml, unsigned char* __restrict__ rec, int rows, int nslices, int slice_len, int Hq, int Hkv, int N_max,
    int n_cap, int budget_max, int t_pitch, long long sb, long long sh, long long sn, float scale_log2e,
    const int32_t* __restrict__ n_ctx_seq, const int32_t* __restrict__ budget_seq, PageMap pm) {
  constexpr int D = kHeadDim;
  constexpr int PT = TPB / 256;                               // tokens per thread
  constexpr int ACC_BYTES = 4 * G * D * 4;                    // [wave][G][D] floats
  constexpr int RES_BYTES = kFuseCandLds * 8 + kHistBins * 4; // candidate list + 4096 digit counters
  static_assert(RES_BYTES >= kFuseRich * 8 + (int)kRecRowBytes, "the records of a row fit the resolve scratch");
  constexpr int BIG = ACC_BYTES > RES_BYTES ? ACC_BYTES : RES_BYTES;
  __shared__ __align__(16) unsigned char big[BIG];            // tile sums, later the resolve's scratch
  __shared__ float sm_m[4][G], sm_l[4][G];
  __shared__ float red[G];
  __shared__ __align__(16) float ex_acc[G][D];                // the last workgroup's own split (candidates)
  __shared__ float ex_m[G], ex_l[G], ex_w[G];
  __shared__ uint32_t wtot[8];
  __shared__ uint32_t bc[4];
  __shared__ uint32_t thr[3];                                 // threshold bin, tokens above it, tokens inside it
  __shared__ uint32_t dh[256];
  __shared__ uint32_t ticket;
  __shared__ __align__(16) float scs[4][16];                  // per wave: rescale factor of each head's running sums
  __shared__ int32_t wl[TPB];                                 // what the gather reads: winners from the front
  __shared__ __align__(16) float cst_s[kStashRecs][kRecLogits];   // this workgroup's candidates: logits
  __shared__ __align__(16) uint4 cst_v[kStashRecs][16];           // ... and V rows, until their records are written
  float (*sm_o)[G][D] = reinterpret_cast<float (*)[G][D]>(big);
  // the merge's split weights live in `big` too: beyond the merge's own partition scratch (< 8 KB); the
  // candidate records staged there are consumed before the weights are written
  static_assert(BIG >= 8192 + G * kMaxSplitsLds * 4, "room for the split weights");
  float* wsm = reinterpret_cast<float*>(big + 8192);

  int row, slice;
  row_slice_of_block(rows, nslices, row, slice);
  const int b = row / Hkv, h = row % Hkv;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int lo = lane & 15, hi = lane >> 4;
  const int N = seq_n_ctx(n_ctx_seq, b, N_max);
  const int bsel = seq_bsel(budget_seq, b, N, budget_max);
  // slice_len <= TPB tokens per workgroup, a multiple of 16: the launch plan cuts a row into equal
  // slices, so that the grid fills the machine evenly whatever the row length
  const int base = slice * slice_len;
  if (base >= N) return;                                      // beyond this sequence (ragged batches only)
  const int n_end = min(N, base + slice_len);                 // this workgroup's tokens: base .. n_end - 1
  const int nvalid = (N + slice_len - 1) / slice_len;         // workgroups of this row that take part
  FASA_T_DECL(10);
  FASA_T(0);

  // ---- 1. loads: scores (S is n_cap long and n_cap a multiple of 64: a whole float4 is always there),
  // histogram, bin definition, queries; a paged cache also looks up where each of its tokens lives ----
  const float* s = S + (size_t)row * n_cap;
  float v[PT];
#pragma unroll
  for (int it = 0; it < PT / 4; ++it) {
    const int n0 = base + (it * 256 + t) * 4;
    const float4 x = *reinterpret_cast<const float4*>(s + (n0 < n_cap ? n0 : 0));
    v[4 * it] = x.x; v[4 * it + 1] = x.y; v[4 * it + 2] = x.z; v[4 * it + 3] = x.w;
  }
  uint32_t* gh = hist + (size_t)row * kHistBins;
  const uint4 h4 = *reinterpret_cast<const uint4*>(gh + 4 * t);
  const float bin_mu = ctl[row].bin_mu, bin_inv = ctl[row].bin_inv;
  MfmaTile<G> tile;
  tile.load_q(q + ((size_t)b * Hq + (size_t)h * G) * D, lo, hi);
  const bool paged = pm.table != nullptr;
  int slot[PT];
  if (paged) {
#pragma unroll
    for (int k = 0; k < PT; ++k)
      slot[k] = kv_slot(pm, b, min(base + ((k >> 2) * 256 + t) * 4 + (k & 3), N - 1));
  }
  if (t == 0) { thr[0] = 0; thr[1] = 0; thr[2] = 0; }
  {
    const uint32_t hb[4] = {h4.x, h4.y, h4.z, h4.w};
    find_bin_256<4>(hb, (uint32_t)bsel, wtot, thr);     // its first barrier orders the zeroing of thr
  }
  const uint32_t tbin = thr[0];
  const uint32_t n_above = thr[1];
  FASA_T(1);

  // ---- 2. classify; winners into the LDS list, then (while the row has few) the candidates ----
  uint32_t key[PT];
  uint32_t win = 0, cnd = 0;  // bit k set: this thread's k-th token is a winner / candidate
#pragma unroll
  for (int k = 0; k < PT; ++k) {
    const int n = base + ((k >> 2) * 256 + t) * 4 + (k & 3);
    key[k] = score_key(v[k]);
    const uint32_t bin = lin_bin(v[k], bin_mu, bin_inv);
    const bool ok = n < n_end;
    win |= (ok && bin > tbin) ? (1u << k) : 0u;
    cnd |= (ok && bin == tbin) ? (1u << k) : 0u;
  }
  uint32_t pw, pc, tw, tc;
  block256_prefix2(__popc(win), __popc(cnd), wtot, pw, pc, tw, tc);
  const int n_win = (int)min(tw, (uint32_t)TPB);
  const bool rich = thr[2] <= (uint32_t)kFuseRich;      // the same decision in every workgroup of the row
  const int n_ride = rich ? (int)min(min(tc, (uint32_t)kStashRecs), (uint32_t)(TPB - n_win)) : 0;
  const bool overflow = rich && tc > (uint32_t)n_ride;   // then the row's last workgroup gathers the taken rows itself
  const int n_list = n_win + n_ride;
  {
    uint32_t p = pw, pcn = tw + pc;
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const int n = base + ((k >> 2) * 256 + t) * 4 + (k & 3);
      if ((win & (1u << k)) && p < (uint32_t)TPB) wl[p++] = paged ? slot[k] : n;
      if ((cnd & (1u << k)) && pcn < (uint32_t)n_list) wl[pcn++] = paged ? slot[k] : n;
    }
  }
  __syncthreads();
  FASA_T(2);
  float* rec_s = reinterpret_cast<float*>(rec + (size_t)row * kRecRowBytes);                      // [kFuseRich][8]
  uint2* rec_v = reinterpret_cast<uint2*>(rec + (size_t)row * kRecRowBytes + kFuseRich * kRecLogits * 4);  // [kFuseRich][32]

  // ---- 3. attention over a list of rows; used for the winners and, by the last workgroup, for the
  // resolved candidates.  State per lane: query head lo, rows 4hi..4hi+3 of every tile. ----
  const int pshift = paged ? pm.shift : 31, pmask = paged ? (1 << pm.shift) - 1 : 0x7fffffff;
  const long long blk_stride = paged ? sb : 0;
  const int slot_max = paged ? (pm.n_pool << pm.shift) - 1 : N - 1;
  const uint16_t* Kb = K + (paged ? 0 : b * sb) + h * sh;
  const uint16_t* Vb = V + (paged ? 0 : b * sb) + h * sh + 8 * lo;

  // One tile = 16 list entries, both products on the matrix cores (mfma_tile.h).
  auto row_off = [&](int e) {
    const int sl = min(max(e, 0), slot_max);   // a stray entry can never become a stray address
    return (long long)(sl >> pshift) * blk_stride + (long long)(sl & pmask) * sn;
  };
  // idx(j): entry j of the list, j already clamped into it
  auto load_kv = [&](auto&& idx, int j0, int cnt) {
    TileKV r;
    const long long koff = row_off(idx(min(j0 + lo, cnt - 1)));
    long long voff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) voff[i] = row_off(idx(min(j0 + 4 * hi + i, cnt - 1)));
#pragma unroll
    for (int i = 0; i < 4; ++i) r.kc[i] = *reinterpret_cast<const uint4*>(Kb + koff + 8 * (hi + 4 * i));
#pragma unroll
    for (int i = 0; i < 4; ++i) r.vr[i] = *reinterpret_cast<const uint4*>(Vb + voff[i]);
    return r;
  };
  // rows j0 .. j0+15 of a list whose first nw entries are attended and whose entries nw .. cnt-1 are
  // candidates: those only leave their logits and V row in the stash, entry (entry - nw)
  auto compute_tile = [&](const TileKV& kv, int j0, int nw, int cnt) {
    float sv[4];
    tile.logits(kv, scale_log2e, sv);
    bool valid[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) valid[e] = j0 + 4 * hi + e < nw;
    if (j0 + 16 > nw && cnt > nw) {   // (wave-uniform) this tile holds candidates
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = j0 + 4 * hi + e - nw;
        if (r >= 0 && r < cnt - nw && r < kStashRecs) {
          if (lo < G) cst_s[r][lo] = sv[e];
          cst_v[r][lo] = kv.vr[e];
        }
      }
    }
    tile.accumulate(kv, sv, valid, &scs[wave][0], lo, hi);
  };
  // Tiles of 16 entries; wave w takes tiles w, w + 4, ...  While a tile is computed the next one's
  // rows are in flight (loads unconditional, the last tile peeled: exact wait counts).  Ends with the
  // workgroup's totals in LDS: sm_m, sm_l and the weighted V sums per wave.
  // under_first_load(): runs once per wave, after the wave's first tile has been requested and before
  // anything waits for it: the place for a memory round trip that nothing else would hide.
  // nw, cnt: see compute_tile.
  auto attend_list = [&](auto&& idx, int nw, int cnt, auto&& under_first_load) {
    tile.reset();
    const int jw = wave * 16;
    if (jw < cnt) {
      const int n_tiles = (cnt - jw + 63) / 64;
      TileKV cur = load_kv(idx, jw, cnt);
      under_first_load();
      for (int i = 0; i + 1 < n_tiles; ++i) {
        const TileKV nxt = load_kv(idx, jw + 64 * (i + 1), cnt);
        compute_tile(cur, jw + 64 * i, nw, cnt);
        cur = nxt;
      }
      compute_tile(cur, jw + 64 * (n_tiles - 1), nw, cnt);
    } else {
      under_first_load();
    }
    tile.finish(&sm_m[wave][0], &sm_l[wave][0], &sm_o[wave][0][0], lo, hi);
    __syncthreads();
  };
  // workgroup totals of thread (query head g, 4 head dims), t < 32 G: max, sum, weighted V
  auto wg_totals = [&](int g, int d4, float& mn, float& ls, float4& a) {
    tile_wg_totals<G>(&sm_m[0][0], &sm_l[0][0], &sm_o[0][0][0], g, d4, mn, ls, a);
  };

  attend_list([&](int j) { return wl[j]; }, n_win, n_list, [&]() {
    // n_sel and n_cand are adjacent: one 64-bit add reserves this workgroup's ranges of T and of the
    // candidate list.  Issued here, its round trip runs under the gather of the first tile (a vector
    // memory result is waited for in issue order: the rows were requested first and are needed next).
    // By the last wave: it has the fewest tiles, so the wait delays no second gather.
    if (t == 192) {
      const unsigned long long r = atomicAdd(reinterpret_cast<unsigned long long*>(&ctl[row].n_sel),
                                             (unsigned long long)tw | ((unsigned long long)tc << 32));
      bc[0] = (uint32_t)r;
      bc[1] = (uint32_t)(r >> 32);
    }
  });
  FASA_T(3);

  // ---- 4. T, candidate list, partial, ticket ----  (bc: attend_list ends with a block barrier)
  int32_t* trow = T + (size_t)row * t_pitch;
  uint2* crow = cand + (size_t)row * n_cap;
  {
    uint32_t bw = bc[0] + pw, bcand = bc[1] + pc;
#pragma unroll
    for (int k = 0; k < PT; ++k) {
      const int n = base + ((k >> 2) * 256 + t) * 4 + (k & 3);
      // the bounds hold by construction of the histogram; they are re-checked so that a histogram
      // that does not match S can never turn into an out-of-range store
      if ((win & (1u << k)) && bw < (uint32_t)bsel) trow[bw++] = n;
      // candidates are read by the row's last workgroup: published with agent-scope stores
      if ((cnd & (1u << k)) && bcand < (uint32_t)n_cap) st_agent(&crow[bcand++], make_uint2(key[k], (uint32_t)n));
    }
    // the stash becomes records at the candidates' places in the list: thread t writes 8 bytes
    // (36 per record: 4 of logits, 32 of the V row)
    for (int i = t; i < n_ride * 36; i += 256) {
      const int r = i / 36, piece = i % 36, place = (int)bc[1] + r;
      if (place < kFuseRich) {
        if (piece < 4) st_agent(reinterpret_cast<uint2*>(rec_s + place * kRecLogits) + piece,
                                reinterpret_cast<const uint2*>(&cst_s[r][0])[piece]);
        else st_agent(&rec_v[place * 32 + piece - 4], reinterpret_cast<const uint2*>(&cst_v[r][0])[piece - 4]);
      }
    }
  }
  const size_t pbase = ((size_t)row * nslices + slice) * G;
  if (t < G * (D / 4)) {
    const int g = t / (D / 4), d4 = t % (D / 4);
    float mn, ls;
    float4 a;
    wg_totals(g, d4, mn, ls, a);
    float2* pa = reinterpret_cast<float2*>(part_acc + (pbase + g) * D + 4 * d4);
    st_agent(pa, make_float2(a.x, a.y));
    st_agent(pa + 1, make_float2(a.z, a.w));
    if (d4 == 0) st_agent(reinterpret_cast<float2*>(part_ml + (pbase + g) * 2), make_float2(mn, ls));
  }
  FASA_T(4);
  publish_barrier();
  // the ticket also collects whether any workgroup had more candidates than it could carry
  if (t == 0) ticket = atomicAdd(&ctl[row].done_att, 1u + (overflow ? 0x10000u : 0u));
  __syncthreads();
  FASA_T(5);
  FASA_T_PRINT(t == 0 && row == 0 && slice == 0, "fused blk0: thr %llu classify %llu tiles(%d rows) %llu store+merge %llu publish+ticket %llu (x10ns)\n",
               FASA_T_D(1, 0), FASA_T_D(2, 1), n_win, FASA_T_D(3, 2), FASA_T_D(4, 3), FASA_T_D(5, 4));
  if ((ticket & 0xffffu) != (uint32_t)nvalid - 1u) return;
  const bool records_complete = rich && !overflow && (ticket >> 16) == 0;

  // ---- 5. the row's last workgroup: candidates of the threshold bin ----
  // their number is the histogram's count of that bin
  const int n_cand = (int)min(thr[2], (uint32_t)n_cap);
  const int need = max(0, min(bsel - (int)n_above, n_cand));
  int32_t* tail = trow + n_above;
  const ExtraSplit ex_lds = {ex_m, ex_l, &ex_acc[0][0], ex_w};
  // leave the row's histogram and counters zeroed for the next call (every workgroup of the row has
  // read what it needed before it took its ticket)
  *reinterpret_cast<uint4*>(gh + 4 * t) = make_uint4(0, 0, 0, 0);
  if (t == 0) { ctl[row].n_sel = 0; ctl[row].n_cand = 0; ctl[row].done_att = 0; }

  if (need > 0 && records_complete) {
    // Every candidate comes with its record.  Requested first, then - inside combine_row - the
    // partials: one round trip for all of it.  Thread t: candidate t, two logits of candidate t / 4,
    // and the t-th eight bytes of every 2 KB of V rows.
    const uint2 ce = ld_agent(&crow[min(t, n_cand - 1)]);
    const float2 cs = ld_agent(reinterpret_cast<const float2*>(rec_s) + min(t, 4 * n_cand - 1));
    constexpr int NV = kFuseRich * 16 / 256;          // 16-byte pieces of V rows per thread
    const __amdgpu_buffer_rsrc_t rv = agent_buffer(rec_v);
    uint4 cv[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u)
      if (u * 256 < 16 * n_cand) cv[u] = agent_load_u128(rv, (uint32_t)min(u * 256 + t, 16 * n_cand - 1) * 16u);
    uint2* lc = reinterpret_cast<uint2*>(big);                                          // [kFuseRich]
    float* lsm = reinterpret_cast<float*>(big + kFuseRich * 8);                          // [kFuseRich][8]
    uint4* lvm = reinterpret_cast<uint4*>(big + kFuseRich * 8 + kFuseRich * kRecLogits * 4);   // [kFuseRich][16]
    int32_t* tk = reinterpret_cast<int32_t*>(dh);                                        // taken candidates, by rank
    auto under_loads = [&]() {
      if (t < kFuseRich) lc[t] = ce;
      reinterpret_cast<float2*>(lsm)[t] = cs;
#pragma unroll
      for (int u = 0; u < NV; ++u)
        if (u * 256 < 16 * n_cand) lvm[u * 256 + t] = cv[u];
      __syncthreads();
      FASA_T(6);
      // rank by counting, four threads per candidate (at most kFuseRich = 64 candidates here)
      static_assert(kFuseRich * 4 <= 256, "four threads per candidate");
      const int ci = t >> 2;
      const int rank = rank_in_list<4>(lc, n_cand, ci);
      if ((t & 3) == 0 && ci < n_cand && rank < need) {
        tail[rank] = (int)lc[ci].y;
        tk[rank] = ci;
      }
      __syncthreads();
      FASA_T(7);
      // the taken candidates as one more split: thread (query head g, 4 head dims), four candidates
      // at a time, running maximum as in the tiles
      if (t < G * (D / 4)) {
        const int g = t / (D / 4), d4 = t % (D / 4);
        float mn = kNegBig, ls = 0.f;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j0 = 0; j0 < need; j0 += 4) {
          int c[4];
          float sj[4];
          uint2 vw[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) c[u] = tk[min(j0 + u, need - 1)];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            sj[u] = j0 + u < need ? lsm[c[u] * kRecLogits + g] : kNegBig;
            vw[u] = reinterpret_cast<const uint2*>(lvm)[c[u] * 32 + d4];
          }
          const float m4 = fmaxf(fmaxf(sj[0], sj[1]), fmaxf(sj[2], sj[3]));
          const float m_new = fmaxf(mn, m4);
          const float sc = exp2f(mn - m_new);
          mn = m_new;
          ls *= sc; a.x *= sc; a.y *= sc; a.z *= sc; a.w *= sc;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float wgt = j0 + u < need ? exp2f(sj[u] - m_new) : 0.f;
            ls += wgt;
            a.x = fmaf(wgt, bf16_lo(vw[u].x), a.x); a.y = fmaf(wgt, bf16_hi(vw[u].x), a.y);
            a.z = fmaf(wgt, bf16_lo(vw[u].y), a.z); a.w = fmaf(wgt, bf16_hi(vw[u].y), a.w);
          }
        }
        *reinterpret_cast<float4*>(&ex_acc[g][4 * d4]) = a;
        if (d4 == 0) { ex_m[g] = mn; ex_l[g] = ls; }
      }
      __syncthreads();
      FASA_T(8);
    };
    combine_row<G, decltype(under_loads)&, kFuseMergeInFlight>(part_acc, part_ml, O, row, b, h, Hq, nvalid, nslices, wsm, red,
                                                               reinterpret_cast<float*>(big), ex_lds, under_loads);
    FASA_T(9);
    FASA_T_PRINT(t == 0 && row == 0, "fused last(row0, slice %d): loads %llu rank(%d of %d) %llu records %llu merge %llu (x10ns)\n",
                 slice, FASA_T_D(6, 5), need, n_cand, FASA_T_D(7, 6), FASA_T_D(8, 7), FASA_T_D(9, 8));
    return;
  }

  ExtraSplit ex = {nullptr, nullptr, nullptr, nullptr};
  if (need > 0) {
    uint2* lc = reinterpret_cast<uint2*>(big);
    uint32_t* dhw = reinterpret_cast<uint32_t*>(big + kFuseCandLds * 8);
    if (t == 0) bc[3] = 0;
    const bool from_lds = n_cand <= kFuseCandLds;
    if (from_lds) {
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
    FASA_T(6);
    if (from_lds) {
      if (n_cand <= kFuseCountMax) {
        // rank by counting: candidate t is taken iff fewer than `need` candidates sort before it
        const int rank = rank_in_list<1>(lc, n_cand, t);
        const bool take = t < n_cand && rank < need;
        if (take) {
          const int tok = (int)lc[t].y;
          tail[rank] = tok;
          wl[rank] = tok;
        }
      } else {
        resolve_candidates<false, 256, 64>(lc, n_cand, need, tail, dh, wtot, bc, dhw, nullptr, pm, b, wl);
      }
    } else {
      resolve_candidates<true, 256, 64>(crow, n_cand, need, tail, dh, wtot, bc, nullptr, nullptr, pm, b, nullptr);
    }
    if (from_lds) __syncthreads();   // wl is complete
    else publish_barrier();          // the tail of T is written and acknowledged: it is read back below
    FASA_T(7);
    if (from_lds) {
      if (paged) {       // the gather reads pool slots
        for (int i = t; i < need; i += 256) wl[i] = kv_slot(pm, b, wl[i]);
        __syncthreads();
      }
      attend_list([&](int j) { return wl[j]; }, need, need, []() {});
    } else if (paged) {
      attend_list([&](int j) { return kv_slot(pm, b, ld_agent(reinterpret_cast<const uint32_t*>(tail) + j)); }, need,
                  need, []() {});
    } else {
      attend_list([&](int j) { return (int)ld_agent(reinterpret_cast<const uint32_t*>(tail) + j); }, need, need,
                  []() {});
    }
    if (t < G * (D / 4)) {
      const int g = t / (D / 4), d4 = t % (D / 4);
      float mn, ls;
      float4 a;
      wg_totals(g, d4, mn, ls, a);
      *reinterpret_cast<float4*>(&ex_acc[g][4 * d4]) = a;
      if (d4 == 0) { ex_m[g] = mn; ex_l[g] = ls; }
    }
    __syncthreads();
    ex = ex_lds;
  }
  FASA_T(8);

  // ---- 6. merge ----
  combine_row<G, NothingUnderLoads, kFuseMergeInFlight>(part_acc, part_ml, O, row, b, h, Hq, nvalid, nslices, wsm, red,
                                                        reinterpret_cast<float*>(big), ex);
  FASA_T(9);
  FASA_T_PRINT(t == 0 && row == 0, "fused last(row0, slice %d): candload %llu resolve %llu attend(%d of %d) %llu combine %llu (x10ns)\n",
               slice, FASA_T_D(6, 5), FASA_T_D(7, 6), need, n_cand, FASA_T_D(8, 7), FASA_T_D(9, 8));
}

// ---------------------------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------------------------
FusePlan plan_fused(const fasa_shape& s, bool by_sequence) {
  FusePlan p{0, 0, 0};
  if (s.dtype != FASA_BF16) return p;                       // float32 caches take the staged kernels
  if (!by_sequence && s.budget >= s.n_ctx) return p;        // everything selected: nothing to select
  const long long rows = (long long)s.batch * s.n_kv_heads;
  const long long N = s.n_ctx;
  // The kernel runs two workgroups per CU, so a grid of up to 2 * 256 workgroups is resident at once and
  // ends together; one workgroup more and a second, nearly empty round doubles the kernel's time.  So a
  // row is cut into EQUAL slices, as many as keep the grid within that bound - small problems are
  // latency-bound and gain from short slices with few winners each - but of at least 1024 tokens (shorter
  // ones measured no gain: more partials to publish and merge) and at most 4096 (what a workgroup can
  // hold in registers).  Rows too long for one round at 4096 tokens per slice take equal slices of at
  // most 4096.  The kernel instance is the smallest that holds a slice.
  const long long cap = 2LL * kAssumedCUs;
  const long long ns_min = (N + 4095) / 4096;
  long long ns = ns_min;
  if (rows * ns_min <= cap) {
    ns = cap / rows;
    if (ns > (N + 1023) / 1024) ns = (N + 1023) / 1024;
    if (ns > kMaxSplitsLds) ns = kMaxSplitsLds;
    if (ns < ns_min) ns = ns_min;
  }
  if (ns > kMaxSplitsLds) return p;                          // rows longer than 256 slices of 4096
  const long long len = ((N + ns - 1) / ns + 15) / 16 * 16;  // <= 4096: ns >= ns_min
  p.slice_len = (int)len;
  p.nslices = (int)((N + len - 1) / len);
  p.tpb = len <= 1024 ? 1024 : (len <= 2048 ? 2048 : (len <= 3072 ? 3072 : 4096));
  return p;
}

template <int G, int TPB>
static hipError_t launch_fused_gt(const fasa_shape& s, const FusePlan& p, const void* q, const void* K,
                                  const void* V, const float* S, uint32_t* hist, RowCtl* ctl, uint2* cand,
                                  int32_t* T, float* O, float* part_acc, float* part_ml, unsigned char* rec,
                                  hipStream_t st, RaggedLens rl, PageMap pm) {
  const int rows = s.batch * s.n_kv_heads;
  const int t_pitch = s.budget < s.n_ctx ? s.budget : s.n_ctx;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)s.head_dim);
  return launch("fasa_select_attend", select_attend_kernel<G, TPB>, dim3(rows * p.nslices), dim3(256), st,
                (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, S, hist, ctl, cand, T, O, part_acc,
                part_ml, rec, rows, p.nslices, p.slice_len, s.n_q_heads, s.n_kv_heads, s.n_ctx, s.n_cap, s.budget, t_pitch,
                (long long)s.kv_stride_b, (long long)s.kv_stride_h, (long long)s.kv_stride_n, scale_log2e,
                rl.n_ctx, rl.budget, pm);
}

template <int G>
static hipError_t launch_fused_g(const fasa_shape& s, const FusePlan& p, const void* q, const void* K,
                                 const void* V, const float* S, uint32_t* hist, RowCtl* ctl, uint2* cand,
                                 int32_t* T, float* O, float* part_acc, float* part_ml, unsigned char* rec,
                                 hipStream_t st, RaggedLens rl, PageMap pm) {
  switch (p.tpb) {
    case 1024: return launch_fused_gt<G, 1024>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 2048: return launch_fused_gt<G, 2048>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 3072: return launch_fused_gt<G, 3072>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 4096: return launch_fused_gt<G, 4096>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_select_attend(const fasa_shape& s, const FusePlan& p, const void* q, const void* K,
                                const void* V, const float* S, uint32_t* hist, RowCtl* ctl, uint2* cand,
                                int32_t* T, float* O, float* part_acc, float* part_ml, unsigned char* rec,
                                hipStream_t st, RaggedLens rl, PageMap pm) {
  switch (s.n_q_heads / s.n_kv_heads) {
    case 1: return launch_fused_g<1>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 2: return launch_fused_g<2>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 3: return launch_fused_g<3>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 4: return launch_fused_g<4>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 5: return launch_fused_g<5>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 6: return launch_fused_g<6>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 7: return launch_fused_g<7>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    case 8: return launch_fused_g<8>(s, p, q, K, V, S, hist, ctl, cand, T, O, part_acc, part_ml, rec, st, rl, pm);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace fasa
