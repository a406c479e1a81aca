// Internal declarations shared by the translation units of libfasa (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstddef>
#include <cstdint>
#include <tuple>
#include <utility>

#include "fasa.h"

namespace fasa {

// ---------------------------------------------------------------------------------------------
// constants of the selection stage
// ---------------------------------------------------------------------------------------------
constexpr int kHistBits = 12;              // coarse bins = top 12 bits of the order-preserving key
constexpr int kHistBins = 1 << kHistBits;  // (sign, 8 exponent bits, 3 mantissa bits)
constexpr int kKeyLowBits = 32 - kHistBits;
constexpr int kHeadDim = 128;
constexpr int kMaxGroup = 8;
// Compute units the launch plans are sized for (MI355X).  A compile-time number because
// fasa_workspace_bytes() has to be a pure host function; a GPU test checks it against the device.
constexpr int kAssumedCUs = 256;

// Per-(b,h) row counters, one 128-byte line per row so that rows served by different XCDs never
// share a line.  All zero between calls: the workgroup that finishes a row resets what it used.
struct RowCtl {
  uint32_t n_sel;     // winners written so far (tokens in bins above the threshold bin)
  uint32_t n_cand;    // candidates collected from the threshold bin
  uint32_t done_sel;  // selection workgroups of this row that finished their slice
  uint32_t done_att;  // attention workgroups of this row that wrote their partial
  float bin_mu;       // adaptive histogram of the fused step: written by the scoring kernel of a call,
  float bin_inv;      // read by its selection kernel (never has to be zero)
  uint32_t pad[26];
};
static_assert(sizeof(RowCtl) == 128, "one line per row");

// Optional per-sequence lengths (DEVICE arrays of `batch` entries, or null = the uniform values of
// the shape).  With them the shape's n_ctx and budget are upper bounds that size the grids, and
// T's row pitch is min(budget, n_ctx) of the shape.
struct RaggedLens {
  const int32_t* n_ctx;
  const int32_t* budget;
};

// Paged K/V cache as the kernels see it.  table == nullptr: contiguous cache, row (b, n) at
// b * kv_stride_b + n * kv_stride_n.  Otherwise row (b, n) lives in pool block
// table[b * max_blocks + (n >> shift)] at offset (n & (page - 1)); kv_stride_b is then the stride
// between pool blocks.  Table entries are clamped into [0, n_pool): a stray entry can never become
// a stray address.
struct PageMap {
  const int32_t* table;
  int max_blocks;
  int shift;     // log2(tokens per block)
  int n_pool;    // blocks in the pool
};
constexpr PageMap kNoPaging = {nullptr, 0, 0, 0};

// pool slot (block * page + offset) of logical token n of sequence b
__device__ __forceinline__ int kv_slot(const PageMap& pm, int b, int n) {
  const int blk = min(max(pm.table[(size_t)b * pm.max_blocks + (n >> pm.shift)], 0), pm.n_pool - 1);
  return (blk << pm.shift) | (n & ((1 << pm.shift) - 1));
}
// element offset of K/V row (b, n), without the head term
__device__ __forceinline__ long long kv_row_offset(const PageMap& pm, int b, int n, long long sb,
                                                   long long sn) {
  if (pm.table == nullptr) return b * sb + (long long)n * sn;
  const int slot = kv_slot(pm, b, n);
  return (long long)(slot >> pm.shift) * sb + (long long)(slot & ((1 << pm.shift) - 1)) * sn;
}

// The two head dims that entry f of KV head h's dominant list names, as lo | hi << 8.  The list
// holds FC numbers (one word per entry) or, for FASA_PAIR_LIST, the dim pairs themselves (two
// words).  Values are clamped into the head: a stray entry can never become a stray LDS index.
__device__ __forceinline__ int list_word(int pairing, int F, int h, int f, int which) {
  return pairing == FASA_PAIR_LIST ? (h * F + f) * 2 + which : h * F + f;
}
__device__ __forceinline__ int pair_dims(int pairing, int a, int b) {
  constexpr int D = kHeadDim;
  const int i = min(max(a, 0), D / 2 - 1);
  int lo = pairing == FASA_PAIR_INTERLEAVED ? 2 * i : i;
  int hi = pairing == FASA_PAIR_INTERLEAVED ? 2 * i + 1 : i + D / 2;
  if (pairing == FASA_PAIR_LIST) {
    lo = min(max(a, 0), D - 1);
    hi = min(max(b, 0), D - 1);
  }
  return lo | (hi << 8);
}

// Workspace carve-up (all offsets 256-byte aligned).
struct WsLayout {
  size_t hist_off, ctl_off, cand_off, part_acc_off, part_ml_off, rec_off, tslot_off, total;
  int rows, max_splits;
};

struct AttendPlan {
  int count;          // tokens attended per row
  int tok_per_split;  // list entries per workgroup
  int n_splits;
};

AttendPlan plan_attend(int rows, int count, int group);

// Fused selection + attention (fused.hip): tokens per workgroup and workgroups per row.
// tpb == 0: this shape takes the staged kernels (float32 cache, everything selected, or a row longer
// than the merge can take slices of).
// Candidates per row of the fused step that are handed over with a record (logits of the group's query
// heads + V row), and the bytes of workspace a row's records take.
constexpr int kFuseRich = 64;
constexpr size_t kFuseRecBytesPerRow = (size_t)kFuseRich * (kMaxGroup * 4 + kHeadDim * 2);

struct FusePlan {
  int tpb;         // kernel instance: most tokens a workgroup can hold (0: the fused step does not apply)
  int nslices;     // workgroups per row
  int slice_len;   // tokens per workgroup, <= tpb, a multiple of 16
};
// by_sequence: lengths and budgets come from device arrays (a budget may then reach its length)
FusePlan plan_fused(const fasa_shape& s, bool by_sequence);
WsLayout ws_layout(const fasa_shape& s);

// ---------------------------------------------------------------------------------------------
// launch helper: plain launch, or a launch bracketed by its own start/stop timestamps
// ---------------------------------------------------------------------------------------------
bool profile_on();
// Hands out a fresh event pair owned by the profiler and remembers it under `name`.
hipError_t profile_events(const char* name, hipEvent_t* start, hipEvent_t* stop);
void set_last_hip_error(hipError_t e);

template <typename... KArgs, typename... Args>
inline hipError_t launch(const char* name, void (*kernel)(KArgs...), dim3 grid, dim3 block,
                         hipStream_t stream, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
  std::tuple<KArgs...> vals{static_cast<KArgs>(std::forward<Args>(args))...};
  void* ptrs[sizeof...(KArgs) ? sizeof...(KArgs) : 1];
  std::apply([&](auto&... v) { size_t i = 0; ((ptrs[i++] = (void*)&v), ...); }, vals);
  hipError_t e;
  if (profile_on()) {
    hipEvent_t a = nullptr, b = nullptr;
    e = profile_events(name, &a, &b);
    if (e == hipSuccess)
      e = hipExtLaunchKernel((const void*)kernel, grid, block, ptrs, 0, stream, a, b, 0);
  } else {
    e = hipLaunchKernel((const void*)kernel, grid, block, ptrs, 0, stream);
  }
  if (e != hipSuccess) set_last_hip_error(e);
  return e;
}

// ---------------------------------------------------------------------------------------------
// stage launchers (defined in pack.hip / score.hip / topk.hip / attend.hip); shapes are already
// validated when these are called
// ---------------------------------------------------------------------------------------------
hipError_t launch_pack(const fasa_shape& s, const void* K, const int32_t* fc_idx, void* Kp,
                       int n_begin, int n_end, hipStream_t st, PageMap pm = kNoPaging);
// A freshly decoded K/V row per (b, h) ([batch][n_kv_heads][head_dim]) that the scoring kernel
// appends at token n_ctx - 1 (K, V: the caches, with the shape's strides; Kp gets the dominant pairs).
// k_new == nullptr: nothing to append.
struct AppendArgs {
  const void* k_new;
  const void* v_new;
  void* K;
  void* V;
  PageMap pm;
};
constexpr AppendArgs kNoAppend = {nullptr, nullptr, nullptr, nullptr, {nullptr, 0, 0, 0}};
// hist == nullptr: scores only.  adaptive_ctl != nullptr (with hist): the adaptive histogram of the
// fused step (bins of lin_bin, location and scale left in the row counters) instead of the
// exponent-based one the stand-alone selection reads.
hipError_t launch_score(const fasa_shape& s, const void* q, const void* Kp, const int32_t* fc_idx,
                        float* S, uint32_t* hist, hipStream_t st, RaggedLens rl = {nullptr, nullptr},
                        AppendArgs ap = kNoAppend, RowCtl* adaptive_ctl = nullptr);
// zeroes the histogram and the row counters (workspace initialisation)
hipError_t launch_ws_clear(const fasa_shape& s, uint32_t* hist, RowCtl* ctl, hipStream_t st);
hipError_t launch_hist(const fasa_shape& s, const float* S, uint32_t* hist, hipStream_t st);
// Tslot (paged caches only, else null): receives the pool slot of every entry of T, same layout
hipError_t launch_select(const fasa_shape& s, const float* S, const uint32_t* hist, RowCtl* ctl,
                         uint2* cand, int32_t* T, hipStream_t st, RaggedLens rl = {nullptr, nullptr},
                         PageMap pm = kNoPaging, int32_t* Tslot = nullptr);
// paged caches: T holds pool slots (launch_select's Tslot), dense must be false
hipError_t launch_attend(const fasa_shape& s, bool dense, const void* q, const void* K,
                         const void* V, const int32_t* T, float* O, RowCtl* ctl, float* part_acc,
                         float* part_ml, hipStream_t st, RaggedLens rl = {nullptr, nullptr},
                         PageMap pm = kNoPaging);

// TopK-I + FAC in one kernel after a scoring pass with the adaptive histogram (launch_score with
// adaptive_ctl); p from plan_fused, p.tpb != 0.  The partial buffers are indexed with p.nslices splits
// per row.  Paged caches are gathered through the table inside the kernel.
hipError_t launch_select_attend(const fasa_shape& s, const FusePlan& p, const void* q, const void* K,
                                const void* V, const float* S, uint32_t* hist, RowCtl* ctl, uint2* cand,
                                int32_t* T, float* O, float* part_acc, float* part_ml, unsigned char* rec,
                                hipStream_t st, RaggedLens rl = {nullptr, nullptr}, PageMap pm = kNoPaging);

// memory-optimised variant (offload.hip)
hipError_t launch_offload_split(const fasa_shape& s, const void* K, const int32_t* fc_idx, void* Kp,
                                void* Knd, int n_begin, int n_end, hipStream_t st);
hipError_t launch_offload_append(const fasa_shape& s, void* Kp, void* Knd, void* Vh,
                                 const int32_t* fc_idx, const void* k_new, const void* v_new,
                                 hipStream_t st);
hipError_t launch_offload_gather(const fasa_shape& s, const void* Kp, const void* Knd, const void* Vh,
                                 const int32_t* fc_idx, const int32_t* T, void* KT, void* VT,
                                 hipStream_t st);

// offline calibration (calib.hip)
hipError_t launch_calib_prepare(const fasa_shape& s, const void* q, void* q_v, int32_t* fc_all,
                                int32_t* fc_v, hipStream_t st);
hipError_t launch_calib_intersect(const fasa_shape& s, const int32_t* T_full, const int32_t* T_v,
                                  float* CA_sum, int kk, hipStream_t st);
int calib_max_ctx();

}  // namespace fasa
