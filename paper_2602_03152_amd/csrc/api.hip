// C-ABI entry points: argument validation (no HIP call before it passes), workspace carve-up,
// stage sequencing on the caller's stream, per-kernel profiler.
#include <algorithm>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "fasa_internal.h"

namespace fasa {

// ---------------------------------------------------------------------------------------------
// last HIP error (per thread)
// ---------------------------------------------------------------------------------------------
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

// ---------------------------------------------------------------------------------------------
// profiler
// ---------------------------------------------------------------------------------------------
struct ProfRec { const char* name; hipEvent_t a, b; };
struct ProfSum { std::string name; int64_t launches; double ms; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof_recs;
static std::vector<ProfSum> g_prof_sums;

bool profile_on() { return g_prof_on; }

hipError_t profile_events(const char* name, hipEvent_t* start, hipEvent_t* stop) {
  hipError_t e = hipEventCreate(start);
  if (e != hipSuccess) return e;
  e = hipEventCreate(stop);
  if (e != hipSuccess) { (void)hipEventDestroy(*start); return e; }
  g_prof_recs.push_back({name, *start, *stop});
  return hipSuccess;
}

static int profile_fold() {
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) { set_last_hip_error(e); return FASA_EHIP; }
  for (auto& r : g_prof_recs) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, r.a, r.b);
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
    if (e != hipSuccess) { set_last_hip_error(e); continue; }
    bool found = false;
    for (auto& s : g_prof_sums)
      if (s.name == r.name) { s.launches++; s.ms += ms; found = true; break; }
    if (!found) g_prof_sums.push_back({r.name, 1, (double)ms});
  }
  g_prof_recs.clear();
  return (int)g_prof_sums.size();
}

// ---------------------------------------------------------------------------------------------
// plans and workspace
// ---------------------------------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

AttendPlan plan_attend(int rows, int count, int group) {
  // The attention kernels are gather-bound and all their workgroups should be resident at once:
  // a second, partly filled round of workgroups costs as much as a full one.  Two workgroups (8 waves)
  // per CU measured best for every workload shape and GQA group (more splits only add partial results
  // to publish and merge).
  (void)group;
  const long long slots = 2LL * kAssumedCUs;
  const long long total = (long long)rows * count;
  const long long by_size = (total + 63) / 64;           // workgroups of at least 64 list entries
  long long nblocks;
  if (by_size <= slots) {
    nblocks = by_size;                                    // small problem: one partial round
  } else {
    const long long rounds = (total + slots * 2048 - 1) / (slots * 2048);   // <= ~2048 entries each
    nblocks = rounds * slots;
  }
  long long n_splits = (nblocks + rows / 2) / rows;
  if (n_splits < 1) n_splits = 1;
  if (n_splits > 256) n_splits = 256;                     // the merging workgroup weights <= 256 splits
  if (n_splits > (count + 15) / 16) n_splits = (count + 15) / 16;
  const long long tps = (count + n_splits - 1) / n_splits;
  AttendPlan p;
  p.count = count;
  p.tok_per_split = (int)tps;
  p.n_splits = (int)((count + tps - 1) / tps);
  return p;
}

WsLayout ws_layout(const fasa_shape& s) {
  WsLayout w{};
  w.rows = s.batch * s.n_kv_heads;
  const int G = s.n_q_heads / s.n_kv_heads;
  const int bsel = s.budget < s.n_ctx ? s.budget : s.n_ctx;
  const int sp_sparse = plan_attend(w.rows, bsel, G).n_splits;
  const int sp_dense = plan_attend(w.rows, s.n_ctx, G).n_splits;
  w.max_splits = sp_sparse > sp_dense ? sp_sparse : sp_dense;
  const int sp_fused = plan_fused(s, true).nslices;      // the fused step: one partial per score slice
  if (sp_fused > w.max_splits) w.max_splits = sp_fused;
  size_t off = 0;
  w.hist_off = off;      off = align256(off + (size_t)w.rows * kHistBins * sizeof(uint32_t));
  w.ctl_off = off;       off = align256(off + (size_t)w.rows * sizeof(RowCtl));
  w.cand_off = off;      off = align256(off + (size_t)w.rows * s.n_cap * sizeof(uint2));
  w.part_acc_off = off;  off = align256(off + (size_t)w.rows * w.max_splits * G * kHeadDim * sizeof(float));
  w.part_ml_off = off;   off = align256(off + (size_t)w.rows * w.max_splits * G * 2 * sizeof(float));
  w.rec_off = off;       off = align256(off + (size_t)w.rows * kFuseRecBytesPerRow);   // candidate records (fused step)
  // pool slots of the selected tokens (paged caches); at the end: earlier offsets do not depend on it
  w.tslot_off = off;     off = align256(off + (size_t)w.rows * (size_t)bsel * sizeof(int32_t));
  w.total = off;
  return w;
}

// ---------------------------------------------------------------------------------------------
// validation
// ---------------------------------------------------------------------------------------------
static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

enum Need : unsigned { kNeedNone = 0, kNeedCtx = 1, kNeedBudget = 2, kNeedFc = 4, kNeedStrides = 8 };

static int check_shape(const fasa_shape* s, unsigned need) {
  if (!s) return FASA_EINVAL;
  if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->head_dim < 2) return FASA_EINVAL;
  if (s->head_dim % 2 != 0 || s->n_q_heads % s->n_kv_heads != 0) return FASA_EINVAL;
  if (s->pairing != FASA_PAIR_ROTATE_HALF && s->pairing != FASA_PAIR_INTERLEAVED && s->pairing != FASA_PAIR_LIST)
    return FASA_EINVAL;
  if (s->dtype != FASA_BF16 && s->dtype != FASA_F32) return FASA_EINVAL;
  if (s->n_cap < 1 || s->n_cap % 64 != 0) return FASA_EINVAL;
  if ((long long)s->batch * s->n_kv_heads > 65535) return FASA_EUNSUPPORTED;
  if (need & kNeedCtx) { if (s->n_ctx < 1 || s->n_ctx > s->n_cap) return FASA_EINVAL; }
  if (need & kNeedBudget) { if (s->budget < 1) return FASA_EINVAL; }
  if (need & kNeedFc) { if (s->n_fc < 1 || s->n_fc > s->head_dim / 2) return FASA_EINVAL; }
  if (need & kNeedStrides) {
    if (s->kv_stride_n < s->head_dim || s->kv_stride_n % 8 != 0) return FASA_EINVAL;
    if (s->kv_stride_h < 0 || s->kv_stride_b < 0 || s->kv_stride_h % 8 != 0 || s->kv_stride_b % 8 != 0)
      return FASA_EINVAL;
  }
  if (s->head_dim != kHeadDim) return FASA_EUNSUPPORTED;
  if (s->n_q_heads / s->n_kv_heads > kMaxGroup) return FASA_EUNSUPPORTED;
  return FASA_OK;
}

// need_slots: the call uses the slot list of a paged cache (the last region of the workspace)
static int check_ws(const fasa_shape* s, const void* ws, size_t ws_bytes, bool need_slots = true) {
  if (!ws || !aligned16(ws)) return FASA_EINVAL;
  const WsLayout w = ws_layout(*s);
  if (ws_bytes < (need_slots ? w.total : w.tslot_off)) return FASA_EWORKSPACE;
  return FASA_OK;
}

// Paged-cache description -> device view.  The table must cover every token the call can touch.
static int check_paging(const fasa_paging* p, const fasa_shape* s, PageMap* out) {
  if (!p || !p->block_table || ((uintptr_t)p->block_table & 3u)) return FASA_EINVAL;
  if (p->reserved != 0) return FASA_EINVAL;
  if (p->page_size < 1 || (p->page_size & (p->page_size - 1)) != 0) return FASA_EINVAL;
  if (p->n_pool_blocks < 1 || p->max_blocks < 1) return FASA_EINVAL;
  if ((long long)p->max_blocks * p->page_size < s->n_ctx) return FASA_EINVAL;
  if ((long long)p->n_pool_blocks * p->page_size > 0x7fffffffLL) return FASA_EUNSUPPORTED;
  int shift = 0;
  while ((1 << shift) < p->page_size) ++shift;
  *out = PageMap{p->block_table, p->max_blocks, shift, p->n_pool_blocks};
  return FASA_OK;
}

#define FASA_HIP(expr) do { if ((expr) != hipSuccess) return FASA_EHIP; } while (0)

// ---------------------------------------------------------------------------------------------
// The library's own workspace for fasa_decode_step_static: one array per GPU, part of the code
// object, held by every device the library is loaded on until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels and clears get the address that
// call returns, looked up once per device.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[FASA_STATIC_WS_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of `scratch` on the current device (nullptr: a HIP call failed, see last error)
static void* scratch_of_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_last_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      set_last_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace fasa

using namespace fasa;

extern "C" {

size_t fasa_workspace_bytes(const fasa_shape* shape) {
  if (check_shape(shape, kNeedCtx | kNeedBudget) != FASA_OK) return 0;
  return ws_layout(*shape).total;
}

int fasa_workspace_init(const fasa_shape* shape, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedBudget);
  if (rc != FASA_OK) return rc;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc != FASA_OK) return rc;
  const WsLayout w = ws_layout(*shape);
  char* base = (char*)ws;
  FASA_HIP(launch_ws_clear(*shape, (uint32_t*)(base + w.hist_off), (RowCtl*)(base + w.ctl_off),
                           (hipStream_t)stream));
  return FASA_OK;
}

int fasa_validate_fc_idx(const fasa_shape* shape, const int32_t* fc_idx_host) {
  int rc = check_shape(shape, kNeedFc);
  if (rc != FASA_OK) return rc;
  if (!fc_idx_host) return FASA_EINVAL;
  // FC numbers in [0, d/2), or (explicit pairs) 2 n_fc dims in [0, d); nothing twice within a head
  const bool pairs = shape->pairing == FASA_PAIR_LIST;
  const int limit = pairs ? shape->head_dim : shape->head_dim / 2;
  const int words = pairs ? 2 * shape->n_fc : shape->n_fc;
  if (limit > 4096) return FASA_EUNSUPPORTED;
  for (int h = 0; h < shape->n_kv_heads; ++h) {
    bool seen[4096] = {false};
    for (int f = 0; f < words; ++f) {
      const int i = fc_idx_host[h * words + f];
      if (i < 0 || i >= limit || seen[i]) return FASA_EINVAL;
      seen[i] = true;
    }
  }
  return FASA_OK;
}

int fasa_pack_kcache(const fasa_shape* shape, const void* K, const int32_t* fc_idx, void* Kp,
                     int32_t n_begin, int32_t n_end, void* stream) {
  int rc = check_shape(shape, kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  if (!K || !fc_idx || !Kp || !aligned16(K) || !aligned16(Kp) || !aligned16(fc_idx)) return FASA_EINVAL;
  if (n_begin < 0 || n_end < n_begin || n_end > shape->n_cap) return FASA_EINVAL;
  if (n_begin == n_end) return FASA_OK;
  FASA_HIP(launch_pack(*shape, K, fc_idx, Kp, n_begin, n_end, (hipStream_t)stream));
  return FASA_OK;
}

int fasa_score(const fasa_shape* shape, const void* q, const void* Kp, const int32_t* fc_idx,
               float* S, void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedFc);
  if (rc != FASA_OK) return rc;
  if (!q || !Kp || !fc_idx || !S) return FASA_EINVAL;
  if (!aligned16(q) || !aligned16(Kp) || !aligned16(fc_idx) || !aligned16(S)) return FASA_EINVAL;
  FASA_HIP(launch_score(*shape, q, Kp, fc_idx, S, nullptr, (hipStream_t)stream));
  return FASA_OK;
}

int fasa_topk(const fasa_shape* shape, const float* S, int32_t* T, void* ws, size_t ws_bytes,
              void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedBudget);
  if (rc != FASA_OK) return rc;
  if (!S || !T || !aligned16(S) || !aligned16(T)) return FASA_EINVAL;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc != FASA_OK) return rc;
  const WsLayout w = ws_layout(*shape);
  char* base = (char*)ws;
  uint32_t* hist = (uint32_t*)(base + w.hist_off);
  RowCtl* ctl = (RowCtl*)(base + w.ctl_off);
  uint2* cand = (uint2*)(base + w.cand_off);
  hipStream_t st = (hipStream_t)stream;
  if (shape->budget < shape->n_ctx) FASA_HIP(launch_hist(*shape, S, hist, st));
  FASA_HIP(launch_select(*shape, S, hist, ctl, cand, T, st));
  return FASA_OK;
}

static int attend_common(const fasa_shape* shape, bool dense, const void* q, const void* K,
                         const void* V, const int32_t* T, float* O, void* ws, size_t ws_bytes,
                         void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedStrides | (dense ? 0u : (unsigned)kNeedBudget));
  if (rc != FASA_OK) return rc;
  if (!q || !K || !V || !O || (!dense && !T)) return FASA_EINVAL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || (!dense && !aligned16(T)))
    return FASA_EINVAL;
  fasa_shape s = *shape;
  if (dense) s.budget = s.n_ctx;
  rc = check_ws(&s, ws, ws_bytes, false);
  if (rc != FASA_OK) return rc;
  const WsLayout w = ws_layout(s);
  char* base = (char*)ws;
  FASA_HIP(launch_attend(s, dense, q, K, V, T, O, (RowCtl*)(base + w.ctl_off),
                         (float*)(base + w.part_acc_off), (float*)(base + w.part_ml_off),
                         (hipStream_t)stream));
  return FASA_OK;
}

int fasa_sparse_attend(const fasa_shape* shape, const void* q, const void* K, const void* V,
                       const int32_t* T, float* O, void* ws, size_t ws_bytes, void* stream) {
  return attend_common(shape, false, q, K, V, T, O, ws, ws_bytes, stream);
}

int fasa_dense_attend(const fasa_shape* shape, const void* q, const void* K, const void* V,
                      float* O, void* ws, size_t ws_bytes, void* stream) {
  return attend_common(shape, true, q, K, V, nullptr, O, ws, ws_bytes, stream);
}

// The three forms of the fused step share one body.  paging == nullptr: contiguous cache.
// by_sequence: lengths (and optionally budgets) come from device arrays; the launch sequence must
// then not depend on them, so the histogram path is always taken (it also covers a sequence whose
// budget reaches its length).
static int decode_step_common(const fasa_shape* shape, const fasa_paging* paging, const void* q, void* K,
                              void* V, void* Kp, const int32_t* fc_idx, const void* k_new,
                              const void* v_new, const int32_t* n_ctx_seq, const int32_t* budget_seq,
                              float* S, int32_t* T, float* O, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedBudget | kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  if (!q || !K || !V || !Kp || !fc_idx || !S || !T || !O) return FASA_EINVAL;
  if ((k_new == nullptr) != (v_new == nullptr)) return FASA_EINVAL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(Kp) || !aligned16(fc_idx) ||
      !aligned16(S) || !aligned16(T) || !aligned16(O) || !aligned16(k_new) || !aligned16(v_new))
    return FASA_EINVAL;
  if (((uintptr_t)n_ctx_seq & 3u) || ((uintptr_t)budget_seq & 3u)) return FASA_EINVAL;
  PageMap pm = kNoPaging;
  if (paging) {
    rc = check_paging(paging, shape, &pm);
    if (rc != FASA_OK) return rc;
  }
  rc = check_ws(shape, ws, ws_bytes, paging != nullptr);
  if (rc != FASA_OK) return rc;
  const WsLayout w = ws_layout(*shape);
  char* base = (char*)ws;
  uint32_t* hist = (uint32_t*)(base + w.hist_off);
  RowCtl* ctl = (RowCtl*)(base + w.ctl_off);
  uint2* cand = (uint2*)(base + w.cand_off);
  int32_t* Tslot = paging ? (int32_t*)(base + w.tslot_off) : nullptr;
  hipStream_t st = (hipStream_t)stream;
  const RaggedLens rl{n_ctx_seq, budget_seq};
  const bool by_sequence = n_ctx_seq != nullptr || budget_seq != nullptr;
  const bool select_all = !by_sequence && shape->budget >= shape->n_ctx;
  // the new row (if any) joins K, V and Kp inside the scoring kernel
  const AppendArgs ap{k_new, v_new, K, V, pm};
  const FusePlan fp = plan_fused(*shape, by_sequence);
  if (fp.tpb != 0) {
    // two launches: scores + adaptive histogram, then selection and attention by token-range ownership
    FASA_HIP(launch_score(*shape, q, Kp, fc_idx, S, hist, st, rl, ap, ctl));
    FASA_HIP(launch_select_attend(*shape, fp, q, K, V, S, hist, ctl, cand, T, O, (float*)(base + w.part_acc_off),
                                  (float*)(base + w.part_ml_off), (unsigned char*)(base + w.rec_off), st, rl, pm));
    return FASA_OK;
  }
  FASA_HIP(launch_score(*shape, q, Kp, fc_idx, S, select_all ? nullptr : hist, st, rl, ap));
  FASA_HIP(launch_select(*shape, S, hist, ctl, cand, T, st, rl, pm, Tslot));
  // paged cache: the attention kernel gathers by pool slot and does not read the table again
  FASA_HIP(launch_attend(*shape, false, q, K, V, paging ? Tslot : T, O, ctl, (float*)(base + w.part_acc_off),
                         (float*)(base + w.part_ml_off), st, rl, pm));
  return FASA_OK;
}

int fasa_decode_step(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                     const int32_t* fc_idx, const void* k_new, const void* v_new, float* S,
                     int32_t* T, float* O, void* ws, size_t ws_bytes, void* stream) {
  return decode_step_common(shape, nullptr, q, K, V, Kp, fc_idx, k_new, v_new, nullptr, nullptr, S, T, O, ws,
                            ws_bytes, stream);
}

int fasa_decode_step_static(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                            const int32_t* fc_idx, const void* k_new, const void* v_new, float* S,
                            int32_t* T, float* O, void* stream) {
  // everything that can be refused is refused before the first HIP call
  int rc = check_shape(shape, kNeedCtx | kNeedBudget | kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  const WsLayout w = ws_layout(*shape);
  if (w.tslot_off > (size_t)FASA_STATIC_WS_BYTES) return FASA_EWORKSPACE;
  if (!q || !K || !V || !Kp || !fc_idx || !S || !T || !O) return FASA_EINVAL;
  void* ws = scratch_of_current_device();
  if (!ws) return FASA_EHIP;
  // The array keeps what the last call left, and that call may have had another layout: the part
  // that has to start at zero is cleared by a kernel (a caller may be capturing this stream).
  FASA_HIP(launch_ws_clear(*shape, (uint32_t*)((char*)ws + w.hist_off), (RowCtl*)((char*)ws + w.ctl_off),
                           (hipStream_t)stream));
  return decode_step_common(shape, nullptr, q, K, V, Kp, fc_idx, k_new, v_new, nullptr, nullptr, S, T, O, ws,
                            w.tslot_off, stream);
}

int fasa_decode_step_ragged(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                            const int32_t* fc_idx, const void* k_new, const void* v_new,
                            const int32_t* n_ctx_seq, const int32_t* budget_seq, float* S, int32_t* T,
                            float* O, void* ws, size_t ws_bytes, void* stream) {
  if (!n_ctx_seq) return FASA_EINVAL;
  return decode_step_common(shape, nullptr, q, K, V, Kp, fc_idx, k_new, v_new, n_ctx_seq, budget_seq, S, T, O,
                            ws, ws_bytes, stream);
}

int fasa_pack_kcache_paged(const fasa_shape* shape, const fasa_paging* paging, const void* K,
                           const int32_t* fc_idx, void* Kp, int32_t n_begin, int32_t n_end, void* stream) {
  int rc = check_shape(shape, kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  if (!K || !fc_idx || !Kp || !aligned16(K) || !aligned16(Kp) || !aligned16(fc_idx)) return FASA_EINVAL;
  if (n_begin < 0 || n_end < n_begin || n_end > shape->n_cap) return FASA_EINVAL;
  fasa_shape cover = *shape;
  cover.n_ctx = n_end;                       // the table has to reach the last token packed
  PageMap pm;
  rc = check_paging(paging, &cover, &pm);
  if (rc != FASA_OK) return rc;
  if (n_begin == n_end) return FASA_OK;
  FASA_HIP(launch_pack(*shape, K, fc_idx, Kp, n_begin, n_end, (hipStream_t)stream, pm));
  return FASA_OK;
}

int fasa_decode_step_paged(const fasa_shape* shape, const fasa_paging* paging, const void* q, void* K,
                           void* V, void* Kp, const int32_t* fc_idx, const void* k_new, const void* v_new,
                           const int32_t* n_ctx_seq, const int32_t* budget_seq, float* S, int32_t* T,
                           float* O, void* ws, size_t ws_bytes, void* stream) {
  if (!paging) return FASA_EINVAL;
  return decode_step_common(shape, paging, q, K, V, Kp, fc_idx, k_new, v_new, n_ctx_seq, budget_seq, S, T, O,
                            ws, ws_bytes, stream);
}

size_t fasa_offload_stage_bytes(const fasa_shape* shape) {
  if (check_shape(shape, kNeedCtx | kNeedBudget) != FASA_OK || shape->pairing == FASA_PAIR_LIST) return 0;
  const size_t e = shape->dtype == FASA_BF16 ? 2 : 4;
  const size_t bsel = (size_t)(shape->budget < shape->n_ctx ? shape->budget : shape->n_ctx);
  return align256(2 * (size_t)shape->batch * shape->n_kv_heads * bsel * shape->head_dim * e);
}

int fasa_offload_split_kcache(const fasa_shape* shape, const void* K, const int32_t* fc_idx, void* Kp,
                              void* Knd_host, int32_t n_begin, int32_t n_end, void* stream) {
  int rc = check_shape(shape, kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  if (shape->pairing == FASA_PAIR_LIST) return FASA_EUNSUPPORTED;   // the split works on FC numbers
  if (!K || !fc_idx || !Kp || !Knd_host) return FASA_EINVAL;
  if (!aligned16(K) || !aligned16(Kp) || !aligned16(fc_idx) || !aligned16(Knd_host)) return FASA_EINVAL;
  if (n_begin < 0 || n_end < n_begin || n_end > shape->n_cap) return FASA_EINVAL;
  if (n_begin == n_end) return FASA_OK;
  FASA_HIP(launch_offload_split(*shape, K, fc_idx, Kp, Knd_host, n_begin, n_end, (hipStream_t)stream));
  return FASA_OK;
}

int fasa_offload_decode_step(const fasa_shape* shape, const void* q, void* Kp, const int32_t* fc_idx,
                             void* Knd_host, void* V_host, const void* k_new, const void* v_new,
                             float* S, int32_t* T, float* O, void* ws, size_t ws_bytes, void* stage,
                             size_t stage_bytes, void* stream) {
  int rc = check_shape(shape, kNeedCtx | kNeedBudget | kNeedFc | kNeedStrides);
  if (rc != FASA_OK) return rc;
  if (shape->pairing == FASA_PAIR_LIST) return FASA_EUNSUPPORTED;
  if (!q || !Kp || !fc_idx || !Knd_host || !V_host || !S || !T || !O || !stage) return FASA_EINVAL;
  if ((k_new == nullptr) != (v_new == nullptr)) return FASA_EINVAL;
  if (!aligned16(q) || !aligned16(Kp) || !aligned16(fc_idx) || !aligned16(Knd_host) || !aligned16(V_host) ||
      !aligned16(S) || !aligned16(T) || !aligned16(O) || !aligned16(k_new) || !aligned16(v_new) ||
      !aligned16(stage))
    return FASA_EINVAL;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc != FASA_OK) return rc;
  if (stage_bytes < fasa_offload_stage_bytes(shape)) return FASA_EWORKSPACE;
  const WsLayout w = ws_layout(*shape);
  char* base = (char*)ws;
  uint32_t* hist = (uint32_t*)(base + w.hist_off);
  RowCtl* ctl = (RowCtl*)(base + w.ctl_off);
  uint2* cand = (uint2*)(base + w.cand_off);
  hipStream_t st = (hipStream_t)stream;
  const bool select_all = shape->budget >= shape->n_ctx;
  const int bsel = shape->budget < shape->n_ctx ? shape->budget : shape->n_ctx;
  const size_t e = shape->dtype == FASA_BF16 ? 2 : 4;
  char* KT = (char*)stage;
  char* VT = KT + (size_t)shape->batch * shape->n_kv_heads * bsel * shape->head_dim * e;
  if (k_new) FASA_HIP(launch_offload_append(*shape, Kp, Knd_host, V_host, fc_idx, k_new, v_new, st));
  FASA_HIP(launch_score(*shape, q, Kp, fc_idx, S, select_all ? nullptr : hist, st));
  FASA_HIP(launch_select(*shape, S, hist, ctl, cand, T, st));
  FASA_HIP(launch_offload_gather(*shape, Kp, Knd_host, V_host, fc_idx, T, KT, VT, st));
  // exact attention over the rebuilt rows: the staging buffer is a dense cache of bsel tokens
  fasa_shape ss = *shape;
  ss.n_ctx = bsel;
  ss.budget = bsel;
  ss.kv_stride_n = shape->head_dim;
  ss.kv_stride_h = (int64_t)bsel * shape->head_dim;
  ss.kv_stride_b = (int64_t)shape->n_kv_heads * bsel * shape->head_dim;
  FASA_HIP(launch_attend(ss, true, q, KT, VT, nullptr, O, ctl, (float*)(base + w.part_acc_off),
                         (float*)(base + w.part_ml_off), st));
  return FASA_OK;
}

// ---- offline calibration -------------------------------------------------------------------------
namespace {
struct CalibLayout {
  fasa_shape full, virt;     // all FCs of the real heads; one FC per virtual head
  size_t fc_all_off, fc_v_off, q_v_off, s_full_off, t_full_off, s_v_off, t_v_off, ws_full_off, ws_virt_off, total;
  int kk;
};

int calib_layout(const fasa_shape* shape, int32_t top_k, CalibLayout* L) {
  int rc = check_shape(shape, kNeedCtx);
  if (rc != FASA_OK) return rc;
  if (top_k < 1) return FASA_EINVAL;
  if (shape->pairing == FASA_PAIR_LIST) return FASA_EUNSUPPORTED;   // agreement is defined per FC number
  const int half = shape->head_dim / 2;
  if ((long long)shape->batch * shape->n_kv_heads * half > 65535) return FASA_EUNSUPPORTED;
  if (shape->n_ctx > calib_max_ctx()) return FASA_EUNSUPPORTED;
  const int kk = top_k < shape->n_ctx ? top_k : shape->n_ctx;
  L->kk = kk;
  L->full = *shape;
  L->full.n_fc = half;
  L->full.budget = kk;
  L->virt = *shape;
  L->virt.n_kv_heads = shape->n_kv_heads * half;
  L->virt.n_q_heads = shape->n_q_heads * half;
  L->virt.n_fc = 1;
  L->virt.budget = kk;
  const size_t e = shape->dtype == FASA_BF16 ? 2 : 4;
  const size_t rows = (size_t)shape->batch * shape->n_kv_heads;
  size_t off = 0;
  L->fc_all_off = off; off = align256(off + (size_t)shape->n_kv_heads * half * 4);
  L->fc_v_off = off;   off = align256(off + (size_t)shape->n_kv_heads * half * 4);
  L->q_v_off = off;    off = align256(off + (size_t)shape->batch * shape->n_q_heads * half * shape->head_dim * e);
  L->s_full_off = off; off = align256(off + rows * shape->n_cap * 4);
  L->t_full_off = off; off = align256(off + rows * kk * 4);
  L->s_v_off = off;    off = align256(off + rows * half * shape->n_cap * 4);
  L->t_v_off = off;    off = align256(off + rows * half * kk * 4);
  // the two selection problems get workspaces of their own: their layouts differ, and what one
  // leaves behind (candidate lists) must never sit where the other expects zeroed counters
  L->ws_full_off = off; off += ws_layout(L->full).total;
  L->ws_virt_off = off; off += ws_layout(L->virt).total;
  L->total = off;
  return FASA_OK;
}
}  // namespace

size_t fasa_calibration_workspace_bytes(const fasa_shape* shape, int32_t top_k) {
  CalibLayout L;
  return calib_layout(shape, top_k, &L) == FASA_OK ? L.total : 0;
}

int fasa_contextual_agreement(const fasa_shape* shape, const void* q, const void* Kp_all, int32_t top_k,
                              float* CA_sum, void* cws, size_t cws_bytes, void* stream) {
  CalibLayout L;
  int rc = calib_layout(shape, top_k, &L);
  if (rc != FASA_OK) return rc;
  if (!q || !Kp_all || !CA_sum || !cws) return FASA_EINVAL;
  if (!aligned16(q) || !aligned16(Kp_all) || !aligned16(CA_sum) || !aligned16(cws)) return FASA_EINVAL;
  if (cws_bytes < L.total) return FASA_EWORKSPACE;
  char* base = (char*)cws;
  int32_t* fc_all = (int32_t*)(base + L.fc_all_off);
  int32_t* fc_v = (int32_t*)(base + L.fc_v_off);
  void* q_v = base + L.q_v_off;
  float* S_full = (float*)(base + L.s_full_off);
  int32_t* T_full = (int32_t*)(base + L.t_full_off);
  float* S_v = (float*)(base + L.s_v_off);
  int32_t* T_v = (int32_t*)(base + L.t_v_off);
  hipStream_t st = (hipStream_t)stream;
  const bool all = L.kk >= shape->n_ctx;
  FASA_HIP(launch_calib_prepare(*shape, q, q_v, fc_all, fc_v, st));
  const WsLayout wv = ws_layout(L.virt);
  {  // full-head scores and their top-K set (Alg. 1: "compute full attention scores")
    char* ws = base + L.ws_full_off;
    const WsLayout w = ws_layout(L.full);
    uint32_t* hist = (uint32_t*)(ws + w.hist_off);
    FASA_HIP(launch_ws_clear(L.full, hist, (RowCtl*)(ws + w.ctl_off), st));
    FASA_HIP(launch_score(L.full, q, Kp_all, fc_all, S_full, all ? nullptr : hist, st));
    FASA_HIP(launch_select(L.full, S_full, hist, (RowCtl*)(ws + w.ctl_off), (uint2*)(ws + w.cand_off), T_full, st));
  }
  {  // single-FC scores of every FC and their top-K sets, as one virtual multi-head problem
    char* ws = base + L.ws_virt_off;
    uint32_t* hist = (uint32_t*)(ws + wv.hist_off);
    FASA_HIP(launch_ws_clear(L.virt, hist, (RowCtl*)(ws + wv.ctl_off), st));
    FASA_HIP(launch_score(L.virt, q_v, Kp_all, fc_v, S_v, all ? nullptr : hist, st));
    FASA_HIP(launch_select(L.virt, S_v, hist, (RowCtl*)(ws + wv.ctl_off), (uint2*)(ws + wv.cand_off), T_v, st));
  }
  FASA_HIP(launch_calib_intersect(*shape, T_full, T_v, CA_sum, L.kk, st));
  return FASA_OK;
}

int fasa_select_dominant_fcs(const fasa_shape* shape, const float* ca_mean_host, int32_t* fc_idx_host_out) {
  int rc = check_shape(shape, kNeedFc);
  if (rc != FASA_OK) return rc;
  if (shape->pairing == FASA_PAIR_LIST) return FASA_EUNSUPPORTED;
  if (!ca_mean_host || !fc_idx_host_out) return FASA_EINVAL;
  const int half = shape->head_dim / 2;
  for (int h = 0; h < shape->n_kv_heads; ++h) {
    std::vector<int> order(half);
    for (int i = 0; i < half; ++i) order[i] = i;
    const float* ca = ca_mean_host + (size_t)h * half;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ca[a] > ca[b]; });
    for (int f = 0; f < shape->n_fc; ++f) fc_idx_host_out[h * shape->n_fc + f] = order[f];
  }
  return FASA_OK;
}

const char* fasa_strerror(int status) {
  switch (status) {
    case FASA_OK: return "ok";
    case FASA_EINVAL: return "invalid argument (null or misaligned pointer, bad shape or index list)";
    case FASA_EUNSUPPORTED: return "request outside what the kernels support (head_dim must be 128, GQA group <= 8, explicit dim pairs only for packing, scoring and the decode steps)";
    case FASA_EWORKSPACE: return "workspace smaller than fasa_workspace_bytes()";
    case FASA_EHIP: return "HIP call failed (see fasa_last_hip_error)";
    default: return "unknown status";
  }
}

int fasa_last_hip_error(void) { return g_last_hip_error; }
int fasa_version(void) { return 1000; }

int fasa_profile_enable(int on) { g_prof_on = on != 0; return FASA_OK; }

int fasa_profile_reset(void) {
  for (auto& r : g_prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof_recs.clear();
  g_prof_sums.clear();
  return FASA_OK;
}

int fasa_profile_collect(void) { return profile_fold(); }

int fasa_profile_entry(int i, char* name_out, size_t name_cap, int64_t* launches_out,
                       double* total_ms_out) {
  if (i < 0 || i >= (int)g_prof_sums.size() || !name_out || name_cap == 0) return FASA_EINVAL;
  const ProfSum& s = g_prof_sums[i];
  std::strncpy(name_out, s.name.c_str(), name_cap - 1);
  name_out[name_cap - 1] = '\0';
  if (launches_out) *launches_out = s.launches;
  if (total_ms_out) *total_ms_out = s.ms;
  return FASA_OK;
}

}  // extern "C"
