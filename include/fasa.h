/*
 * fasa.h -- C ABI of the MI355X (gfx950) FASA decode hot path.
 *
 * FASA = frequency-aware sparse attention.  One decode step of one attention layer does
 *   (1) TIP   : score every cached token with a partial dot product over the KV head's
 *               dominant RoPE frequency chunks (FCs)                     (paper Sec. 4.1)
 *   (2) TopK-I: keep the indices of the B best-scored tokens per KV head (paper Sec. 4.1)
 *   (3) FAC   : exact softmax attention over the gathered B rows of K, V (paper Sec. 4.2)
 * The dominant-FC list I_dom is an input (it comes from an offline calibration, Alg. 1).
 *
 * Conventions that hold for every entry point
 *   - All tensor pointers are DEVICE pointers (HBM) unless the name ends in _host.  The caller owns
 *     every buffer, including the workspace; the library allocates and frees nothing on the device.
 *     A workspace is prepared once with fasa_workspace_init and then reused call after call.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream).  No entry
 *     point synchronises the host.  Calls that share a workspace must be ordered by the stream.
 *   - Return value: FASA_OK (0) or a negative fasa_status.  Arguments are validated before the
 *     first HIP call, so error paths work on a host without a GPU.  Inputs must be finite; the
 *     ranking of NaN scores is unspecified.
 *   - FC i of a d-dim head vector is the rotation pair (dim i, dim i + d/2) ("rotate-half"
 *     storage of the FC of paper Sec. 3.1) unless shape->pairing says otherwise (fasa_pairing
 *     below); FCs are never split (paper App. D.2).
 *   - GQA: query head hq reads KV head hq / G, G = n_q_heads / n_kv_heads.  There is one score
 *     vector and one index set per KV head; scores are summed over the G query heads of the group.
 *   - Layouts (row-major, innermost last):
 *       q      [batch][n_q_heads][head_dim]                 dtype
 *       K, V   [batch][n_kv_heads][>= n_ctx tokens][head_dim] dtype, element strides kv_stride_{b,h,n},
 *                                                            K holds post-RoPE keys
 *       fc_idx [n_kv_heads][n_fc]                           int32, distinct values in [0, head_dim/2)
 *              ([n_kv_heads][n_fc][2], distinct dims in [0, head_dim), with FASA_PAIR_LIST)
 *       Kp     [batch][n_kv_heads][n_fc][n_cap][2]          dtype, FC-major copy of the dominant K dims
 *       S      [batch][n_kv_heads][n_cap]                   float32, entries >= n_ctx untouched
 *       T      [batch][n_kv_heads][min(budget, n_ctx)]      int32, a SET: order unspecified, no duplicates
 *       O      [batch][n_q_heads][head_dim]                 float32
 *   - Alignment: every pointer 16-byte aligned; n_cap a multiple of 64; kv_stride_n a multiple of 8
 *     elements and >= head_dim; head_dim == 128; 1 <= G <= 8.
 */
#ifndef FASA_H
#define FASA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FASA_OK = 0,
  FASA_EINVAL = -1,       /* null pointer, bad shape, misaligned pointer, bad fc_idx */
  FASA_EUNSUPPORTED = -2, /* valid request outside what the kernels are built for      */
  FASA_EWORKSPACE = -3,   /* workspace smaller than fasa_workspace_bytes()             */
  FASA_EHIP = -4          /* a HIP call failed; see fasa_last_hip_error()              */
} fasa_status;

typedef enum { FASA_BF16 = 0, FASA_F32 = 1 } fasa_dtype;

/* Which two head dims entry f of a head's dominant list names (paper Sec. 3.1 defines an FC as a
 * 2-D rotation subspace; where its two components are stored is a property of the model's weights):
 *   FASA_PAIR_ROTATE_HALF  the entry is an FC number i, stored at dims (i, i + d/2);
 *   FASA_PAIR_INTERLEAVED  the entry is an FC number i, stored at dims (2i, 2i + 1), the indexing
 *                          Sec. 3.1 itself writes;
 *   FASA_PAIR_LIST         the entry is the dim pair itself, fc_idx being [n_kv_heads][n_fc][2]: heads
 *                          whose rotary encoding covers only part of the dims, or whose dominant
 *                          components are single dims rather than rotation pairs (paper Sec. 6,
 *                          partial-RoPE and ALiBi heads); any grouping of the listed dims into pairs
 *                          gives the same scores.
 * Every entry point that takes fc_idx reads it this way, the packed copy Kp holding
 * (K[.., lo_f], K[.., hi_f]) per entry.  The memory-optimised variant, the calibration entry points
 * and fasa_select_dominant_fcs work on FC numbers: they return FASA_EUNSUPPORTED for FASA_PAIR_LIST. */
typedef enum { FASA_PAIR_ROTATE_HALF = 0, FASA_PAIR_INTERLEAVED = 1, FASA_PAIR_LIST = 2 } fasa_pairing;

typedef struct fasa_shape {
  int32_t batch;       /* Bt                                                            */
  int32_t n_q_heads;   /* Hq                                                            */
  int32_t n_kv_heads;  /* Hkv, divides Hq                                               */
  int32_t head_dim;    /* d                                                             */
  int32_t n_fc;        /* F = |I_dom| per KV head (paper: N_tip), 1 .. d/2              */
  int32_t n_ctx;       /* N: valid cached tokens this step (paper: t), 1 .. n_cap       */
  int32_t n_cap;       /* token capacity of the Kp and S planes                         */
  int32_t budget;      /* B (paper: N_fac) >= 1; B >= N selects every token             */
  int32_t dtype;       /* fasa_dtype of q, K, V, Kp                                     */
  int32_t pairing;     /* fasa_pairing; 0 = rotate-half                                 */
  int64_t kv_stride_b; /* element strides of K and V; the head_dim stride is 1          */
  int64_t kv_stride_h;
  int64_t kv_stride_n;
} fasa_shape;

/* Bytes of device workspace that any entry point below needs for `shape` (host-only, pure).
 * Returns 0 if the shape is invalid. */
size_t fasa_workspace_bytes(const fasa_shape* shape);

/* Prepares a workspace: zeroes the counters and histograms the selection and attention stages
 * count in.  Call once after allocating (or after anything else wrote to) the workspace, and again
 * after a call that returned an error.  Every successful fasa_topk / fasa_sparse_attend /
 * fasa_dense_attend / fasa_decode_step leaves the workspace prepared for the next call, so a decode
 * loop initialises once.  The workspace layout depends on batch * n_kv_heads only for the part
 * that must be zero, so one prepared workspace serves calls whose n_ctx and budget vary, as long
 * as it is at least fasa_workspace_bytes() of each call's shape. */
int fasa_workspace_init(const fasa_shape* shape, void* ws, size_t ws_bytes, void* stream);

/* Host-side check of a dominant-FC list (HOST pointer [n_kv_heads][n_fc]): every value in
 * [0, head_dim/2), no duplicates within a head (an FC is selected whole or not at all,
 * paper App. D.2).  FASA_PAIR_LIST: [n_kv_heads][n_fc][2], every value in [0, head_dim), no dim
 * twice within a head. */
int fasa_validate_fc_idx(const fasa_shape* shape, const int32_t* fc_idx_host);

/* Dominant-key cache maintenance (paper Alg. 2: Split + UpdateCache of k^dom).
 * For tokens n in [n_begin, n_end), 0 <= n_begin <= n_end <= n_cap:
 *     Kp[b,h,f,n,0] = K[b,h,n,i],  Kp[b,h,f,n,1] = K[b,h,n,i + d/2],  i = fc_idx[h,f]
 * (the two dims shape->pairing names, in general).  A bit-exact copy.  Full pack after prefill: [0, N); append of one decoded token: [N-1, N).
 * shape->n_ctx and shape->budget are not used. */
int fasa_pack_kcache(const fasa_shape* shape, const void* K, const int32_t* fc_idx, void* Kp,
                     int32_t n_begin, int32_t n_end, void* stream);

/* TIP scoring (paper Sec. 4.1, S_t = sum over I_dom of single-FC scores; Alg. 2: q^dom (K^dom)^T):
 *     S[b,h,n] = sum_{g<G} sum_{f<F} ( q[b,hG+g,i_f] Kp[b,h,f,n,0] + q[b,hG+g,i_f+d/2] Kp[b,h,f,n,1] )
 * for n < n_ctx (i_f, i_f + d/2: in general the two dims shape->pairing names for entry f).
 * Raw logits: no 1/sqrt(d), no softmax.  float32 accumulation. */
int fasa_score(const fasa_shape* shape, const void* q, const void* Kp, const int32_t* fc_idx,
               float* S, void* stream);

/* TopK-I (paper Sec. 4.1, T_t = TopK-I(S_t, N_fac)): for each (b,h) the index set of the
 * min(budget, n_ctx) largest S[b,h,0:n_ctx].  Equal scores are resolved towards the lower index;
 * -0 and +0 are equal.  Needs a prepared workspace (fasa_workspace_init) and leaves it prepared. */
int fasa_topk(const fasa_shape* shape, const float* S, int32_t* T, void* ws, size_t ws_bytes,
              void* stream);

/* FAC (paper Sec. 4.2, eq. fac_output): for every query head hq, h = hq / G,
 *     O[b,hq] = softmax_j( q[b,hq] . K[b,h,T[b,h,j]] / sqrt(d) ) V[b,h,T[b,h,j]]
 * over the min(budget, n_ctx) entries of T[b,h].  Rows are used as cached (no re-rotation).
 * float32 accumulation and output.  T entries must lie in [0, n_ctx); entries outside are clamped
 * into that range before use (memory safety only: the result is then unspecified). */
int fasa_sparse_attend(const fasa_shape* shape, const void* q, const void* K, const void* V,
                       const int32_t* T, float* O, void* ws, size_t ws_bytes, void* stream);

/* Full-KV decode attention over tokens [0, n_ctx) (the paper's FKV baseline, Sec. 4.4); same
 * kernel family as fasa_sparse_attend with contiguous loads.  budget and n_fc are not used. */
int fasa_dense_attend(const fasa_shape* shape, const void* q, const void* K, const void* V,
                      float* O, void* ws, size_t ws_bytes, void* stream);

/* One whole decode step on one stream without host round trips (paper Sec. 4.1-4.2; Alg. 2 order:
 * the new key joins the dominant cache before scoring):
 *   if k_new != NULL: K[b,h,n_ctx-1,:] = k_new[b,h,:], V[b,h,n_ctx-1,:] = v_new[b,h,:]
 *                     ([batch][n_kv_heads][head_dim], dtype) and the row's dominant FCs go to Kp;
 *                     k_new and v_new must be both NULL or both non-NULL;
 *   then S, T and O exactly as fasa_score -> S, fasa_topk -> T, fasa_sparse_attend -> O define them
 *   (T the same set, ties towards the lower index; O up to the order of float32 additions).
 * S and T are outputs the caller may inspect (S doubles as the score scratch).
 * How it runs: bf16 caches take two launches - the scoring kernel, which also counts a histogram of
 * the scores, then one kernel in which every workgroup classifies a range of tokens against the
 * B-th score's histogram bin and attends at once over the winners it owns, the row's last workgroup
 * settling the ties of that bin and merging the partial results.  float32 caches, rows longer than
 * 2^20 tokens and budget >= n_ctx run the three stand-alone kernels back to back. */
int fasa_decode_step(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                     const int32_t* fc_idx, const void* k_new, const void* v_new, float* S,
                     int32_t* T, float* O, void* ws, size_t ws_bytes, void* stream);

/* fasa_decode_step for callers that cannot allocate device memory or hand over a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is an array inside the library, FASA_STATIC_WS_BYTES per GPU, held by every GPU the
 * library is loaded on until the process ends.  The call allocates and frees nothing; it launches one
 * small clearing kernel (no memset node) and then the kernels of fasa_decode_step.
 *   - Shapes whose workspace (fasa_workspace_bytes without the paged-cache slot list) exceeds
 *     FASA_STATIC_WS_BYTES are refused with FASA_EWORKSPACE before any HIP call.
 *   - No fasa_workspace_init is needed: every call clears what must start at zero.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race.  Order them on one stream.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress) and must not be
 *     made while the stream is being captured; later calls may be.
 * Arguments and results otherwise as fasa_decode_step. */
#define FASA_STATIC_WS_BYTES (32u << 20)
int fasa_decode_step_static(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                            const int32_t* fc_idx, const void* k_new, const void* v_new, float* S,
                            int32_t* T, float* O, void* stream);

/* fasa_decode_step for a batch whose sequences differ in length (paper Sec. 4.1-4.2 per sequence;
 * the decode loop of Alg. 2 where t advances every step): the lengths live on the DEVICE, so the
 * same call - or one captured HIP graph of it - serves every step of a growing, ragged batch.
 *   n_ctx_seq  DEVICE int32[batch], required: valid tokens of sequence b, clamped by the kernels into
 *              [1, shape->n_ctx];
 *   budget_seq DEVICE int32[batch] or NULL: token budget of sequence b, clamped into
 *              [1, shape->budget]; NULL = shape->budget for all.
 * shape->n_ctx and shape->budget are UPPER BOUNDS: they size the launches and the workspace, and fix
 * the row pitch of T at P = min(shape->budget, shape->n_ctx).  For sequence b, with N_b and
 * B_b = min(budget_b, N_b) after clamping:
 *   k_new/v_new (if given) go to position N_b - 1; S[b,h,0:N_b] and T[b,h,0:B_b] (at T + (b*Hkv+h)*P)
 *   are written, entries beyond are left as they were; O[b] attends over exactly those B_b tokens.
 * The arrays are read by the kernels when they run, not at call time: they must stay valid and
 * unchanged until the step has finished on the stream.  Needs a prepared workspace and leaves it
 * prepared.  All other arguments as fasa_decode_step. */
int fasa_decode_step_ragged(const fasa_shape* shape, const void* q, void* K, void* V, void* Kp,
                            const int32_t* fc_idx, const void* k_new, const void* v_new,
                            const int32_t* n_ctx_seq, const int32_t* budget_seq, float* S, int32_t* T,
                            float* O, void* ws, size_t ws_bytes, void* stream);

/* ---- paged K/V cache (serving engines that hand out the cache in fixed-size blocks) --------------
 * The rows of K and V live in one pool of blocks of `page_size` tokens; sequence b's logical block j
 * (tokens j*page_size .. (j+1)*page_size - 1) is pool block block_table[b*max_blocks + j].  Row (b, h, n):
 *     K + block_table[b*max_blocks + n / page_size] * kv_stride_b + h * kv_stride_h
 *       + (n % page_size) * kv_stride_n
 * i.e. kv_stride_b is the element stride between POOL BLOCKS; any block layout with these three
 * strides works ([block][token][head][dim], [block][head][token][dim], ...).  V uses the same table
 * and strides.  The packed copy Kp, S and T stay as described above (logical token numbers).
 * Table entries outside [0, n_pool_blocks) are clamped into it before use (memory safety only). */
typedef struct fasa_paging {
  const int32_t* block_table; /* DEVICE int32 [batch][max_blocks]                                  */
  int32_t max_blocks;         /* row pitch of block_table; max_blocks * page_size >= tokens touched */
  int32_t page_size;          /* tokens per block, a power of two                                   */
  int32_t n_pool_blocks;      /* blocks in the pool; n_pool_blocks * page_size < 2^31               */
  int32_t reserved;           /* must be 0                                                          */
} fasa_paging;

/* fasa_pack_kcache reading a paged K (paper Alg. 2, Split + UpdateCache of k^dom, as above). */
int fasa_pack_kcache_paged(const fasa_shape* shape, const fasa_paging* paging, const void* K,
                           const int32_t* fc_idx, void* Kp, int32_t n_begin, int32_t n_end, void* stream);

/* fasa_decode_step / fasa_decode_step_ragged on a paged K/V cache (paper Sec. 4.1-4.2, Alg. 2 order).
 * n_ctx_seq and budget_seq are optional here (both NULL: the uniform values of the shape).  The
 * selection stage also records the pool slot of every selected token in the workspace, so the
 * attention stage gathers rows without reading the table again.  T receives logical token numbers. */
int fasa_decode_step_paged(const fasa_shape* shape, const fasa_paging* paging, const void* q, void* K,
                           void* V, void* Kp, const int32_t* fc_idx, const void* k_new, const void* v_new,
                           const int32_t* n_ctx_seq, const int32_t* budget_seq, float* S, int32_t* T,
                           float* O, void* ws, size_t ws_bytes, void* stream);

/* ---- memory-optimised variant (paper Sec. 4.3 and Alg. 2: "FASA-M") -----------------------------
 * Only the dominant key dims (Kp) stay on the device.  The non-dominant key dims and all values
 * live in PINNED HOST memory that the device can address (hipHostMalloc / a pinned torch tensor):
 *     Knd_host [batch][n_kv_heads][n_cap][head_dim - 2*n_fc]   dtype, non-dominant dims of each key,
 *                                                               ascending dim order
 *     V_host   [batch][n_kv_heads][tokens][head_dim]           dtype, strides kv_stride_{b,h,n}
 * Per step the device itself fetches the selected rows over PCIe (Alg. 2: SelectTokens,
 * TransferToGPU), rebuilds the full key rows from both parts (Combine) into `stage`, a DEVICE
 * buffer of fasa_offload_stage_bytes(), and runs the same attention over it.  Results equal those
 * of fasa_decode_step on the same cache (same T; O up to float32 summation order). */

/* Bytes of the device staging buffer for the gathered rows (host-only, pure; 0 on a bad shape). */
size_t fasa_offload_stage_bytes(const fasa_shape* shape);

/* Alg. 2 Split + UpdateCache for tokens [n_begin, n_end): reads K (DEVICE, strides kv_stride_*),
 * writes the dominant pairs to Kp (DEVICE) and the remaining dims to Knd_host (HOST, pinned). */
int fasa_offload_split_kcache(const fasa_shape* shape, const void* K, const int32_t* fc_idx, void* Kp,
                              void* Knd_host, int32_t n_begin, int32_t n_end, void* stream);

/* One decode step of the memory-optimised variant.  k_new / v_new ([batch][n_kv_heads][head_dim],
 * DEVICE, both NULL or both set) are split and appended at position n_ctx - 1 first (Alg. 2 order).
 * Needs a prepared workspace like fasa_decode_step. */
int fasa_offload_decode_step(const fasa_shape* shape, const void* q, void* Kp, const int32_t* fc_idx,
                             void* Knd_host, void* V_host, const void* k_new, const void* v_new,
                             float* S, int32_t* T, float* O, void* ws, size_t ws_bytes, void* stage,
                             size_t stage_bytes, void* stream);

/* ---- offline calibration (paper Sec. 3.3 eq. ca_k, Sec. 4.1 objective, Alg. 1) ---------------------
 * Contextual agreement of every single FC with the full head for one query (one calibration
 * sample):   CA[b,h,i] = | TopK-I(alpha, K) & TopK-I(alpha^(i), K) | / K,
 * alpha = full-head raw scores, alpha^(i) = scores of FC i alone, both summed over the GQA group of
 * KV head h, ranked like fasa_topk (ties towards the lower index), K = min(top_k, n_ctx).
 *   Kp_all  DEVICE [batch][n_kv_heads][head_dim/2][n_cap][2]: fasa_pack_kcache with n_fc = head_dim/2
 *           and fc_idx[h] = 0, 1, .., head_dim/2 - 1 (same shape->pairing as this call)
 *   CA_sum  DEVICE float [batch][n_kv_heads][head_dim/2]: the call ADDS this sample's CA to it, so a
 *           loop over samples leaves the sum; divide by the number of samples for the mean
 *   cws     DEVICE scratch of fasa_calibration_workspace_bytes(); needs no preparation
 * shape->n_fc and shape->budget are not used.  n_ctx <= 262144 and batch * n_kv_heads * head_dim/2
 * <= 65535, else FASA_EUNSUPPORTED. */
size_t fasa_calibration_workspace_bytes(const fasa_shape* shape, int32_t top_k);
int fasa_contextual_agreement(const fasa_shape* shape, const void* q, const void* Kp_all, int32_t top_k,
                              float* CA_sum, void* cws, size_t cws_bytes, void* stream);

/* Alg. 1, stage 2 (host-only): fc_idx_host_out[h][0..n_fc) = the n_fc FCs of KV head h with the
 * largest mean CA, ca_mean_host being HOST float [n_kv_heads][head_dim/2]; equal values go to the
 * lower FC index; descending order of CA. */
int fasa_select_dominant_fcs(const fasa_shape* shape, const float* ca_mean_host, int32_t* fc_idx_host_out);

/* Static description of a status code. */
const char* fasa_strerror(int status);
/* hipError_t value of the last failed HIP call on this thread (0 if none). */
int fasa_last_hip_error(void);
/* Library version, major * 1000 + minor. */
int fasa_version(void);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch records the GPU
 * timestamps of its own start and end (kernel execution only, no launch gap).
 * fasa_profile_collect() synchronises the device, folds the recorded launches into per-kernel
 * totals and returns the number of distinct kernels seen since the last reset;
 * fasa_profile_entry() reads entry i: kernel name (copied, NUL-terminated), launches, total ms.
 * Not thread-safe; meant for a single benchmarking thread. */
int fasa_profile_enable(int on);
int fasa_profile_reset(void);
int fasa_profile_collect(void);
int fasa_profile_entry(int i, char* name_out, size_t name_cap, int64_t* launches_out,
                       double* total_ms_out);

#ifdef __cplusplus
}
#endif
#endif /* FASA_H */
