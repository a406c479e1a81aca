// Host-side exerciser of the C ABI for sanitizer builds (paper_2602_03152_amd/build.py --sanitize):
// walks every entry point's argument validation and the pure host functions - workspace sizes and
// launch plans over a sweep of shapes, the dominant-list checker, the dominant-FC choice - without a
// GPU.  Compiled together with the library's sources with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side (device code is untouched); any report fails the run.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fasa.h"

#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static fasa_shape shape(int batch, int hq, int hkv, int f, int n, int cap, int budget, int dtype = FASA_BF16) {
  fasa_shape s{};
  s.batch = batch; s.n_q_heads = hq; s.n_kv_heads = hkv; s.head_dim = 128; s.n_fc = f; s.n_ctx = n; s.n_cap = cap;
  s.budget = budget; s.dtype = dtype; s.pairing = FASA_PAIR_ROTATE_HALF;
  s.kv_stride_n = 128; s.kv_stride_h = (int64_t)cap * 128; s.kv_stride_b = (int64_t)hkv * cap * 128;
  return s;
}

int main() {
  void* A = reinterpret_cast<void*>(0x10000);   // a fake aligned "device pointer": validation must fail before it is touched
  // ---- workspace sizes and launch plans over a sweep of shapes (pure host arithmetic) ----
  size_t checked = 0;
  for (int batch : {1, 2, 3, 8, 16, 64})
    for (int hkv : {1, 2, 3, 4, 8})
      for (int g : {1, 2, 4, 7, 8})
        for (int n : {1, 2, 63, 64, 1000, 4096, 32768, 33279, 131072, (1 << 20) + 77})
          for (int budget : {1, 2, 255, 2048, 6193, 1 << 21}) {
            const int cap = (n + 63) / 64 * 64;
            fasa_shape s = shape(batch, hkv * g, hkv, 16, n, cap, budget);
            const size_t b = fasa_workspace_bytes(&s);
            EXPECT(b > 0 && b % 256 == 0);
            EXPECT(fasa_offload_stage_bytes(&s) % 256 == 0);
            // argument validation of the step with too small a workspace, then with a null pointer
            EXPECT(fasa_decode_step(&s, A, A, A, A, (const int32_t*)A, nullptr, nullptr, (float*)A, (int32_t*)A, (float*)A, A,
                                    b / 2, nullptr) == FASA_EWORKSPACE);
            EXPECT(fasa_workspace_init(&s, A, b - 1, nullptr) == FASA_EWORKSPACE);
            EXPECT(fasa_decode_step(&s, nullptr, A, A, A, (const int32_t*)A, nullptr, nullptr, (float*)A, (int32_t*)A,
                                    (float*)A, A, b, nullptr) == FASA_EINVAL);
            ++checked;
          }
  // ---- bad shapes ----
  {
    fasa_shape s = shape(1, 32, 8, 16, 1000, 1024, 100);
    fasa_shape t = s; t.n_cap = 1000;          EXPECT(fasa_workspace_bytes(&t) == 0);
    t = s; t.n_ctx = 2000;                     EXPECT(fasa_workspace_bytes(&t) == 0);
    t = s; t.budget = 0;                       EXPECT(fasa_workspace_bytes(&t) == 0);
    t = s; t.head_dim = 64;                    EXPECT(fasa_topk(&t, (const float*)A, (int32_t*)A, A, 1 << 30, nullptr) == FASA_EUNSUPPORTED);
    t = s; t.n_q_heads = 30;                   EXPECT(fasa_score(&t, A, A, (const int32_t*)A, (float*)A, nullptr) == FASA_EINVAL);
    t = s; t.pairing = 7;                      EXPECT(fasa_score(&t, A, A, (const int32_t*)A, (float*)A, nullptr) == FASA_EINVAL);
    EXPECT(fasa_workspace_bytes(nullptr) == 0);
    EXPECT(fasa_pack_kcache(&s, A, (const int32_t*)A, A, 5, 4, nullptr) == FASA_EINVAL);
    EXPECT(fasa_pack_kcache(&s, A, (const int32_t*)A, A, 7, 7, nullptr) == FASA_OK);     // empty range: nothing launched
    EXPECT(fasa_decode_step_static(&s, nullptr, A, A, A, (const int32_t*)A, nullptr, nullptr, (float*)A, (int32_t*)A,
                                   (float*)A, nullptr) == FASA_EINVAL);
    fasa_shape big = shape(64, 32, 8, 16, 65536, 65536, 4096);
    EXPECT(fasa_decode_step_static(&big, A, A, A, A, (const int32_t*)A, nullptr, nullptr, (float*)A, (int32_t*)A, (float*)A,
                                   nullptr) == FASA_EWORKSPACE);
    fasa_paging pg{(const int32_t*)A, 4, 16, 100, 0};
    EXPECT(fasa_pack_kcache_paged(&s, &pg, A, (const int32_t*)A, A, 0, 65, nullptr) == FASA_EINVAL);   // table ends at 64
    pg.page_size = 12;
    EXPECT(fasa_pack_kcache_paged(&s, &pg, A, (const int32_t*)A, A, 0, 16, nullptr) == FASA_EINVAL);   // not a power of two
    EXPECT(fasa_calibration_workspace_bytes(&s, 0) == 0);
    EXPECT(fasa_calibration_workspace_bytes(&s, 64) > 0);
  }
  // ---- dominant-list checker and dominant-FC choice (host arrays) ----
  {
    fasa_shape s = shape(1, 8, 2, 4, 100, 128, 10);
    std::vector<int32_t> fc = {0, 5, 63, 7, 1, 2, 3, 4};
    EXPECT(fasa_validate_fc_idx(&s, fc.data()) == FASA_OK);
    fc[3] = 64;  EXPECT(fasa_validate_fc_idx(&s, fc.data()) == FASA_EINVAL);
    fc[3] = 5;   EXPECT(fasa_validate_fc_idx(&s, fc.data()) == FASA_EINVAL);   // twice in one head
    fc[3] = -1;  EXPECT(fasa_validate_fc_idx(&s, fc.data()) == FASA_EINVAL);
    s.pairing = FASA_PAIR_LIST;
    std::vector<int32_t> pairs = {0, 64, 1, 127, 2, 3, 9, 10,  5, 6, 7, 8, 100, 101, 11, 12};
    EXPECT(fasa_validate_fc_idx(&s, pairs.data()) == FASA_OK);
    pairs[15] = 128; EXPECT(fasa_validate_fc_idx(&s, pairs.data()) == FASA_EINVAL);
    s.pairing = FASA_PAIR_ROTATE_HALF;
    std::vector<float> ca(2 * 64);
    for (int i = 0; i < 128; ++i) ca[i] = (float)((i * 37) % 64) / 64.f;
    std::vector<int32_t> out(8, -1);
    EXPECT(fasa_select_dominant_fcs(&s, ca.data(), out.data()) == FASA_OK);
    EXPECT(fasa_validate_fc_idx(&s, out.data()) == FASA_OK);
    EXPECT(fasa_select_dominant_fcs(&s, nullptr, out.data()) == FASA_EINVAL);
  }
  for (int c : {0, -1, -2, -3, -4, -99}) EXPECT(fasa_strerror(c) != nullptr);
  char name[8];
  EXPECT(fasa_profile_entry(0, name, sizeof name, nullptr, nullptr) == FASA_EINVAL);
  std::printf("abi_host_check: %zu shapes, all checks passed\n", checked);
  return 0;
}
