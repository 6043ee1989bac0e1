// Host-side walk through the C ABI's argument validation, for a build of the library whose host code is
// instrumented with AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_abi_sanitizers.py builds both
// and runs this program; no GPU is needed: every call here is rejected, or accepted as a no-op, on the host).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "dsmoe.h"

static int failures = 0;
#define EXPECT(expr, want)                                                                 \
  do {                                                                                     \
    const long got_ = (long)(expr);                                                        \
    if (got_ != (long)(want)) {                                                            \
      std::fprintf(stderr, "line %d: %s = %ld, wanted %ld\n", __LINE__, #expr, got_, (long)(want)); \
      ++failures;                                                                          \
    }                                                                                      \
  } while (0)

int main() {
  void* fake = reinterpret_cast<void*>(0x1000);   // aligned, never dereferenced on these paths
  void* odd = reinterpret_cast<void*>(0x1004);
  float* ff = static_cast<float*>(fake);
  int32_t* fi = static_cast<int32_t*>(fake);
  uint64_t* fu = static_cast<uint64_t*>(fake);

  dsmoe_desc d = {256, 64, 8, DSMOE_F32, 128, 1024};
  dsmoe_ctx* c = nullptr;
  EXPECT(dsmoe_create(nullptr, &c), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_create(&d, nullptr), DSMOE_ERR_INVALID_ARG);
  for (int bad = 0; bad < 7; ++bad) {
    dsmoe_desc b = d;
    int32_t want = DSMOE_ERR_UNSUPPORTED;
    switch (bad) {
      case 0: b.n_experts = 128; break;
      case 1: b.n_experts = 12; break;
      case 2: b.d_model = 250; break;
      case 3: b.d_ff = 40; break;
      case 4: b.dtype = 7; break;
      case 5: b.d_model = 0; want = DSMOE_ERR_INVALID_ARG; break;
      default: b.max_rows = 128 * 8 + 1; want = DSMOE_ERR_INVALID_ARG; break;
    }
    dsmoe_ctx* t = nullptr;
    EXPECT(dsmoe_create(&b, &t), want);
    EXPECT(t == nullptr, 1);
  }
  EXPECT(dsmoe_create(&d, &c), DSMOE_OK);
  size_t n = 0;
  EXPECT(dsmoe_workspace_bytes(c, &n), DSMOE_OK);
  EXPECT(n > 0, 1);
  EXPECT(dsmoe_workspace_bytes(c, nullptr), DSMOE_ERR_INVALID_ARG);

  EXPECT(dsmoe_route(c, nullptr, fake, nullptr, 4, ff, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(std::strstr(dsmoe_last_error(c), "null pointer") != nullptr, 1);
  EXPECT(dsmoe_route(c, odd, fake, nullptr, 4, ff, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_route(c, fake, fake, nullptr, -1, ff, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_route(c, fake, fake, nullptr, 129, ff, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_route(c, fake, fake, nullptr, 0, ff, nullptr), DSMOE_OK);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_TOPK, 0, 0.f, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_TOPK, 9, 0.f, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_THRESHOLD, 0, -0.5f, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_THRESHOLD, 0, NAN, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_THRESHOLD | DSMOE_SEL_NORMALISED, 0, INFINITY, fu, nullptr, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_TOPK | DSMOE_SEL_NORMALISED, 2, 0.5f, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, 5, 1, 0.f, fu, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_select(c, ff, 4, DSMOE_SEL_THRESHOLD_TOPK, 0, 0.1f, fu, nullptr, nullptr), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_select(c, ff, 0, DSMOE_SEL_THRESHOLD, 0, 0.1f, fu, nullptr, nullptr), DSMOE_OK);
  EXPECT(dsmoe_sparse_fwd(c, fake, fake, nullptr, fake, fake, fake, 4, DSMOE_SEL_TOPK, 2, 0.f, fake, nullptr), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_sparse_fwd_uses_persistent_kernel(c, 32, DSMOE_SEL_TOPK, 4, 0.f), 0);
  EXPECT(dsmoe_sparse_fwd_path(c, 32, DSMOE_SEL_TOPK, 4, 0.f), -1);          // no workspace yet
  EXPECT(dsmoe_sparse_fwd_path(nullptr, 32, DSMOE_SEL_TOPK, 4, 0.f), -1);
  EXPECT(dsmoe_expert_ffn(c, fake, nullptr, fi, fi, fake, fake, fake, fake, nullptr), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_combine(c, nullptr, ff, fi, fi, 4, fake, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_combine(c, fake, ff, fi, fi, 0, fake, nullptr), DSMOE_OK);
  EXPECT(dsmoe_dispatch(c, fake, ff, fu, 4, fi, fi, ff, fi, fi, fi, nullptr, nullptr), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_dispatch_static(c, fake, ff, fu, -1, fi, fi, ff, fi, fi, fi, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_dispatch_static(c, fake, nullptr, fu, 4, fi, fi, ff, fi, fi, fi, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_dispatch_static(c, fake, ff, fu, 4, fi, fi, ff, static_cast<int32_t*>(odd), fi, fi, nullptr, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_mi_loss(c, ff, 4, ff, ff, nullptr), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_set_expert_kind(c, 7), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_set_expert_kind(c, DSMOE_EXPERT_GELU), DSMOE_OK);
  EXPECT(dsmoe_set_expert_kind(c, DSMOE_EXPERT_SWIGLU), DSMOE_OK);
  EXPECT(dsmoe_set_sync_spin_limit(c, -1), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_set_sync_spin_limit(c, 100), DSMOE_OK);
  EXPECT(dsmoe_dense_bwd_mi(c, fake, fake, fake, fake, fake, fake, fake, 4, fake, fake, ff, nullptr, ff, ff, ff, INFINITY, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_dense_bwd(c, fake, fake, fake, fake, fake, fake, fake, 4, fake, fake, nullptr, nullptr, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);
  size_t nb = 0;
  EXPECT(dsmoe_dense_saved_bytes(c, 16, &nb), DSMOE_OK);
  EXPECT(dsmoe_dense_bwd_scratch_bytes(c, 16, &nb), DSMOE_OK);
  EXPECT(dsmoe_dense_saved_bytes(c, -1, &nb), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_profile_enable(c, -1), DSMOE_ERR_INVALID_ARG);
  int32_t nc = 0;
  float a = 0, b = 0;
  EXPECT(dsmoe_profile_read(c, &nc, &a, &b), DSMOE_OK);
  EXPECT(dsmoe_profile_read(c, nullptr, &a, &b), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_set_workspace(c, nullptr, 1 << 20), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_set_workspace(c, reinterpret_cast<void*>(0x1010), (size_t)1 << 30), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_set_workspace(c, fake, 16), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_poll_error(nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_destroy(c), DSMOE_OK);
  EXPECT(dsmoe_destroy(nullptr), DSMOE_OK);
  EXPECT(std::strcmp(dsmoe_last_error(nullptr), "null context"), 0);

  dsmoe_desc big = {256, 64, 8, DSMOE_BF16, 1 << 17, 16};
  EXPECT(dsmoe_create(&big, &c), DSMOE_OK);
  EXPECT(dsmoe_dispatch_static(c, fake, ff, fu, DSMOE_STATIC_DISPATCH_MAX_TOKENS + 1, fi, fi, ff, fi, fi, fi, nullptr, nullptr),
         DSMOE_ERR_UNSUPPORTED);
  EXPECT(dsmoe_destroy(c), DSMOE_OK);

  EXPECT(dsmoe_bench_mfma(nullptr, fake, 8, 8, &a, nullptr, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_bench_stream(fake, 16, 0, 8, fake, &a, &nb, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_bench_xcc_ids(nullptr, 8, nullptr), DSMOE_ERR_INVALID_ARG);

  dsmoe_moa_desc md = {256, 8, 2, 64, DSMOE_BF16, 64};
  dsmoe_moa_ctx* m = nullptr;
  dsmoe_moa_desc mb = md;
  mb.d_head = 96;
  EXPECT(dsmoe_moa_create(&mb, &m), DSMOE_ERR_UNSUPPORTED);
  mb = md;
  mb.n_head = 0;
  EXPECT(dsmoe_moa_create(&mb, &m), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_create(&md, &m), DSMOE_OK);
  EXPECT(dsmoe_moa_workspace_bytes(m, &nb), DSMOE_OK);
  EXPECT(dsmoe_moa_fwd(m, fake, fake, nullptr, fake, fake, fake, fake, 4, 8, DSMOE_SEL_TOPK, 2, 0.f, 1.f, fake, nullptr),
         DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_moa_set_workspace(m, fake, 16), DSMOE_ERR_WORKSPACE);
  EXPECT(dsmoe_moa_set_workspace(m, fake, nb), DSMOE_OK);
  EXPECT(dsmoe_moa_fwd(m, fake, fake, nullptr, fake, fake, fake, fake, 65, 80, DSMOE_SEL_TOPK, 2, 0.f, 1.f, fake, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_fwd(m, fake, fake, nullptr, fake, fake, fake, fake, 4, 3, DSMOE_SEL_TOPK, 2, 0.f, 1.f, fake, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_fwd(m, nullptr, fake, nullptr, fake, fake, fake, fake, 4, 8, DSMOE_SEL_TOPK, 2, 0.f, 1.f, fake, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_fwd(m, fake, fake, nullptr, fake, fake, fake, fake, 4, 8, DSMOE_SEL_TOPK, 2, 0.f, NAN, fake, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_fwd(m, fake, fake, nullptr, fake, fake, fake, fake, 0, 8, DSMOE_SEL_TOPK, 2, 0.f, 1.f, fake, nullptr), DSMOE_OK);
  // backward: size query, and every refusal that happens on the host
  size_t sb = 0;
  EXPECT(dsmoe_moa_bwd_scratch_bytes(m, 4, 8, &sb), DSMOE_OK);
  EXPECT(sb > 0, 1);
  EXPECT(dsmoe_moa_bwd_scratch_bytes(m, 4, 8, nullptr), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd_scratch_bytes(m, 9, 8, &sb), DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd(nullptr, fake, fake, fake, fake, fake, fake, fake, 4, 8, 1.f, fake, fake, ff, nullptr, ff, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd(m, fake, fake, fake, fake, fake, fake, fake, 0, 8, 1.f, fake, fake, ff, nullptr, ff, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd(m, fake, fake, fake, fake, fake, fake, fake, 4, 3, 1.f, fake, fake, ff, nullptr, ff, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd(m, fake, fake, fake, fake, fake, fake, fake, 4, 8, INFINITY, fake, fake, ff, nullptr, ff, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);
  EXPECT(dsmoe_moa_bwd(m, fake, fake, fake, fake, fake, fake, fake, 4, 8, 1.f, fake, fake, ff, nullptr, ff, ff, ff, ff, nullptr),
         DSMOE_ERR_INVALID_ARG);   // no dense forward came before
  EXPECT(std::strstr(dsmoe_moa_last_error(m), "dsmoe_moa_fwd") != nullptr, 1);
  EXPECT(dsmoe_moa_destroy(m), DSMOE_OK);

  if (failures) {
    std::fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  std::puts("abi sanitizer driver: all checks passed");
  return 0;
}
