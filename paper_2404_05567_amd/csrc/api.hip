// C-ABI entry points of libdsmoe: argument validation, workspace carve-up and kernel sequencing.
// All arithmetic lives in the kernels; nothing here touches tensor data on the host.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.h"

using namespace dsmoe;

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int32_t fail(dsmoe_ctx* c, int32_t code, const char* fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

int32_t hip_fail(dsmoe_ctx* c, hipError_t e, const char* what) {
  return fail(c, DSMOE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

WorkspaceLayout make_layout(const dsmoe_desc& d, size_t esize) {
  WorkspaceLayout w{};
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
  const size_t nblk = (size_t)(d.max_tokens + kDispatchTokensPerBlock - 1) / kDispatchTokensPerBlock + 1;
  const size_t E = (size_t)d.n_experts, rows = (size_t)d.max_rows, T = (size_t)d.max_tokens;
  w.err_flag = take(16);
  w.blk_cnt = take(nblk * E * 4);
  w.blk_tok = take(nblk * 4);
  w.h = take(rows * d.d_ff * esize);
  w.probs = take(T * E * 4);
  w.mask = take(T * 8);
  w.cnt_tok = take(T * 4);
  w.expert_off = take((E + 1) * 4);
  w.row_token = take(rows * 4);
  w.row_weight = take(rows * 4);
  w.tok_off = take((T + 1) * 4);
  w.tok_rows = take(rows * 4);
  w.nnz = take(4);
  w.y_perm = take(rows * d.d_model * esize);
  w.stat_part = take((size_t)kStatMaxBlocks * 128 * 4);
  w.k_dev = take(4);
  const size_t dec_rows = d.dtype == DSMOE_BF16 ? (size_t)std::min<int64_t>(d.max_tokens, kDecodeMaxTokens) * E : 0;
  w.dec_info = take(32);
  w.dec_arrivals = take(decode_arrival_slots(d) * 4);
  w.dec_p1 = take(dec_rows * 2 * d.d_ff * 4);
  w.dec_p2 = take(dec_rows * d.d_model * 4);
  w.dec_ht = take((d.dtype == DSMOE_BF16 ? (size_t)std::min<int64_t>(d.max_tokens, kDecodeMaxTokens) : 0) * E * d.d_ff * 2);
  w.dec_sync = take(kDenseSyncTotalWords * 4);
  w.tiny_p1 = take(decode_tiny_p1_bytes(d));
  w.tiny_p2 = take(decode_tiny_p2_bytes(d));
  w.total = o;
  return w;
}

// counters of the all-expert decode kernel at zero, its publication words at "not yet published"
hipError_t reset_dense_sync(dsmoe_ctx* c, hipStream_t s) {
  char* base = c->workspace + c->ws.dec_sync;
  if (hipError_t e = hipMemsetAsync(base, 0, (size_t)kDensePubWeight * 4, s)) return e;
  return hipMemsetAsync(base + (size_t)kDensePubWeight * 4, 0xff, (size_t)128 * 64 * 4, s);
}

// checks shared by every call that enqueues work
int32_t check_call(dsmoe_ctx* c, int32_t T, bool needs_ws) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (T < 0) return fail(c, DSMOE_ERR_INVALID_ARG, "T must be >= 0 (got %d)", T);
  if (T > c->desc.max_tokens)
    return fail(c, DSMOE_ERR_INVALID_ARG, "T = %d exceeds max_tokens = %d", T, c->desc.max_tokens);
  if (needs_ws && !c->workspace) return fail(c, DSMOE_ERR_WORKSPACE, "no workspace set (dsmoe_set_workspace)");
  return DSMOE_OK;
}

// Validates a selection request and resolves DSMOE_SEL_NORMALISED: on return `mode` is one of the three base
// modes and `eps` the raw-probability threshold (the paper's normalised threshold divided by N, Sec. 4.2).
int32_t check_select_args(dsmoe_ctx* c, int32_t& mode, int32_t k, float& eps) {
  if (mode & DSMOE_SEL_NORMALISED) {
    mode &= ~DSMOE_SEL_NORMALISED;
    if (mode != DSMOE_SEL_THRESHOLD && mode != DSMOE_SEL_THRESHOLD_TOPK)
      return fail(c, DSMOE_ERR_INVALID_ARG, "DSMOE_SEL_NORMALISED goes with a threshold mode (got mode %d)", mode);
    if (!(eps >= 0.f) || std::isinf(eps)) return fail(c, DSMOE_ERR_INVALID_ARG, "eps must be finite and >= 0");
    eps = eps / static_cast<float>(c->desc.n_experts);
  }
  if (mode == DSMOE_SEL_TOPK) {
    if (k < 1 || k > c->desc.n_experts)
      return fail(c, DSMOE_ERR_INVALID_ARG, "k = %d outside [1, %d]", k, c->desc.n_experts);
  } else if (mode == DSMOE_SEL_THRESHOLD || mode == DSMOE_SEL_THRESHOLD_TOPK) {
    if (!(eps >= 0.f) || std::isinf(eps)) return fail(c, DSMOE_ERR_INVALID_ARG, "eps must be finite and >= 0");
  } else {
    return fail(c, DSMOE_ERR_INVALID_ARG, "unknown selection mode %d", mode);
  }
  return DSMOE_OK;
}

#define REQUIRE_PTR(c, p)                                                                         \
  do {                                                                                            \
    if ((p) == nullptr) return fail((c), DSMOE_ERR_INVALID_ARG, "null pointer: %s", #p);           \
    if (misaligned(p)) return fail((c), DSMOE_ERR_INVALID_ARG, "pointer not 16-byte aligned: %s", #p); \
  } while (0)
#define OPTIONAL_PTR(c, p)                                                                        \
  do {                                                                                            \
    if ((p) != nullptr && misaligned(p))                                                          \
      return fail((c), DSMOE_ERR_INVALID_ARG, "pointer not 16-byte aligned: %s", #p);              \
  } while (0)
// the expert's weight matrices: the two-matrix GeLU expert has no w_up (the argument is ignored)
#define REQUIRE_EXPERT_WEIGHTS(c, w_gate, w_up, w_down)                                            \
  do {                                                                                            \
    REQUIRE_PTR(c, w_gate);                                                                       \
    if ((c)->expert_kind == DSMOE_EXPERT_SWIGLU) REQUIRE_PTR(c, w_up);                             \
    REQUIRE_PTR(c, w_down);                                                                       \
  } while (0)
#define HIP_TRY(c, expr)                                    \
  do {                                                      \
    hipError_t e_ = (expr);                                 \
    if (e_ != hipSuccess) return hip_fail((c), e_, #expr);  \
  } while (0)

}  // namespace

extern "C" {

int32_t dsmoe_create(const dsmoe_desc* desc, dsmoe_ctx** out) {
  if (!desc || !out) return DSMOE_ERR_INVALID_ARG;
  *out = nullptr;
  if (desc->d_model <= 0 || desc->d_ff <= 0 || desc->n_experts <= 0 || desc->max_tokens < 0 || desc->max_rows < 0)
    return DSMOE_ERR_INVALID_ARG;
  if (desc->dtype != DSMOE_F32 && desc->dtype != DSMOE_BF16) return DSMOE_ERR_UNSUPPORTED;
  if (desc->n_experts > kMaxExperts || desc->n_experts % 8 != 0) return DSMOE_ERR_UNSUPPORTED;
  if (desc->d_model % 64 != 0 || desc->d_ff % 64 != 0) return DSMOE_ERR_UNSUPPORTED;
  if (desc->max_rows > (int64_t)desc->max_tokens * desc->n_experts) return DSMOE_ERR_INVALID_ARG;
  if (desc->max_rows >= (int64_t)1 << 31) return DSMOE_ERR_UNSUPPORTED;
  dsmoe_ctx* c = new (std::nothrow) dsmoe_ctx();
  if (!c) return DSMOE_ERR_INVALID_ARG;
  c->desc = *desc;
  c->esize = desc->dtype == DSMOE_BF16 ? 2 : 4;
  c->ws = make_layout(c->desc, c->esize);
  c->workspace = nullptr;
  c->workspace_bytes = 0;
  c->err[0] = 0;
  c->expert_kind = DSMOE_EXPERT_SWIGLU;
  c->spin_limit = kDefaultSpinLimit;
  c->routing_pending_T = -1;
  c->n_cu = 256;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
      prop.multiProcessorCount > 0)
    c->n_cu = prop.multiProcessorCount;
  else
    (void)hipGetLastError();   // no device visible: keep the MI355X default
  *out = c;
  return DSMOE_OK;
}

static void release_events(dsmoe_ctx* c) {
  if (c->prof.ev) {
    for (int i = 0; i < 3 * c->prof.max_calls; ++i) (void)hipEventDestroy(c->prof.ev[i]);
    delete[] c->prof.ev;
  }
  c->prof = dsmoe_profile();
}

int32_t dsmoe_profile_enable(dsmoe_ctx* c, int32_t max_calls) {
  if (!c || max_calls < 0 || max_calls > (1 << 20)) return DSMOE_ERR_INVALID_ARG;
  release_events(c);
  if (max_calls == 0) return DSMOE_OK;
  c->prof.ev = new (std::nothrow) hipEvent_t[3 * (size_t)max_calls];
  if (!c->prof.ev) return fail(c, DSMOE_ERR_INVALID_ARG, "out of host memory");
  for (int i = 0; i < 3 * max_calls; ++i) {
    hipError_t e = hipEventCreate(&c->prof.ev[i]);
    if (e != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(c->prof.ev[j]);
      delete[] c->prof.ev;
      c->prof = dsmoe_profile();
      return hip_fail(c, e, "hipEventCreate");
    }
  }
  c->prof.max_calls = max_calls;
  return DSMOE_OK;
}

int32_t dsmoe_profile_read(dsmoe_ctx* c, int32_t* n_calls, float* gateup_ms, float* down_ms) {
  if (!c || !n_calls || !gateup_ms || !down_ms) return DSMOE_ERR_INVALID_ARG;
  *n_calls = 0; *gateup_ms = 0.f; *down_ms = 0.f;
  for (int i = 0; i < c->prof.n; ++i) {
    hipEvent_t* ev = c->prof.ev + 3 * i;
    float a = 0.f, b = 0.f;
    HIP_TRY(c, hipEventSynchronize(ev[2]));
    HIP_TRY(c, hipEventElapsedTime(&a, ev[0], ev[1]));
    HIP_TRY(c, hipEventElapsedTime(&b, ev[1], ev[2]));
    *gateup_ms += a; *down_ms += b;
  }
  *n_calls = c->prof.n;
  c->prof.n = 0;
  return DSMOE_OK;
}

int32_t dsmoe_destroy(dsmoe_ctx* ctx) {
  if (ctx) release_events(ctx);
  delete ctx;
  return DSMOE_OK;
}

const char* dsmoe_last_error(const dsmoe_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int32_t dsmoe_set_expert_kind(dsmoe_ctx* c, int32_t kind) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (kind != DSMOE_EXPERT_SWIGLU && kind != DSMOE_EXPERT_GELU)
    return fail(c, DSMOE_ERR_INVALID_ARG, "unknown expert kind %d", kind);
  c->expert_kind = kind;
  return DSMOE_OK;
}

int32_t dsmoe_set_sync_spin_limit(dsmoe_ctx* c, int32_t polls) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (polls < 0) return fail(c, DSMOE_ERR_INVALID_ARG, "polls must be >= 0");
  c->spin_limit = polls;
  return DSMOE_OK;
}

#ifdef DSMOE_TRACE
size_t dsmoe_trace_offset(const dsmoe_ctx* c) { return c->ws.dec_p1; }   // development builds only
#endif

int32_t dsmoe_workspace_bytes(const dsmoe_ctx* ctx, size_t* bytes) {
  if (!ctx || !bytes) return DSMOE_ERR_INVALID_ARG;
  *bytes = ctx->ws.total;
  return DSMOE_OK;
}

int32_t dsmoe_set_workspace(dsmoe_ctx* c, void* dptr, size_t bytes) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (!dptr) return fail(c, DSMOE_ERR_INVALID_ARG, "null workspace");
  if (reinterpret_cast<uintptr_t>(dptr) & 255u) return fail(c, DSMOE_ERR_INVALID_ARG, "workspace not 256-byte aligned");
  if (bytes < c->ws.total)
    return fail(c, DSMOE_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", bytes, c->ws.total);
  c->workspace = static_cast<char*>(dptr);
  c->workspace_bytes = bytes;
  // the deferred status word starts cleared
  HIP_TRY(c, hipMemsetAsync(c->workspace + c->ws.err_flag, 0, 16, nullptr));
  // arrival counters of the weight-streaming path: every call leaves them at zero again
  HIP_TRY(c, hipMemsetAsync(c->workspace + c->ws.dec_arrivals, 0, decode_arrival_slots(c->desc) * 4, nullptr));
  HIP_TRY(c, reset_dense_sync(c, nullptr));
  c->routing_pending_T = -1;
  HIP_TRY(c, hipStreamSynchronize(nullptr));
  return DSMOE_OK;
}

int32_t dsmoe_poll_error(dsmoe_ctx* c, void* stream) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  // two deferred status words: the workspace's, and the one of dsmoe_dispatch_static once it has run on this device
  int32_t* flags[2] = {nullptr, nullptr};
  if (c->workspace) flags[0] = reinterpret_cast<int32_t*>(c->workspace + c->ws.err_flag);
  HIP_TRY(c, static_dispatch_flag(&flags[1]));
  if (!flags[0] && !flags[1]) return fail(c, DSMOE_ERR_WORKSPACE, "no workspace set");
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t status = DSMOE_OK;
  int32_t diag[kDenseDiagWords] = {0};
  for (int32_t* dflag : flags) {
    if (!dflag) continue;
    int32_t flag = 0;
    HIP_TRY(c, hipMemcpyAsync(&flag, dflag, 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    if (flag != 0) {
      HIP_TRY(c, hipMemsetAsync(dflag, 0, 4, s));
      if (flag == DSMOE_ERR_INTERNAL && dflag == flags[0]) {   // a wait between blocks gave up: counters may be off
        HIP_TRY(c, hipMemcpyAsync(diag, c->workspace + c->ws.dec_sync + kDenseSyncWords * 4, sizeof(diag),
                                  hipMemcpyDeviceToHost, s));
        HIP_TRY(c, hipStreamSynchronize(s));
        HIP_TRY(c, reset_dense_sync(c, s));
      }
      HIP_TRY(c, hipStreamSynchronize(s));
      status = flag;
    }
  }
  if (status == DSMOE_ERR_INTERNAL)
    return fail(c, status, "decode kernel: %s (block %d, XCD %d, counter %d read %d, wanted %d); the call's output "
                           "is undefined", diag[0] == 3 ? "an XCD did not run all of its work items"
                                                        : "a block gave up waiting for its peers",
                diag[1], diag[2], diag[3], diag[4], diag[5]);
  if (status != DSMOE_OK)
    return fail(c, status, "dispatched rows exceeded max_rows = %lld", (long long)c->desc.max_rows);
  return DSMOE_OK;
}

int32_t dsmoe_route(dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, int32_t T, float* probs,
                    void* stream) {
  if (int32_t rc = check_call(c, T, false)) return rc;
  if (T == 0) return DSMOE_OK;
  REQUIRE_PTR(c, x); REQUIRE_PTR(c, w_r); OPTIONAL_PTR(c, b_r); REQUIRE_PTR(c, probs);
  HIP_TRY(c, launch_route(c, x, w_r, b_r, T, probs, -1, 0, 0.f, nullptr, nullptr, static_cast<hipStream_t>(stream)));
  return DSMOE_OK;
}

int32_t dsmoe_select(dsmoe_ctx* c, const float* probs, int32_t T, int32_t mode, int32_t k, float eps,
                     uint64_t* mask, int32_t* cnt_tok, void* stream) {
  if (int32_t rc = check_call(c, T, false)) return rc;
  if (int32_t rc = check_select_args(c, mode, k, eps)) return rc;
  if (mode == DSMOE_SEL_THRESHOLD_TOPK)
    if (int32_t rc = check_call(c, T, true)) return rc;   // the counts and K of the first pass live in the workspace
  if (T == 0) return DSMOE_OK;
  REQUIRE_PTR(c, probs); REQUIRE_PTR(c, mask);
  if (cnt_tok && (reinterpret_cast<uintptr_t>(cnt_tok) & 3u)) return fail(c, DSMOE_ERR_INVALID_ARG, "cnt_tok misaligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (mode == DSMOE_SEL_THRESHOLD_TOPK) {
    // threshold counts -> K on the device -> top-K; the counts of the first pass live in the workspace
    int32_t* cnt_ws = reinterpret_cast<int32_t*>(c->workspace + c->ws.cnt_tok);
    int32_t* k_dev = reinterpret_cast<int32_t*>(c->workspace + c->ws.k_dev);
    HIP_TRY(c, launch_select(c, probs, T, DSMOE_SEL_THRESHOLD, 0, eps, mask, cnt_ws, s));
    HIP_TRY(c, launch_threshold_topk_k(c, cnt_ws, T, k_dev, s));
    HIP_TRY(c, launch_select(c, probs, T, DSMOE_SEL_TOPK, 1, 0.f, mask, cnt_tok, s, k_dev));
    return DSMOE_OK;
  }
  HIP_TRY(c, launch_select(c, probs, T, mode, k, eps, mask, cnt_tok, s));
  return DSMOE_OK;
}

int32_t dsmoe_dispatch(dsmoe_ctx* c, const void* x, const float* probs, const uint64_t* mask, int32_t T,
                       int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                       int32_t* tok_rows, int32_t* nnz, void* x_perm, void* stream) {
  if (int32_t rc = check_call(c, T, true)) return rc;
  REQUIRE_PTR(c, expert_off); REQUIRE_PTR(c, tok_off); REQUIRE_PTR(c, nnz);
  if (T > 0) {
    REQUIRE_PTR(c, probs); REQUIRE_PTR(c, mask); REQUIRE_PTR(c, row_token); REQUIRE_PTR(c, row_weight);
    REQUIRE_PTR(c, tok_rows); OPTIONAL_PTR(c, x_perm);
    if (x_perm) REQUIRE_PTR(c, x);
  }
  HIP_TRY(c, launch_dispatch(c, x, probs, mask, T, expert_off, row_token, row_weight, tok_off, tok_rows, nnz,
                             x_perm, static_cast<hipStream_t>(stream)));
  return DSMOE_OK;
}

int32_t dsmoe_expert_ffn(dsmoe_ctx* c, const void* x, const void* x_perm, const int32_t* row_token,
                         const int32_t* expert_off, const void* w_gate, const void* w_up, const void* w_down,
                         void* y_perm, void* stream) {
  if (int32_t rc = check_call(c, 0, true)) return rc;
  if (c->desc.max_rows == 0) return DSMOE_OK;
  if (!x_perm) { REQUIRE_PTR(c, x); REQUIRE_PTR(c, row_token); }
  OPTIONAL_PTR(c, x_perm);
  REQUIRE_PTR(c, expert_off); REQUIRE_EXPERT_WEIGHTS(c, w_gate, w_up, w_down);
  REQUIRE_PTR(c, y_perm);
  HIP_TRY(c, launch_expert_ffn(c, x, x_perm, row_token, expert_off, w_gate, w_up, w_down, y_perm,
                               static_cast<hipStream_t>(stream)));
  return DSMOE_OK;
}

int32_t dsmoe_combine(dsmoe_ctx* c, const void* y_perm, const float* row_weight, const int32_t* tok_off,
                      const int32_t* tok_rows, int32_t T, void* out, void* stream) {
  if (int32_t rc = check_call(c, T, false)) return rc;
  if (T == 0) return DSMOE_OK;
  REQUIRE_PTR(c, y_perm); REQUIRE_PTR(c, row_weight); REQUIRE_PTR(c, tok_off); REQUIRE_PTR(c, tok_rows);
  REQUIRE_PTR(c, out);
  HIP_TRY(c, launch_combine(c, y_perm, row_weight, tok_off, tok_rows, T, out, static_cast<hipStream_t>(stream)));
  return DSMOE_OK;
}

int32_t dsmoe_sparse_fwd(dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                         const void* w_up, const void* w_down, int32_t T, int32_t mode, int32_t k, float eps,
                         void* out, void* stream) {
  if (int32_t rc = check_call(c, T, true)) return rc;
  if (int32_t rc = check_select_args(c, mode, k, eps)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* w = c->workspace;
  if (T == 0) {   // publish an empty routing; nothing else to do
    HIP_TRY(c, launch_dispatch(c, nullptr, nullptr, nullptr, 0, reinterpret_cast<int32_t*>(w + c->ws.expert_off),
                               nullptr, nullptr, reinterpret_cast<int32_t*>(w + c->ws.tok_off), nullptr,
                               reinterpret_cast<int32_t*>(w + c->ws.nnz), nullptr, s));
    return DSMOE_OK;
  }
  REQUIRE_PTR(c, x); REQUIRE_PTR(c, w_r); OPTIONAL_PTR(c, b_r); REQUIRE_EXPERT_WEIGHTS(c, w_gate, w_up, w_down);
  REQUIRE_PTR(c, out);
  float* probs = reinterpret_cast<float*>(w + c->ws.probs);
  uint64_t* mask = reinterpret_cast<uint64_t*>(w + c->ws.mask);
  int32_t* cnt_tok = reinterpret_cast<int32_t*>(w + c->ws.cnt_tok);
  int32_t* expert_off = reinterpret_cast<int32_t*>(w + c->ws.expert_off);
  int32_t* row_token = reinterpret_cast<int32_t*>(w + c->ws.row_token);
  float* row_weight = reinterpret_cast<float*>(w + c->ws.row_weight);
  int32_t* tok_off = reinterpret_cast<int32_t*>(w + c->ws.tok_off);
  int32_t* tok_rows = reinterpret_cast<int32_t*>(w + c->ws.tok_rows);
  int32_t* nnz = reinterpret_cast<int32_t*>(w + c->ws.nnz);
  void* y_perm = w + c->ws.y_perm;
  c->routing_pending_T = -1;
  if (decode_dense_applies(c, T, mode, k, eps)) {
    // decode-sized batch that selects nearly every expert: one persistent kernel, router included
    HIP_TRY(c, launch_decode_dense(c, x, w_r, b_r, w_gate, w_up, w_down, T, mode, k, eps, out, s));
    c->routing_pending_T = T;
    return DSMOE_OK;
  }
  if (decode_tiny_applies(c, T, mode)) {
    // a handful of tokens: three kernels, router included, that stream the selected experts' weight rows
    HIP_TRY(c, launch_decode_tiny(c, x, w_r, b_r, w_gate, w_up, w_down, T, mode, k, eps, out, s));
    c->routing_pending_T = T;
    return DSMOE_OK;
  }
  if (mode == DSMOE_SEL_THRESHOLD_TOPK) {
    int32_t* k_dev = reinterpret_cast<int32_t*>(w + c->ws.k_dev);
    HIP_TRY(c, launch_route(c, x, w_r, b_r, T, probs, DSMOE_SEL_THRESHOLD, 0, eps, mask, cnt_tok, s));
    HIP_TRY(c, launch_threshold_topk_k(c, cnt_tok, T, k_dev, s));
    HIP_TRY(c, launch_select(c, probs, T, DSMOE_SEL_TOPK, 1, 0.f, mask, cnt_tok, s, k_dev));
  } else {
    HIP_TRY(c, launch_route(c, x, w_r, b_r, T, probs, mode, k, eps, mask, cnt_tok, s));
  }
  if (c->desc.dtype == DSMOE_BF16 && T <= kDecodeMaxTokens) {
    // decode-sized batch: weight-streaming kernels that derive the dispatch from the masks themselves
    HIP_TRY(c, launch_decode_fwd(c, x, w_gate, w_up, w_down, T, out, s));
    return DSMOE_OK;
  }
  HIP_TRY(c, launch_dispatch(c, x, probs, mask, T, expert_off, row_token, row_weight, tok_off, tok_rows, nnz,
                             nullptr, s));
  if (c->desc.max_rows > 0)
    HIP_TRY(c, launch_expert_ffn(c, x, nullptr, row_token, expert_off, w_gate, w_up, w_down, y_perm, s));
  HIP_TRY(c, launch_combine(c, y_perm, row_weight, tok_off, tok_rows, T, out, s));
  return DSMOE_OK;
}

int32_t dsmoe_sparse_fwd_uses_persistent_kernel(const dsmoe_ctx* c, int32_t T, int32_t mode, int32_t k, float eps) {
  if (!c || !c->workspace) return 0;
  if (mode & DSMOE_SEL_NORMALISED) {
    mode &= ~DSMOE_SEL_NORMALISED;
    eps = eps / static_cast<float>(c->desc.n_experts);
  }
  return decode_dense_applies(c, T, mode, k, eps) ? 1 : 0;
}

int32_t dsmoe_sparse_fwd_path(const dsmoe_ctx* c, int32_t T, int32_t mode, int32_t k, float eps) {
  if (!c || !c->workspace || T < 0 || T > c->desc.max_tokens) return -1;
  if (mode & DSMOE_SEL_NORMALISED) {
    mode &= ~DSMOE_SEL_NORMALISED;
    eps = eps / static_cast<float>(c->desc.n_experts);
  }
  if (mode != DSMOE_SEL_TOPK && mode != DSMOE_SEL_THRESHOLD && mode != DSMOE_SEL_THRESHOLD_TOPK) return -1;
  if (decode_dense_applies(c, T, mode, k, eps)) return DSMOE_PATH_ALL_EXPERTS;
  if (decode_tiny_applies(c, T, mode)) return DSMOE_PATH_FEW_TOKENS;
  if (c->desc.dtype == DSMOE_BF16 && T >= 1 && T <= kDecodeMaxTokens) return DSMOE_PATH_STREAMING;
  return DSMOE_PATH_GROUPED;
}

int32_t dsmoe_sparse_fwd_routing(dsmoe_ctx* c, int32_t T, float* probs, uint64_t* mask, int32_t* expert_off,
                                 int32_t* row_token, void* stream) {
  if (int32_t rc = check_call(c, T, true)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t E = (size_t)c->desc.n_experts;
  char* w = c->workspace;
  if (c->routing_pending_T >= 0) {
    // the last forward kept only scores and masks (its kernels need no dispatch): derive the rest now
    const int Tp = c->routing_pending_T;
    HIP_TRY(c, launch_dispatch(c, nullptr, reinterpret_cast<const float*>(w + c->ws.probs),
                               reinterpret_cast<const uint64_t*>(w + c->ws.mask), Tp,
                               reinterpret_cast<int32_t*>(w + c->ws.expert_off), reinterpret_cast<int32_t*>(w + c->ws.row_token),
                               reinterpret_cast<float*>(w + c->ws.row_weight), reinterpret_cast<int32_t*>(w + c->ws.tok_off),
                               reinterpret_cast<int32_t*>(w + c->ws.tok_rows), reinterpret_cast<int32_t*>(w + c->ws.nnz),
                               nullptr, s));
    c->routing_pending_T = -1;
  }
  if (probs && T) HIP_TRY(c, hipMemcpyAsync(probs, w + c->ws.probs, (size_t)T * E * 4, hipMemcpyDeviceToDevice, s));
  if (mask && T) HIP_TRY(c, hipMemcpyAsync(mask, w + c->ws.mask, (size_t)T * 8, hipMemcpyDeviceToDevice, s));
  if (expert_off) HIP_TRY(c, hipMemcpyAsync(expert_off, w + c->ws.expert_off, (E + 1) * 4, hipMemcpyDeviceToDevice, s));
  if (row_token && c->desc.max_rows)
    HIP_TRY(c, hipMemcpyAsync(row_token, w + c->ws.row_token, (size_t)c->desc.max_rows * 4, hipMemcpyDeviceToDevice, s));
  return DSMOE_OK;
}

int32_t dsmoe_dense_saved_bytes(const dsmoe_ctx* c, int32_t T, size_t* bytes) {
  if (!c || !bytes || T < 0) return DSMOE_ERR_INVALID_ARG;
  *bytes = dense_saved_bytes(c, T);
  return DSMOE_OK;
}

int32_t dsmoe_dense_bwd_scratch_bytes(const dsmoe_ctx* c, int32_t T, size_t* bytes) {
  if (!c || !bytes || T < 0) return DSMOE_ERR_INVALID_ARG;
  *bytes = dense_bwd_scratch_bytes(c, T);
  return DSMOE_OK;
}

int32_t dsmoe_dense_fwd(dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                        const void* w_up, const void* w_down, int32_t T, void* out, float* probs, void* saved,
                        void* stream) {
  if (int32_t rc = check_call(c, T, true)) return rc;
  if (T == 0) return DSMOE_OK;
  REQUIRE_PTR(c, x); REQUIRE_PTR(c, w_r); OPTIONAL_PTR(c, b_r); REQUIRE_EXPERT_WEIGHTS(c, w_gate, w_up, w_down);
  REQUIRE_PTR(c, out); OPTIONAL_PTR(c, probs); OPTIONAL_PTR(c, saved);
  if (!saved && (int64_t)T * c->desc.n_experts > c->desc.max_rows)
    return fail(c, DSMOE_ERR_WORKSPACE, "dense forward without a `saved` buffer keeps T * E = %lld hidden rows in the "
                "workspace, which holds max_rows = %lld", (long long)T * c->desc.n_experts, (long long)c->desc.max_rows);
  hipError_t e = launch_dense_fwd(c, x, w_r, b_r, w_gate, w_up, w_down, T, out, probs, saved,
                                  static_cast<hipStream_t>(stream));
  if (e == hipErrorNotSupported) return fail(c, DSMOE_ERR_NOT_IMPL, "dense forward not implemented");
  HIP_TRY(c, e);
  return DSMOE_OK;
}

int32_t dsmoe_dense_bwd_mi(dsmoe_ctx* c, const void* x, const void* w_r, const void* w_gate, const void* w_up,
                           const void* w_down, const void* saved, const void* d_out, int32_t T, void* scratch,
                           void* dx, float* dw_r, float* db_r, float* dw_gate, float* dw_up, float* dw_down,
                           float mi_alpha, void* stream) {
  if (int32_t rc = check_call(c, T, false)) return rc;
  if (!std::isfinite(mi_alpha)) return fail(c, DSMOE_ERR_INVALID_ARG, "mi_alpha must be finite");
  const bool swiglu = c->expert_kind == DSMOE_EXPERT_SWIGLU;   // the two-matrix expert has no w_up and no dw_up
  REQUIRE_PTR(c, dw_r); OPTIONAL_PTR(c, db_r); REQUIRE_PTR(c, dw_gate); REQUIRE_PTR(c, dw_down);
  if (swiglu) REQUIRE_PTR(c, dw_up);
  if (T == 0) {   // no tokens: every weight gradient is zero
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
    HIP_TRY(c, hipMemsetAsync(dw_r, 0, d * E * 4, s));
    if (db_r) HIP_TRY(c, hipMemsetAsync(db_r, 0, E * 4, s));
    HIP_TRY(c, hipMemsetAsync(dw_gate, 0, E * d * f * 4, s));
    if (swiglu) HIP_TRY(c, hipMemsetAsync(dw_up, 0, E * d * f * 4, s));
    HIP_TRY(c, hipMemsetAsync(dw_down, 0, E * d * f * 4, s));
    return DSMOE_OK;
  }
  REQUIRE_PTR(c, x); REQUIRE_PTR(c, w_r); REQUIRE_EXPERT_WEIGHTS(c, w_gate, w_up, w_down);
  REQUIRE_PTR(c, saved); REQUIRE_PTR(c, d_out); REQUIRE_PTR(c, scratch); REQUIRE_PTR(c, dx);
  hipError_t e = launch_dense_bwd(c, x, w_r, w_gate, w_up, w_down, saved, d_out, T, scratch, dx, dw_r, db_r,
                                  dw_gate, dw_up, dw_down, mi_alpha, static_cast<hipStream_t>(stream));
  if (e == hipErrorNotSupported) return fail(c, DSMOE_ERR_NOT_IMPL, "dense backward not implemented");
  HIP_TRY(c, e);
  return DSMOE_OK;
}

int32_t dsmoe_dense_bwd(dsmoe_ctx* c, const void* x, const void* w_r, const void* w_gate, const void* w_up,
                        const void* w_down, const void* saved, const void* d_out, int32_t T, void* scratch,
                        void* dx, float* dw_r, float* db_r, float* dw_gate, float* dw_up, float* dw_down,
                        void* stream) {
  return dsmoe_dense_bwd_mi(c, x, w_r, w_gate, w_up, w_down, saved, d_out, T, scratch, dx, dw_r, db_r, dw_gate, dw_up,
                            dw_down, 0.f, stream);
}

int32_t dsmoe_mi_loss(dsmoe_ctx* c, const float* probs, int32_t T, float* loss, float* p_mean, void* stream) {
  if (int32_t rc = check_call(c, T, true)) return rc;
  if (T == 0) return fail(c, DSMOE_ERR_INVALID_ARG, "the loss is a mean over tokens: T must be >= 1");
  REQUIRE_PTR(c, probs);
  if (!loss && !p_mean) return fail(c, DSMOE_ERR_INVALID_ARG, "nothing to write: loss and p_mean are both null");
  if ((reinterpret_cast<uintptr_t>(loss) | reinterpret_cast<uintptr_t>(p_mean)) & 3u)
    return fail(c, DSMOE_ERR_INVALID_ARG, "loss / p_mean misaligned");
  HIP_TRY(c, launch_mi_loss(c, probs, T, reinterpret_cast<float*>(c->workspace + c->ws.stat_part), p_mean, loss,
                            static_cast<hipStream_t>(stream)));
  return DSMOE_OK;
}

}  // extern "C"
