// Internal declarations shared by the HIP sources of libdsmoe (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dsmoe.h"

namespace dsmoe {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Hardware id of the XCD (accelerator complex die, each with its own L2) the calling wave runs on: bits 3:0 of
// the XCC_ID hardware register (register 20).
__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u; }

constexpr int kMaxExperts = 64;
// counters of the all-expert decode kernel (decode_dense.hip)
constexpr int kDenseClaimWords = 32;      // bitmap words per XCD and phase: at most 1024 items
constexpr int kDenseSyncClaim1 = 16;                                        // + 32 XCD: claimed first-phase items
constexpr int kDenseSyncClaim2 = kDenseSyncClaim1 + 8 * kDenseClaimWords;   // + 32 XCD: claimed second-phase items
constexpr int kDenseSyncDone1 = kDenseSyncClaim2 + 8 * kDenseClaimWords;    // + 32 XCD: first-phase items whose hidden
                                                                            // columns are in the XCD's L2
constexpr int kDenseSyncDone2 = kDenseSyncDone1 + 8 * kDenseClaimWords;     // + 32 XCD: finished second-phase items
constexpr int kDenseSyncWords = kDenseSyncDone2 + 8 * kDenseClaimWords;
// behind the counters and the diagnostics: what the in-kernel router publishes for the other blocks
constexpr int kDensePubCount = kDenseSyncWords + 8;                      // i32 [128]: selected experts of a token (0: not yet)
constexpr int kDensePubWeight = kDensePubCount + 128;                    // u32 [128][64]: combine weights (all ones: not yet)
constexpr int kDenseSyncTotalWords = kDensePubWeight + 128 * 64;
constexpr int kDenseDiagWords = 8;        // behind the counters: what the first failing block saw (reason, block, ...)
constexpr int kDefaultSpinLimit = 1 << 20;   // polls before a block gives up waiting for its peers
constexpr int kDispatchTokensPerBlock = 256;  // tokens handled by one block of the dispatch kernels
constexpr int kDecodeMaxTokens = 128;         // largest batch served by the weight-streaming (decode) path
constexpr int kStaticDispatchMaxTokens = DSMOE_STATIC_DISPATCH_MAX_TOKENS;   // largest T of dsmoe_dispatch_static

// Workspace carve-up (byte offsets into the caller's buffer).
struct WorkspaceLayout {
  size_t err_flag;    // int32[4]: [0] deferred status
  size_t blk_cnt;     // int32 [n_dispatch_blocks][E]   per-block expert histogram
  size_t blk_tok;     // int32 [n_dispatch_blocks]      per-block number of (token, expert) pairs
  size_t h;           // dtype [max_rows][f]            silu(G)*U rows between the two grouped GEMMs
  // routing objects and permuted output owned by dsmoe_sparse_fwd
  size_t probs;       // f32 [max_tokens][E]
  size_t mask;        // u64 [max_tokens]
  size_t cnt_tok;     // i32 [max_tokens]
  size_t expert_off;  // i32 [E+1]
  size_t row_token;   // i32 [max_rows]
  size_t row_weight;  // f32 [max_rows]
  size_t tok_off;     // i32 [max_tokens+1]
  size_t tok_rows;    // i32 [max_rows]
  size_t nnz;         // i32 [1]
  size_t y_perm;      // dtype [max_rows][d]
  size_t stat_part;   // f32 [256][128]: per-block partial sums of the score statistics
  size_t k_dev;       // i32 [1]: K of Threshold-TopK selection
  // weight-streaming (decode) path, bf16 only
  size_t dec_info;    // i32 [8]: rows, active experts, K split of gate/up, K split of down
  size_t dec_arrivals;   // i32 [decode_arrival_slots]: blocks that have finished a shared result; zero between calls
  size_t dec_p1;      // f32 [decode_row_cap][2 f]      K-chunk partial sums of gate | up
  size_t dec_p2;      // f32 [decode_row_cap][d]        K-chunk partial sums of the down projection
  size_t dec_ht;      // bf16 [min(max_tokens, 128)][E f]   weighted hidden activations of the all-expert decode kernel
  size_t dec_sync;    // i32 [kDenseSyncWords]: counters of the all-expert decode kernel; zero between calls
  size_t tiny_p1;     // f32 [2 * 256][min(max_tokens, 4)][2 f]   partial gate | up sums of the few-token kernels
  size_t tiny_p2;     // f32 [256][min(max_tokens, 4)][d]         their partial outputs
  size_t total;
};

}  // namespace dsmoe

struct dsmoe_profile {
  int max_calls = 0, n = 0;
  hipEvent_t* ev = nullptr;   // 3 events per call: before gate/up, between, after down
};

struct dsmoe_ctx {
  dsmoe_desc desc;
  mutable dsmoe_profile prof;
  size_t esize;  // bytes per dtype element
  dsmoe::WorkspaceLayout ws;
  char* workspace;
  size_t workspace_bytes;
  int n_cu;
  int expert_kind;   // DSMOE_EXPERT_SWIGLU or DSMOE_EXPERT_GELU
  int spin_limit;    // polls a block of the all-expert decode kernel waits for its peers
  int routing_pending_T;   // >= 0: the last dsmoe_sparse_fwd (of that many tokens) left scores and masks only;
                           // dsmoe_sparse_fwd_routing derives the dispatch objects from them on demand
  char err[256];
};

namespace dsmoe {

// arrival counters of the decode path: one per (expert, 64-column slice of the hidden width), plus one
// per 32-token group of the router
inline size_t decode_arrival_slots(const dsmoe_desc& d) {
  return (size_t)d.n_experts * ((d.d_ff + 63) / 64) + 64;
}

// rows of K-chunk partial sums the decode path may keep (K split times dispatched rows)
inline int decode_row_cap(const dsmoe_ctx* c) {
  return (c->desc.max_tokens < kDecodeMaxTokens ? c->desc.max_tokens : kDecodeMaxTokens) * c->desc.n_experts;
}

// ---- kernel launchers (each validates nothing: the C-ABI layer has done so) -------------------
// router.hip
hipError_t launch_route(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, int T,
                        float* probs, int mode /* <0: no selection */, int k, float eps, uint64_t* mask,
                        int32_t* cnt_tok, hipStream_t s);
hipError_t launch_select(const dsmoe_ctx* c, const float* probs, int T, int mode, int k, float eps,
                         uint64_t* mask, int32_t* cnt_tok, hipStream_t s, const int32_t* k_dev = nullptr);
// router_stats.hip
constexpr int kStatMaxBlocks = 256;
int mi_blocks(int T);   // rows of 128 floats that launch_mi_loss needs in `part` (at most kStatMaxBlocks)
hipError_t launch_mi_loss(const dsmoe_ctx* c, const float* S, int T, float* part, float* p_mean, float* loss,
                          hipStream_t s);
hipError_t launch_threshold_topk_k(const dsmoe_ctx* c, const int32_t* cnt_tok, int T, int32_t* k_out, hipStream_t s);
// dispatch.hip
hipError_t launch_dispatch(const dsmoe_ctx* c, const void* x, const float* probs, const uint64_t* mask, int T,
                           int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                           int32_t* tok_rows, int32_t* nnz, void* x_perm, hipStream_t s);
// expert_ffn.hip
hipError_t launch_expert_ffn(const dsmoe_ctx* c, const void* x, const void* x_perm, const int32_t* row_token,
                             const int32_t* expert_off, const void* w_gate, const void* w_up,
                             const void* w_down, void* y_perm, hipStream_t s);
hipError_t launch_down_dense(const dsmoe_ctx* c, const void* h, int T, int k_total, const void* w, void* out,
                             hipStream_t s);
hipError_t launch_shared_rows_gemm(const dsmoe_ctx* c, const void* x, int groups, int rows, int k, int n,
                                   const void* w, void* out, hipStream_t s);
// address of the deferred status word of dsmoe_dispatch_static on the current device; null while that entry
// point has not run there
hipError_t static_dispatch_flag(int32_t** flag);
// dispatch.hip (combine)
hipError_t launch_combine(const dsmoe_ctx* c, const void* y_perm, const float* row_weight,
                          const int32_t* tok_off, const int32_t* tok_rows, int T, void* out, hipStream_t s);
// decode.hip: expert FFN + combine of dsmoe_sparse_fwd for at most kDecodeMaxTokens bf16 tokens, from the
// probabilities and masks the router left in the workspace; also publishes the routing objects there
hipError_t launch_decode_fwd(const dsmoe_ctx* c, const void* x, const void* w_gate, const void* w_up,
                             const void* w_down, int T, void* out, hipStream_t s);
// decode_dense.hip: the whole sparse forward (router included) for decode-sized batches that select nearly
// every expert; leaves scores and masks in the workspace
bool decode_dense_applies(const dsmoe_ctx* c, int T, int mode, int k, float eps);
// decode_tiny.hip: at most 4 tokens, router included, weights streamed through the vector ALUs
size_t decode_tiny_p1_bytes(const dsmoe_desc& d);
size_t decode_tiny_p2_bytes(const dsmoe_desc& d);
bool decode_tiny_applies(const dsmoe_ctx* c, int T, int mode);
hipError_t launch_decode_tiny(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                              const void* w_up, const void* w_down, int T, int mode, int k, float eps, void* out,
                              hipStream_t s);
hipError_t launch_decode_dense(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                               const void* w_up, const void* w_down, int T, int mode, int k, float eps, void* out,
                               hipStream_t s);
// dense.hip
size_t dense_saved_bytes(const dsmoe_ctx* c, int T);
size_t dense_bwd_scratch_bytes(const dsmoe_ctx* c, int T);
hipError_t launch_dense_fwd(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r,
                            const void* w_gate, const void* w_up, const void* w_down, int T, void* out,
                            float* probs, void* saved, hipStream_t s);
hipError_t launch_dense_bwd(const dsmoe_ctx* c, const void* x, const void* w_r, const void* w_gate,
                            const void* w_up, const void* w_down, const void* saved, const void* d_out, int T,
                            void* scratch, void* dx, float* dw_r, float* db_r, float* dw_gate, float* dw_up,
                            float* dw_down, float mi_alpha, hipStream_t s);

}  // namespace dsmoe
