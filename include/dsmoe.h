/*
 * dsmoe.h - C ABI of the MI355X (gfx950) implementation of the DS-MoE expert layer
 * ("Dense Training, Sparse Inference", arXiv 2404.05567).
 *
 * The layer (paper Sec. 3.1, Eq. 1): a router h gives every token X a score vector
 * S = softmax(h(X)) over N experts; sparse inference evaluates only a selected index set A of
 * experts and returns O = sum_{i in A} S_i * e_i(X).  Dense training (Sec. 3.2, Eq. 3) evaluates
 * every expert on every token, O = sum_{j=1..N} S_j * e_j(X), and back-propagates through all of them.
 *
 * Conventions shared by every call
 *   - All tensor arguments are DEVICE pointers (HIP global memory) unless marked "host".  They must be
 *     16-byte aligned and are owned by the caller; the library never allocates, frees or retains them
 *     beyond the asynchronous work it enqueues.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work and
 *     return; they never synchronise the stream (dsmoe_poll_error excepted).
 *   - Layouts are row-major: X[T,d], W_r[d,E], b_r[E], W_gate[E,d,f], W_up[E,d,f], W_down[E,f,d],
 *     with d = d_model, E = n_experts, f = d_ff.  Limits: E <= 64 and a multiple of 8 (selection sets are
 *     64-bit masks; bits at or above E of a caller's mask are ignored), d and f multiples of 64.  "dtype" tensors hold fp32 or bf16 values as chosen
 *     in the descriptor; router probabilities, row weights and all accumulators are fp32.
 *   - The expert is a SwiGLU MLP without biases: e(x) = (silu(x W_gate) * (x W_up)) W_down (default), or the
 *     paper's two-matrix GeLU MLP (dsmoe_set_expert_kind).
 *   - T = 0 is a valid no-op.
 *   - A context and its workspace serve one call at a time: calls that use the workspace (or the same
 *     `saved` / `scratch` buffers) must be ordered on one stream or by events; a context is not
 *     thread-safe.  Work of one call is ordered after the previous call's on the same stream.
 *   - Return value: DSMOE_OK or a negative dsmoe_status; dsmoe_last_error() gives a message for the
 *     last failing call on that context.  Errors found on the host (bad arguments) enqueue nothing.
 *     A capacity overflow (more dispatched rows than max_rows) is found on the device: the dispatch
 *     then publishes an empty routing (every later stage does no work) and raises a flag that
 *     dsmoe_poll_error() reports.
 */
#ifndef DSMOE_H_
#define DSMOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dsmoe_ctx dsmoe_ctx;

typedef enum { DSMOE_F32 = 0, DSMOE_BF16 = 1 } dsmoe_dtype;
typedef enum { DSMOE_SEL_TOPK = 0, DSMOE_SEL_THRESHOLD = 1, DSMOE_SEL_THRESHOLD_TOPK = 2 } dsmoe_sel_mode;
/* OR into DSMOE_SEL_THRESHOLD or DSMOE_SEL_THRESHOLD_TOPK: `eps` is then the paper's normalised threshold
 * (Sec. 4.2, footnote: an expert is kept when N * S_i exceeds it, N = n_experts; the paper's example value is
 * 0.48).  The library tests S_i > eps / N with the quotient rounded once to fp32.  Without the flag `eps` is
 * compared with the raw probability S_i. */
#define DSMOE_SEL_NORMALISED 0x100
typedef enum { DSMOE_EXPERT_SWIGLU = 0, DSMOE_EXPERT_GELU = 1 } dsmoe_expert_kind;

typedef enum {
  DSMOE_OK = 0,
  DSMOE_ERR_INVALID_ARG = -1, /* null pointer, negative size, k outside [1,E], eps < 0 or NaN, misaligned */
  DSMOE_ERR_UNSUPPORTED = -2, /* E > 64 or not a multiple of 8, d_model or d_ff not a multiple of 64, unknown
                                 dtype, a size beyond a stated limit of the call */
  DSMOE_ERR_WORKSPACE = -3,   /* workspace missing or too small */
  DSMOE_ERR_CAPACITY = -4,    /* device-side: dispatched rows exceeded max_rows */
  DSMOE_ERR_HIP = -5,         /* a HIP runtime call failed */
  DSMOE_ERR_NOT_IMPL = -6,
  DSMOE_ERR_INTERNAL = -7     /* device-side: blocks of a kernel that cooperate through one XCD's L2 did not run
                                 where expected, or a bounded wait between blocks gave up; output undefined */
} dsmoe_status;

/* Layer description (host struct). max_tokens bounds T of every call; max_rows bounds the number of
 * dispatched (token, expert) pairs nnz = sum_t |A(t)| (at most max_tokens * n_experts). */
typedef struct {
  int32_t d_model;
  int32_t d_ff;
  int32_t n_experts;
  int32_t dtype; /* dsmoe_dtype */
  int32_t max_tokens;
  int64_t max_rows;
} dsmoe_desc;

/* Create / destroy a context (host object; no device memory is allocated). */
int32_t dsmoe_create(const dsmoe_desc* desc, dsmoe_ctx** out);
int32_t dsmoe_destroy(dsmoe_ctx* ctx);
const char* dsmoe_last_error(const dsmoe_ctx* ctx);

/* The expert e_i of Eq. 1.  DSMOE_EXPERT_SWIGLU (default): e(x) = (silu(x W_gate) * (x W_up)) W_down.
 * DSMOE_EXPERT_GELU: the paper's own two-matrix MLP (Sec. 4.1), e(x) = gelu(x W_1) W_2 with the exact
 * GeLU g * Phi(g); W_1 is passed as w_gate, W_2 as w_down; w_up and, in the backward pass, dw_up are
 * ignored (may be NULL).  Applies to every call that evaluates experts. */
int32_t dsmoe_set_expert_kind(dsmoe_ctx* ctx, int32_t kind);

/* Decode-sized dsmoe_sparse_fwd calls may run as one persistent kernel whose blocks hand results to each other;
 * a block polls at most `polls` times (default 2^20, roughly a second) for its peers before it gives up and
 * raises DSMOE_ERR_INTERNAL through dsmoe_poll_error.  Every wait is bounded: the kernel always ends.
 * polls = 0 makes every such wait give up at once (for tests of the error path). */
int32_t dsmoe_set_sync_spin_limit(dsmoe_ctx* ctx, int32_t polls);

/* Scratch memory the library needs (intermediate H = silu(G)*U rows, block histograms, the routing
 * objects and permuted outputs of dsmoe_sparse_fwd).  The caller allocates `bytes` of device memory,
 * 256-byte aligned, and lends it with dsmoe_set_workspace; it must stay valid until the last enqueued
 * call has finished.  Calls on one context share the workspace and therefore must be issued on one
 * stream (or otherwise serialised). */
int32_t dsmoe_workspace_bytes(const dsmoe_ctx* ctx, size_t* bytes /* host */);
int32_t dsmoe_set_workspace(dsmoe_ctx* ctx, void* dptr, size_t bytes);

/* Synchronises `stream`, then returns and clears the deferred device status (DSMOE_OK or
 * DSMOE_ERR_CAPACITY). */
int32_t dsmoe_poll_error(dsmoe_ctx* ctx, void* stream);

/* Router, Eq. 1 first half: probs[T,E] = softmax over all E experts of X W_r (+ b_r).
 * x: dtype [T,d]; w_r: dtype [d,E]; b_r: dtype [E] or NULL; probs: fp32 [T,E] (written). */
int32_t dsmoe_route(dsmoe_ctx* ctx, const void* x, const void* w_r, const void* b_r, int32_t T,
                    float* probs, void* stream);

/* Expert selection (Sec. 3.1: the K best-scored experts; Sec. 3.2 "Sparse Inference": the experts whose
 * score passes a threshold eps).  TOPK keeps the k highest probabilities, equal values going to the lower
 * expert index.  THRESHOLD keeps {e : probs[t,e] > eps} (raw probability, strict; with DSMOE_SEL_NORMALISED
 * eps is the paper's normalised threshold of Sec. 4.2 and the test is probs[t,e] > eps / E) and falls back
 * to the arg-max expert (lowest index) when that set is empty.  THRESHOLD_TOPK (Sec. 4.3 "Threshold-TopK"): the threshold rule gives every
 * token a count; K = the batch mean of the counts rounded half up, clamped to [1, E], computed on the
 * device; every token then keeps its top K (k is ignored; needs the workspace).
 * probs: fp32 [T,E]; mask: u64 [T], bit e set <=> expert e selected (written);
 * cnt_tok: i32 [T] number of selected experts (written; may be NULL). */
int32_t dsmoe_select(dsmoe_ctx* ctx, const float* probs, int32_t T, int32_t mode, int32_t k, float eps,
                     uint64_t* mask, int32_t* cnt_tok, void* stream);

/* Token-to-expert dispatch (the first of the two overheads of dynamic inference named in Sec. 4.4: every
 * token is duplicated once per selected expert): groups the
 * (token, expert) pairs by expert, experts ascending, tokens ascending inside an expert.
 * Written: expert_off i32 [E+1] exclusive prefix sum of tokens per expert (expert_off[E] = nnz);
 * row_token i32 [max_rows] token of each row; row_weight fp32 [max_rows] = probs[token, expert];
 * tok_off i32 [T+1] exclusive prefix sum of cnt_tok; tok_rows i32 [max_rows] rows of each token in
 * ascending expert order; nnz i32 [1].  Entries past nnz are left untouched.
 * x_perm: dtype [max_rows,d] or NULL; when given, row r receives a copy of x[row_token[r], :]. */
int32_t dsmoe_dispatch(dsmoe_ctx* ctx, const void* x, const float* probs, const uint64_t* mask, int32_t T,
                       int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                       int32_t* tok_rows, int32_t* nnz, void* x_perm, void* stream);

/* dsmoe_dispatch for callers that cannot allocate device memory or lend a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error behaviour
 * as dsmoe_dispatch, but no workspace is needed: the scratch of its kernels (per-block expert histograms,
 * about 65 KB, and the deferred status word) is a device array inside the library, which every GPU the
 * library runs on holds until the process ends.  The call allocates nothing and frees nothing.
 * Limits: T <= DSMOE_STATIC_DISPATCH_MAX_TOKENS (beyond it: DSMOE_ERR_UNSUPPORTED, nothing enqueued).
 * All calls on one GPU share that GPU's array, whatever their context or stream: calls that overlap in time
 * on one GPU race and must be serialised by the caller.  Nothing in the array has to start at zero (every
 * histogram entry a call reads it has written first); the status word is set only by a capacity overflow
 * and cleared by dsmoe_poll_error, which also reports it (and needs no workspace for that). */
#define DSMOE_STATIC_DISPATCH_MAX_TOKENS 65536
int32_t dsmoe_dispatch_static(dsmoe_ctx* ctx, const void* x, const float* probs, const uint64_t* mask,
                              int32_t T, int32_t* expert_off, int32_t* row_token, float* row_weight,
                              int32_t* tok_off, int32_t* tok_rows, int32_t* nnz, void* x_perm, void* stream);

/* Per-expert SwiGLU FFN on the dispatched rows (the e_i(X) of Eq. 1):
 * y_perm[r,:] = e_{expert(r)}(x[row_token[r],:]) for r < expert_off[E].
 * Rows are read from x_perm when it is non-NULL, otherwise gathered from x through row_token.
 * y_perm: dtype [max_rows,d] (rows < nnz written). */
int32_t dsmoe_expert_ffn(dsmoe_ctx* ctx, const void* x, const void* x_perm, const int32_t* row_token,
                         const int32_t* expert_off, const void* w_gate, const void* w_up,
                         const void* w_down, void* y_perm, void* stream);

/* Probability-weighted combine and un-permute (Eq. 1 second half; the second overhead named in Sec. 4.4:
 * the expert outputs of a token are gathered and added up): out[t,:] = sum_j row_weight[r_j] * y_perm[r_j,:] over the rows
 * r_j = tok_rows[tok_off[t] .. tok_off[t+1]) in that (ascending expert) order, fp32 accumulation.
 * out: dtype [T,d] (written). */
int32_t dsmoe_combine(dsmoe_ctx* ctx, const void* y_perm, const float* row_weight, const int32_t* tok_off,
                      const int32_t* tok_rows, int32_t T, void* out, void* stream);

/* Whole sparse-inference forward (Eq. 1): route, select, dispatch, expert FFN and combine in one call,
 * with the intermediate routing objects kept in the workspace.  Same results as the five staged calls.
 * out: dtype [T,d] (written). */
int32_t dsmoe_sparse_fwd(dsmoe_ctx* ctx, const void* x, const void* w_r, const void* b_r,
                         const void* w_gate, const void* w_up, const void* w_down, int32_t T,
                         int32_t mode, int32_t k, float eps, void* out, void* stream);

/* 1 if dsmoe_sparse_fwd would serve a call of T tokens with this selection by its persistent decode kernel (a
 * bf16 batch of at most 64 tokens that together select nearly every expert: top-K with at most a tenth of the
 * experts expected idle, or at least 8 tokens under a normalised threshold of at most 1), which streams the
 * weights of ALL experts once; 0 otherwise (also without a workspace).  Informational. */
int32_t dsmoe_sparse_fwd_uses_persistent_kernel(const dsmoe_ctx* ctx, int32_t T, int32_t mode, int32_t k, float eps);

/* Which kernels dsmoe_sparse_fwd would run for a call of T tokens with this selection (Sec. 4.4 separates the
 * compute-bound prefill from the I/O-bound decoding; the library picks by batch size).  Informational; -1 for an
 * invalid request or without a workspace.  All paths compute Eq. 1 on the same routing. */
#define DSMOE_PATH_GROUPED 0     /* dispatch + grouped MFMA GEMMs + combine (prefill) */
#define DSMOE_PATH_STREAMING 1   /* at most 128 tokens (bf16): weight-streaming MFMA kernels, K-split partial sums */
#define DSMOE_PATH_ALL_EXPERTS 2 /* the persistent kernel of dsmoe_sparse_fwd_uses_persistent_kernel */
#define DSMOE_PATH_FEW_TOKENS 3  /* at most 4 tokens (bf16, top-K or threshold): three kernels, router included, that
                                  * stream the selected experts' weight rows through the vector ALUs */
int32_t dsmoe_sparse_fwd_path(const dsmoe_ctx* ctx, int32_t T, int32_t mode, int32_t k, float eps);

/* Copies the routing objects of the last dsmoe_sparse_fwd out of the workspace (any argument may be
 * NULL; after a decode-sized call whose kernels need no dispatch, the dispatch objects are derived here, on
 * `stream`, from the scores and masks that call left): probs fp32 [T,E], mask u64 [T], expert_off i32 [E+1], row_token i32 [max_rows]. */
int32_t dsmoe_sparse_fwd_routing(dsmoe_ctx* ctx, int32_t T, float* probs, uint64_t* mask,
                                 int32_t* expert_off, int32_t* row_token, void* stream);

/* Dense-training forward (Sec. 3.2 "Dense Training"): out[t,:] = sum_{j=1..E} S[t,j] * e_j(x[t,:]),
 * every expert on every token.  `saved` (dsmoe_dense_saved_bytes(T) bytes, caller-owned, layout
 * private) receives what the backward pass needs; NULL skips it.  probs: fp32 [T,E] or NULL. */
int32_t dsmoe_dense_saved_bytes(const dsmoe_ctx* ctx, int32_t T, size_t* bytes /* host */);
int32_t dsmoe_dense_fwd(dsmoe_ctx* ctx, const void* x, const void* w_r, const void* b_r,
                        const void* w_gate, const void* w_up, const void* w_down, int32_t T, void* out,
                        float* probs, void* saved, void* stream);

/* Dense-training backward (Eq. 3: grad S = [e_1(X)..e_N(X)]^T grad O, grad e_j(X) = S_j grad O, then
 * the chain rule through the experts, the softmax and the router).
 * d_out: dtype [T,d].  scratch: dsmoe_dense_bwd_scratch_bytes(T) bytes of caller-owned device memory.
 * Written (overwritten, not accumulated): dx dtype [T,d]; fp32 gradients dw_r [d,E], db_r [E]
 * (NULL allowed), dw_gate [E,d,f], dw_up [E,d,f], dw_down [E,f,d]. */
int32_t dsmoe_dense_bwd_scratch_bytes(const dsmoe_ctx* ctx, int32_t T, size_t* bytes /* host */);
int32_t dsmoe_dense_bwd(dsmoe_ctx* ctx, const void* x, const void* w_r, const void* w_gate,
                        const void* w_up, const void* w_down, const void* saved, const void* d_out,
                        int32_t T, void* scratch, void* dx, float* dw_r, float* db_r, float* dw_gate,
                        float* dw_up, float* dw_down, void* stream);

/* Mutual-information load-balance loss of the router (Sec. 3.2, Eq. 4-6):
 *   L_MI = -H(e) + (1/T) sum_t H(e | x_t),  H(e) = -sum_i p_i log p_i with p_i the batch mean of
 *   probs[:,i],  H(e | x_t) = -sum_i probs[t,i] log probs[t,i]  (0 log 0 = 0).
 * probs: fp32 [T,E] (T >= 1).  Written: loss, device fp32 [1] (may be NULL); p_mean, device fp32 [E], the
 * batch means p_i (may be NULL; not both).  Needs the workspace.  Two-stage reduction in a fixed order. */
int32_t dsmoe_mi_loss(dsmoe_ctx* ctx, const float* probs, int32_t T, float* loss, float* p_mean,
                      void* stream);

/* dsmoe_dense_bwd for the total loss L = L_LM + mi_alpha * L_MI (Sec. 3.2, Eq. 6): the score gradient
 * of Eq. 3 gets the term mi_alpha * dL_MI/dS[t,i] = mi_alpha * (log p_i - log S[t,i]) / T before the
 * softmax backward, so dx, dw_r and db_r include the load-balance term; the expert-weight gradients do
 * not depend on it.  mi_alpha = 0 is dsmoe_dense_bwd.  Same arguments, buffers and error behaviour. */
int32_t dsmoe_dense_bwd_mi(dsmoe_ctx* ctx, const void* x, const void* w_r, const void* w_gate,
                           const void* w_up, const void* w_down, const void* saved, const void* d_out,
                           int32_t T, void* scratch, void* dx, float* dw_r, float* db_r, float* dw_gate,
                           float* dw_up, float* dw_down, float mi_alpha, void* stream);

/* Kernel timing for benchmarks (not part of the layer's definition).  While enabled, every call that
 * runs the expert FFN (dsmoe_expert_ffn, dsmoe_sparse_fwd) brackets its two grouped-GEMM kernels with
 * HIP events recorded on the call's stream, for at most max_calls calls.  dsmoe_profile_read waits for
 * the recorded events, returns the number of calls and the summed durations in milliseconds of the
 * gate/up kernel and of the down kernel (host pointers), and starts a new series.
 * max_calls = 0 disables timing and releases the events. */
int32_t dsmoe_profile_enable(dsmoe_ctx* ctx, int32_t max_calls);
int32_t dsmoe_profile_read(dsmoe_ctx* ctx, int32_t* n_calls /* host */, float* gateup_ms /* host */,
                           float* down_ms /* host */);

/* Measured ceilings for benchmarks (not part of the layer; each call synchronises `stream`).
 * dsmoe_bench_mfma: `blocks` blocks of eight waves run `iters` x 8 independent 32x32x16 bf16 MFMAs per wave on
 *   register operands taken from `seed` (device, 16 KiB: zeros or random bf16 values - the sustained clock
 *   depends on the bits that toggle); `sink`: device, blocks * 2 KiB.  Returns milliseconds and the flop count.
 * dsmoe_bench_stream: `blocks` blocks read (write = 0) or write (write = 1) the window [window, window + bytes)
 *   once with 16-byte accesses; `moved` receives the bytes actually touched.  `sink`: device, >= 4 bytes.
 * dsmoe_bench_xcc_ids: out[b] (device int32 [blocks]) = hardware id of the XCD that ran block b of a launch. */
int32_t dsmoe_bench_mfma(const void* seed, void* sink, int32_t blocks, int32_t iters, float* ms /* host */,
                         double* flop /* host */, void* stream);
int32_t dsmoe_bench_stream(void* window, size_t bytes, int32_t write, int32_t blocks, void* sink,
                           float* ms /* host */, size_t* moved /* host */, void* stream);
int32_t dsmoe_bench_xcc_ids(int32_t* out, int32_t blocks, void* stream);

/* ---- Mixture-of-Attention-heads layer (Sec. 3.2, "Mixture of Attention Head", Eq. 7-8) -------------
 * bf16 only.  E experts; expert i has a query projection W_q[i] and an output projection
 * W_o[i]; the n_head key/value heads of the cache are shared by all experts (grouped-query attention:
 * head j of every expert attends to K[j], V[j]).  For a token x with router scores S (softmax of
 * x W_r + b_r, as in the MLP layer) and selected set A:
 *     Q_i = x W_q[i],   O_ij = softmax(scale * Q_ij K_j^T) V_j W_o[i][j]   (Eq. 7)
 *     out = sum_{i in A} S_i sum_j O_ij                                    (Eq. 8)
 * The T tokens of a call are the last T positions of the cache (position of token t = L - T + t) and a
 * token attends to positions <= its own (causal); the caller has already written their keys and values
 * into the cache.  `scale`: Eq. 7 prints no factor (scale = 1); 1/sqrt(d_head) is the usual one.
 * Every expert is computed for every token (the paper runs this layer densely at inference, Sec. 4.4);
 * the selection only zeroes the weights of the experts outside A.
 *
 * Layouts (device, row-major, 16-byte aligned): x [T,d]; w_r [d,E]; b_r [E] or NULL;
 * w_q [E, d, n_head*d_head]; k_cache, v_cache [n_head, L, d_head]; w_o [E, n_head*d_head, d]; out [T,d].
 * Limits: E a multiple of 8 and <= 64, d a multiple of 64, d_head 64 or 128, L >= T >= 0,
 * T <= max_tokens.  The context owns no device memory; dsmoe_moa_set_workspace lends it
 * dsmoe_moa_workspace_bytes bytes (router scores, masks, Q, the attention outputs with and without their
 * weights, the softmax denominators).
 * mode: DSMOE_SEL_TOPK (k), DSMOE_SEL_THRESHOLD (eps) or DSMOE_SEL_ALL.  Errors as for the MLP layer
 * (status code, message from dsmoe_moa_last_error); one call at a time per context. */
#define DSMOE_SEL_ALL (-1)
typedef struct dsmoe_moa_desc {
  int32_t d_model, n_experts, n_head, d_head, dtype /* DSMOE_BF16 */, max_tokens;
} dsmoe_moa_desc;
typedef struct dsmoe_moa_ctx dsmoe_moa_ctx;
int32_t dsmoe_moa_create(const dsmoe_moa_desc* desc /* host */, dsmoe_moa_ctx** out /* host */);
int32_t dsmoe_moa_destroy(dsmoe_moa_ctx* ctx);
const char* dsmoe_moa_last_error(const dsmoe_moa_ctx* ctx);
int32_t dsmoe_moa_workspace_bytes(const dsmoe_moa_ctx* ctx, size_t* bytes /* host */);
int32_t dsmoe_moa_set_workspace(dsmoe_moa_ctx* ctx, void* workspace /* device, 256-byte aligned */, size_t bytes);
int32_t dsmoe_moa_fwd(dsmoe_moa_ctx* ctx, const void* x, const void* w_r, const void* b_r, const void* w_q,
                      const void* k_cache, const void* v_cache, const void* w_o, int32_t T, int32_t L,
                      int32_t mode, int32_t k, float eps, float scale, void* out, void* stream);
/* Copies the router scores (fp32 [T,E]) and selection masks (bit e of mask[t]; all experts for
 * DSMOE_SEL_ALL) of the last dsmoe_moa_fwd call out of the workspace; either pointer may be NULL. */
int32_t dsmoe_moa_routing(dsmoe_moa_ctx* ctx, int32_t T, float* probs, uint64_t* mask, void* stream);

/* Dense-training backward of the attention layer (Sec. 3.2, "Dense Training": every expert active and
 * weighted by its score; gradients of Eq. 7-8, the score gradient as in Eq. 3 with the attention experts in
 * the place of the MLP experts).  For the upstream gradient d_out [T,d] of
 *     out = sum_i S_i sum_j softmax(scale Q_ij K_j^T) V_j W_o[i][j]
 * it returns the gradients with respect to x, the router, both projections and the shared cache:
 *     dx [T,d] bf16;  dw_r [d,E], db_r [E] (may be NULL), dw_q [E, d, n_head*d_head],
 *     dw_o [E, n_head*d_head, d], dk and dv [n_head, L, d_head]: fp32, overwritten (not accumulated).
 * It must directly follow, on the same stream, the dsmoe_moa_fwd call with mode DSMOE_SEL_ALL and the same
 * x, weights, cache, T, L and scale: that call leaves the scores, the queries, the attention outputs and
 * the logarithms of the softmax denominators in the workspace, and this one reads them (any other call
 * in between, or another T, L or scale, is DSMOE_ERR_INVALID_ARG).  T >= 1.
 * `scratch`: caller-owned device memory of dsmoe_moa_bwd_scratch_bytes(T, L) bytes, 256-byte aligned,
 * contents irrelevant before and after (its largest part is the attention probabilities of all experts,
 * E * T * n_head * L bf16 values).  No floating-point atomics: sums over experts and tokens are
 * contractions in a fixed order, results are bitwise reproducible.  All pointers device, 16-byte aligned;
 * nothing is allocated; work is enqueued on `stream`. */
int32_t dsmoe_moa_bwd_scratch_bytes(const dsmoe_moa_ctx* ctx, int32_t T, int32_t L, size_t* bytes /* host */);
int32_t dsmoe_moa_bwd(dsmoe_moa_ctx* ctx, const void* x, const void* w_r, const void* w_q, const void* k_cache,
                      const void* v_cache, const void* w_o, const void* d_out, int32_t T, int32_t L, float scale,
                      void* scratch, void* dx, float* dw_r, float* db_r, float* dw_q, float* dw_o, float* dk,
                      float* dv, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DSMOE_H_ */
