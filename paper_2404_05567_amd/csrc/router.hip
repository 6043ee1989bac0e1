// Router of the MoE layer: S = softmax(h(X)) over all N experts (paper Eq. 1), fused with the
// inference-time expert selection (top-K of Sec. 3.1, score threshold of Sec. 3.2 "Sparse Inference").
//
// One block owns 32 tokens.  The waves split K, read their X fragments straight from global memory
// into the MFMA token operand through a deep register ring (the kernel is bound by the X read), and
// bring the matching W_r slice into the expert operand through LDS.  Partial logits are reduced
// across waves in a fixed order, then each wave finishes its share of the tokens with one lane per
// expert: max, exp, sum by butterfly reductions, and the selection as a ballot.
//   fp32: four waves share every 128-byte K slice; W_r is transposed in registers (route_kernel).
//   bf16: eight waves own contiguous K ranges and never synchronise inside the K loop: each stages
//         its own 16 x E slice of W_r as stored and reads it back with the transposing LDS load; with
//         16 slices in flight per wave a decode-sized call needs one memory round trip (route_bf16_kernel).
#include "gemm_dma.h"
#include "router_common.h"

namespace dsmoe {

constexpr int kRouterTokens = 32;   // tokens per block
constexpr int kRouterRing = 16;     // K slices of X kept in flight per wave

template <typename T, int EP>   // EP: experts padded to 32 or 64
__global__ void __launch_bounds__(kThreads)
route_kernel(const T* __restrict__ x, const T* __restrict__ w_r, const T* __restrict__ b_r, int T_tokens, int d, int E,
             float* __restrict__ probs, int mode, int k, float eps, unsigned long long* __restrict__ mask,
             int32_t* __restrict__ cnt_tok) {
  constexpr int BK = ElemTraits<T>::BK;
  constexpr int ET = EP / 32;
  __shared__ __align__(16) char sW[2][EP * kLdsPitch];
  __shared__ float sPart[4][kRouterTokens][EP + 1];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * kRouterTokens;
  const int nkt = d / BK;

  // X fragment of this lane: token t0 + lane%32, bytes [wave*32 + (lane/32)*16, +16) of each K slice
  const int trow = min(t0 + (lane & 31), T_tokens - 1);
  const char* xp = reinterpret_cast<const char*>(x + (size_t)trow * d) + wave * 32 + (lane >> 5) * 16;
  const char* fW = &sW[0][0] + (lane & 31) * kLdsPitch + wave * 32 + (lane >> 5) * 16;

  SrcCols<T, EP> W;
  W.base = reinterpret_cast<const char*>(w_r);
  W.ld_bytes = (size_t)E * sizeof(T);
  W.seg_stride = 0;
  W.rows_valid = E;
  W.k_valid = d;

  f32x16 acc[ET];
#pragma unroll
  for (int et = 0; et < ET; ++et)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[et][i] = 0.f;

  u32x4 xr[kRouterRing];
#pragma unroll
  for (int j = 0; j < kRouterRing; ++j)
    if (j < nkt) xr[j] = ldg16(xp + (size_t)j * kRowBytes);
  u32x4 wr[SrcCols<T, EP>::NV];
  W.load(wr, 0, 0);

  for (int kt0 = 0; kt0 < nkt; kt0 += kRouterRing) {
#pragma unroll
    for (int j = 0; j < kRouterRing; ++j) {
      const int kt = kt0 + j;
      if (kt < nkt) {
        W.store(wr, sW[kt & 1]);
        if (kt + 1 < nkt) W.load(wr, 0, kt + 1);
        __syncthreads();
#pragma unroll
        for (int et = 0; et < ET; ++et) {
          const u32x4 wf =
              *reinterpret_cast<const u32x4*>(fW + (kt & 1) * (EP * kLdsPitch) + et * 32 * kLdsPitch);
          Mma<T>::run(acc[et], wf, xr[j]);
        }
        if (kt + kRouterRing < nkt) xr[j] = ldg16(xp + (size_t)(kt + kRouterRing) * kRowBytes);
      }
    }
  }

  // partial logits of this wave: lane owns token lane%32; register 4q+i <-> expert 8q + 4*(lane/32) + i
#pragma unroll
  for (int et = 0; et < ET; ++et)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      sPart[wave][lane & 31][et * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3)] = acc[et][i];
  __syncthreads();

  const float bias = (b_r != nullptr && lane < E) ? to_f32(b_r[lane]) : 0.f;
  for (int tt = wave * 8; tt < wave * 8 + 8; ++tt) {
    const int t = t0 + tt;
    if (t >= T_tokens) break;
    float z = -INFINITY;
    if (lane < E) z = ((sPart[0][tt][lane] + sPart[1][tt][lane]) + (sPart[2][tt][lane] + sPart[3][tt][lane])) + bias;
    const float zmax = wave_max(z);
    const float ez = lane < E ? expf(z - zmax) : 0.f;
    const float p = ez / wave_sum(ez);
    if (lane < E) probs[(size_t)t * E + lane] = p;
    if (mode >= 0) {
      const unsigned long long m = select_wave(lane < E ? p : -1.f, lane, E, mode, k, eps);
      if (lane == 0) {
        mask[t] = m;
        if (cnt_tok) cnt_tok[t] = __popcll(m);
      }
    }
  }
}


template <int EP, int TOK>
__global__ void __launch_bounds__(kThreads2)
route_bf16_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w_r, const bf16_t* __restrict__ b_r,
                  int T_tokens, int d, int E, float* __restrict__ probs, int mode, int k, float eps,
                  unsigned long long* __restrict__ mask, int32_t* __restrict__ cnt_tok) {
  extern __shared__ __align__(16) char smem[];
  route_bf16_tile<EP, TOK>(x, w_r, b_r, T_tokens, d, E, probs, mode, k, eps, mask, cnt_tok, blockIdx.x * TOK, smem);
}

template <int EP, int TOK>
static hipError_t launch_route_bf16(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, int T_tokens,
                                    float* probs, int mode, int k, float eps, uint64_t* mask, int32_t* cnt_tok,
                                    hipStream_t s) {
  constexpr int lds = route_bf16_lds<EP, TOK>();
  static bool attr_set = false;
  if (!attr_set) {
    if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&route_bf16_kernel<EP, TOK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds))
      return e;
    attr_set = true;
  }
  const int grid = (T_tokens + TOK - 1) / TOK;
  route_bf16_kernel<EP, TOK><<<dim3(grid), dim3(kThreads2), lds, s>>>(
      (const bf16_t*)x, (const bf16_t*)w_r, (const bf16_t*)b_r, T_tokens, c->desc.d_model, c->desc.n_experts, probs,
      mode, k, eps, (unsigned long long*)mask, cnt_tok);
  return hipGetLastError();
}

__global__ void __launch_bounds__(kThreads)
select_kernel(const float* __restrict__ probs, int T_tokens, int E, int mode, int k, float eps,
              unsigned long long* __restrict__ mask, int32_t* __restrict__ cnt_tok, const int32_t* __restrict__ k_dev) {
  if (k_dev != nullptr) k = k_dev[0];   // K computed on the device (Threshold-TopK)
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T_tokens) return;
  const float p = lane < E ? probs[(size_t)t * E + lane] : -1.f;
  const unsigned long long m = select_wave(p, lane, E, mode, k, eps);
  if (lane == 0) {
    mask[t] = m;
    if (cnt_tok) cnt_tok[t] = __popcll(m);
  }
}

template <typename T>
static hipError_t launch_route_t(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, int T_tokens,
                                 float* probs, int mode, int k, float eps, uint64_t* mask, int32_t* cnt_tok,
                                 hipStream_t s) {
  const int d = c->desc.d_model, E = c->desc.n_experts;
  const int grid = (T_tokens + kRouterTokens - 1) / kRouterTokens;
  if (E <= 32)
    hipLaunchKernelGGL((route_kernel<T, 32>), dim3(grid), dim3(kThreads), 0, s, (const T*)x, (const T*)w_r,
                       (const T*)b_r, T_tokens, d, E, probs, mode, k, eps, (unsigned long long*)mask, cnt_tok);
  else
    hipLaunchKernelGGL((route_kernel<T, 64>), dim3(grid), dim3(kThreads), 0, s, (const T*)x, (const T*)w_r,
                       (const T*)b_r, T_tokens, d, E, probs, mode, k, eps, (unsigned long long*)mask, cnt_tok);
  return hipGetLastError();
}

hipError_t launch_route(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, int T_tokens,
                        float* probs, int mode, int k, float eps, uint64_t* mask, int32_t* cnt_tok, hipStream_t s) {
  if (T_tokens == 0) return hipSuccess;
  if (c->desc.dtype == DSMOE_BF16) {
    // tokens per block: as few as still give at most one block per CU (a shorter selection tail); a full
    // tile for large calls, since every block reads all of W_r and issues the same loads whatever its tokens
    const int tok = T_tokens <= 8 * c->n_cu ? 8 : T_tokens <= 16 * c->n_cu ? 16 : 32;
#define DSMOE_ROUTE_BF16(EP, TOK) \
  launch_route_bf16<EP, TOK>(c, x, w_r, b_r, T_tokens, probs, mode, k, eps, mask, cnt_tok, s)
    if (c->desc.n_experts <= 32)
      return tok == 8 ? DSMOE_ROUTE_BF16(32, 8) : tok == 16 ? DSMOE_ROUTE_BF16(32, 16) : DSMOE_ROUTE_BF16(32, 32);
    return tok == 8 ? DSMOE_ROUTE_BF16(64, 8) : tok == 16 ? DSMOE_ROUTE_BF16(64, 16) : DSMOE_ROUTE_BF16(64, 32);
#undef DSMOE_ROUTE_BF16
  }
  return launch_route_t<float>(c, x, w_r, b_r, T_tokens, probs, mode, k, eps, mask, cnt_tok, s);
}

hipError_t launch_select(const dsmoe_ctx* c, const float* probs, int T_tokens, int mode, int k, float eps,
                         uint64_t* mask, int32_t* cnt_tok, hipStream_t s, const int32_t* k_dev) {
  if (T_tokens == 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3((T_tokens + 3) / 4), dim3(kThreads), 0, s, probs, T_tokens,
                     c->desc.n_experts, mode, k, eps, (unsigned long long*)mask, cnt_tok, k_dev);
  return hipGetLastError();
}

}  // namespace dsmoe
