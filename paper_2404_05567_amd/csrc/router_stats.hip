// Batch statistics of the router scores S[T,E]:
//   * the mutual-information load-balance loss of Sec. 3.2 (Eq. 4-6): L_MI = -H(e) + mean_t H(e | x_t), with
//     p(e_i) the batch mean of S[:,i] and H(e | x_t) the entropy of one token's scores (the printed Eq. 4 has
//     lost the index of p(e); this is the reading under which Eq. 5 follows from it);
//   * the K of Threshold-TopK selection (Sec. 4.3): the batch mean of the per-token expert counts that the
//     threshold gives, rounded half up, used as a fixed top-K.
// Both are reductions over tokens done in two deterministic stages (per-block partial sums added in block order).
#include <algorithm>

#include "common.h"

namespace dsmoe {

namespace {

constexpr int kStatThreads = 256;

// part[b][0..64): column sums of S over the block's tokens; part[b][64..128): sums of S log S per expert.
// One lane per expert, the block's four waves take tokens 4 b + w, 4 (b + grid) + w, ...
__global__ void __launch_bounds__(kStatThreads)
mi_partial_kernel(const float* __restrict__ S, int T, int E, float* __restrict__ part) {
  __shared__ float sh[kStatThreads / 64][128];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float cs = 0.f, en = 0.f;
  if (lane < E)
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
      const float s = S[(size_t)t * E + lane];
      cs += s;
      en += s > 0.f ? s * logf(s) : 0.f;       // 0 log 0 = 0
    }
  sh[wave][lane] = cs;
  sh[wave][64 + lane] = en;
  __syncthreads();
  if (threadIdx.x < 128)
    part[(size_t)blockIdx.x * 128 + threadIdx.x] =
        (sh[0][threadIdx.x] + sh[1][threadIdx.x]) + (sh[2][threadIdx.x] + sh[3][threadIdx.x]);
}

__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

// p_mean[i] = (sum_b part[b][i]) / T;  loss = sum_i p_i log p_i - (1/T) sum_i sum_b part[b][64 + i]
__global__ void __launch_bounds__(64)
mi_final_kernel(const float* __restrict__ part, int nb, int T, int E, float* __restrict__ p_mean,
                float* __restrict__ loss) {
  const int lane = threadIdx.x;
  float cs = 0.f, en = 0.f;
  for (int b = 0; b < nb; ++b) {
    cs += part[(size_t)b * 128 + lane];
    en += part[(size_t)b * 128 + 64 + lane];
  }
  const float inv = 1.f / (float)T;
  const float p = cs * inv;
  const float plogp = (lane < E && p > 0.f) ? p * logf(p) : 0.f;
  const float total = wave_sum64(plogp) - wave_sum64(lane < E ? en : 0.f) * inv;
  if (p_mean != nullptr && lane < E) p_mean[lane] = p;
  if (loss != nullptr && lane == 0) loss[0] = total;
}

// k_out[0] = clamp(floor(mean(cnt_tok) + 1/2), 1, E), in integers: floor((2 sum + T) / (2 T))
__global__ void __launch_bounds__(kStatThreads)
threshold_topk_k_kernel(const int32_t* __restrict__ cnt_tok, int T, int E, int32_t* __restrict__ k_out) {
  __shared__ long long sh[kStatThreads / 64];
  long long sum = 0;
  for (int t = threadIdx.x; t < T; t += kStatThreads) sum += cnt_tok[t];
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) sum += __shfl_xor(sum, s, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    const long long tot = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    const long long k = (2 * tot + T) / (2ll * T);
    k_out[0] = (int32_t)std::min<long long>(std::max<long long>(k, 1), E);
  }
}

}  // namespace

int mi_blocks(int T) { return std::max(1, std::min(kStatMaxBlocks, (T + 63) / 64)); }

hipError_t launch_mi_loss(const dsmoe_ctx* c, const float* S, int T, float* part, float* p_mean, float* loss,
                          hipStream_t s) {
  const int nb = mi_blocks(T), E = c->desc.n_experts;
  mi_partial_kernel<<<dim3(nb), dim3(kStatThreads), 0, s>>>(S, T, E, part);
  if (hipError_t e = hipGetLastError()) return e;
  mi_final_kernel<<<dim3(1), dim3(64), 0, s>>>(part, nb, T, E, p_mean, loss);
  return hipGetLastError();
}

hipError_t launch_threshold_topk_k(const dsmoe_ctx* c, const int32_t* cnt_tok, int T, int32_t* k_out, hipStream_t s) {
  threshold_topk_k_kernel<<<dim3(1), dim3(kStatThreads), 0, s>>>(cnt_tok, T, c->desc.n_experts, k_out);
  return hipGetLastError();
}

}  // namespace dsmoe
