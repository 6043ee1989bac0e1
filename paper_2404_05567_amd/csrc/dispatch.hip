// Token-to-expert dispatch and the weighted combine: the two "overheads of dynamic inference" the
// paper names in Sec. 4.4 (duplication of intermediate tokens, aggregation of expert outputs).
//
// Dispatch is a stable counting sort of the (token, expert) pairs by expert: a per-block histogram,
// then a scatter pass in which every block re-derives its own base offsets from the histogram table
// (a few KB) instead of waiting for a separate scan kernel.  Ranks inside a block come from wave
// ballots, so the order (experts ascending, tokens ascending inside an expert) is deterministic.
#include <algorithm>

#include "gemm_core.h"

namespace dsmoe {

constexpr int kDB = kDispatchTokensPerBlock;   // 256 tokens = 4 waves of 64

__global__ void __launch_bounds__(kDB)
dispatch_hist_kernel(const unsigned long long* __restrict__ mask, int T, int E, int32_t* __restrict__ blk_cnt,
                     int32_t* __restrict__ blk_tok) {
  __shared__ int sCnt[4][kMaxExperts];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * kDB + threadIdx.x;
  const unsigned long long m = t < T ? mask[t] : 0ull;
  int mine = 0;
  for (int e = 0; e < E; ++e) {
    const int c = __popcll(__ballot((m >> e) & 1ull));
    if (lane == e) mine = c;
  }
  sCnt[wave][lane] = mine;
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = threadIdx.x < E ? sCnt[0][lane] + sCnt[1][lane] + sCnt[2][lane] + sCnt[3][lane] : 0;
    if (threadIdx.x < E) blk_cnt[(size_t)blockIdx.x * E + threadIdx.x] = c;
    int tot = c;
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) tot += __shfl_xor(tot, s, 64);
    if (threadIdx.x == 0) blk_tok[blockIdx.x] = tot;
  }
}

__global__ void __launch_bounds__(kDB)
dispatch_scatter_kernel(const unsigned long long* __restrict__ mask, const float* __restrict__ probs, int T, int E,
                        const int32_t* __restrict__ blk_cnt, const int32_t* __restrict__ blk_tok, long long max_rows,
                        int32_t* __restrict__ expert_off, int32_t* __restrict__ row_token, float* __restrict__ row_weight,
                        int32_t* __restrict__ tok_off, int32_t* __restrict__ tok_rows, int32_t* __restrict__ nnz_out,
                        int32_t* __restrict__ err_flag) {
  __shared__ int sRowBase[kMaxExperts];    // first row of this block's tokens inside each expert
  __shared__ int sWave[4][kMaxExperts];    // per-wave expert counts
  __shared__ int sWaveTok[4];
  __shared__ int sTokBase, sNnz;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nblk = gridDim.x, b = blockIdx.x;

  if (threadIdx.x < 64) {
    int total = 0, before = 0;
    if (lane < E)
      for (int bb = 0; bb < nblk; ++bb) {
        const int c = blk_cnt[(size_t)bb * E + lane];
        total += c;
        if (bb < b) before += c;
      }
    int incl = total;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(incl, s, 64);
      if (lane >= s) incl += o;
    }
    const int nnz = __shfl(incl, 63, 64);
    const bool overflow = (long long)nnz > max_rows;
    const int off = overflow ? 0 : incl - total;
    if (lane < E) sRowBase[lane] = off + before;
    if (b == 0) {
      if (lane < E) expert_off[lane] = off;
      if (lane == 0) {
        expert_off[E] = overflow ? 0 : nnz;
        nnz_out[0] = overflow ? 0 : nnz;
        if (overflow) err_flag[0] = DSMOE_ERR_CAPACITY;
      }
    }
    if (lane == 0) sNnz = overflow ? -1 : nnz;
  } else if (threadIdx.x < 128) {
    int before = 0;
    for (int bb = lane; bb < b; bb += 64) before += blk_tok[bb];
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) before += __shfl_xor(before, s, 64);
    if (lane == 0) sTokBase = before;
  }

  const int t = b * kDB + threadIdx.x;
  const unsigned long long m = t < T ? mask[t] : 0ull;
  const unsigned long long lt = (1ull << lane) - 1ull;
  int mine = 0;
  for (int e = 0; e < E; ++e) {
    const int c = __popcll(__ballot((m >> e) & 1ull));
    if (lane == e) mine = c;
  }
  sWave[wave][lane] = mine;
  // exclusive scan of the per-token counts inside the wave
  const int cnt = __popcll(m);
  int incl = cnt;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const int o = __shfl_up(incl, s, 64);
    if (lane >= s) incl += o;
  }
  if (lane == 63) sWaveTok[wave] = incl;
  __syncthreads();

  const bool overflow = sNnz < 0;
  int tbase = overflow ? 0 : sTokBase + incl - cnt;
  for (int w = 0; w < wave; ++w) tbase += overflow ? 0 : sWaveTok[w];
  if (t < T) tok_off[t] = tbase;
  if (t == T - 1) tok_off[T] = overflow ? 0 : sNnz;
  if (overflow) return;

  for (int e = 0; e < E; ++e) {
    const unsigned long long bits = __ballot((m >> e) & 1ull);
    if ((m >> e) & 1ull) {
      int row = sRowBase[e] + __popcll(bits & lt);
      for (int w = 0; w < wave; ++w) row += sWave[w][e];
      row_token[row] = t;
      row_weight[row] = probs[(size_t)t * E + e];
      tok_rows[tbase + __popcll(m & ((1ull << e) - 1ull))] = row;
    }
  }
}

// x_perm[r,:] = x[row_token[r],:] for r < nnz (optional materialised permutation)
__global__ void __launch_bounds__(kThreads)
gather_rows_kernel(const char* __restrict__ x, const int32_t* __restrict__ row_token, const int32_t* __restrict__ nnz,
                   char* __restrict__ x_perm, int row_bytes) {
  const int n = nnz[0];
  for (int r = blockIdx.x; r < n; r += gridDim.x) {
    const char* src = x + (size_t)row_token[r] * row_bytes;
    char* dst = x_perm + (size_t)r * row_bytes;
    for (int o = threadIdx.x * 16; o < row_bytes; o += kThreads * 16)
      *reinterpret_cast<u32x4*>(dst + o) = ldg16(src + o);
  }
}

__global__ void empty_routing_kernel(int E, int32_t* expert_off, int32_t* tok_off, int32_t* nnz) {
  if (threadIdx.x <= E) expert_off[threadIdx.x] = 0;
  if (threadIdx.x == 0) { tok_off[0] = 0; nnz[0] = 0; }
}

hipError_t launch_dispatch(const dsmoe_ctx* c, const void* x, const float* probs, const uint64_t* mask, int T,
                           int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                           int32_t* tok_rows, int32_t* nnz, void* x_perm, hipStream_t s) {
  const int E = c->desc.n_experts;
  if (T == 0) {
    hipLaunchKernelGGL(empty_routing_kernel, dim3(1), dim3(128), 0, s, E, expert_off, tok_off, nnz);
    return hipGetLastError();
  }
  const int nblk = (T + kDB - 1) / kDB;
  int32_t* blk_cnt = reinterpret_cast<int32_t*>(c->workspace + c->ws.blk_cnt);
  int32_t* blk_tok = reinterpret_cast<int32_t*>(c->workspace + c->ws.blk_tok);
  int32_t* err_flag = reinterpret_cast<int32_t*>(c->workspace + c->ws.err_flag);
  hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblk), dim3(kDB), 0, s, (const unsigned long long*)mask, T, E,
                     blk_cnt, blk_tok);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(nblk), dim3(kDB), 0, s, (const unsigned long long*)mask, probs, T,
                     E, blk_cnt, blk_tok, (long long)c->desc.max_rows, expert_off, row_token, row_weight, tok_off,
                     tok_rows, nnz, err_flag);
  err = hipGetLastError();
  if (err != hipSuccess || x_perm == nullptr) return err;
  const long grid = std::min<long>(c->desc.max_rows, (long)c->n_cu * 8);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)std::max<long>(grid, 1)), dim3(kThreads), 0, s,
                     (const char*)x, row_token, nnz, (char*)x_perm, (int)(c->desc.d_model * c->esize));
  return hipGetLastError();
}

// ---- combine -----------------------------------------------------------------------------------
// out[t,:] = sum over the token's rows (ascending expert) of row_weight * y_perm[row,:], fp32 accumulate.
template <typename T>
__global__ void __launch_bounds__(kThreads)
combine_kernel(const T* __restrict__ y, const float* __restrict__ row_weight, const int32_t* __restrict__ tok_off,
               const int32_t* __restrict__ tok_rows, int d, T* __restrict__ out) {
  constexpr int VEC = ElemTraits<T>::VEC;
  const int t = blockIdx.x;
  const int lo = tok_off[t], hi = tok_off[t + 1];
  for (int c0 = threadIdx.x * VEC; c0 < d; c0 += kThreads * VEC) {
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    for (int j = lo; j < hi; ++j) {
      const int row = tok_rows[j];
      const float w = row_weight[row];
      const u32x4 v = ldg16(y + (size_t)row * d + c0);
      if constexpr (VEC == 4) {
        const f32x4 vf = __builtin_bit_cast(f32x4, v);
        acc[0] = fmaf(w, vf.x, acc[0]);
        acc[1] = fmaf(w, vf.y, acc[1]);
        acc[2] = fmaf(w, vf.z, acc[2]);
        acc[3] = fmaf(w, vf.w, acc[3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] = fmaf(w, __uint_as_float(v[i] << 16), acc[2 * i]);
          acc[2 * i + 1] = fmaf(w, __uint_as_float(v[i] & 0xffff0000u), acc[2 * i + 1]);
        }
      }
    }
    if constexpr (VEC == 4) {
      store4(reinterpret_cast<float*>(out) + (size_t)t * d + c0, acc[0], acc[1], acc[2], acc[3]);
    } else {
      u32x4 o = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]), pack_bf16x2(acc[4], acc[5]),
                 pack_bf16x2(acc[6], acc[7])};
      *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(out) + (size_t)t * d + c0) = o;
    }
  }
}

hipError_t launch_combine(const dsmoe_ctx* c, const void* y_perm, const float* row_weight, const int32_t* tok_off,
                          const int32_t* tok_rows, int T, void* out, hipStream_t s) {
  if (T == 0) return hipSuccess;
  const int d = c->desc.d_model;
  if (c->desc.dtype == DSMOE_BF16)
    hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(T), dim3(kThreads), 0, s, (const bf16_t*)y_perm, row_weight,
                       tok_off, tok_rows, d, (bf16_t*)out);
  else
    hipLaunchKernelGGL(combine_kernel<float>, dim3(T), dim3(kThreads), 0, s, (const float*)y_perm, row_weight,
                       tok_off, tok_rows, d, (float*)out);
  return hipGetLastError();
}

}  // namespace dsmoe
