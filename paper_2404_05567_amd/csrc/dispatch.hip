// Token-to-expert dispatch and the weighted combine: the two costs that Sec. 4.4 of the paper attributes to
// dynamic (sparse) inference - a token is copied once per selected expert, and its expert outputs are
// collected and summed afterwards.
//
// Dispatch is a stable counting sort of the (token, expert) pairs by expert: a per-block histogram,
// then a scatter pass in which every block re-derives its own base offsets from the histogram table
// (a few KB) instead of waiting for a separate scan kernel.  Ranks inside a block come from wave
// ballots, so the order (experts ascending, tokens ascending inside an expert) is deterministic.
#include <algorithm>
#include <cstdio>
#include <mutex>

#include "gemm_core.h"

namespace dsmoe {

constexpr int kDB = kDispatchTokensPerBlock;   // 256 tokens = 4 waves of 64

// Bits of a selection mask that name an expert.  A caller's mask may carry stray bits above E; they are dropped
// where a mask is loaded, so that the per-token counts (a population count) and the per-expert counts (bits
// below E) always agree and no row index can pass the counted total.
__device__ __forceinline__ unsigned long long expert_bits(int E) { return E >= 64 ? ~0ull : (1ull << E) - 1ull; }

__global__ void __launch_bounds__(kDB)
dispatch_hist_kernel(const unsigned long long* __restrict__ mask, int T, int E, int32_t* __restrict__ blk_cnt,
                     int32_t* __restrict__ blk_tok) {
  __shared__ int sCnt[4][kMaxExperts];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * kDB + threadIdx.x;
  const unsigned long long m = t < T ? mask[t] & expert_bits(E) : 0ull;
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

// One block per 256 tokens, 1024 threads: the first four waves hold one token per lane (ballots, scans), then
// four threads share a token and walk its experts, every probability read of a thread in flight at once.
constexpr int kScatterThreads = 4 * kDB;
__global__ void __launch_bounds__(kScatterThreads)
dispatch_scatter_kernel(const unsigned long long* __restrict__ mask, const float* __restrict__ probs, int T, int E,
                        const int32_t* __restrict__ blk_cnt, const int32_t* __restrict__ blk_tok, long long max_rows,
                        int32_t* __restrict__ expert_off, int32_t* __restrict__ row_token, float* __restrict__ row_weight,
                        int32_t* __restrict__ tok_off, int32_t* __restrict__ tok_rows, int32_t* __restrict__ nnz_out,
                        int32_t* __restrict__ err_flag) {
  constexpr int NW = kScatterThreads / 64;
  __shared__ int sRowBase[kMaxExperts];    // first row of this block's tokens inside each expert
  __shared__ int sWave[4][kMaxExperts];    // per-wave expert counts (token waves)
  __shared__ int sWaveTok[4];
  __shared__ int sTokBase, sNnz;
  __shared__ int sPartTotal[NW][64], sPartBefore[NW][64], sPartTok[NW];
  __shared__ unsigned long long sBits[4][kMaxExperts];   // per token wave and expert: which tokens selected it
  __shared__ unsigned long long sMask[kDB];
  __shared__ int sTokOff[kDB];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nblk = gridDim.x, b = blockIdx.x;

  // column sums of the histogram table: wave w adds blocks w, w + NW, ... (eight reads in flight)
  {
    int total = 0, before = 0;
    for (int bb0 = wave; bb0 < nblk; bb0 += NW * 8) {
      int cv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int bb = bb0 + NW * u;
        cv[u] = (bb < nblk && lane < E) ? blk_cnt[(size_t)bb * E + lane] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        total += cv[u];
        if (bb0 + NW * u < b) before += cv[u];
      }
    }
    sPartTotal[wave][lane] = total;
    sPartBefore[wave][lane] = before;
    int tb = 0;
    for (int bb = threadIdx.x; bb < b; bb += kScatterThreads) tb += blk_tok[bb];
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) tb += __shfl_xor(tb, s, 64);
    if (lane == 0) sPartTok[wave] = tb;
  }

  // token waves: one token per lane
  const int t = b * kDB + threadIdx.x;
  int cnt = 0, incl = 0;
  if (wave < 4) {
    const unsigned long long m = t < T ? mask[t] & expert_bits(E) : 0ull;
    int mine = 0;
    for (int e = 0; e < E; ++e) {
      const unsigned long long bits = __ballot((m >> e) & 1ull);
      if (lane == e) {
        mine = __popcll(bits);
        sBits[wave][e] = bits;
      }
    }
    sWave[wave][lane] = mine;
    sMask[threadIdx.x] = m;
    cnt = __popcll(m);
    incl = cnt;                            // inclusive scan of the per-token counts inside the wave
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(incl, s, 64);
      if (lane >= s) incl += o;
    }
    if (lane == 63) sWaveTok[wave] = incl;
  }
  __syncthreads();

  if (threadIdx.x < 64) {
    int total = 0, before = 0, tb = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      total += sPartTotal[w][lane];
      before += sPartBefore[w][lane];
      tb += sPartTok[w];
    }
    int inc = total;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(inc, s, 64);
      if (lane >= s) inc += o;
    }
    const int nnz = __shfl(inc, 63, 64);
    const bool overflow = (long long)nnz > max_rows;
    const int off = overflow ? 0 : inc - total;
    if (lane < E) sRowBase[lane] = off + before;
    if (b == 0) {
      if (lane < E) expert_off[lane] = off;
      if (lane == 0) {
        expert_off[E] = overflow ? 0 : nnz;
        nnz_out[0] = overflow ? 0 : nnz;
        if (overflow) err_flag[0] = DSMOE_ERR_CAPACITY;
      }
    }
    if (lane == 0) {
      sNnz = overflow ? -1 : nnz;
      sTokBase = tb;
    }
  }
  __syncthreads();

  const bool overflow = sNnz < 0;
  if (wave < 4) {
    int tbase = overflow ? 0 : sTokBase + incl - cnt;
    for (int w = 0; w < wave; ++w) tbase += overflow ? 0 : sWaveTok[w];
    sTokOff[threadIdx.x] = tbase;
    if (t < T) tok_off[t] = tbase;
    if (t == T - 1) tok_off[T] = overflow ? 0 : sNnz;
  }
  if (overflow) return;
  __syncthreads();

  // Thread (token tl, quarter q) owns experts q, q + 4, ...  A pair's row is the block's base inside the
  // expert plus the number of earlier tokens of the block that selected the expert (from the ballots).
  const int tl = threadIdx.x >> 2, q = threadIdx.x & 3, tg = b * kDB + tl;
  const unsigned long long mt = sMask[tl];    // 0 beyond T
  float pv[kMaxExperts / 4];
#pragma unroll
  for (int j = 0; j < kMaxExperts / 4; ++j) {
    const int e = q + 4 * j;
    pv[j] = (e < E && ((mt >> e) & 1ull)) ? probs[(size_t)tg * E + e] : 0.f;
  }
  const int tw = tl >> 6;
  const unsigned long long below = (1ull << (tl & 63)) - 1ull;
  const int tbase = sTokOff[tl];
#pragma unroll
  for (int j = 0; j < kMaxExperts / 4; ++j) {
    const int e = q + 4 * j;
    if (e < E && ((mt >> e) & 1ull)) {
      int row = sRowBase[e] + __popcll(sBits[tw][e] & below);
      for (int w = 0; w < tw; ++w) row += sWave[w][e];
      row_token[row] = tg;
      row_weight[row] = pv[j];
      tok_rows[tbase + __popcll(mt & ((1ull << e) - 1ull))] = row;
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

// blk_cnt [n_blocks][E], blk_tok [n_blocks] and the deferred status word: scratch of the two passes
static hipError_t launch_dispatch_with(const dsmoe_ctx* c, int32_t* blk_cnt, int32_t* blk_tok, int32_t* err_flag,
                                       const void* x, const float* probs, const uint64_t* mask, int T,
                                       int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                                       int32_t* tok_rows, int32_t* nnz, void* x_perm, hipStream_t s) {
  const int E = c->desc.n_experts;
  if (T == 0) {
    hipLaunchKernelGGL(empty_routing_kernel, dim3(1), dim3(128), 0, s, E, expert_off, tok_off, nnz);
    return hipGetLastError();
  }
  const int nblk = (T + kDB - 1) / kDB;
  hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblk), dim3(kDB), 0, s, (const unsigned long long*)mask, T, E,
                     blk_cnt, blk_tok);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(nblk), dim3(kScatterThreads), 0, s, (const unsigned long long*)mask, probs, T,
                     E, blk_cnt, blk_tok, (long long)c->desc.max_rows, expert_off, row_token, row_weight, tok_off,
                     tok_rows, nnz, err_flag);
  err = hipGetLastError();
  if (err != hipSuccess || x_perm == nullptr) return err;
  const long grid = std::min<long>(c->desc.max_rows, (long)c->n_cu * 8);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)std::max<long>(grid, 1)), dim3(kThreads), 0, s,
                     (const char*)x, row_token, nnz, (char*)x_perm, (int)(c->desc.d_model * c->esize));
  return hipGetLastError();
}

hipError_t launch_dispatch(const dsmoe_ctx* c, const void* x, const float* probs, const uint64_t* mask, int T,
                           int32_t* expert_off, int32_t* row_token, float* row_weight, int32_t* tok_off,
                           int32_t* tok_rows, int32_t* nnz, void* x_perm, hipStream_t s) {
  return launch_dispatch_with(c, reinterpret_cast<int32_t*>(c->workspace + c->ws.blk_cnt),
                              reinterpret_cast<int32_t*>(c->workspace + c->ws.blk_tok),
                              reinterpret_cast<int32_t*>(c->workspace + c->ws.err_flag), x, probs, mask, T, expert_off,
                              row_token, row_weight, tok_off, tok_rows, nnz, x_perm, s);
}

// ---- dispatch for callers that cannot allocate ------------------------------------------------------
// The scratch of the two passes (per-block histograms, the deferred status word) lives in a device array of
// the library instead of a caller-lent workspace.  Every GPU holds its own copy of the array at its own
// address; host code never uses the array's name as an address, only what hipGetSymbolAddress returned for
// the device that was current.
constexpr int kStaticBlocks = kStaticDispatchMaxTokens / kDB;
constexpr size_t kStaticFlagOff = 0;                                        // int32 [4]
constexpr size_t kStaticCntOff = 256;                                       // int32 [kStaticBlocks][kMaxExperts]
constexpr size_t kStaticTokOff = kStaticCntOff + (size_t)kStaticBlocks * kMaxExperts * 4;   // int32 [kStaticBlocks]
constexpr size_t kStaticBytes = (kStaticTokOff + (size_t)kStaticBlocks * 4 + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static char* g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, once asked for

// Address of the current device's copy of the array (asked for once per device, with that device current).
static hipError_t static_scratch(char** out, bool create) {
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev)) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev] && create) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
    g_scratch_ptr[dev] = static_cast<char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

hipError_t static_dispatch_flag(int32_t** flag) {
  char* p = nullptr;
  if (hipError_t e = static_scratch(&p, false)) return e;
  *flag = p ? reinterpret_cast<int32_t*>(p + kStaticFlagOff) : nullptr;
  return hipSuccess;
}

}  // namespace dsmoe

extern "C" int32_t dsmoe_dispatch_static(dsmoe_ctx* c, const void* x, const float* probs, const uint64_t* mask,
                                         int32_t T, int32_t* expert_off, int32_t* row_token, float* row_weight,
                                         int32_t* tok_off, int32_t* tok_rows, int32_t* nnz, void* x_perm,
                                         void* stream) {
  using namespace dsmoe;
  if (!c) return DSMOE_ERR_INVALID_ARG;
  auto fail = [&](int32_t code, const char* msg) {
    snprintf(c->err, sizeof(c->err), "dsmoe_dispatch_static: %s", msg);
    return code;
  };
  if (T < 0 || T > c->desc.max_tokens) return fail(DSMOE_ERR_INVALID_ARG, "T outside [0, max_tokens]");
  if (T > kStaticDispatchMaxTokens)
    return fail(DSMOE_ERR_UNSUPPORTED, "T exceeds DSMOE_STATIC_DISPATCH_MAX_TOKENS (the library's own scratch array "
                                       "holds histograms for that many tokens); use dsmoe_dispatch with a workspace");
  auto bad = [](const void* p, bool required) {
    return (required && p == nullptr) || (reinterpret_cast<uintptr_t>(p) & 15u) != 0;
  };
  if (bad(expert_off, true) || bad(tok_off, true) || bad(nnz, true))
    return fail(DSMOE_ERR_INVALID_ARG, "expert_off, tok_off and nnz must be non-null and 16-byte aligned");
  if (T > 0 && (bad(probs, true) || bad(mask, true) || bad(row_token, true) || bad(row_weight, true) ||
                bad(tok_rows, true) || bad(x_perm, false) || (x_perm && bad(x, true))))
    return fail(DSMOE_ERR_INVALID_ARG, "null or misaligned pointer");
  char* base = nullptr;
  if (hipError_t e = static_scratch(&base, true)) {
    snprintf(c->err, sizeof(c->err), "dsmoe_dispatch_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    return DSMOE_ERR_HIP;
  }
  hipError_t e = launch_dispatch_with(c, reinterpret_cast<int32_t*>(base + kStaticCntOff),
                                      reinterpret_cast<int32_t*>(base + kStaticTokOff),
                                      reinterpret_cast<int32_t*>(base + kStaticFlagOff), x, probs, mask, T, expert_off,
                                      row_token, row_weight, tok_off, tok_rows, nnz, x_perm,
                                      static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    snprintf(c->err, sizeof(c->err), "dsmoe_dispatch_static: launch: %s", hipGetErrorString(e));
    return DSMOE_ERR_HIP;
  }
  return DSMOE_OK;
}

namespace dsmoe {

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
