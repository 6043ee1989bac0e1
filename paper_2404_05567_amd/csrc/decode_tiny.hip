// Sparse-inference forward for a handful of tokens (at most 4: single-sequence decoding and the smallest decode
// batches).  The layer is then nothing but reading the selected experts' weights once (paper Sec. 4.4: decoding
// is I/O-bound), and there is too little arithmetic per weight byte for the matrix cores to matter, so these
// kernels keep every CU streaming whole, contiguous weight rows through the vector ALUs:
//
//   kernel 1  router (every block computes the scores and the selection of all tokens itself: no launch and no
//             wait between the router and the experts), then gate / up: the rows [k] of the active experts'
//             W_gate, W_up ([d][f], a row is f contiguous values) are dealt out in equal contiguous runs, one
//             run per block; a block leaves fp32 partial sums  sum_{k in run} x[t][k] W[k][:]  per segment
//             (a run touches at most two experts);
//   kernel 2  adds the partial sums of the hidden columns it needs, applies the activation and the combine
//             weight (h = S_e silu(G) U, Eq. 1), and streams the rows [c] of the active experts' W_down ([f][d])
//             the same way: one fp32 partial output  sum_{(e,c) in run} h[t][e][c] W_down[e][c][:]  per block;
//   kernel 3  adds the blocks' partial outputs.
//
// All sums run in a fixed order (no floating-point atomics): results are bitwise reproducible.  Nothing waits
// for another block inside a kernel.
#include "gemm_core.h"
#include "router_common.h"

namespace dsmoe {

namespace {

constexpr int kTinyMaxTokens = 4;   // beyond, the vector ALUs (no packed fp32 here) cannot keep up with the weight stream
constexpr int kTinyBlocks = 256;       // most blocks (runs of weight rows) per kernel
constexpr int kTinyRows = 1024;        // most weight rows of a run

struct TinyArgs {
  const bf16_t *x, *w_r, *b_r, *w_gate, *w_up, *w_down;
  float* probs; unsigned long long* mask; int32_t* cnt_tok;   // the call's routing, kept for dsmoe_sparse_fwd_routing
  float *p1, *p2;
  bf16_t* out;
  int32_t* err_flag;
  int T, d, f, E, mode, k;
  float eps;
  long long max_rows;
};

__host__ __device__ inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Rows are dealt out in units of `rp` rows (what one pass of a block covers); every active expert has upe units.
// Block b takes the units [b upb, (b + 1) upb) of the U upe units of all active experts, upb <= upe: at most
// two experts.  Segment s (0, 1) of the block: rank u of the expert and the unit range [lo, hi) inside it
// (empty when lo >= hi).
__device__ __forceinline__ void tiny_segment(int U, int upe, int upb, int b, int s, int& u, int& lo, int& hi) {
  const int total = U * upe, first = min(b * upb, total), last = min(first + upb, total);
  u = first / upe + s;
  const int e_lo = u * upe;
  lo = max(first, e_lo) - e_lo;
  hi = min(last, e_lo + upe) - e_lo;
}

// Active experts (ascending) and their number from the selection masks; nothing is active after a capacity
// overflow (more selected pairs than max_rows: the call then returns zeros and reports DSMOE_ERR_CAPACITY).
// Called by the first wave; `overflow` is valid in lane 0.
__device__ __forceinline__ void tiny_plan(const unsigned long long* m, int T, int E, long long max_rows, int* act, int* U,
                                          bool& overflow) {
  const int lane = threadIdx.x;
  unsigned long long any = 0ull;
  int nnz = 0;
  for (int t = 0; t < T; ++t) {
    any |= m[t];
    nnz += __popcll(m[t]);
  }
  overflow = nnz > max_rows;
  if (overflow) any = 0ull;
  if (lane < E && ((any >> lane) & 1ull)) act[__popcll(any & ((1ull << lane) - 1ull))] = lane;
  if (lane == 0) *U = __popcll(any);
}

// ---- kernel 1: router, then partial gate / up sums ------------------------------------------------------
template <bool GELU, int EP, int TT>
__global__ void __launch_bounds__(kThreads2) tiny_gateup_kernel(const TinyArgs a) {
  __shared__ __align__(16) char sRoute[route_bf16_lds<EP, 8>()];
  __shared__ float sProbs[kTinyMaxTokens * kMaxExperts];
  __shared__ unsigned long long sMask[kTinyMaxTokens];
  __shared__ int sCnt[kTinyMaxTokens];
  __shared__ int sAct[kMaxExperts];
  __shared__ int sU;
  __shared__ float sX[TT][kTinyRows];
  __shared__ __align__(16) float sRed[kThreads2 * 16];
  const int tid = threadIdx.x, T = a.T, d = a.d, f = a.f, E = a.E;

  route_bf16_tile<EP, 8>(a.x, a.w_r, a.b_r, T, d, E, sProbs, a.mode, a.k, a.eps, sMask, sCnt, 0, sRoute);
  __syncthreads();
  if (tid < 64) {
    bool overflow;
    tiny_plan(sMask, T, E, a.max_rows, sAct, &sU, overflow);
    if (blockIdx.x == 0 && tid == 0 && overflow) a.err_flag[0] = DSMOE_ERR_CAPACITY;
  }
  if (blockIdx.x == 0) {
    for (int i = tid; i < T * E; i += kThreads2) a.probs[i] = sProbs[i];
    if (tid < T) {
      a.mask[tid] = sMask[tid];
      a.cnt_tok[tid] = sCnt[tid];
    }
  }
  __syncthreads();

  constexpr int NM = GELU ? 1 : 2;                 // weight matrices of the first product
  const int W = NM * f;                            // values of a partial-sum row
  const int cols8 = f / 8, rp = kThreads2 / cols8; // 16-byte chunks of a weight row; rows per pass
  const bool active = tid < rp * cols8;
  const int r = tid / cols8, q = tid % cols8;
  const int U = sU, upe = cdiv(d, rp), upb = cdiv(U * upe, (int)gridDim.x);
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  for (int s = 0; s < 2; ++s) {
    int u, lo, hi;
    tiny_segment(U, upe, upb, blockIdx.x, s, u, lo, hi);
    if (lo >= hi) continue;
    const int e = sAct[u];
    const int k0 = lo * rp, k1 = min(d, hi * rp), nk = k1 - k0, n_pass = hi - lo;
    const size_t wo = ((size_t)e * d + k0 + r) * f + (size_t)q * 8;
    const bf16_t* wg = a.w_gate + wo;
    const bf16_t* wu = GELU ? nullptr : a.w_up + wo;
    // four passes (8 or 4 loads of 16 bytes per thread) are requested before the four before them are used
    auto request = [&](int i0, u32x4 (&raw)[NM][4]) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = active && i0 + j < n_pass && k0 + r + rp * (i0 + j) < k1;
        const size_t ro = (size_t)rp * (i0 + j) * f;
        raw[0][j] = ok ? ldg16(wg + ro) : zero4;
        if constexpr (!GELU) raw[1][j] = ok ? ldg16(wu + ro) : zero4;
      }
    };
    u32x4 cur[NM][4], nxt[NM][4];
    request(0, cur);                               // the first weights travel while the token rows are staged
    __syncthreads();                               // the previous segment no longer reads sX
    for (int i = tid; i < TT * nk; i += kThreads2) {
      const int t = i / nk, kk = i % nk;
      sX[t][kk] = t < T ? to_f32(a.x[(size_t)t * d + k0 + kk]) : 0.f;
    }
    __syncthreads();
    float acc[NM][TT][8];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[m][t][c] = 0.f;
    if (active) {
      for (int i0 = 0; i0 < n_pass; i0 += 4) {
        if (i0 + 4 < n_pass) request(i0 + 4, nxt);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int kk = min(r + rp * (i0 + j), nk - 1);      // rows past the end carry zero weights
          float xv[TT];
#pragma unroll
          for (int t = 0; t < TT; ++t) xv[t] = sX[t][kk];
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            float w8[8];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              w8[2 * c] = __uint_as_float(cur[m][j][c] << 16);
              w8[2 * c + 1] = __uint_as_float(cur[m][j][c] & 0xffff0000u);
            }
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
              for (int c = 0; c < 8; ++c) acc[m][t][c] = fmaf(xv[t], w8[c], acc[m][t][c]);
          }
        }
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
          for (int j = 0; j < 4; ++j) cur[m][j] = nxt[m][j];
      }
    }
    // the rp row groups of the block add up, token by token, in order
    float* dst = a.p1 + (size_t)(2 * blockIdx.x + s) * T * W;
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      if (t >= T) break;
      __syncthreads();
      if (active) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          float* p = sRed + (size_t)r * W + m * f + q * 8;
          *reinterpret_cast<f32x4*>(p) = f32x4{acc[m][t][0], acc[m][t][1], acc[m][t][2], acc[m][t][3]};
          *reinterpret_cast<f32x4*>(p + 4) = f32x4{acc[m][t][4], acc[m][t][5], acc[m][t][6], acc[m][t][7]};
        }
      }
      __syncthreads();
      for (int o = tid * 4; o < W; o += kThreads2 * 4) {
        f32x4 sum = *reinterpret_cast<const f32x4*>(sRed + o);
        for (int rr = 1; rr < rp; ++rr) sum += *reinterpret_cast<const f32x4*>(sRed + (size_t)rr * W + o);
        store4(dst + (size_t)t * W + o, sum.x, sum.y, sum.z, sum.w);
      }
    }
  }
}

// ---- kernel 2: hidden activations from the partial sums, then partial outputs ------------------------------
// CH: 16-byte chunks of a W_down row per thread (rows of more than 4096 values)
template <bool GELU, int TT, int CH>
__global__ void __launch_bounds__(kThreads2) tiny_down_kernel(const TinyArgs a, int nb1) {
  __shared__ int sAct[kMaxExperts];
  __shared__ int sU;
  __shared__ float sWt[TT][kMaxExperts];
  __shared__ float sH[TT][kTinyRows];
  __shared__ __align__(16) float sRed[kThreads2 * 8 * CH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, T = a.T, d = a.d, f = a.f, E = a.E;
  if (tid < 64) {
    bool overflow;
    tiny_plan(a.mask, T, E, a.max_rows, sAct, &sU, overflow);
  }
  for (int i = tid; i < TT * kMaxExperts; i += kThreads2) {
    const int t = i / kMaxExperts, e = i % kMaxExperts;
    sWt[t][e] = (t < T && e < E && ((a.mask[t] >> e) & 1ull)) ? a.probs[(size_t)t * E + e] : 0.f;
  }
  __syncthreads();

  constexpr int NM = GELU ? 1 : 2;
  const int W = NM * f, U = sU;
  // how kernel 1 dealt out the rows of W_gate / W_up
  const int rp1 = kThreads2 / (f / 8), upe1 = cdiv(d, rp1), upb1 = cdiv(U * upe1, nb1);
  // this kernel's rows of W_down
  const int tpr = d / 8 / CH, rp = kThreads2 / tpr;     // threads per row, rows per pass
  const bool active = tid < rp * tpr;
  const int r = tid / tpr, q = tid % tpr;
  const int upe = cdiv(f, rp), upb = cdiv(U * upe, (int)gridDim.x);
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  float acc[TT][8 * CH];
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int c = 0; c < 8 * CH; ++c) acc[t][c] = 0.f;

  for (int s = 0; s < 2; ++s) {
    int u, lo, hi;
    tiny_segment(U, upe, upb, blockIdx.x, s, u, lo, hi);
    if (lo >= hi) continue;
    const int e = sAct[u];
    const int c0 = lo * rp, c1 = min(f, hi * rp), nc = c1 - c0, n_pass = hi - lo;
    const bf16_t* wd = a.w_down + ((size_t)e * f + c0 + r) * d + (size_t)q * 8;
    auto request = [&](int i0, u32x4 (&raw)[4][CH]) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = active && i0 + j < n_pass && c0 + r + rp * (i0 + j) < c1;
#pragma unroll
        for (int cc = 0; cc < CH; ++cc)
          raw[j][cc] = ok ? ldg16(wd + (size_t)rp * (i0 + j) * d + (size_t)cc * tpr * 8) : zero4;
      }
    };
    u32x4 cur[4][CH], nxt[4][CH];
    request(0, cur);                               // the first weights travel while the hidden activations are formed
    // h[t][c] = S_e act(sum of the partial sums), one wave per (token, hidden column), four of them in flight;
    // a lane adds the partial sums of the blocks b0 + lane, b0 + lane + 64, ...
    const int b0 = (u * upe1) / upb1, b1 = ((u + 1) * upe1 - 1) / upb1;
    __syncthreads();                               // the previous segment no longer reads sH
    for (int p0 = wave; p0 < nc * TT; p0 += 8 * 4) {
      float g[4], up[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        g[j] = up[j] = 0.f;
        const int p = p0 + 8 * j, t = p / nc, c = c0 + p % nc;
        if (p < nc * TT && t < T)
          for (int bb = b0 + lane; bb <= b1; bb += 64) {
            const int seg = 2 * bb + ((bb * upb1) / upe1 == u ? 0 : 1);
            const float* pp = a.p1 + ((size_t)seg * T + t) * W + c;
            g[j] += pp[0];
            if constexpr (!GELU) up[j] += pp[f];
          }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = p0 + 8 * j, t = p / nc;
        if (p >= nc * TT) break;
        const float gs = wave_sum(g[j]);
        float h;
        if constexpr (GELU) {
          h = gelu_f(gs);
        } else {
          h = silu_f(gs) * wave_sum(up[j]);
        }
        if (lane == 0) sH[t][p % nc] = t < T ? sWt[t][e] * h : 0.f;
      }
    }
    __syncthreads();
    if (active) {
      for (int i0 = 0; i0 < n_pass; i0 += 4) {
        if (i0 + 4 < n_pass) request(i0 + 4, nxt);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ci = min(r + rp * (i0 + j), nc - 1);
          float hv[TT];
#pragma unroll
          for (int t = 0; t < TT; ++t) hv[t] = sH[t][ci];
#pragma unroll
          for (int cc = 0; cc < CH; ++cc) {
            float w8[8];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              w8[2 * c] = __uint_as_float(cur[j][cc][c] << 16);
              w8[2 * c + 1] = __uint_as_float(cur[j][cc][c] & 0xffff0000u);
            }
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
              for (int c = 0; c < 8; ++c) acc[t][8 * cc + c] = fmaf(hv[t], w8[c], acc[t][8 * cc + c]);
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int cc = 0; cc < CH; ++cc) cur[j][cc] = nxt[j][cc];
      }
    }
  }
  // the block's partial output: the rp row groups add up in order; every block stores one (zeros without rows)
  float* dst = a.p2 + (size_t)blockIdx.x * T * d;
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    if (t >= T) break;
    __syncthreads();
    if (active) {
#pragma unroll
      for (int cc = 0; cc < CH; ++cc) {
        float* p = sRed + (size_t)r * d + ((size_t)cc * tpr + q) * 8;
        *reinterpret_cast<f32x4*>(p) = f32x4{acc[t][8 * cc], acc[t][8 * cc + 1], acc[t][8 * cc + 2], acc[t][8 * cc + 3]};
        *reinterpret_cast<f32x4*>(p + 4) = f32x4{acc[t][8 * cc + 4], acc[t][8 * cc + 5], acc[t][8 * cc + 6], acc[t][8 * cc + 7]};
      }
    }
    __syncthreads();
    for (int o = tid * 4; o < d; o += kThreads2 * 4) {
      f32x4 sum = *reinterpret_cast<const f32x4*>(sRed + o);
      for (int rr = 1; rr < rp; ++rr) sum += *reinterpret_cast<const f32x4*>(sRed + (size_t)rr * d + o);
      store4(dst + (size_t)t * d + o, sum.x, sum.y, sum.z, sum.w);
    }
  }
}

// ---- kernel 3: out[t][:] = sum of the blocks' partial outputs ----------------------------------------------
// Block: 32 columns of one token.  Wave w adds the partial outputs 64 w .. 64 w + 63: eight lanes cover the 128
// bytes of one partial, a lane adds every eighth one in order, then the eight lane groups and the four waves
// add up along a fixed tree.
__global__ void __launch_bounds__(256) tiny_reduce_kernel(const float* __restrict__ p2, int nb, int T, int d,
                                                         bf16_t* __restrict__ out) {
  __shared__ f32x4 sPart[4][8];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, pg = lane >> 3, c4 = lane & 7;
  const int t = blockIdx.y, n = blockIdx.x * 32 + 4 * c4;
  f32x4 v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int p = 64 * wave + 8 * i + pg;
    v[i] = (p < nb && n < d) ? __builtin_bit_cast(f32x4, ldg16(p2 + ((size_t)p * T + t) * d + n)) : f32x4{0.f, 0.f, 0.f, 0.f};
  }
  f32x4 sum = v[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) sum += v[i];
#pragma unroll
  for (int o = 8; o < 64; o <<= 1) {
    sum.x += __shfl_xor(sum.x, o, 64);
    sum.y += __shfl_xor(sum.y, o, 64);
    sum.z += __shfl_xor(sum.z, o, 64);
    sum.w += __shfl_xor(sum.w, o, 64);
  }
  if (lane < 8) sPart[wave][lane] = sum;
  __syncthreads();
  if (threadIdx.x < 8 && n < d) {
    const f32x4 r = sPart[0][threadIdx.x] + sPart[1][threadIdx.x] + sPart[2][threadIdx.x] + sPart[3][threadIdx.x];
    store4(out + (size_t)t * d + n, r.x, r.y, r.z, r.w);
  }
}

int tiny_blocks(const dsmoe_ctx* c) { return std::min(c->n_cu / 8 * 8, kTinyBlocks); }

template <bool GELU, int EP>
hipError_t launch_gateup(const TinyArgs& a, int grid, hipStream_t s) {
  if (a.T == 1) tiny_gateup_kernel<GELU, EP, 1><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
  else if (a.T == 2) tiny_gateup_kernel<GELU, EP, 2><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
  else tiny_gateup_kernel<GELU, EP, 4><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
  return hipGetLastError();
}
template <bool GELU, int CH>
hipError_t launch_down(const TinyArgs& a, int grid, hipStream_t s) {
  if (a.T == 1) tiny_down_kernel<GELU, 1, CH><<<dim3(grid), dim3(kThreads2), 0, s>>>(a, grid);
  else if (a.T == 2) tiny_down_kernel<GELU, 2, CH><<<dim3(grid), dim3(kThreads2), 0, s>>>(a, grid);
  else tiny_down_kernel<GELU, 4, CH><<<dim3(grid), dim3(kThreads2), 0, s>>>(a, grid);
  return hipGetLastError();
}

}  // namespace

size_t decode_tiny_p1_bytes(const dsmoe_desc& d) {
  if (d.dtype != DSMOE_BF16) return 0;
  return (size_t)2 * kTinyBlocks * std::min<int64_t>(d.max_tokens, kTinyMaxTokens) * 2 * d.d_ff * 4;
}
size_t decode_tiny_p2_bytes(const dsmoe_desc& d) {
  if (d.dtype != DSMOE_BF16) return 0;
  return (size_t)kTinyBlocks * std::min<int64_t>(d.max_tokens, kTinyMaxTokens) * d.d_model * 4;
}

bool decode_tiny_applies(const dsmoe_ctx* c, int T, int mode) {
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  if (c->desc.dtype != DSMOE_BF16 || T < 1 || T > kTinyMaxTokens) return false;
  if (mode != DSMOE_SEL_TOPK && mode != DSMOE_SEL_THRESHOLD) return false;
  const int nb = tiny_blocks(c);
  if (nb < kMaxExperts) return false;                       // a run of rows touches at most two experts
  if (d % 64 != 0 || f % 8 != 0 || f / 8 > kThreads2) return false;
  const int ch = d / 8 > kThreads2 ? 2 : 1;
  if (d / 8 > 2 * kThreads2 || (d / 8) % ch != 0) return false;
  // rows of a run when every expert is active
  const int rp1 = kThreads2 / (f / 8), rows1 = cdiv(E * cdiv(d, rp1), nb) * rp1;
  const int rp2 = kThreads2 / (d / 8 / ch), rows2 = cdiv(E * cdiv(f, rp2), nb) * rp2;
  return rows1 <= kTinyRows && rows2 <= kTinyRows;
}

hipError_t launch_decode_tiny(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                              const void* w_up, const void* w_down, int T, int mode, int k, float eps, void* out,
                              hipStream_t s) {
  char* w = c->workspace;
  TinyArgs a;
  a.x = (const bf16_t*)x; a.w_r = (const bf16_t*)w_r; a.b_r = (const bf16_t*)b_r;
  a.w_gate = (const bf16_t*)w_gate; a.w_up = (const bf16_t*)w_up; a.w_down = (const bf16_t*)w_down;
  a.probs = reinterpret_cast<float*>(w + c->ws.probs);
  a.mask = reinterpret_cast<unsigned long long*>(w + c->ws.mask);
  a.cnt_tok = reinterpret_cast<int32_t*>(w + c->ws.cnt_tok);
  a.p1 = reinterpret_cast<float*>(w + c->ws.tiny_p1);
  a.p2 = reinterpret_cast<float*>(w + c->ws.tiny_p2);
  a.out = (bf16_t*)out;
  a.err_flag = reinterpret_cast<int32_t*>(w + c->ws.err_flag);
  a.T = T; a.d = c->desc.d_model; a.f = c->desc.d_ff; a.E = c->desc.n_experts;
  a.mode = mode; a.k = k; a.eps = eps;
  a.max_rows = c->desc.max_rows;
  const int grid = tiny_blocks(c);
  const bool gelu = c->expert_kind == DSMOE_EXPERT_GELU;
  hipError_t e;
  if (a.E <= 32) e = gelu ? launch_gateup<true, 32>(a, grid, s) : launch_gateup<false, 32>(a, grid, s);
  else e = gelu ? launch_gateup<true, 64>(a, grid, s) : launch_gateup<false, 64>(a, grid, s);
  if (e != hipSuccess) return e;
  if (a.d / 8 > kThreads2) e = gelu ? launch_down<true, 2>(a, grid, s) : launch_down<false, 2>(a, grid, s);
  else e = gelu ? launch_down<true, 1>(a, grid, s) : launch_down<false, 1>(a, grid, s);
  if (e != hipSuccess) return e;
  tiny_reduce_kernel<<<dim3((a.d + 31) / 32, T), dim3(256), 0, s>>>(a.p2, grid, T, a.d, a.out);
  return hipGetLastError();
}

}  // namespace dsmoe
