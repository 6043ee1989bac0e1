// Sparse-inference forward for decode-sized batches (at most 128 tokens): the expert FFN of Eq. 1 is then
// bound by reading the selected experts' weights once from HBM, not by arithmetic (paper Sec. 4.4 calls
// the decoding phase I/O-bound), so the kernels here are laid out to keep every CU streaming weights:
//
//   * no dispatch kernels: every block derives the routing (tokens per expert, row offsets) from the
//     selection bitmasks of the <= 128 tokens itself; the last block also publishes the usual routing objects;
//   * a work item is (active expert, column slice, K chunk).  The K split is chosen on the device from the
//     number of active experts: none when the unsplit items already cover half the CUs, else enough chunks
//     for one item per CU even when a single token activates four experts;
//   * K chunks leave fp32 partial sums that are added in a fixed order (no floating-point atomics: results
//     are bitwise reproducible).  For gate/up the block that stores the last chunk of an (expert, slice)
//     adds them and applies the activation; an unsplit item writes H = silu(G) * U straight from its
//     accumulators.  Down-projection chunks are added by the weighted combine.
#include <algorithm>

#include "gemm.h"

namespace dsmoe {

namespace {

constexpr int kDecT = kDecodeMaxTokens;
// Hidden-width columns per gate/up item: 64 (128-byte pieces of a weight row) gives one item per CU without a
// K split when all 32 experts of a 512-wide layer are active.
constexpr int kDecSlice = 64;

struct DecodePlan {
  unsigned long long tokbits[kMaxExperts][2];   // tokens 0..63 / 64..127 that selected the expert
  unsigned long long tokmask[kDecT];            // selection mask of each token
  int cnt[kMaxExperts];        // tokens per expert
  int cnt_w0[kMaxExperts];     // ... of which among tokens 0..63
  int off[kMaxExperts + 1];    // exclusive prefix sum of cnt (all zero after a capacity overflow)
  int act[kMaxExperts];        // active experts, ascending
  int U, nnz, ks1, ks2;        // active experts, rows, K split of the gate/up and of the down products
};

// K split: the smallest power of two that gives at least `blocks` items, limited by the partial-sum
// buffer (ks * nnz <= row_cap rows) and by the K steps available (ks divides ksteps, two steps per chunk).
// Adding up the chunks costs device-wide fences, so a layer that occupies half the CUs unsplit stays unsplit.
__device__ __forceinline__ int choose_ksplit(int U, int slices, int blocks, int nnz, int row_cap, int ksteps) {
  if (2 * U * slices > blocks) return 1;
  int ks = 1;
  while (U * slices * ks < blocks && 2 * ks * nnz <= row_cap && (ksteps & (2 * ks - 1)) == 0 && ksteps >= 4 * ks)
    ks *= 2;
  return ks;
}

// Called by every thread of the block; returns the selection mask of token threadIdx.x (0 beyond T and for
// threads >= 128).  Each wave reads all masks and counts the experts e = wave, wave + 8, ...
__device__ __forceinline__ unsigned long long build_plan(DecodePlan& p, const unsigned long long* __restrict__ mask,
                                                         int T, int E, int blocks, long long max_rows, int row_cap,
                                                         int ns1, int ns2, int d, int f) {
  __shared__ int sCnt[kMaxExperts];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long m0 = lane < T ? mask[lane] : 0ull, m1 = lane + 64 < T ? mask[lane + 64] : 0ull;
  if (wave < 2) p.tokmask[threadIdx.x] = wave == 0 ? m0 : m1;
  for (int e = wave; e < E; e += kThreads2 / 64) {
    const unsigned long long b0 = __ballot((m0 >> e) & 1ull), b1 = __ballot((m1 >> e) & 1ull);
    if (lane == 0) {
      p.tokbits[e][0] = b0;
      p.tokbits[e][1] = b1;
      p.cnt_w0[e] = __popcll(b0);
      sCnt[e] = __popcll(b0) + __popcll(b1);
    }
  }
  __syncthreads();
  if (wave == 0) {
    const int c = lane < E ? sCnt[lane] : 0;
    int incl = c;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(incl, s, 64);
      if (lane >= s) incl += o;
    }
    const int nnz = __shfl(incl, 63, 64);
    const bool overflow = (long long)nnz > max_rows;
    const unsigned long long actm = overflow ? 0ull : __ballot(c > 0);
    p.cnt[lane] = overflow ? 0 : c;
    p.off[lane] = overflow ? 0 : incl - c;
    if (c > 0 && !overflow) p.act[__popcll(actm & ((1ull << lane) - 1ull))] = lane;
    if (lane == 0) {
      const int U = __popcll(actm), n = overflow ? 0 : nnz;
      p.off[64] = n;
      p.U = U;
      p.nnz = overflow ? -1 : nnz;
      p.ks1 = choose_ksplit(U, ns1, blocks, n, row_cap, d / kBK2);
      p.ks2 = choose_ksplit(U, ns2, blocks, n, row_cap, f / kBK2);
    }
  }
  __syncthreads();
  return wave == 0 ? m0 : wave == 1 ? m1 : 0ull;
}

// Counts the blocks that have finished their share of a result; true in the block that arrives last, which
// then sees every earlier block's global stores.  The counter is left at zero for the next call.
// Called by every thread of the block.
__device__ __forceinline__ bool arrive_last(int32_t* counter, int expected) {
  __shared__ int s_last;
  __syncthreads();                         // every wave's partial sums are on their way to the L2 ...
  if (threadIdx.x < 64) {                  // ... and one wave publishes them: the device-wide fences are costly
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    int last = 0;
    if (threadIdx.x == 0) {
      last = atomicAdd(counter, 1) == expected - 1;
      if (last) atomicExch(counter, 0);
      s_last = last;
    }
    if (__shfl(last, 0, 64)) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  __syncthreads();
  return s_last != 0;
}

// ---- gate / up: partial G, U over one K chunk ----------------------------------------------------------
// GELU: the two-matrix expert, H = gelu(x W_1) with W_1 passed as w_gate; items are 128-column slices of one product.
template <bool GELU>
__global__ void __launch_bounds__(kThreads2)
decode_gateup_kernel(const bf16_t* __restrict__ x, const unsigned long long* __restrict__ mask,
                     const float* __restrict__ probs, const bf16_t* __restrict__ w_gate,
                     const bf16_t* __restrict__ w_up, float* __restrict__ P1, bf16_t* __restrict__ H,
                     int32_t* __restrict__ arrivals, int T, int d, int f, int E,
                     long long max_rows, int row_cap, int32_t* __restrict__ info, int32_t* __restrict__ expert_off,
                     int32_t* __restrict__ row_token, float* __restrict__ row_weight, int32_t* __restrict__ tok_off,
                     int32_t* __restrict__ tok_rows, int32_t* __restrict__ nnz_out, int32_t* __restrict__ err_flag) {
  constexpr int BNS = GELU ? 2 * kDecSlice : kDecSlice;   // hidden-width columns per item
  // six stages: more weight bytes in flight; 128 token rows x 128 weight columns (64 gate + 64 up, or 128 of W_1)
  typedef std::conditional_t<GELU, Tile3<kDecT, 2 * kDecSlice, 1, false, true, false, 6, 2>,
                             Tile3<kDecT, 2 * kDecSlice, 2, false, true, false, 6, 2>> TL;
  DSMOE_TILE3_STAGES(TL, st);
  __shared__ DecodePlan plan;
  __shared__ int toks[kDecT];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ns1 = (f + BNS - 1) / BNS, ns2 = (d + 255) / 256;
  const unsigned long long m = build_plan(plan, mask, T, E, gridDim.x, max_rows, row_cap, ns1, ns2, d, f);
  const bool overflow = plan.nnz < 0;
  const int items = plan.U * ns1 * plan.ks1;
  const int kc = d / plan.ks1;                   // K elements per chunk
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int c = item % plan.ks1, j = (item / plan.ks1) % ns1, e = plan.act[item / (plan.ks1 * ns1)];
    const int Me = plan.cnt[e], n0 = j * BNS;
    __syncthreads();                             // the previous item no longer reads toks
    if (wave < 2 && ((m >> e) & 1ull))
      toks[__popcll(plan.tokbits[e][wave] & ((1ull << lane) - 1ull)) + (wave == 1 ? plan.cnt_w0[e] : 0)] = threadIdx.x;
    __syncthreads();
    typename TL::LSrc L;
    L.init(Me, 0, [&](int r) { return x + (size_t)toks[r] * d + (size_t)c * kc; });
    typename TL::RSrc R;
    const size_t wo = (size_t)e * d * f + (size_t)c * kc * f + n0;
    if constexpr (GELU) {
      const bf16_t* const base[1] = {w_gate + wo};
      R.init(base, f, min(BNS, f - n0), kc);
    } else {
      const bf16_t* const base[2] = {w_gate + wo, w_up + wo};
      R.init(base, f, min(BNS, f - n0), kc);
    }
    typename TL::Acc acc;
    TL::zero(acc);
    TL::mainloop(acc, L, R, kc / kBK2, 1 << 30, st);
    const int hrow0 = plan.off[e];
    if (plan.ks1 == 1) {   // the whole K range: H = silu(G) * U straight from the accumulators
#pragma unroll
      for (int mt = 0; mt < TL::MT; ++mt) {
        const int mrow = TL::acc_m(mt);
        if (mrow >= Me) continue;
        bf16_t* hrow = H + (size_t)(hrow0 + mrow) * f;
        if constexpr (GELU) {
#pragma unroll
          for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int n = n0 + TL::acc_n(nt, g);
              if (n >= f) continue;
              const f32x16& G = acc[nt][mt];
              store4(hrow + n, gelu_f(G[4 * g]), gelu_f(G[4 * g + 1]), gelu_f(G[4 * g + 2]), gelu_f(G[4 * g + 3]));
            }
          continue;
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + TL::acc_n(0, g);
          if (n >= f) continue;
          const f32x16& G = acc[0][mt];
          const f32x16& Uv = acc[1][mt];
          store4(hrow + n, silu_f(G[4 * g]) * Uv[4 * g], silu_f(G[4 * g + 1]) * Uv[4 * g + 1],
                 silu_f(G[4 * g + 2]) * Uv[4 * g + 2], silu_f(G[4 * g + 3]) * Uv[4 * g + 3]);
        }
      }
      continue;
    }
    // fp32 partial sums of this K chunk, stored straight from the accumulator layout
#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt) {
      const int mrow = TL::acc_m(mt);
      if (mrow >= Me) continue;
      float* prow = P1 + ((size_t)c * plan.nnz + hrow0 + mrow) * (2 * (size_t)f);
      if constexpr (GELU) {
#pragma unroll
        for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int n = n0 + TL::acc_n(nt, g);
            if (n >= f) continue;
            const f32x16& G = acc[nt][mt];
            store4(prow + n, G[4 * g], G[4 * g + 1], G[4 * g + 2], G[4 * g + 3]);
          }
        continue;
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + TL::acc_n(0, g);
        if (n >= f) continue;
        const f32x16& G = acc[0][mt];
        const f32x16& Uv = acc[1][mt];
        store4(prow + n, G[4 * g], G[4 * g + 1], G[4 * g + 2], G[4 * g + 3]);
        store4(prow + f + n, Uv[4 * g], Uv[4 * g + 1], Uv[4 * g + 2], Uv[4 * g + 3]);
      }
    }
    // the block that stores the last chunk of (expert, column slice) adds the chunks in ascending order
    if (!arrive_last(arrivals + e * ns1 + j, plan.ks1)) continue;
    constexpr int QPR = BNS / 4;                  // column quads per row of the slice
    for (int idx = threadIdx.x; idx < Me * QPR; idx += kThreads2) {
      const int r = idx / QPR, n = n0 + (idx % QPR) * 4;
      if (n >= f) continue;
      const float* p = P1 + (size_t)(hrow0 + r) * (2 * (size_t)f) + n;
      const size_t cstride = (size_t)plan.nnz * 2 * f;
      f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = g;
      for (int c0 = 0; c0 < plan.ks1; c0 += 4) {
        f32x4 gv[4], uv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (c0 + q < plan.ks1) {
            gv[q] = __builtin_bit_cast(f32x4, ldg16(p + (size_t)(c0 + q) * cstride));
            if constexpr (!GELU) uv[q] = __builtin_bit_cast(f32x4, ldg16(p + (size_t)(c0 + q) * cstride + f));
          }
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (c0 + q < plan.ks1) {
            g += gv[q];
            if constexpr (!GELU) u += uv[q];
          }
      }
      if constexpr (GELU)
        store4(H + (size_t)(hrow0 + r) * f + n, gelu_f(g.x), gelu_f(g.y), gelu_f(g.z), gelu_f(g.w));
      else
        store4(H + (size_t)(hrow0 + r) * f + n, silu_f(g.x) * u.x, silu_f(g.y) * u.y, silu_f(g.z) * u.z,
               silu_f(g.w) * u.w);
    }
  }
  if (blockIdx.x == gridDim.x - 1) {   // publish the routing objects of this call: later kernels read them,
                                       // so the block does it after its own items
    if ((int)threadIdx.x <= E) expert_off[threadIdx.x] = threadIdx.x == E ? plan.off[64] : plan.off[threadIdx.x];
    if (threadIdx.x == 0) {
      nnz_out[0] = overflow ? 0 : plan.nnz;
      info[0] = overflow ? 0 : plan.nnz; info[1] = plan.U; info[2] = plan.ks1; info[3] = plan.ks2;
      if (overflow) err_flag[0] = DSMOE_ERR_CAPACITY;
    }
    __shared__ int sTokOff[kDecT + 1];
    __shared__ int sTok0;
    const int cnt = __popcll(m);
    int incl = cnt;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(incl, s, 64);
      if (lane >= s) incl += o;
    }
    if (threadIdx.x == 63) sTok0 = incl;
    __syncthreads();
    if (wave < 2) {
      const int tbase = overflow ? 0 : incl - cnt + (wave == 1 ? sTok0 : 0);
      sTokOff[threadIdx.x] = tbase;
      if ((int)threadIdx.x < T) tok_off[threadIdx.x] = tbase;
      if ((int)threadIdx.x == T - 1) tok_off[T] = overflow ? 0 : plan.nnz;
    }
    __syncthreads();
    // one (token, expert) pair per thread and pass: every probability load of a pass is in flight at once
    constexpr int kPairs = kDecT * kMaxExperts / kThreads2;
    const int npairs = overflow ? 0 : T * E;
    float pw[kPairs];
#pragma unroll
    for (int i = 0; i < kPairs; ++i) {
      const int idx = threadIdx.x + i * kThreads2;
      pw[i] = idx < npairs ? probs[idx] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kPairs; ++i) {
      const int idx = threadIdx.x + i * kThreads2;
      if (idx >= npairs) continue;
      const int t = idx / E, e = idx - t * E;
      const unsigned long long mt = plan.tokmask[t];
      if (!((mt >> e) & 1ull)) continue;
      const unsigned long long b0 = plan.tokbits[e][0], b1 = plan.tokbits[e][1];
      const int rank = t < 64 ? __popcll(b0 & ((1ull << t) - 1ull)) : __popcll(b0) + __popcll(b1 & ((1ull << (t - 64)) - 1ull));
      const int row = plan.off[e] + rank;
      row_token[row] = t;
      row_weight[row] = pw[i];
      tok_rows[sTokOff[t] + __popcll(mt & ((1ull << e) - 1ull))] = row;
    }
  }
}

// ---- down: partial Y over one chunk of the hidden width -------------------------------------------------
__global__ void __launch_bounds__(kThreads2)
decode_down_kernel(const bf16_t* __restrict__ H, const int32_t* __restrict__ info,
                   const int32_t* __restrict__ expert_off, const bf16_t* __restrict__ w_down,
                   float* __restrict__ P2, int d, int f, int E) {
  constexpr int BN = 256;
  typedef Tile3<kDecT, BN, 1, false, true, false, 6> TL;
  DSMOE_TILE3_STAGES(TL, st);
  __shared__ int sOff[kMaxExperts + 1], sAct[kMaxExperts];
  __shared__ int sU;
  if (threadIdx.x < 64) {
    const int e = threadIdx.x;
    const int lo = e < E ? expert_off[e] : 0, hi = e < E ? expert_off[e + 1] : 0;
    const unsigned long long actm = __ballot(hi > lo);
    sOff[e] = lo;
    if (e == E - 1) sOff[E] = hi;
    if (hi > lo) sAct[__popcll(actm & ((1ull << e) - 1ull))] = e;
    if (e == 0) sU = __popcll(actm);
  }
  __syncthreads();
  const int nnz = info[0], ks2 = info[3];
  const int ns2 = (d + BN - 1) / BN;
  const int items = sU * ns2 * ks2;
  const int kc = f / ks2;
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int c = item % ks2, j = (item / ks2) % ns2, e = sAct[item / (ks2 * ns2)];
    const int row0 = sOff[e], Me = sOff[e + 1] - row0, n0 = j * BN;
    typename TL::LSrc L;
    L.init(Me, 0, [&](int r) { return H + (size_t)(row0 + r) * f + (size_t)c * kc; });
    typename TL::RSrc R;
    const bf16_t* const base[1] = {w_down + (size_t)e * f * d + (size_t)c * kc * d + n0};
    R.init(base, d, min(BN, d - n0), kc);
    typename TL::Acc acc;
    TL::zero(acc);
    TL::mainloop(acc, L, R, kc / kBK2, 1 << 30, st);
#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt) {
      const int mrow = TL::acc_m(mt);
      if (mrow >= Me) continue;
      float* prow = P2 + ((size_t)c * nnz + row0 + mrow) * (size_t)d;
#pragma unroll
      for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + TL::acc_n(nt, g);
          if (n >= d) continue;
          const f32x16& A = acc[nt][mt];
          store4(prow + n, A[4 * g], A[4 * g + 1], A[4 * g + 2], A[4 * g + 3]);
        }
    }
  }
}

// ---- combine: out[t,:] = sum over the token's rows (ascending expert) of weight * (sum of down partials) ----
// Block (t, column chunk).  The (row, K chunk) partials are read eight at a time so that their latencies
// overlap; they are added in a fixed order: K chunks ascending within a row, rows by ascending expert.
constexpr int kCombCols = 512;   // columns per block: 128 threads x 4
__global__ void __launch_bounds__(kCombCols / 4)
decode_combine_kernel(const float* __restrict__ P2, const int32_t* __restrict__ info,
                      const float* __restrict__ row_weight, const int32_t* __restrict__ tok_off,
                      const int32_t* __restrict__ tok_rows, int d, bf16_t* __restrict__ out) {
  __shared__ int sRow[kMaxExperts];
  __shared__ float sW[kMaxExperts];
  const int t = blockIdx.x, c0 = blockIdx.y * kCombCols + threadIdx.x * 4;
  const int nnz = info[0], ks2 = info[3];
  const int lo = tok_off[t], n = tok_off[t + 1] - lo;
  if ((int)threadIdx.x < n) {
    const int row = tok_rows[lo + threadIdx.x];
    sRow[threadIdx.x] = row;
    sW[threadIdx.x] = row_weight[row];
  }
  __syncthreads();
  if (c0 >= d) return;
  const size_t chunk_stride = (size_t)nnz * d;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f}, y = acc;
  const int total = n * ks2;
  int j = 0, c = 0;                         // position of the next partial to add
  for (int i0 = 0; i0 < total; i0 += 8) {
    f32x4 v[8];
    int jj = j, cc = c;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool ok = i0 + u < total;
      const float* p = P2 + (size_t)cc * chunk_stride + (size_t)sRow[ok ? jj : 0] * d + c0;
      v[u] = ok ? __builtin_bit_cast(f32x4, ldg16(p)) : f32x4{0.f, 0.f, 0.f, 0.f};
      if (++cc == ks2) { cc = 0; ++jj; }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (i0 + u >= total) break;
      y = c == 0 ? v[u] : y + v[u];
      if (++c == ks2) {
        const float w = sW[j];
        acc.x = fmaf(w, y.x, acc.x);
        acc.y = fmaf(w, y.y, acc.y);
        acc.z = fmaf(w, y.z, acc.z);
        acc.w = fmaf(w, y.w, acc.w);
        c = 0; ++j;
      }
    }
  }
  store4(out + (size_t)t * d + c0, acc.x, acc.y, acc.z, acc.w);
}

}  // namespace

hipError_t launch_decode_fwd(const dsmoe_ctx* c, const void* x, const void* w_gate, const void* w_up,
                             const void* w_down, int T, void* out, hipStream_t s) {
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  char* w = c->workspace;
  const float* probs = reinterpret_cast<const float*>(w + c->ws.probs);
  const unsigned long long* mask = reinterpret_cast<const unsigned long long*>(w + c->ws.mask);
  int32_t* info = reinterpret_cast<int32_t*>(w + c->ws.dec_info);
  float* P1 = reinterpret_cast<float*>(w + c->ws.dec_p1);
  float* P2 = reinterpret_cast<float*>(w + c->ws.dec_p2);
  bf16_t* H = reinterpret_cast<bf16_t*>(w + c->ws.h);
  int32_t* expert_off = reinterpret_cast<int32_t*>(w + c->ws.expert_off);
  int32_t* row_token = reinterpret_cast<int32_t*>(w + c->ws.row_token);
  float* row_weight = reinterpret_cast<float*>(w + c->ws.row_weight);
  int32_t* tok_off = reinterpret_cast<int32_t*>(w + c->ws.tok_off);
  int32_t* tok_rows = reinterpret_cast<int32_t*>(w + c->ws.tok_rows);
  int32_t* nnz = reinterpret_cast<int32_t*>(w + c->ws.nnz);
  int32_t* err_flag = reinterpret_cast<int32_t*>(w + c->ws.err_flag);
  int32_t* arrivals = reinterpret_cast<int32_t*>(w + c->ws.dec_arrivals);
  const int grid = (c->n_cu + 7) / 8 * 8;
  const int row_cap = decode_row_cap(c);

  if (c->expert_kind == DSMOE_EXPERT_GELU)
    decode_gateup_kernel<true><<<dim3(grid), dim3(kThreads2), 0, s>>>(
        (const bf16_t*)x, mask, probs, (const bf16_t*)w_gate, nullptr, P1, H, arrivals, T, d, f, E,
        (long long)c->desc.max_rows, row_cap, info, expert_off, row_token, row_weight, tok_off, tok_rows, nnz, err_flag);
  else
    decode_gateup_kernel<false><<<dim3(grid), dim3(kThreads2), 0, s>>>(
        (const bf16_t*)x, mask, probs, (const bf16_t*)w_gate, (const bf16_t*)w_up, P1, H, arrivals, T, d, f, E,
        (long long)c->desc.max_rows, row_cap, info, expert_off, row_token, row_weight, tok_off, tok_rows, nnz, err_flag);
  if (hipError_t e = hipGetLastError()) return e;
  decode_down_kernel<<<dim3(grid), dim3(kThreads2), 0, s>>>(H, info, expert_off, (const bf16_t*)w_down,
                                                                         P2, d, f, E);
  if (hipError_t e = hipGetLastError()) return e;
  decode_combine_kernel<<<dim3(T, (d + kCombCols - 1) / kCombCols), dim3(kCombCols / 4), 0, s>>>(P2, info, row_weight, tok_off, tok_rows, d, (bf16_t*)out);
  return hipGetLastError();
}

}  // namespace dsmoe
