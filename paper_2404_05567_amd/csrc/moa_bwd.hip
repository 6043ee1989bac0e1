// Dense-training backward of the Mixture-of-Attention-heads layer (paper Sec. 3.2: Eq. 7-8 under the dense
// gradient of Eq. 3), bf16 storage with fp32 accumulation.  Every expert is active and weighted by its score:
//
//   forward (moa.hip, selection "all")   Q_e = X W_q[e];  C[t,e,j] = softmax_l(scale Q_ej K_j^T) V_j;
//                                        Cs = S C;  O = Cs W_o  (W_o read as one [E hd, d] matrix, hd = n_head d_head)
//   kept by the forward for this pass    S, Q, C (unweighted), Cs, and lse = log2 sum_l 2^(scale log2e Q K^T) per row
//
//   dCs = dO W_o^T                                    grad S[t,e] = <C[t,e], dCs[t,e]>   (Eq. 3),  dC = S dCs
//   dW_o[e] = Cs_e^T dO                               delta[e,j,t] = <dC[t,e,j], C[t,e,j]>
//   P = 2^(scale log2e Q K^T - lse) (recomputed)      dV_j = sum_e P_ej^T dC_ej
//   dA = P (dC V_j^T - delta) scale  (in place of P)  dQ_ej = dA_ej K_j,  dK_j = sum_e dA_ej^T Q_ej
//   dW_q[e] = X^T dQ_e                                dX = sum_e dQ_e W_q[e]^T + dZ W_r^T
//   dZ = S (dS - sum_k S_k dS_k), dW_r = X^T dZ, db_r = sum_t dZ      (softmax and router, as in the MLP layer)
//
// The attention probabilities of one call are materialised once ([E T, n_head L] in bf16, in the caller's
// scratch buffer) so that every product above is a plain batched contraction on the library's bf16 MFMA core;
// tiles that lie wholly behind the causal diagonal are not multiplied.  The sums over experts that the shared
// key/value heads need (dK, dV) are contractions over the stacked (expert, token) rows: a fixed order, no
// floating-point atomics, bitwise reproducible.
#include <algorithm>
#include <cmath>

#include "gemm.h"
#include "moa_internal.h"

using namespace dsmoe;

namespace {

enum { kEpiPlain = 0, kEpiProbs = 1, kEpiSoftmaxBwd = 2 };

// out[b][m][n] = alpha * sum_k L_b[m][k] R_b[k][n], b = (b1, b2), with optional epilogues.
// "rows" operands are k-contiguous (element [m][k] at base + m ld + k), "cols" operands are stored [k][m].
struct BatchedArgs {
  const bf16_t* L; const bf16_t* R; void* out;
  long long ldl, ldr, ldo;
  long long sL1, sL2, sR1, sR2, sO1, sO2;     // batch strides in elements
  int nb1, nb2, M, N, K;
  int seg_k;                                  // rows x rows only: K is cut in segments of seg_k ...
  long long segL, segR;                       // ... that lie segL / segR elements apart (0: one contiguous run)
  float alpha;
  int tiles_per_batch;                        // tiles of a batch member that are computed (causal epilogues leave some out)
  const float* rowv;                          // kEpiProbs: lse [b][M];  kEpiSoftmaxBwd: delta [b][M]
  int pos0;                                   // both: column n is visible to row m iff n <= pos0 + m
  int causal_k;                               // the left operand is zero for k > pos0 + m: stop the contraction there
  int causal_k0;                              // cols x cols: the left operand is zero for k < m - pos0: start there
  const void* zeros;
};

template <bool LK, bool RK, bool OUT_F32, int EPI>
__global__ void __launch_bounds__(kThreads2) batched_gemm_kernel(const BatchedArgs a) {
  typedef Gemm<bf16_t, 256, 256, 1, LK, RK, LK || RK> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (a.M + GM::BM - 1) / GM::BM, n_nt = (a.N + GM::BN - 1) / GM::BN;
  (void)n_mt;
  TileWalker tw;
  constexpr bool causal = EPI == kEpiProbs || EPI == kEpiSoftmaxBwd;
  tw.init(a.nb1 * a.nb2 * a.tiles_per_batch);
  int idx;
  while (tw.next(idx)) {
    // A tile wholly behind the causal diagonal would hold zeros.  It is neither computed nor stored (the products
    // that read the probabilities leave the same tiles out: causal_k, causal_k0), and not dealt out either: row
    // tile mt has the column tiles up to its last visible key.
    const int b = idx / a.tiles_per_batch;
    int nt = idx % a.tiles_per_batch, mt = 0;
    if constexpr (causal) {
      for (; mt < n_mt - 1; ++mt) {
        const int c = min(n_nt, (a.pos0 + mt * GM::BM + GM::BM - 1) / GM::BN + 1);
        if (nt < c) break;
        nt -= c;
      }
    } else {
      mt = nt / n_nt;
      nt = nt % n_nt;
    }
    const int b1 = b / a.nb2, b2 = b % a.nb2;
    const int m0 = mt * GM::BM, n0 = nt * GM::BN;
    const bf16_t* Lb = a.L + b1 * a.sL1 + b2 * a.sL2;
    const bf16_t* Rb = a.R + b1 * a.sR1 + b2 * a.sR2;
    char* Ob = static_cast<char*>(a.out) + (size_t)(b1 * a.sO1 + b2 * a.sO2) * (OUT_F32 ? 4 : 2);
    typename GM::Acc acc;
    GM::zero(acc);
    {
      typename GM::LSrc L;
      typename GM::RSrc R;
      int K = a.K;
      if constexpr (LK && RK) {
        if (a.causal_k0) {
          const int k0 = max(0, m0 - a.pos0) / GM::BK * GM::BK;
          Lb += (size_t)k0 * a.ldl;
          Rb += (size_t)k0 * a.ldr;
          K -= k0;
        }
      }
      if constexpr (LK) GM::l_cols(L, Lb + m0, (size_t)a.ldl, a.M - m0, K, a.zeros);
      else GM::l_rows(L, min(GM::BM, a.M - m0), (size_t)a.segL * 2, [&](int r) { return Lb + (size_t)(m0 + r) * a.ldl; });
      if constexpr (RK) {
        const bf16_t* const base[1] = {Rb + n0};
        GM::r_cols(R, base, (size_t)a.ldr, a.N - n0, K, a.zeros);
      } else {
        GM::r_rows(R, min(GM::BN, a.N - n0), (size_t)a.segR * 2, [&](int r) { return Rb + (size_t)(n0 + r) * a.ldr; });
      }
      const int k_end = a.causal_k ? min(K, a.pos0 + m0 + GM::BM) : K;
      const int nkt = (k_end + GM::BK - 1) / GM::BK;
      GM::mainloop(acc, L, R, nkt, a.seg_k > 0 ? a.seg_k / GM::BK : 1 << 30, st);
    }
    // what a chunk's epilogue reads from memory is requested a 32-row block ahead of its use
    float rv[GM::NJ];
    u32x4 q0[GM::NJ];
    GM::for_each_chunk_loaded(
        acc, st,
        [&](int j, int m, int n) {
          const int row = m0 + m, col = n0 + n;
          if (row >= a.M || col >= a.N) return;
          if constexpr (EPI == kEpiProbs || EPI == kEpiSoftmaxBwd) rv[j] = a.rowv[(size_t)b * a.M + row];
          if constexpr (EPI == kEpiSoftmaxBwd) q0[j] = load_raw(reinterpret_cast<const bf16_t*>(Ob) + (size_t)row * a.ldo + col);
        },
        [&](int j, int m, int n, const float (&v)[1][GM::CHUNK]) {
          const int row = m0 + m, col = n0 + n;
          if (row >= a.M || col >= a.N) return;
          float o[GM::CHUNK];
          if constexpr (EPI == kEpiProbs) {
#pragma unroll
            for (int i = 0; i < GM::CHUNK; ++i)
              o[i] = col + i <= a.pos0 + row ? __builtin_amdgcn_exp2f(fminf(v[0][i] * a.alpha - rv[j], 0.f)) : 0.f;
          } else if constexpr (EPI == kEpiSoftmaxBwd) {
            float p[GM::CHUNK];
            unpack_chunk(q0[j], p, (const bf16_t*)nullptr);
#pragma unroll
            for (int i = 0; i < GM::CHUNK; ++i) o[i] = col + i <= a.pos0 + row ? p[i] * (v[0][i] - rv[j]) * a.alpha : 0.f;
          } else {
#pragma unroll
            for (int i = 0; i < GM::CHUNK; ++i) o[i] = v[0][i] * a.alpha;
          }
          if constexpr (OUT_F32) store_chunk(reinterpret_cast<float*>(Ob) + (size_t)row * a.ldo + col, o);
          else store_chunk(reinterpret_cast<bf16_t*>(Ob) + (size_t)row * a.ldo + col, o);
        });
  }
}

template <bool LK, bool RK, bool OUT_F32, int EPI = kEpiPlain>
hipError_t launch_batched(const dsmoe_ctx* c, const BatchedArgs& a, hipStream_t s) {
  const int n_mt = (a.M + 255) / 256, n_nt = (a.N + 255) / 256;
  BatchedArgs b = a;
  b.tiles_per_batch = 0;
  for (int mt = 0; mt < n_mt; ++mt)
    b.tiles_per_batch += EPI == kEpiPlain ? n_nt : std::min(n_nt, (a.pos0 + mt * 256 + 255) / 256 + 1);
  const long tiles = (long)a.nb1 * a.nb2 * b.tiles_per_batch;
  const int grid = (int)((std::min<long>(tiles, c->n_cu) + 7) / 8 * 8);
  batched_gemm_kernel<LK, RK, OUT_F32, EPI><<<dim3(grid), dim3(kThreads2), 0, s>>>(b);
  return hipGetLastError();
}

BatchedArgs plain_args() {
  BatchedArgs a{};
  a.nb1 = a.nb2 = 1;
  a.alpha = 1.f;
  return a;
}

// One wave per (token, expert): grad S = <C, dCs> (Eq. 3), dC = S dCs in the [E][T][hd] layout of Q, and the
// per-head terms delta = <dC, C> of the softmax backward.  A lane owns 8 consecutive values; the d_head / 8 lanes
// of a head add up along a fixed shuffle tree.
// dCs arrives as n_part fp32 partial sums (K split of its product), part_stride values apart.
__global__ void __launch_bounds__(256) moa_score_grad_kernel(const bf16_t* __restrict__ C, const float* __restrict__ dCs,
                                                            int n_part, size_t part_stride,
                                                            const float* __restrict__ S, float* __restrict__ dS,
                                                            bf16_t* __restrict__ dC, float* __restrict__ delta, int T,
                                                            int E, int NH, int DH) {
  const int lane = threadIdx.x & 63;
  const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= (long)T * E) return;
  const int t = (int)(w / E), e = (int)(w % E), hd = NH * DH, lph = DH / 8;     // lanes per head: 8 or 16
  const float s = S[(size_t)t * E + e];
  const bf16_t* c = C + ((size_t)t * E + e) * hd;
  const float* g = dCs + ((size_t)t * E + e) * hd;
  bf16_t* o = dC + ((size_t)e * T + t) * hd;
  float total = 0.f;
  for (int c0 = 0; c0 < hd; c0 += 512) {                 // 64 lanes x 8 values per pass
    const int i = c0 + 8 * lane;
    float part = 0.f;
    if (i < hd) {
      float cv[8], gv[8], gw[8], ov[8];
      load_chunk(c + i, cv);
      load_chunk(g + i, gv);
      if (n_part == 2) {
        load_chunk(g + part_stride + i, gw);
#pragma unroll
        for (int k = 0; k < 8; ++k) gv[k] += gw[k];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        part = fmaf(cv[k], gv[k], part);
        ov[k] = s * gv[k];
      }
      store_chunk(o + i, ov);
    }
    for (int sft = 1; sft < lph; sft <<= 1) part += __shfl_xor(part, sft, 64);   // the lanes of one head
    if (i < hd && lane % lph == 0) delta[((size_t)e * NH + i / DH) * T + t] = s * part;
    float all = lane % lph == 0 ? part : 0.f;                                     // one value per head
#pragma unroll
    for (int sft = 32; sft > 0; sft >>= 1) all += __shfl_xor(all, sft, 64);
    total += all;
  }
  if (lane == 0) dS[(size_t)t * E + e] = total;
}

// dZ = S (dS - sum_k S_k dS_k): one wave per token, one lane per expert
__global__ void __launch_bounds__(256) moa_softmax_bwd_kernel(const float* __restrict__ S, const float* __restrict__ dS,
                                                             int T, int E, float* __restrict__ dZ,
                                                             unsigned* __restrict__ zeros) {
  if (blockIdx.x == 0 && threadIdx.x < 64) zeros[threadIdx.x] = 0u;   // the zero page of the token-contracted products
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const float s = lane < E ? S[(size_t)t * E + lane] : 0.f, ds = lane < E ? dS[(size_t)t * E + lane] : 0.f;
  float dot = s * ds;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
  const float dz = s * (ds - dot);
  if (lane < E) dZ[(size_t)t * E + lane] = dz;
}

// dX = (sum_e dQ_e W_q[e]^T, handed over in fp32) + dZ W_r^T, rounded once: dx[t][n] = dxf[t][n] + sum_e dZ[t][e] W_r[n][e].
// A thread keeps its row of W_r in registers and walks kRouterTok tokens, whose dZ rows are the same for the whole block.
constexpr int kRouterTok = 32;
__global__ void __launch_bounds__(256) moa_router_dx_kernel(const float* __restrict__ dZ, const bf16_t* __restrict__ w_r, int T,
                                                           int d, int E, const float* __restrict__ dxf,
                                                           int n_part, bf16_t* __restrict__ dx) {
  const int n = blockIdx.y * 256 + threadIdx.x, t0 = blockIdx.x * kRouterTok;
  if (n >= d) return;
  float w[kMaxExperts];
#pragma unroll
  for (int c = 0; c < kMaxExperts / 8; ++c) {
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (8 * c < E) load_chunk(w_r + (size_t)n * E + 8 * c, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) w[8 * c + i] = v[i];
  }
  for (int t = t0; t < min(T, t0 + kRouterTok); ++t) {
    const float* z = dZ + (size_t)t * E;
    float acc = dxf[(size_t)t * d + n];
    if (n_part == 2) acc += dxf[(size_t)T * d + (size_t)t * d + n];
#pragma unroll
    for (int c = 0; c < kMaxExperts / 8; ++c)
      if (8 * c < E) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(z[8 * c + i], w[8 * c + i], acc);
      }
    dx[(size_t)t * d + n] = (bf16_t)acc;
  }
}

// dW_r = X^T dZ as partial sums over token ranges: part[split][n][e] = sum over the split's tokens of
// X[t][n] dZ[t][e]; a thread owns two neighbouring columns n and eight experts (blockIdx.z picks the eight).
__global__ void __launch_bounds__(256) moa_router_dw_kernel(const bf16_t* __restrict__ x, const float* __restrict__ dZ, int T,
                                                           int d, int E, int tok_per_split, float* __restrict__ part) {
  const int n = 2 * (blockIdx.x * 256 + threadIdx.x), e0 = 8 * blockIdx.z;
  if (n >= d) return;
  const int t0 = blockIdx.y * tok_per_split, t1 = min(T, t0 + tok_per_split);
  float a0[8], a1[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a0[i] = a1[i] = 0.f;
#pragma unroll 8
  for (int t = t0; t < t1; ++t) {
    const unsigned xv = *reinterpret_cast<const unsigned*>(x + (size_t)t * d + n);
    const float x0 = __uint_as_float(xv << 16), x1 = __uint_as_float(xv & 0xffff0000u);
    const float* z = dZ + (size_t)t * E + e0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a0[i] = fmaf(x0, z[i], a0[i]);
      a1[i] = fmaf(x1, z[i], a1[i]);
    }
  }
  float* o = part + ((size_t)blockIdx.y * d + n) * E + e0;
  store4(o, a0[0], a0[1], a0[2], a0[3]);
  store4(o + 4, a0[4], a0[5], a0[6], a0[7]);
  store4(o + E, a1[0], a1[1], a1[2], a1[3]);
  store4(o + E + 4, a1[4], a1[5], a1[6], a1[7]);
}

// out[g][i] = sum over s < n_part of part[(g * n_part + s) * n + i], in order; g = blockIdx.y, 4 values per thread
__global__ void __launch_bounds__(256) moa_sum_parts_kernel(const float* __restrict__ part, int n_part, size_t n,
                                                           float* __restrict__ out) {
  const size_t i = 4 * ((size_t)blockIdx.x * 256 + threadIdx.x);
  if (i >= n) return;
  const float* p = part + (size_t)blockIdx.y * n_part * n + i;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int sp = 0; sp < n_part; ++sp) acc += __builtin_bit_cast(f32x4, ldg16(p + sp * n));
  store4(out + (size_t)blockIdx.y * n + i, acc.x, acc.y, acc.z, acc.w);
}

// db_r[e] = sum_t dZ[t][e]: one block per expert, strided partial sums, then a fixed-order tree
__global__ void __launch_bounds__(256) moa_router_db_kernel(const float* __restrict__ dZ, int T, int E, float* __restrict__ db_r) {
  __shared__ float sSum[256];
  const int e = blockIdx.x;
  float s = 0.f;
  for (int t = threadIdx.x; t < T; t += 256) s += dZ[(size_t)t * E + e];
  sSum[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sSum[threadIdx.x] += sSum[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) db_r[e] = sSum[0];
}

// columns [L, Lp) of the probability matrix are multiplied (as zeros) by the products that contract over keys
__global__ void __launch_bounds__(256) moa_zero_pad_kernel(bf16_t* __restrict__ P, long rows, int L, int Lp, int NH) {
  const int pad = Lp - L;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * NH * pad) return;
  const long r = i / (NH * pad);
  const int j = (int)(i / pad % NH), c = (int)(i % pad);
  P[(size_t)r * NH * Lp + (size_t)j * Lp + L + c] = (bf16_t)0.f;
}

size_t al256(size_t v) { return (v + 255) / 256 * 256; }

struct BwdScratch { size_t zeros, dcs, dc, delta, ds, p, dq, dz, dxf, part, total; int Lp, tok_per_split, n_split; };
BwdScratch bwd_scratch(const dsmoe_moa_desc& d, int T, int L) {
  const size_t E = d.n_experts, hd = (size_t)d.n_head * d.d_head, Tn = T;
  BwdScratch l;
  l.Lp = (L + 31) / 32 * 32;
  l.tok_per_split = std::max(64, (T + 63) / 64);          // token ranges of the router weight gradient: at most 64
  l.n_split = (T + l.tok_per_split - 1) / l.tok_per_split;
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o = al256(o + bytes); return at; };
  l.zeros = take(256);
  l.dcs = take(2 * Tn * E * hd * 4);            // two K halves in fp32
  l.dc = take(E * Tn * hd * 2);
  l.delta = take(E * d.n_head * Tn * 4);
  l.ds = take(Tn * E * 4);
  l.p = take(E * Tn * d.n_head * (size_t)l.Lp * 2);
  l.dq = take(E * Tn * hd * 2);
  l.dz = take(Tn * E * 4);
  l.dxf = take(2 * Tn * (size_t)d.d_model * 4);
  // per-expert partial sums of dK / dV ([n_head][E][L][d_head]), then the router weight gradient's ([n_split][d][E])
  l.part = take(std::max(E * (size_t)L * hd * 4, (size_t)l.n_split * d.d_model * E * 4));
  l.total = o;
  return l;
}

}  // namespace

extern "C" {

int32_t dsmoe_moa_bwd_scratch_bytes(const dsmoe_moa_ctx* c, int32_t T, int32_t L, size_t* bytes) {
  if (!c || !bytes || T < 0 || L < T) return DSMOE_ERR_INVALID_ARG;
  *bytes = bwd_scratch(c->desc, T, L).total;
  return DSMOE_OK;
}

int32_t dsmoe_moa_bwd(dsmoe_moa_ctx* c, const void* x, const void* w_r, const void* w_q, const void* k_cache,
                      const void* v_cache, const void* w_o, const void* d_out, int32_t T, int32_t L, float scale,
                      void* scratch, void* dx, float* dw_r, float* db_r, float* dw_q, float* dw_o, float* dk, float* dv,
                      void* stream) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  auto fail = [&](int32_t code, const char* msg) {
    snprintf(c->err, sizeof(c->err), "dsmoe_moa_bwd: %s", msg);
    return code;
  };
  if (T < 1 || T > c->desc.max_tokens) return fail(DSMOE_ERR_INVALID_ARG, "T outside [1, max_tokens]");
  if (L < T) return fail(DSMOE_ERR_INVALID_ARG, "the cache holds the T tokens themselves: L >= T");
  if (!std::isfinite(scale)) return fail(DSMOE_ERR_INVALID_ARG, "scale must be finite");
  if (!c->workspace) return fail(DSMOE_ERR_WORKSPACE, "no workspace set (dsmoe_moa_set_workspace)");
  if (c->saved_T != T || c->saved_L != L || c->saved_scale != scale)
    return fail(DSMOE_ERR_INVALID_ARG, "needs the dsmoe_moa_fwd call of the same T, L and scale with selection "
                                       "DSMOE_SEL_ALL right before (its scores, queries and attention outputs are kept)");
  const void* ptrs[] = {x, w_r, w_q, k_cache, v_cache, w_o, d_out, scratch, dx, dw_r, dw_q, dw_o, dk, dv};
  for (const void* p : ptrs)
    if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u)) return fail(DSMOE_ERR_INVALID_ARG, "null or misaligned pointer");
  if (db_r && (reinterpret_cast<uintptr_t>(db_r) & 3u)) return fail(DSMOE_ERR_INVALID_ARG, "db_r misaligned");

  hipStream_t s = static_cast<hipStream_t>(stream);
  const dsmoe_ctx* ic = &c->inner;
  const int E = c->desc.n_experts, d = c->desc.d_model, NH = c->desc.n_head, DH = c->desc.d_head, hd = NH * DH;
  const BwdScratch sc = bwd_scratch(c->desc, T, L);
  char* w = static_cast<char*>(scratch);
  const float* S = reinterpret_cast<const float*>(c->workspace + c->o_probs);
  const bf16_t* Q = reinterpret_cast<const bf16_t*>(c->workspace + c->o_q);
  const bf16_t* Cs = reinterpret_cast<const bf16_t*>(c->workspace + c->o_cs);
  const bf16_t* C = reinterpret_cast<const bf16_t*>(c->workspace + c->o_c);
  const float* lse = reinterpret_cast<const float*>(c->workspace + c->o_lse);
  float* dCs = reinterpret_cast<float*>(w + sc.dcs);
  bf16_t* dC = reinterpret_cast<bf16_t*>(w + sc.dc);
  float* delta = reinterpret_cast<float*>(w + sc.delta);
  float* dS = reinterpret_cast<float*>(w + sc.ds);
  bf16_t* P = reinterpret_cast<bf16_t*>(w + sc.p);
  bf16_t* dQ = reinterpret_cast<bf16_t*>(w + sc.dq);
  float* dZ = reinterpret_cast<float*>(w + sc.dz);
  float* part = reinterpret_cast<float*>(w + sc.part);
  float* dxf = reinterpret_cast<float*>(w + sc.dxf);
  const void* zeros = w + sc.zeros;
  const long long ldp = (long long)NH * sc.Lp;
  const int pos0 = L - T;
  const float sl2e = scale * 1.4426950408889634f;
  const bf16_t* X = static_cast<const bf16_t*>(x);
  const bf16_t* dO = static_cast<const bf16_t*>(d_out);
  const bf16_t* Kc = static_cast<const bf16_t*>(k_cache);
  const bf16_t* Vc = static_cast<const bf16_t*>(v_cache);
#define MOA_TRY(expr)                                                                                \
  do {                                                                                               \
    hipError_t e_ = (expr);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      snprintf(c->err, sizeof(c->err), "dsmoe_moa_bwd: %s: %s", #expr, hipGetErrorString(e_));        \
      return DSMOE_ERR_HIP;                                                                          \
    }                                                                                                \
  } while (0)

  // The two products with only T x d or T x E hd outputs are cut in two K halves when their tiles would leave half
  // the CUs idle; the halves are fp32 partial sums that the next kernel adds.
  auto k_halves = [&](long m, long n) { return 2 * ((m + 255) / 256) * ((n + 255) / 256) <= ic->n_cu ? 2 : 1; };
  // dCs = dO W_o^T  ([T, d] x [E hd, d]^T)
  const int ks_c = k_halves(T, (long)E * hd);
  {
    BatchedArgs a = plain_args();
    a.L = dO; a.ldl = d; a.sL2 = d / ks_c; a.R = static_cast<const bf16_t*>(w_o); a.ldr = d; a.sR2 = d / ks_c;
    a.out = dCs; a.ldo = (long long)E * hd; a.sO2 = (long long)T * E * hd;
    a.nb2 = ks_c; a.M = T; a.N = E * hd; a.K = d / ks_c;
    MOA_TRY((launch_batched<false, false, true>(ic, a, s)));
  }
  moa_score_grad_kernel<<<dim3((unsigned)(((long)T * E + 3) / 4)), dim3(256), 0, s>>>(C, dCs, ks_c, (size_t)T * E * hd, S, dS, dC,
                                                                                  delta, T, E, NH, DH);
  MOA_TRY(hipGetLastError());
  moa_softmax_bwd_kernel<<<dim3((T + 3) / 4), dim3(256), 0, s>>>(S, dS, T, E, dZ,
                                                                 reinterpret_cast<unsigned*>(w + sc.zeros));
  MOA_TRY(hipGetLastError());
  // dW_o[e] = Cs_e^T dO  (contraction over tokens)
  {
    BatchedArgs a = plain_args();
    a.L = Cs; a.ldl = (long long)E * hd; a.sL1 = hd; a.R = dO; a.ldr = d; a.out = dw_o; a.ldo = d; a.sO1 = (long long)hd * d;
    a.nb1 = E; a.M = hd; a.N = d; a.K = T; a.zeros = zeros;
    MOA_TRY((launch_batched<true, true, true>(ic, a, s)));
  }
  // P[(e,t)][(j,l)] = 2^(scale log2e Q_ej K_j^T - lse), zero behind the causal diagonal
  if (sc.Lp > L) {
    const long n = (long)E * T * NH * (sc.Lp - L);
    moa_zero_pad_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(P, (long)E * T, L, sc.Lp, NH);
    MOA_TRY(hipGetLastError());
  }
  {
    BatchedArgs a = plain_args();
    a.L = Q; a.ldl = hd; a.sL1 = (long long)T * hd; a.sL2 = DH;
    a.R = Kc; a.ldr = DH; a.sR2 = (long long)L * DH;
    a.out = P; a.ldo = ldp; a.sO1 = (long long)T * ldp; a.sO2 = sc.Lp;
    a.nb1 = E; a.nb2 = NH; a.M = T; a.N = L; a.K = DH; a.alpha = sl2e; a.rowv = lse; a.pos0 = pos0;
    MOA_TRY((launch_batched<false, false, false, kEpiProbs>(ic, a, s)));
  }
  // dV_j = sum_e P_ej^T dC_ej: one contraction over tokens per (head, expert) into fp32 partial sums, added in
  // expert order afterwards.  Tokens before the key tile's first position see none of its keys: they are left out.
  const size_t kv_elems = (size_t)L * DH;
  auto sum_over_experts = [&](float* out) {
    moa_sum_parts_kernel<<<dim3((unsigned)((kv_elems / 4 + 255) / 256), NH), dim3(256), 0, s>>>(part, E, kv_elems, out);
    return hipGetLastError();
  };
  {
    BatchedArgs a = plain_args();
    a.L = P; a.ldl = ldp; a.sL1 = sc.Lp; a.sL2 = (long long)T * ldp;
    a.R = dC; a.ldr = hd; a.sR1 = DH; a.sR2 = (long long)T * hd;
    a.out = part; a.ldo = DH; a.sO1 = (long long)E * kv_elems; a.sO2 = (long long)kv_elems;
    a.nb1 = NH; a.nb2 = E; a.M = L; a.N = DH; a.K = T; a.zeros = zeros; a.causal_k0 = 1; a.pos0 = pos0;
    MOA_TRY((launch_batched<true, true, true>(ic, a, s)));
    MOA_TRY(sum_over_experts(dv));
  }
  // dA = P (dC V_j^T - delta) scale, in place of P
  {
    BatchedArgs a = plain_args();
    a.L = dC; a.ldl = hd; a.sL1 = (long long)T * hd; a.sL2 = DH;
    a.R = Vc; a.ldr = DH; a.sR2 = (long long)L * DH;
    a.out = P; a.ldo = ldp; a.sO1 = (long long)T * ldp; a.sO2 = sc.Lp;
    a.nb1 = E; a.nb2 = NH; a.M = T; a.N = L; a.K = DH; a.alpha = scale; a.rowv = delta; a.pos0 = pos0;
    MOA_TRY((launch_batched<false, false, false, kEpiSoftmaxBwd>(ic, a, s)));
  }
  // dQ_ej = dA_ej K_j  (contraction over keys; the pad columns of dA are zero, the cache rows past L read as zero)
  {
    BatchedArgs a = plain_args();
    a.L = P; a.ldl = ldp; a.sL1 = (long long)T * ldp; a.sL2 = sc.Lp;
    a.R = Kc; a.ldr = DH; a.sR2 = (long long)L * DH;
    a.out = dQ; a.ldo = hd; a.sO1 = (long long)T * hd; a.sO2 = DH;
    a.nb1 = E; a.nb2 = NH; a.M = T; a.N = DH; a.K = L; a.zeros = zeros; a.causal_k = 1; a.pos0 = pos0;
    MOA_TRY((launch_batched<false, true, false>(ic, a, s)));
  }
  // dK_j = sum_e dA_ej^T Q_ej, the same way
  {
    BatchedArgs a = plain_args();
    a.L = P; a.ldl = ldp; a.sL1 = sc.Lp; a.sL2 = (long long)T * ldp;
    a.R = Q; a.ldr = hd; a.sR1 = DH; a.sR2 = (long long)T * hd;
    a.out = part; a.ldo = DH; a.sO1 = (long long)E * kv_elems; a.sO2 = (long long)kv_elems;
    a.nb1 = NH; a.nb2 = E; a.M = L; a.N = DH; a.K = T; a.zeros = zeros; a.causal_k0 = 1; a.pos0 = pos0;
    MOA_TRY((launch_batched<true, true, true>(ic, a, s)));
    MOA_TRY(sum_over_experts(dk));
  }
  // dW_q[e] = X^T dQ_e
  {
    BatchedArgs a = plain_args();
    a.L = X; a.ldl = d; a.R = dQ; a.ldr = hd; a.sR1 = (long long)T * hd; a.out = dw_q; a.ldo = hd; a.sO1 = (long long)d * hd;
    a.nb1 = E; a.M = d; a.N = hd; a.K = T; a.zeros = zeros;
    MOA_TRY((launch_batched<true, true, true>(ic, a, s)));
  }
  // router: dW_r = X^T dZ (partial sums over token ranges, added in order), db_r = sum_t dZ, and its term of dX
  moa_router_dw_kernel<<<dim3((d / 2 + 255) / 256, sc.n_split, E / 8), dim3(256), 0, s>>>(X, dZ, T, d, E, sc.tok_per_split, part);
  MOA_TRY(hipGetLastError());
  moa_sum_parts_kernel<<<dim3((unsigned)(((size_t)d * E / 4 + 255) / 256)), dim3(256), 0, s>>>(part, sc.n_split, (size_t)d * E,
                                                                                           dw_r);
  MOA_TRY(hipGetLastError());
  if (db_r) {
    moa_router_db_kernel<<<dim3(E), dim3(256), 0, s>>>(dZ, T, E, db_r);
    MOA_TRY(hipGetLastError());
  }
  // dX = sum_e dQ_e W_q[e]^T (one contraction over (expert, hd) in E segments, fp32) + dZ W_r^T
  const int ks_x = k_halves(T, d);
  {
    BatchedArgs a = plain_args();
    a.L = dQ; a.ldl = hd; a.segL = (long long)T * hd;
    a.R = static_cast<const bf16_t*>(w_q); a.ldr = hd; a.segR = (long long)d * hd;
    a.seg_k = hd; a.out = dxf; a.ldo = d; a.M = T; a.N = d;
    a.nb2 = ks_x; a.K = E / ks_x * hd; a.sL2 = (long long)(E / ks_x) * a.segL; a.sR2 = (long long)(E / ks_x) * a.segR;
    a.sO2 = (long long)T * d;
    MOA_TRY((launch_batched<false, false, true>(ic, a, s)));
  }
  moa_router_dx_kernel<<<dim3((T + kRouterTok - 1) / kRouterTok, (d + 255) / 256), dim3(256), 0, s>>>(
      dZ, static_cast<const bf16_t*>(w_r), T, d, E, dxf, ks_x, static_cast<bf16_t*>(dx));
  MOA_TRY(hipGetLastError());
#undef MOA_TRY
  return DSMOE_OK;
}

}  // extern "C"
