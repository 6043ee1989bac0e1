// Dense-training forward and backward of the MoE layer (paper Sec. 3.2 "Dense Training", Eq. 3):
// every expert runs on every token, O = sum_j S_j e_j(X), and the gradient flows through all of them.
//
// Forward      G_j = X W_gate[j], U_j = X W_up[j]              (kernel dense_gateup, grouped over j)
//              Ht[:, j] = S_j * silu(G_j) * U_j                (its epilogue; G, U, Ht kept for backward)
//              O = Ht [W_down[0]; ...; W_down[N-1]]             (one product over the concatenated width)
// Backward     Eq. 3: grad e_j(X) = S_j dO and grad S_j = <e_j(X), dO>.  With D_j = dO W_down[j]^T the
//              second is grad S_j = sum_c H_j[:, c] D_j[:, c] (H_j = silu(G_j) U_j), so the retained
//              expert outputs e_j(X) of the paper's formulation are never materialised.
//              dH_j = S_j D_j, dU_j = dH_j silu(G_j), dG_j = dH_j U_j silu'(G_j)    (kernel dense_bwd_dh)
//              dW_down[j] = Ht_j^T dO                                               (kernel dense_bwd_dwdown)
//              dW_gate[j] = X^T dG_j, dW_up[j] = X^T dU_j                           (kernel dense_bwd_dwgu)
//              dZ = S (dS - sum_k S_k dS_k)   (softmax), dW_r = X^T dZ, db_r = sum_t dZ
//              dX = sum_j dU_j W_up[j]^T + dG_j W_gate[j]^T + dZ W_r^T              (kernel dense_bwd_dx; the
//                   router term is one more K segment of the same contraction, with dZ in the storage type)
// All reductions have a fixed order: results are bitwise reproducible.
#include <algorithm>

#include "gemm.h"

namespace dsmoe {

namespace {

size_t al256(size_t v) { return (v + 255) / 256 * 256; }

template <typename T> struct DenseTiles;
template <> struct DenseTiles<float> { static constexpr int BM = 128, BN1 = 128, BN2 = 128; };
template <> struct DenseTiles<bf16_t> { static constexpr int BM = 256, BN1 = 256, BN2 = 128; };

struct SavedLayout { size_t S, G, U, Ht, total; };
SavedLayout saved_layout(const dsmoe_ctx* c, int T) {
  const size_t n = (size_t)T * c->desc.n_experts, nf = n * c->desc.d_ff * c->esize;
  SavedLayout l;
  size_t o = 0;
  l.S = o; o = al256(o + n * 4);
  l.G = o; o = al256(o + nf);
  l.U = o; o = al256(o + nf);
  l.Ht = o; o = al256(o + nf);
  l.total = o;
  return l;
}

constexpr int kWrTokens = 256;   // tokens per slab of the router weight-gradient kernel

// dU and dG are [T][E f + EP] matrices: the EP pad columns of dG hold dZ in the storage type, so that the
// router term of dX is one more K segment of the dG rows; W_r is repacked as [d][f] (first EP columns used)
// so that its rows have the pitch of the expert weights' rows.
struct ScratchLayout { size_t zeros, dU, dG, dS_part, dZ, WrP, dWr_part, mi_part, p_mean, total; int ntb, nsplit, EP; size_t ldg; };
ScratchLayout scratch_layout(const dsmoe_ctx* c, int T) {
  const size_t E = c->desc.n_experts, n = (size_t)T * E;
  const int bn1 = c->desc.dtype == DSMOE_BF16 ? DenseTiles<bf16_t>::BN1 : DenseTiles<float>::BN1;
  ScratchLayout l;
  l.ntb = (c->desc.d_ff + bn1 - 1) / bn1;
  l.nsplit = std::max(1, (T + kWrTokens - 1) / kWrTokens);
  l.EP = (c->desc.n_experts + 31) / 32 * 32;   // the router term of dX runs through the MFMA core: K padded to 32
  l.ldg = E * c->desc.d_ff + l.EP;
  const size_t nf = (size_t)T * l.ldg * c->esize;
  size_t o = 0;
  l.zeros = o; o = al256(o + 256);   // read in place of token rows past T by the token-contracted products
  l.dU = o; o = al256(o + nf);
  l.dG = o; o = al256(o + nf);
  l.dS_part = o; o = al256(o + n * l.ntb * 4);
  l.dZ = o; o = al256(o + n * 4);
  l.WrP = o; o = al256(o + (size_t)c->desc.d_model * c->desc.d_ff * c->esize);
  l.dWr_part = o; o = al256(o + (size_t)l.nsplit * c->desc.d_model * E * 4);
  l.mi_part = o; o = al256(o + (size_t)kStatMaxBlocks * 128 * 4);   // score statistics for the MI-loss gradient
  l.p_mean = o; o = al256(o + 64 * 4);
  l.total = o;
  return l;
}

__device__ __forceinline__ float sigmoid_f(float g) { return __builtin_amdgcn_rcpf(1.f + __expf(-g)); }
// exact GeLU g * Phi(g) and its derivative Phi(g) + g * phi(g) (the two-matrix expert of Sec. 4.1)
// Phi(g) and gelu'(g) = Phi(g) + g phi(g); for bf16 storage the cheaper Phi of gemm_core.h
template <typename T>
__device__ __forceinline__ float gelu_cdf_f(float g) {
  if constexpr (std::is_same_v<T, bf16_t>) return gelu_cdf_bf16_f(g);
  else return 0.5f * (1.f + erff(g * 0.70710678118654752f));
}
template <typename T>
__device__ __forceinline__ float gelu_prime_f(float g) {
  return gelu_cdf_f<T>(g) + g * 0.3989422804014327f * __expf(-0.5f * g * g);
}

// ---- forward: gate / up products of every expert on every token --------------------------------------
template <typename T>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN2, 2, false, true>::THREADS))
dense_gateup_kernel(const T* __restrict__ x, const T* __restrict__ w_gate, const T* __restrict__ w_up,
                    const float* __restrict__ S, T* __restrict__ G, T* __restrict__ U, T* __restrict__ Ht, int Tn,
                    int d, int f, int E) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN2, 2, false, true> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (Tn + GM::BM - 1) / GM::BM, n_nt = (f + GM::BN - 1) / GM::BN;
  const size_t EF = (size_t)E * f;
  TileWalker tw;
  tw.init(E * n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = (idx / n_nt) % n_mt, e = idx / (n_nt * n_mt);
    const int t0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::LSrc L;
    GM::l_rows(L, min(GM::BM, Tn - t0), 0, [&](int r) { return x + (size_t)(t0 + r) * d; });
    typename GM::RSrc R;
    const T* const base[2] = {w_gate + (size_t)e * d * f + n0, w_up + (size_t)e * d * f + n0};
    GM::r_cols(R, base, f, f - n0, d);
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, d / GM::BK, 1 << 30, st);
    if constexpr (std::is_same<T, bf16_t>::value) {
      // bf16: the three outputs are formed in the accumulator layout and cross the LDS already rounded
      // the scores of this lane's rows, read before the first store of the epilogue
      float srow[GM::TL::MT];
#pragma unroll
      for (int i = 0; i < GM::TL::MT; ++i) {
        const int t = t0 + GM::TL::acc_m(i);
        srow[i] = t < Tn ? S[(size_t)t * E + e] : 0.f;
      }
      auto pre = [&](int mt_i, int, int, const float (&v)[2][4], auto& out) {
        const float s = srow[mt_i];
        constexpr int NO = sizeof(out) / sizeof(out[0]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          out[NO - 1][i] = s * silu_f(v[0][i]) * v[1][i];
          if constexpr (NO == 3) { out[0][i] = v[0][i]; out[1][i] = v[1][i]; }
        }
      };
      if (G != nullptr)
        GM::TL::template for_each_chunk_bf16<3>(acc, st, pre, [&](int m, int n, const u32x4 (&p)[3]) {
          const int t = t0 + m, col = n0 + n;
          if (t >= Tn || col >= f) return;
          const size_t o = (size_t)t * EF + (size_t)e * f + col;
          stg16(G + o, p[0]);
          stg16(U + o, p[1]);
          stg16(Ht + o, p[2]);
        });
      else
        GM::TL::template for_each_chunk_bf16<1>(acc, st, pre, [&](int m, int n, const u32x4 (&p)[1]) {
          const int t = t0 + m, col = n0 + n;
          if (t >= Tn || col >= f) return;
          stg16(Ht + (size_t)t * EF + (size_t)e * f + col, p[0]);
        });
    } else {
      GM::for_each_chunk(acc, st, [&](int m, int n, const float (&v)[2][GM::CHUNK]) {
        const int t = t0 + m, col = n0 + n;
        if (t >= Tn || col >= f) return;
        const float s = S[(size_t)t * E + e];
        const size_t o = (size_t)t * EF + (size_t)e * f + col;
        if (G != nullptr) {
          store_chunk(G + o, v[0]);
          store_chunk(U + o, v[1]);
        }
        float h[GM::CHUNK];
#pragma unroll
        for (int i = 0; i < GM::CHUNK; ++i) h[i] = s * silu_f(v[0][i]) * v[1][i];
        store_chunk(Ht + o, h);
      });
    }
  }
}

// ---- forward, two-matrix GeLU expert: G = X W_1 of every expert on every token, Ht = S gelu(G) -----------
template <typename T>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, true>::THREADS))
dense_gelu1_kernel(const T* __restrict__ x, const T* __restrict__ w_1, const float* __restrict__ S, T* __restrict__ G,
                   T* __restrict__ Ht, int Tn, int d, int f, int E) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, true> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (Tn + GM::BM - 1) / GM::BM, n_nt = (f + GM::BN - 1) / GM::BN;
  const size_t EF = (size_t)E * f;
  TileWalker tw;
  tw.init(E * n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = (idx / n_nt) % n_mt, e = idx / (n_nt * n_mt);
    const int t0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::LSrc L;
    GM::l_rows(L, min(GM::BM, Tn - t0), 0, [&](int r) { return x + (size_t)(t0 + r) * d; });
    typename GM::RSrc R;
    const T* const base[1] = {w_1 + (size_t)e * d * f + n0};
    GM::r_cols(R, base, f, f - n0, d);
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, d / GM::BK, 1 << 30, st);
    float sq[GM::NJ];
    GM::for_each_chunk_loaded(
        acc, st,
        [&](int j, int m, int) { sq[j] = t0 + m < Tn ? S[(size_t)(t0 + m) * E + e] : 0.f; },
        [&](int j, int m, int n, const float (&v)[1][GM::CHUNK]) {
          const int t = t0 + m, col = n0 + n;
          if (t >= Tn || col >= f) return;
          const size_t o = (size_t)t * EF + (size_t)e * f + col;
          if (G != nullptr) store_chunk(G + o, v[0]);
          float h[GM::CHUNK];
#pragma unroll
          for (int i = 0; i < GM::CHUNK; ++i) h[i] = sq[j] * v[0][i] * gelu_cdf_f<T>(v[0][i]);
          store_chunk(Ht + o, h);
        });
  }
}

// ---- backward: D_j = dO W_down[j]^T, then the SwiGLU backward and the score-gradient partial sums -----
// GELU: the expert is gelu(x W_1) W_2: dG = S D gelu'(G), grad S partial = sum gelu(G) D; U and dU are not touched.
template <typename T, bool GELU>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, false>::THREADS))
dense_bwd_dh_kernel(const T* __restrict__ d_out, const T* __restrict__ w_down, const float* __restrict__ S,
                    const T* __restrict__ G, const T* __restrict__ U, T* __restrict__ dU, T* __restrict__ dG,
                    float* __restrict__ dS_part, int Tn, int d, int f, int E, size_t ldg) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, false> GM;
  DSMOE_GEMM_STAGES(GM, st);
  __shared__ float red[GM::WAVES_N][GM::BM];
  const int n_mt = (Tn + GM::BM - 1) / GM::BM, n_nt = (f + GM::BN - 1) / GM::BN;
  const size_t EF = (size_t)E * f;
  TileWalker tw;
  tw.init(E * n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = (idx / n_nt) % n_mt, e = idx / (n_nt * n_mt);
    const int t0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::LSrc L;
    GM::l_rows(L, min(GM::BM, Tn - t0), 0, [&](int r) { return d_out + (size_t)(t0 + r) * d; });
    typename GM::RSrc R;
    GM::r_rows(R, min(GM::BN, f - n0), 0, [&](int r) { return w_down + ((size_t)e * f + n0 + r) * d; });
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, d / GM::BK, 1 << 30, st);

    // calls for one tile row come in a run; the lanes sharing the row add their partial sums at its end
    float part = 0.f;
    int cur_m = -1;
    auto flush = [&]() {
      if (cur_m < 0) return;
      const float p = GM::row_sum(part);
      if (GM::row_leader()) red[GM::wave_n()][cur_m] = p;
    };
    // saved activations and the score of each chunk, requested a 32-row block ahead of their use
    u32x4 gq[GM::NJ], uq[GM::NJ];
    float sq[GM::NJ];
    GM::for_each_chunk_loaded(
        acc, st,
        [&](int j, int m, int n) {
          const int t = t0 + m, col = n0 + n;
          if (t >= Tn || col >= f) return;
          const size_t o = (size_t)t * EF + (size_t)e * f + col;
          gq[j] = load_raw(G + o);
          if constexpr (!GELU) uq[j] = load_raw(U + o);
          sq[j] = S[(size_t)t * E + e];
        },
        [&](int j, int m, int n, const float (&v)[1][GM::CHUNK]) {
          if (m != cur_m) { flush(); cur_m = m; part = 0.f; }
          const int t = t0 + m, col = n0 + n;
          if (t >= Tn || col >= f) return;
          const float s = sq[j];
          const size_t od = (size_t)t * ldg + (size_t)e * f + col;
          float g[GM::CHUNK], u[GM::CHUNK], du[GM::CHUNK], dg[GM::CHUNK];
          unpack_chunk(gq[j], g, (const T*)nullptr);
          if constexpr (GELU) {
#pragma unroll
            for (int i = 0; i < GM::CHUNK; ++i) {
              part = fmaf(g[i] * gelu_cdf_f<T>(g[i]), v[0][i], part);
              dg[i] = s * v[0][i] * gelu_prime_f<T>(g[i]);
            }
            store_chunk(dG + od, dg);
            return;
          }
          unpack_chunk(uq[j], u, (const T*)nullptr);
#pragma unroll
          for (int i = 0; i < GM::CHUNK; ++i) {
            const float sg = sigmoid_f(g[i]), sl = g[i] * sg;
            part = fmaf(sl * u[i], v[0][i], part);
            const float dh = s * v[0][i];
            du[i] = dh * sl;
            dg[i] = dh * u[i] * (sg * (1.f + g[i] * (1.f - sg)));
          }
          store_chunk(dU + od, du);
          store_chunk(dG + od, dg);
        });
    flush();
    __syncthreads();
    for (int m = threadIdx.x; m < GM::BM; m += GM::THREADS) {
      const int t = t0 + m;
      if (t >= Tn) continue;
      float p = red[0][m];
#pragma unroll
      for (int w = 1; w < GM::WAVES_N; ++w) p += red[w][m];
      dS_part[((size_t)t * E + e) * n_nt + nt] = p;
    }
    // the next tile's main loop passes barriers before `red` is written again
  }
}

// ---- backward: out[j] = A_j^T B_j, contraction over tokens ------------------------------------------------
// A_j = A[:, j * a_es .. + M), B_j = B[:, j * b_es .. + N) (row pitches lda, ldb); out[j] is [M][N].
// dW_down[j] = Ht_j^T dO (a_es = f, b_es = 0) and, for the two-matrix expert, dW_1[j] = X^T dG_j (a_es = 0, b_es = f).
template <typename T>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, true, true, true>::THREADS))
dense_bwd_dwdown_kernel(const T* __restrict__ A, size_t lda, int a_es, int M, const T* __restrict__ B, size_t ldb,
                        int b_es, int N, float* __restrict__ out, int Tn, int E, const void* __restrict__ zeros) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, true, true, true> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (M + GM::BM - 1) / GM::BM, n_nt = (N + GM::BN - 1) / GM::BN;
  TileWalker tw;
  tw.init(E * n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = (idx / n_nt) % n_mt, e = idx / (n_nt * n_mt);
    const int m0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::LSrc L;
    GM::l_cols(L, A + (size_t)e * a_es + m0, lda, M - m0, Tn, zeros);
    typename GM::RSrc R;
    const T* const base[1] = {B + (size_t)e * b_es + n0};
    GM::r_cols(R, base, ldb, N - n0, Tn, zeros);
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, (Tn + GM::BK - 1) / GM::BK, 1 << 30, st);
    GM::for_each_chunk(acc, st, [&](int m, int n, const float (&v)[1][GM::CHUNK]) {
      if (m0 + m >= M || n0 + n >= N) return;
      store_chunk(out + ((size_t)e * M + m0 + m) * N + n0 + n, v[0]);
    });
  }
}

// ---- backward: dW_gate[j] = X^T dG_j, dW_up[j] = X^T dU_j ---------------------------------------------
template <typename T>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN2, 2, true, true, true>::THREADS))
dense_bwd_dwgu_kernel(const T* __restrict__ x, const T* __restrict__ dG, const T* __restrict__ dU,
                      float* __restrict__ dw_gate, float* __restrict__ dw_up, int Tn, int d, int f, int E,
                      size_t ldg, const void* __restrict__ zeros) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN2, 2, true, true, true> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (d + GM::BM - 1) / GM::BM, n_nt = (f + GM::BN - 1) / GM::BN;
  TileWalker tw;
  tw.init(E * n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = (idx / n_nt) % n_mt, e = idx / (n_nt * n_mt);
    const int m0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::LSrc L;
    GM::l_cols(L, x + m0, d, d - m0, Tn, zeros);
    typename GM::RSrc R;
    const T* const base[2] = {dG + (size_t)e * f + n0, dU + (size_t)e * f + n0};
    GM::r_cols(R, base, ldg, f - n0, Tn, zeros);
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, (Tn + GM::BK - 1) / GM::BK, 1 << 30, st);
    GM::for_each_chunk(acc, st, [&](int m, int n, const float (&v)[2][GM::CHUNK]) {
      if (m0 + m >= d || n0 + n >= f) return;
      const size_t o = ((size_t)e * d + m0 + m) * f + n0 + n;
      store_chunk(dw_gate + o, v[0]);
      store_chunk(dw_up + o, v[1]);
    });
  }
}

// ---- backward: dX = sum_j dU_j W_up[j]^T + dG_j W_gate[j]^T + dZ W_r^T -----------------------------------
// GELU: dX = sum_j dG_j W_1[j]^T + dZ W_r^T (no up projection).
template <typename T, bool GELU>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, false>::THREADS))
dense_bwd_dx_kernel(const T* __restrict__ dU, const T* __restrict__ dG, const T* __restrict__ w_up,
                    const T* __restrict__ w_gate, const T* __restrict__ w_rp, T* __restrict__ dx, int Tn, int d, int f,
                    int E, int EP, size_t ldg) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, false> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (Tn + GM::BM - 1) / GM::BM, n_nt = (d + GM::BN - 1) / GM::BN;
  const size_t EF = (size_t)E * f;
  const T* dZt = dG + EF;   // the pad columns of dG
  TileWalker tw;
  tw.init(n_mt * n_nt);
  int idx;
  while (tw.next(idx)) {
    const int nt = idx % n_nt, mt = idx / n_nt;
    const int t0 = mt * GM::BM, n0 = nt * GM::BN;
    typename GM::Acc acc;
    GM::zero(acc);
    if constexpr (std::is_same<T, bf16_t>::value) {
      // One K loop over 2 E + 1 segments: dU_j W_up[j]^T (j < E), dG_j W_gate[j]^T, then the router term
      // dZ W_r^T.  The token side runs on from dU into dG (segment E) and on into dG's pad columns; the weight
      // side runs on from W_up into W_gate and then into the repacked W_r: the row pitches are the same, so
      // each switch is a uniform address offset.
      typename GM::LSrc L;
      typename GM::RSrc R;
      const long long segL = (long long)f * sizeof(T), segR = (long long)d * f * sizeof(T);
      if constexpr (GELU) {
        // E segments dG_j W_1[j]^T, then dG's pad columns against the repacked W_r
        GM::l_rows(L, min(GM::BM, Tn - t0), (size_t)segL, [&](int r) { return dG + (size_t)(t0 + r) * ldg; });
        GM::r_rows(R, min(GM::BN, d - n0), (size_t)segR, [&](int r) { return w_gate + (size_t)(n0 + r) * f; });
        R.set_jump(0, E, ((const char*)w_rp - (const char*)w_gate) - E * segR);
        GM::mainloop(acc, L, R, (int)(EF / GM::BK) + EP / GM::BK, f / GM::BK, st);
      } else {
        GM::l_rows(L, min(GM::BM, Tn - t0), (size_t)segL, [&](int r) { return dU + (size_t)(t0 + r) * ldg; });
        GM::r_rows(R, min(GM::BN, d - n0), (size_t)segR, [&](int r) { return w_up + (size_t)(n0 + r) * f; });
        const long long dL = (const char*)dG - (const char*)dU, dR1 = (const char*)w_gate - (const char*)w_up,
                        dR2 = (const char*)w_rp - (const char*)w_up;
        L.set_jump(0, E, dL - E * segL);
        R.set_jump(0, E, dR1 - E * segR);
        R.set_jump(1, 2 * E, dR2 - dR1 - E * segR);
        GM::mainloop(acc, L, R, 2 * (int)(EF / GM::BK) + EP / GM::BK, f / GM::BK, st);
      }
    } else {
#pragma unroll 1
      for (int part = GELU ? 1 : 0; part < 3; ++part) {
        typename GM::LSrc L;
        typename GM::RSrc R;
        if (part < 2) {
          // K runs over (expert, hidden unit): one segment of f per expert on both sides
          const T* a = part ? dG : dU;
          const T* w = part ? w_gate : w_up;
          GM::l_rows(L, min(GM::BM, Tn - t0), (size_t)f * sizeof(T), [&](int r) { return a + (size_t)(t0 + r) * ldg; });
          GM::r_rows(R, min(GM::BN, d - n0), (size_t)d * f * sizeof(T), [&](int r) { return w + (size_t)(n0 + r) * f; });
          GM::mainloop(acc, L, R, (int)(EF / GM::BK), f / GM::BK, st);
        } else {
          // router path: K runs over the (padded) experts
          GM::l_rows(L, min(GM::BM, Tn - t0), 0, [&](int r) { return dZt + (size_t)(t0 + r) * ldg; });
          GM::r_rows(R, min(GM::BN, d - n0), 0, [&](int r) { return w_rp + (size_t)(n0 + r) * f; });
          GM::mainloop(acc, L, R, EP / GM::BK, 1 << 30, st);
        }
      }
    }
    GM::for_each_chunk(acc, st, [&](int m, int n, const float (&v)[1][GM::CHUNK]) {
      const int t = t0 + m, col = n0 + n;
      if (t >= Tn || col >= d) return;
      store_chunk(dx + (size_t)t * d + col, v[0]);
    });
  }
}

// ---- softmax backward: dZ = S (dS - sum_k S_k dS_k), one wave per token, one lane per expert -------------
template <typename T>
__global__ void __launch_bounds__(kThreads)
dense_softmax_bwd_kernel(const float* __restrict__ S, const float* __restrict__ dS_part, int ntb, int Tn, int E, int EP,
                         float* __restrict__ dZ, T* __restrict__ dZt, size_t ldz, unsigned* __restrict__ zeros,
                         const float* __restrict__ p_mean, float alpha_over_T) {
  if (blockIdx.x == 0 && threadIdx.x < 64) zeros[threadIdx.x] = 0u;   // the zero page of the later kernels
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  float s = 0.f, ds = 0.f;
  if (lane < E) {
    s = S[(size_t)t * E + lane];
    for (int j = 0; j < ntb; ++j) ds += dS_part[((size_t)t * E + lane) * ntb + j];
    // gradient of alpha * L_MI w.r.t. the score (Eq. 4-6): alpha (log p_i - log S[t,i]) / T; a score that
    // underflowed to 0 gets none (its factor S in the softmax backward is 0 anyway)
    if (p_mean != nullptr && s > 0.f) ds += alpha_over_T * (logf(p_mean[lane]) - logf(s));
  }
  float dot = s * ds;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
  const float dz = s * (ds - dot);
  if (lane < E) dZ[(size_t)t * E + lane] = dz;
  if (lane < EP) dZt[(size_t)t * ldz + lane] = (T)(lane < E ? dz : 0.f);
}

// ---- router weight gradient: partial dW_r = X^T dZ over a slab of tokens, through the MFMA core ---------------
// (dZ in the storage type, padded to EP columns); the slabs are added in order by the reduce kernel.
template <typename T>
__global__ void __launch_bounds__((Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, true, true, true>::THREADS))
dense_router_dw_kernel(const T* __restrict__ x, const T* __restrict__ dZt, size_t ldz, int Tn, int d, int E, int EP,
                       int nsplit, float* __restrict__ dWr_part, const void* __restrict__ zeros) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, true, true, true> GM;
  DSMOE_GEMM_STAGES(GM, st);
  const int n_mt = (d + GM::BM - 1) / GM::BM;
  TileWalker tw;
  tw.init(n_mt * nsplit);
  int idx;
  while (tw.next(idx)) {
    const int mt = idx % n_mt, ks = idx / n_mt;
    const int m0 = mt * GM::BM, k0 = ks * kWrTokens, kv = min(kWrTokens, Tn - k0);
    typename GM::LSrc L;
    GM::l_cols(L, x + (size_t)k0 * d + m0, d, d - m0, kv, zeros);
    typename GM::RSrc R;
    const T* const base[1] = {dZt + (size_t)k0 * ldz};
    GM::r_cols(R, base, ldz, EP, kv, zeros);
    typename GM::Acc acc;
    GM::zero(acc);
    GM::mainloop(acc, L, R, (kv + GM::BK - 1) / GM::BK, 1 << 30, st);
    float* out = dWr_part + (size_t)ks * d * E;
    GM::for_each_chunk(acc, st, [&](int m, int n, const float (&v)[1][GM::CHUNK]) {
      if (m0 + m >= d || n >= E) return;
      store_chunk(out + (size_t)(m0 + m) * E + n, v[0]);
    });
  }
}

__global__ void __launch_bounds__(kThreads)
dense_router_dw_reduce_kernel(const float* __restrict__ dWr_part, int nsplit, int n, float* __restrict__ dw_r) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int k = 0; k < nsplit; ++k) s += dWr_part[(size_t)k * n + i];
  dw_r[i] = s;
}

// db_r[e] = sum_t dZ[t, e]: one block per expert, strided partial sums, then a fixed-order tree
__global__ void __launch_bounds__(kThreads)
dense_router_db_kernel(const float* __restrict__ dZ, int Tn, int E, float* __restrict__ db_r) {
  __shared__ float sSum[kThreads];
  const int e = blockIdx.x;
  float s = 0.f;
  for (int t = threadIdx.x; t < Tn; t += kThreads) s += dZ[(size_t)t * E + e];
  sSum[threadIdx.x] = s;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sSum[threadIdx.x] += sSum[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) db_r[e] = sSum[0];
}

// w_rp[i][0..EP) = w_r[i][0..E) followed by zeros; rows of pitch ld
template <typename T>
__global__ void __launch_bounds__(kThreads)
dense_pad_wr_kernel(const T* __restrict__ w_r, int d, int E, int EP, int ld, T* __restrict__ w_rp) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= d * EP) return;
  const int row = i / EP, e = i % EP;
  w_rp[(size_t)row * ld + e] = e < E ? w_r[(size_t)row * E + e] : (T)0.f;
}

template <typename K>
hipError_t set_lds(K kernel, int bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

int grid_for(const dsmoe_ctx* c, long tiles, int blocks_per_cu) {
  const long full = (long)c->n_cu * blocks_per_cu;
  return (int)((std::min(tiles, full) + 7) / 8 * 8);
}

template <typename T>
hipError_t dense_fwd_t(const dsmoe_ctx* c, const void* x, const void* w_gate, const void* w_up, const void* w_down,
                       int Tn, const float* S, T* G, T* U, T* Ht, void* out, hipStream_t s) {
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN2, 2, false, true> GM;
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  constexpr int bpc = sizeof(T) == 4 ? 2 : 1;
  typedef Gemm<T, DenseTiles<T>::BM, DenseTiles<T>::BN1, 1, false, true> GM1;
  static bool attrs = false;
  if (!attrs) {
    if (hipError_t e = set_lds(dense_gateup_kernel<T>, GM::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_gelu1_kernel<T>, GM1::LDS_BYTES)) return e;
    attrs = true;
  }
  if (c->expert_kind == DSMOE_EXPERT_GELU) {
    const long tiles = (long)E * ((Tn + GM1::BM - 1) / GM1::BM) * ((f + GM1::BN - 1) / GM1::BN);
    dense_gelu1_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GM1::THREADS), GM1::LDS_BYTES, s>>>(
        (const T*)x, (const T*)w_gate, S, G, Ht, Tn, d, f, E);
  } else {
    const long tiles = (long)E * ((Tn + GM::BM - 1) / GM::BM) * ((f + GM::BN - 1) / GM::BN);
    dense_gateup_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GM::THREADS), GM::LDS_BYTES, s>>>(
        (const T*)x, (const T*)w_gate, (const T*)w_up, S, G, U, Ht, Tn, d, f, E);
  }
  if (hipError_t e = hipGetLastError()) return e;
  return launch_down_dense(c, Ht, Tn, E * f, w_down, out, s);
}

template <typename T>
hipError_t dense_bwd_t(const dsmoe_ctx* c, const void* x, const void* w_r, const void* w_gate, const void* w_up,
                       const void* w_down, const char* saved, const void* d_out, int Tn, char* scratch, void* dx,
                       float* dw_r, float* db_r, float* dw_gate, float* dw_up, float* dw_down, float mi_alpha,
                       hipStream_t s) {
  typedef DenseTiles<T> DT;
  typedef Gemm<T, DT::BM, DT::BN1, 1, false, false> GRR;
  typedef Gemm<T, DT::BM, DT::BN1, 1, true, true, true> GCC1;
  typedef Gemm<T, DT::BM, DT::BN2, 2, true, true, true> GCC2;
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  constexpr int bpc = sizeof(T) == 4 ? 2 : 1;
  const SavedLayout sv = saved_layout(c, Tn);
  const ScratchLayout sc = scratch_layout(c, Tn);
  const float* S = reinterpret_cast<const float*>(saved + sv.S);
  const T* G = reinterpret_cast<const T*>(saved + sv.G);
  const T* U = reinterpret_cast<const T*>(saved + sv.U);
  const T* Ht = reinterpret_cast<const T*>(saved + sv.Ht);
  T* dU = reinterpret_cast<T*>(scratch + sc.dU);
  T* dG = reinterpret_cast<T*>(scratch + sc.dG);
  float* dS_part = reinterpret_cast<float*>(scratch + sc.dS_part);
  float* dZ = reinterpret_cast<float*>(scratch + sc.dZ);
  T* dZt = dG + (size_t)E * f;   // the pad columns of dG, row pitch sc.ldg
  T* w_rp = reinterpret_cast<T*>(scratch + sc.WrP);
  float* dWr_part = reinterpret_cast<float*>(scratch + sc.dWr_part);
  auto cdiv = [](long a, long b) { return (a + b - 1) / b; };

  static bool attrs = false;
  if (!attrs) {
    if (hipError_t e = set_lds(dense_bwd_dh_kernel<T, false>, GRR::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_bwd_dh_kernel<T, true>, GRR::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_bwd_dx_kernel<T, false>, GRR::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_bwd_dx_kernel<T, true>, GRR::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_bwd_dwdown_kernel<T>, GCC1::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_router_dw_kernel<T>, GCC1::LDS_BYTES)) return e;
    if (hipError_t e = set_lds(dense_bwd_dwgu_kernel<T>, GCC2::LDS_BYTES)) return e;
    attrs = true;
  }

  const bool gelu = c->expert_kind == DSMOE_EXPERT_GELU;
  long tiles = E * cdiv(Tn, DT::BM) * cdiv(f, DT::BN1);
  if (gelu)
    dense_bwd_dh_kernel<T, true><<<dim3(grid_for(c, tiles, bpc)), dim3(GRR::THREADS), GRR::LDS_BYTES, s>>>(
        (const T*)d_out, (const T*)w_down, S, G, U, dU, dG, dS_part, Tn, d, f, E, sc.ldg);
  else
    dense_bwd_dh_kernel<T, false><<<dim3(grid_for(c, tiles, bpc)), dim3(GRR::THREADS), GRR::LDS_BYTES, s>>>(
        (const T*)d_out, (const T*)w_down, S, G, U, dU, dG, dS_part, Tn, d, f, E, sc.ldg);
  if (hipError_t e = hipGetLastError()) return e;

  const float* p_mean = nullptr;
  if (mi_alpha != 0.f) {   // batch means of the scores for the gradient of the MI loss
    float* pm = reinterpret_cast<float*>(scratch + sc.p_mean);
    if (hipError_t e = launch_mi_loss(c, S, Tn, reinterpret_cast<float*>(scratch + sc.mi_part), pm, nullptr, s)) return e;
    p_mean = pm;
  }
  dense_softmax_bwd_kernel<T><<<dim3((Tn + 3) / 4), dim3(kThreads), 0, s>>>(
      S, dS_part, sc.ntb, Tn, E, sc.EP, dZ, dZt, sc.ldg, reinterpret_cast<unsigned*>(scratch + sc.zeros), p_mean,
      mi_alpha / (float)Tn);
  if (hipError_t e = hipGetLastError()) return e;

  dense_pad_wr_kernel<T><<<dim3((d * sc.EP + kThreads - 1) / kThreads), dim3(kThreads), 0, s>>>(
      (const T*)w_r, d, E, sc.EP, f, w_rp);
  if (hipError_t e = hipGetLastError()) return e;
  tiles = cdiv(d, DT::BM) * sc.nsplit;
  dense_router_dw_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GCC1::THREADS), GCC1::LDS_BYTES, s>>>(
      (const T*)x, dZt, sc.ldg, Tn, d, E, sc.EP, sc.nsplit, dWr_part, scratch + sc.zeros);
  if (hipError_t e = hipGetLastError()) return e;
  dense_router_dw_reduce_kernel<<<dim3((d * E + kThreads - 1) / kThreads), dim3(kThreads), 0, s>>>(dWr_part, sc.nsplit,
                                                                                                  d * E, dw_r);
  if (hipError_t e = hipGetLastError()) return e;
  if (db_r != nullptr) {
    dense_router_db_kernel<<<dim3(E), dim3(kThreads), 0, s>>>(dZ, Tn, E, db_r);
    if (hipError_t e = hipGetLastError()) return e;
  }

  tiles = E * cdiv(f, DT::BM) * cdiv(d, DT::BN1);
  dense_bwd_dwdown_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GCC1::THREADS), GCC1::LDS_BYTES, s>>>(
      Ht, (size_t)E * f, f, f, (const T*)d_out, (size_t)d, 0, d, dw_down, Tn, E, scratch + sc.zeros);
  if (hipError_t e = hipGetLastError()) return e;

  if (gelu) {   // dW_1[j] = X^T dG_j
    tiles = E * cdiv(d, DT::BM) * cdiv(f, DT::BN1);
    dense_bwd_dwdown_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GCC1::THREADS), GCC1::LDS_BYTES, s>>>(
        (const T*)x, (size_t)d, 0, d, dG, sc.ldg, f, f, dw_gate, Tn, E, scratch + sc.zeros);
  } else {
    tiles = E * cdiv(d, DT::BM) * cdiv(f, DT::BN2);
    dense_bwd_dwgu_kernel<T><<<dim3(grid_for(c, tiles, bpc)), dim3(GCC2::THREADS), GCC2::LDS_BYTES, s>>>(
        (const T*)x, dG, dU, dw_gate, dw_up, Tn, d, f, E, sc.ldg, scratch + sc.zeros);
  }
  if (hipError_t e = hipGetLastError()) return e;

  tiles = cdiv(Tn, DT::BM) * cdiv(d, DT::BN1);
  if (gelu)
    dense_bwd_dx_kernel<T, true><<<dim3(grid_for(c, tiles, bpc)), dim3(GRR::THREADS), GRR::LDS_BYTES, s>>>(
        dU, dG, (const T*)w_up, (const T*)w_gate, w_rp, (T*)dx, Tn, d, f, E, sc.EP, sc.ldg);
  else
    dense_bwd_dx_kernel<T, false><<<dim3(grid_for(c, tiles, bpc)), dim3(GRR::THREADS), GRR::LDS_BYTES, s>>>(
        dU, dG, (const T*)w_up, (const T*)w_gate, w_rp, (T*)dx, Tn, d, f, E, sc.EP, sc.ldg);
  return hipGetLastError();
}

}  // namespace

size_t dense_saved_bytes(const dsmoe_ctx* c, int T) { return saved_layout(c, T).total; }
size_t dense_bwd_scratch_bytes(const dsmoe_ctx* c, int T) { return scratch_layout(c, T).total; }

hipError_t launch_dense_fwd(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                            const void* w_up, const void* w_down, int T, void* out, float* probs, void* saved,
                            hipStream_t s) {
  const int E = c->desc.n_experts;
  char* sv = static_cast<char*>(saved);
  const SavedLayout l = saved_layout(c, T);
  float* S = sv ? reinterpret_cast<float*>(sv + l.S) : (probs ? probs : reinterpret_cast<float*>(c->workspace + c->ws.probs));
  if (hipError_t e = launch_route(c, x, w_r, b_r, T, S, -1, 0, 0.f, nullptr, nullptr, s)) return e;
  if (probs != nullptr && probs != S)
    if (hipError_t e = hipMemcpyAsync(probs, S, (size_t)T * E * 4, hipMemcpyDeviceToDevice, s)) return e;
  void* G = sv ? sv + l.G : nullptr;
  void* U = sv ? sv + l.U : nullptr;
  void* Ht = sv ? sv + l.Ht : c->workspace + c->ws.h;
  if (c->desc.dtype == DSMOE_BF16)
    return dense_fwd_t<bf16_t>(c, x, w_gate, w_up, w_down, T, S, (bf16_t*)G, (bf16_t*)U, (bf16_t*)Ht, out, s);
  return dense_fwd_t<float>(c, x, w_gate, w_up, w_down, T, S, (float*)G, (float*)U, (float*)Ht, out, s);
}

hipError_t launch_dense_bwd(const dsmoe_ctx* c, const void* x, const void* w_r, const void* w_gate, const void* w_up,
                            const void* w_down, const void* saved, const void* d_out, int T, void* scratch, void* dx,
                            float* dw_r, float* db_r, float* dw_gate, float* dw_up, float* dw_down, float mi_alpha,
                            hipStream_t s) {
  if (c->desc.dtype == DSMOE_BF16)
    return dense_bwd_t<bf16_t>(c, x, w_r, w_gate, w_up, w_down, (const char*)saved, d_out, T, (char*)scratch, dx, dw_r,
                               db_r, dw_gate, dw_up, dw_down, mi_alpha, s);
  return dense_bwd_t<float>(c, x, w_r, w_gate, w_up, w_down, (const char*)saved, d_out, T, (char*)scratch, dx, dw_r,
                            db_r, dw_gate, dw_up, dw_down, mi_alpha, s);
}

}  // namespace dsmoe
