// Grouped per-expert SwiGLU FFN on dispatched rows: the e_i(X) of Eq. 1 (paper Sec. 3.1), evaluated
// only for the (token, expert) pairs kept by the selection (Sec. 3.2 "Sparse Inference").
//
//   kernel 1 (gate/up):  H[r,:] = silu(x_r W_gate[e]) * (x_r W_up[e])   rows r of expert e
//   kernel 2 (down):     Y[r,:] = H[r,:] W_down[e]
//
// With the paper's own two-matrix GeLU expert (Sec. 4.1) kernel 1 is the same grouped product as kernel 2 with
// gathered rows and the activation in its epilogue:  H[r,:] = gelu(x_r W_1[e]),  Y[r,:] = H[r,:] W_2[e].
//
// Both are persistent grids walking a tile list derived on the device from expert_off, so no host
// synchronisation is needed to learn the data-dependent row counts.  Token rows are gathered
// through row_token while staging the L operand (no permuted copy of X is required).
#include <algorithm>

#include "gemm.h"

namespace dsmoe {

template <typename T, int BM, int BN>
__global__ void __launch_bounds__(kThreads, 2)
gateup_kernel(const T* __restrict__ x, const T* __restrict__ x_perm, const int32_t* __restrict__ row_token,
              const int32_t* __restrict__ expert_off, const T* __restrict__ w_gate, const T* __restrict__ w_up,
              T* __restrict__ h, int d, int f, int E) {
  typedef Tile<T, BM, BN, 2> TL;
  extern __shared__ __align__(16) char smem[];
  __shared__ GroupTiles gt;
  build_group_tiles(gt, expert_off, E, BM);
  const int n_tiles = (f + BN - 1) / BN;
  TileWalker tw;
  tw.init(gt.tile_off[E] * n_tiles);
  int idx;
  while (tw.next(idx)) {
    const int nt_blk = idx % n_tiles, mg = idx / n_tiles;
    const int e = find_group(gt, E, mg);
    const int m0 = (mg - gt.tile_off[e]) * BM;
    const int row0 = gt.row_off[e] + m0;
    const int valid = min(BM, gt.row_off[e + 1] - row0);
    const int n0 = nt_blk * BN;

    SrcRows<T, BM> L;
    L.seg_stride = 0;
#pragma unroll
    for (int i = 0; i < SrcRows<T, BM>::NV; ++i) {
      const int r = min((int)(threadIdx.x >> 3) + 32 * i, valid - 1);
      const T* src = x_perm ? x_perm + (size_t)(row0 + r) * d : x + (size_t)row_token[row0 + r] * d;
      L.p[i] = reinterpret_cast<const char*>(src) + (threadIdx.x & 7) * 16;
    }
    SrcCols<T, BN> R[2];
    R[0].base = reinterpret_cast<const char*>(w_gate + (size_t)e * d * f + n0);
    R[1].base = reinterpret_cast<const char*>(w_up + (size_t)e * d * f + n0);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      R[b].ld_bytes = (size_t)f * sizeof(T);
      R[b].seg_stride = 0;
      R[b].rows_valid = min(BN, f - n0);
      R[b].k_valid = d;
    }
    typename TL::Acc acc;
    TL::zero(acc);
    TL::mainloop(acc, L, R, d / TL::BK, 1 << 30, smem);

#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt) {
      const int m = TL::acc_m(mt);
      if (m >= valid) continue;
      T* hrow = h + (size_t)(row0 + m) * f + n0;
#pragma unroll
      for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = TL::acc_n(nt, g);
          if (n0 + n >= f) continue;
          const f32x16& G = acc[0][nt][mt];
          const f32x16& U = acc[1][nt][mt];
          store4(hrow + n, silu_f(G[4 * g]) * U[4 * g], silu_f(G[4 * g + 1]) * U[4 * g + 1],
                 silu_f(G[4 * g + 2]) * U[4 * g + 2], silu_f(G[4 * g + 3]) * U[4 * g + 3]);
        }
    }
  }
}

// Grouped product out[r, 0..d) = act(in[row(r), 0..f) W[e]) over the rows r of each expert e: the down projection
// (GELU = false, rows read in place) and the first product of the GeLU expert (GELU = true, rows gathered
// through row_token when GATHER).  d: output width, f: contraction length.
template <typename T, int BM, int BN, bool GELU = false, bool GATHER = false>
__global__ void __launch_bounds__(kThreads, 2)
down_kernel(const T* __restrict__ h, const int32_t* __restrict__ row_token, const int32_t* __restrict__ expert_off,
            const T* __restrict__ w_down, T* __restrict__ y, int d, int f, int E, int uniform_rows) {
  typedef Tile<T, BM, BN, 1> TL;
  extern __shared__ __align__(16) char smem[];
  __shared__ GroupTiles gt;
  build_group_tiles(gt, expert_off, E, BM, uniform_rows);
  const int n_tiles = (d + BN - 1) / BN;
  TileWalker tw;
  tw.init(gt.tile_off[E] * n_tiles);
  int idx;
  while (tw.next(idx)) {
    const int nt_blk = idx % n_tiles, mg = idx / n_tiles;
    const int e = find_group(gt, E, mg);
    const int m0 = (mg - gt.tile_off[e]) * BM;
    const int row0 = gt.row_off[e] + m0;
    const int valid = min(BM, gt.row_off[e + 1] - row0);
    const int n0 = nt_blk * BN;

    SrcRows<T, BM> L;
    L.seg_stride = 0;
#pragma unroll
    for (int i = 0; i < SrcRows<T, BM>::NV; ++i) {
      const int r = min((int)(threadIdx.x >> 3) + 32 * i, valid - 1);
      const size_t src_row = GATHER ? (size_t)row_token[row0 + r] : (size_t)(row0 + r);
      L.p[i] = reinterpret_cast<const char*>(h + src_row * f) + (threadIdx.x & 7) * 16;
    }
    SrcCols<T, BN> R[1];
    R[0].base = reinterpret_cast<const char*>(w_down + (size_t)e * f * d + n0);
    R[0].ld_bytes = (size_t)d * sizeof(T);
    R[0].seg_stride = 0;
    R[0].rows_valid = min(BN, d - n0);
    R[0].k_valid = f;
    typename TL::Acc acc;
    TL::zero(acc);
    TL::mainloop(acc, L, R, f / TL::BK, 1 << 30, smem);

#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt) {
      const int m = TL::acc_m(mt);
      if (m >= valid) continue;
      T* yrow = y + (size_t)(row0 + m) * d + n0;
#pragma unroll
      for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = TL::acc_n(nt, g);
          if (n0 + n >= d) continue;
          const f32x16& A = acc[0][nt][mt];
          if (GELU) store4(yrow + n, gelu_f(A[4 * g]), gelu_f(A[4 * g + 1]), gelu_f(A[4 * g + 2]), gelu_f(A[4 * g + 3]));
          else store4(yrow + n, A[4 * g], A[4 * g + 1], A[4 * g + 2], A[4 * g + 3]);
        }
    }
  }
}

// ---- bf16: 256-row tiles, 8 waves, direct global -> LDS loads -------------------------------------------
// Both kernels walk their tiles in two passes (SplitWalker): 256-row tiles, then 128-row tiles for the short
// ends of experts and for an uneven last turn of the grid.  Each pass is software-pipelined over its tiles:
// the first K steps of the next tile are requested before the epilogue of the current one.
template <class TL, class Next, class Setup, class Epi>
__device__ __forceinline__ void tile_pipeline(const Stages3& st, int nkt, Next next, Setup setup, Epi epi) {
  RowTile cur;
  if (!next(cur)) return;
  typename TL::LSrc L;
  typename TL::RSrc R;
  typename TL::Iter it;
  setup(cur, L, R);
  TL::prefetch(L, R, it, nkt, 1 << 30, st);
  while (true) {
    typename TL::Acc acc;
    TL::zero(acc);
    TL::run(acc, L, R, it, nkt, 1 << 30, st);
    RowTile nxt;
    typename TL::LSrc Ln;
    typename TL::RSrc Rn;
    typename TL::Iter itn;
    const bool more = next(nxt);
    if (more) {
      setup(nxt, Ln, Rn);
      TL::prefetch(Ln, Rn, itn, nkt, 1 << 30, st);
    }
    epi(cur, acc);
    if (!more) break;
    cur = nxt; L = Ln; R = Rn; it = itn;
  }
}

// The same walk with the load pipeline running on from tile to tile (Tile3::run_chain): the next tile is set
// up before the current one starts, and epi may use stage NST-1 only.
template <class TL, class Next, class Setup, class Epi>
__device__ __forceinline__ void tile_chain(const Stages3& st, int nkt, Next next, Setup setup, Epi epi) {
  RowTile cur;
  if (!next(cur)) return;
  typename TL::LSrc L;
  typename TL::RSrc R;
  typename TL::Iter it;
  setup(cur, L, R);
  TL::chain_begin(L, R, it, nkt, st);
  while (true) {
    RowTile nxt;
    typename TL::LSrc Ln = L;
    typename TL::RSrc Rn = R;
    typename TL::Iter itn = it;
    const bool more = next(nxt);
    if (more) {
      setup(nxt, Ln, Rn);
      itn.seg = 0; itn.kin = 0; itn.next = 0;
    }
    typename TL::Acc acc;
    TL::zero(acc);
    TL::run_chain(acc, L, R, it, Ln, Rn, itn, nkt, st);
    epi(cur, acc);
    if (!more) break;
    cur = nxt; L = Ln; R = Rn; it = itn;
  }
}

template <int BM>
__global__ void __launch_bounds__(kThreads2)
gateup_bf16_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ x_perm, const int32_t* __restrict__ row_token,
                   const int32_t* __restrict__ expert_off, const bf16_t* __restrict__ w_gate,
                   const bf16_t* __restrict__ w_up, bf16_t* __restrict__ h, int d, int f, int E) {
  constexpr int BNS = 128;                         // columns per source (gate, up) and block
  typedef Tile3<BM, 2 * BNS, 2> TL;
  typedef Tile3<BM / 2, 2 * BNS, 2> TH;            // the half tile runs in the same stages
  static_assert(TH::NST == TL::NST && TH::LDS_R == TL::LDS_R && TH::LDS_L <= TL::LDS_L, "stages serve both");
  DSMOE_TILE3_STAGES(TL, st);
  __shared__ SplitTiles gt;
  build_split_tiles(gt, expert_off, E, BM / 2);
  const int nkt = d / TL::BK;
  SplitWalker tw;
  tw.init(gt, E, (f + BNS - 1) / BNS, BM / 2);
  auto setup = [&](const RowTile& t, auto& L, auto& R) {
    const int row0 = t.row0, n0 = t.nt * BNS;
    L.init(t.valid, 0, [&](int r) {
      return x_perm ? x_perm + (size_t)(row0 + r) * d : x + (size_t)row_token[row0 + r] * d;
    });
    const bf16_t* const base[2] = {w_gate + (size_t)t.e * d * f + n0, w_up + (size_t)t.e * d * f + n0};
    R.init(base, f, min(BNS, f - n0), d);
  };
  auto epilogue = [&](auto tile, auto last_stage, const RowTile& t, const auto& acc) {
    typedef decltype(tile) TT;
    const int n0 = t.nt * BNS;
    TT::template for_each_chunk_bf16<1, decltype(last_stage)::value>(
        acc, st,
        [&](int, int, int, const float (&v)[2][4], float (&o)[1][4]) {
#pragma unroll
          for (int i = 0; i < 4; ++i) o[0][i] = silu_f(v[0][i]) * v[1][i];
        },
        [&](int m, int n, const u32x4 (&p)[1]) {
          if (m >= t.valid || n0 + n >= f) return;
          stg16(h + (size_t)(t.row0 + m) * f + n0 + n, p[0]);
        });
  };
  if (TL::chainable(nkt))
    tile_chain<TL>(
        st, nkt, [&](RowTile& t) { return tw.next_full(gt, E, t); }, setup,
        [&](const RowTile& t, const typename TL::Acc& acc) { epilogue(TL{}, std::true_type{}, t, acc); });
  else
    tile_pipeline<TL>(
        st, nkt, [&](RowTile& t) { return tw.next_full(gt, E, t); }, setup,
        [&](const RowTile& t, const typename TL::Acc& acc) { epilogue(TL{}, std::false_type{}, t, acc); });
  tile_pipeline<TH>(
      st, nkt, [&](RowTile& t) { return tw.next_half(gt, E, t); }, setup,
      [&](const RowTile& t, const typename TH::Acc& acc) { epilogue(TH{}, std::false_type{}, t, acc); });
}

// GATHER: 0 = row r of group e is row row_off[e] + r of h, 1 = row row_token[row_off[e] + r], 2 = row r (every
// group reads the same rows)
template <int BM, bool GELU = false, int GATHER = 0>
__global__ void __launch_bounds__(kThreads2)
down_bf16_kernel(const bf16_t* __restrict__ h, const int32_t* __restrict__ row_token,
                 const int32_t* __restrict__ expert_off, const bf16_t* __restrict__ w_down, bf16_t* __restrict__ y,
                 int d, int f, int E, int uniform_rows) {
  constexpr int BN = 256;
  typedef Tile3<BM, BN> TL;
  typedef Tile3<BM / 2, BN> TH;
  static_assert(TH::NST == TL::NST && TH::LDS_R == TL::LDS_R && TH::LDS_L <= TL::LDS_L, "stages serve both");
  DSMOE_TILE3_STAGES(TL, st);
  __shared__ SplitTiles gt;
  build_split_tiles(gt, expert_off, E, BM / 2, uniform_rows);
  const int nkt = f / TL::BK;
  SplitWalker tw;
  tw.init(gt, E, (d + BN - 1) / BN, BM / 2);
  auto setup = [&](const RowTile& t, auto& L, auto& R) {
    const int row0 = t.row0, n0 = t.nt * BN, group0 = gt.row_off[t.e];
    L.init(t.valid, 0, [&](int r) {
      if constexpr (GATHER == 2) return h + (size_t)(row0 - group0 + r) * f;
      return h + (GATHER == 1 ? (size_t)row_token[row0 + r] : (size_t)(row0 + r)) * f;
    });
    const bf16_t* const base[1] = {w_down + (size_t)t.e * f * d + n0};
    R.init(base, d, min(BN, d - n0), f);
  };
  auto epilogue = [&](auto tile, auto last_stage, const RowTile& t, const auto& acc) {
    typedef decltype(tile) TT;
    const int n0 = t.nt * BN;
    TT::template for_each_chunk_bf16<1, decltype(last_stage)::value>(
        acc, st,
        [&](int, int, int, const float (&v)[1][4], float (&o)[1][4]) {
#pragma unroll
          for (int i = 0; i < 4; ++i) o[0][i] = GELU ? gelu_bf16_f(v[0][i]) : v[0][i];
        },
        [&](int m, int n, const u32x4 (&p)[1]) {
          if (m >= t.valid || n0 + n >= d) return;
          stg16(y + (size_t)(t.row0 + m) * d + n0 + n, p[0]);
        });
  };
  if (TL::chainable(nkt))
    tile_chain<TL>(
        st, nkt, [&](RowTile& t) { return tw.next_full(gt, E, t); }, setup,
        [&](const RowTile& t, const typename TL::Acc& acc) { epilogue(TL{}, std::true_type{}, t, acc); });
  else
    tile_pipeline<TL>(
        st, nkt, [&](RowTile& t) { return tw.next_full(gt, E, t); }, setup,
        [&](const RowTile& t, const typename TL::Acc& acc) { epilogue(TL{}, std::false_type{}, t, acc); });
  tile_pipeline<TH>(
      st, nkt, [&](RowTile& t) { return tw.next_half(gt, E, t); }, setup,
      [&](const RowTile& t, const typename TH::Acc& acc) { epilogue(TH{}, std::false_type{}, t, acc); });
}

static hipError_t launch_ffn_bf16(const dsmoe_ctx* c, const void* x, const void* x_perm, const int32_t* row_token,
                                  const int32_t* expert_off, const void* w_gate, const void* w_up,
                                  const void* w_down, void* y_perm, hipStream_t s) {
  constexpr int BM = 256;
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  bf16_t* h = reinterpret_cast<bf16_t*>(c->workspace + c->ws.h);
  const long max_mt = (c->desc.max_rows + BM - 1) / BM + E;
  const long t1 = max_mt * ((f + 127) / 128), t2 = max_mt * ((d + 255) / 256);
  const int g1 = (int)((std::min<long>(t1, c->n_cu) + 7) / 8 * 8), g2 = (int)((std::min<long>(t2, c->n_cu) + 7) / 8 * 8);
  hipEvent_t* ev = (c->prof.ev && c->prof.n < c->prof.max_calls) ? c->prof.ev + 3 * c->prof.n++ : nullptr;
  if (ev) (void)hipEventRecord(ev[0], s);
  if (c->expert_kind == DSMOE_EXPERT_GELU) {
    // H = gelu(rows W_1): output width f, contraction over d, 256-column tiles
    const int g1g = (int)((std::min<long>(max_mt * ((f + 255) / 256), c->n_cu) + 7) / 8 * 8);
    if (x_perm)
      down_bf16_kernel<BM, true, 0><<<dim3(g1g), dim3(kThreads2), 0, s>>>(
          (const bf16_t*)x_perm, nullptr, expert_off, (const bf16_t*)w_gate, h, f, d, E, 0);
    else
      down_bf16_kernel<BM, true, 1><<<dim3(g1g), dim3(kThreads2), 0, s>>>(
          (const bf16_t*)x, row_token, expert_off, (const bf16_t*)w_gate, h, f, d, E, 0);
  } else {
    gateup_bf16_kernel<BM><<<dim3(g1), dim3(kThreads2), 0, s>>>(
        (const bf16_t*)x, (const bf16_t*)x_perm, row_token, expert_off, (const bf16_t*)w_gate, (const bf16_t*)w_up, h,
        d, f, E);
  }
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  if (ev) (void)hipEventRecord(ev[1], s);
  down_bf16_kernel<BM><<<dim3(g2), dim3(kThreads2), 0, s>>>(h, nullptr, expert_off, (const bf16_t*)w_down,
                                                                        (bf16_t*)y_perm, d, f, E, 0);
  err = hipGetLastError();
  if (ev) (void)hipEventRecord(ev[2], s);
  return err;
}

template <typename T>
static hipError_t launch_ffn_t(const dsmoe_ctx* c, const void* x, const void* x_perm, const int32_t* row_token,
                               const int32_t* expert_off, const void* w_gate, const void* w_up, const void* w_down,
                               void* y_perm, hipStream_t s) {
  constexpr int BM = 128, BN1 = 128, BN2 = 256;
  const int d = c->desc.d_model, f = c->desc.d_ff, E = c->desc.n_experts;
  T* h = reinterpret_cast<T*>(c->workspace + c->ws.h);
  // upper bound of row tiles: every expert may add one ragged tile
  const long max_mt = (c->desc.max_rows + BM - 1) / BM + E;
  const long t1 = max_mt * ((f + BN1 - 1) / BN1), t2 = max_mt * ((d + BN2 - 1) / BN2);
  const int full = c->n_cu * 2;
  const int g1 = (int)((std::min<long>(t1, full) + 7) / 8 * 8), g2 = (int)((std::min<long>(t2, full) + 7) / 8 * 8);
  constexpr int lds1 = Tile<T, BM, BN1, 2>::LDS_BYTES, lds2 = Tile<T, BM, BN2, 1>::LDS_BYTES;
  hipEvent_t* ev = (c->prof.ev && c->prof.n < c->prof.max_calls) ? c->prof.ev + 3 * c->prof.n++ : nullptr;
  if (ev) (void)hipEventRecord(ev[0], s);
  if (c->expert_kind == DSMOE_EXPERT_GELU) {
    const int g1g = (int)((std::min<long>(max_mt * ((f + BN2 - 1) / BN2), full) + 7) / 8 * 8);
    if (x_perm)
      down_kernel<T, BM, BN2, true, false><<<dim3(g1g), dim3(kThreads), lds2, s>>>(
          (const T*)x_perm, nullptr, expert_off, (const T*)w_gate, h, f, d, E, 0);
    else
      down_kernel<T, BM, BN2, true, true><<<dim3(g1g), dim3(kThreads), lds2, s>>>(
          (const T*)x, row_token, expert_off, (const T*)w_gate, h, f, d, E, 0);
  } else {
    gateup_kernel<T, BM, BN1><<<dim3(g1), dim3(kThreads), lds1, s>>>(
        (const T*)x, (const T*)x_perm, row_token, expert_off, (const T*)w_gate, (const T*)w_up, h, d, f, E);
  }
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  if (ev) (void)hipEventRecord(ev[1], s);
  down_kernel<T, BM, BN2><<<dim3(g2), dim3(kThreads), lds2, s>>>((const T*)h, nullptr, expert_off, (const T*)w_down,
                                                                 (T*)y_perm, d, f, E, 0);
  err = hipGetLastError();
  if (ev) (void)hipEventRecord(ev[2], s);
  return err;
}

// out[t,:] = h[t,:] W for ONE group of T rows: h is [T, k_total], w is [k_total, d].  Used by the dense
// layer, whose down projection over all experts is one product over the concatenated hidden width.
hipError_t launch_down_dense(const dsmoe_ctx* c, const void* h, int T, int k_total, const void* w, void* out,
                             hipStream_t s) {
  const int d = c->desc.d_model;
  if (c->desc.dtype == DSMOE_BF16) {
    const long tiles = (long)((T + 255) / 256) * ((d + 255) / 256);
    const int g = (int)((std::min<long>(tiles, c->n_cu) + 7) / 8 * 8);
    down_bf16_kernel<256><<<dim3(g), dim3(kThreads2), 0, s>>>((const bf16_t*)h, nullptr, nullptr, (const bf16_t*)w,
                                                                          (bf16_t*)out, d, k_total, 1, T);
  } else {
    constexpr int BM = 128, BN = 256;
    const long tiles = (long)((T + BM - 1) / BM) * ((d + BN - 1) / BN);
    const int g = (int)((std::min<long>(tiles, c->n_cu * 2) + 7) / 8 * 8);
    down_kernel<float, BM, BN><<<dim3(g), dim3(kThreads), Tile<float, BM, BN, 1>::LDS_BYTES, s>>>(
        (const float*)h, nullptr, nullptr, (const float*)w, (float*)out, d, k_total, 1, T);
  }
  return hipGetLastError();
}

// out[g][r][:] = x[r][:] W[g] for `groups` matrices W[g] of [k][n] and the same `rows` rows of x in every group
// (bf16 only): the query projections of the attention experts.
hipError_t launch_shared_rows_gemm(const dsmoe_ctx* c, const void* x, int groups, int rows, int k, int n,
                                   const void* w, void* out, hipStream_t s) {
  const long tiles = (long)groups * ((rows + 255) / 256 + 1) * ((n + 255) / 256);
  const int g = (int)((std::min<long>(tiles, c->n_cu) + 7) / 8 * 8);
  down_bf16_kernel<256, false, 2><<<dim3(g), dim3(kThreads2), 0, s>>>(
      (const bf16_t*)x, nullptr, nullptr, (const bf16_t*)w, (bf16_t*)out, n, k, groups, rows);
  return hipGetLastError();
}

hipError_t launch_expert_ffn(const dsmoe_ctx* c, const void* x, const void* x_perm, const int32_t* row_token,
                             const int32_t* expert_off, const void* w_gate, const void* w_up,
                             const void* w_down, void* y_perm, hipStream_t s) {
  if (c->desc.dtype == DSMOE_BF16)
    return launch_ffn_bf16(c, x, x_perm, row_token, expert_off, w_gate, w_up, w_down, y_perm, s);
  return launch_ffn_t<float>(c, x, x_perm, row_token, expert_off, w_gate, w_up, w_down, y_perm, s);
}

}  // namespace dsmoe
