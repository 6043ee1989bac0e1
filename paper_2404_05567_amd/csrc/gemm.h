// One front end for the two MFMA contraction cores, so that a kernel body is written once for both
// storage types:
//   float  -> Tile  (gemm_core.h): 256 threads, [row][k] LDS tiles, fp32 MFMA (exact fp32 products)
//   bf16_t -> Tile3 (gemm_dma.h): 512 threads, direct global -> LDS loads, k-major tiles read with the
//             transposing LDS load
//
//   Out[m][n] = sum_k L[m][k] * R_s[k][n]      for NSRC weight-side sources s sharing one L tile
//
// Either operand can come from memory in one of two layouts:
//   "rows": every row (m or n index) is k-contiguous   (activations, or a weight used transposed)
//   "cols": stored [k][row] with rows contiguous       (a weight matrix, or X^T / dY for weight gradients)
// LK / RK select the "cols" layout for the L / R side.  KTAIL zero-fills k >= k_valid of "cols"
// operands (contractions over tokens, whose count need not be a multiple of the K step).
// BN is the number of columns per source.
#pragma once

#include <type_traits>

#include "gemm_dma.h"

namespace dsmoe {

// ---- source set-up, one overload per source type ---------------------------------------------------
// row_base(r) returns the address of element [row r][k = 0] of K segment 0; rows >= valid re-read row valid-1.
template <typename T, int ROWS, class F>
__device__ __forceinline__ void init_rows(SrcRows<T, ROWS>& s, int valid, size_t seg_stride_bytes, F row_base) {
  s.seg_stride = seg_stride_bytes;
#pragma unroll
  for (int i = 0; i < SrcRows<T, ROWS>::NV; ++i) {
    const int r = min((int)(threadIdx.x >> 3) + 32 * i, valid - 1);
    s.p[i] = reinterpret_cast<const char*>(row_base(r)) + (threadIdx.x & 7) * 16;
  }
}
template <int ROWS, class F>
__device__ __forceinline__ void init_rows(LRows2<ROWS>& s, int valid, size_t seg_stride_bytes, F row_base) {
  s.seg_stride = seg_stride_bytes;
#pragma unroll
  for (int i = 0; i < LRows2<ROWS>::NV; ++i) {
    const int r = min((int)(threadIdx.x >> 2) + 128 * i, valid - 1);
    s.p[i] = reinterpret_cast<const char*>(row_base(r)) + (threadIdx.x & 3) * 16;
  }
}

// base: element [k = 0][first row of the tile]; ld: elements between consecutive k;
// rows_valid: rows of the matrix that exist from the tile's first row on; k_valid: extent of K.
template <typename T, int ROWS>
__device__ __forceinline__ void init_cols(SrcCols<T, ROWS>& s, const T* base, size_t ld, int rows_valid, int k_valid) {
  s.base = reinterpret_cast<const char*>(base);
  s.ld_bytes = ld * sizeof(T);
  s.seg_stride = 0;
  s.rows_valid = min(ROWS, rows_valid);
  s.k_valid = k_valid;
}

template <typename T, int BM_, int BN_, int NSRC_, bool LK, bool RK, bool KTAIL = false>
struct Gemm;

// ---- fp32 ----------------------------------------------------------------------------------------
template <int BM_, int BN_, int NSRC_, bool LK, bool RK, bool KTAIL>
struct Gemm<float, BM_, BN_, NSRC_, LK, RK, KTAIL> {
  typedef float T;
  typedef Tile<float, BM_, BN_, NSRC_> TL;
  static constexpr int BM = BM_, BN = BN_, NSRC = NSRC_, BK = TL::BK, THREADS = kThreads, LDS_BYTES = TL::LDS_BYTES;
  static constexpr int WAVES_N = 2;   // waves side by side along n
  typedef std::conditional_t<LK, SrcCols<float, BM>, SrcRows<float, BM>> LSrc;
  typedef std::conditional_t<RK, SrcCols<float, BN>, SrcRows<float, BN>> RSrc1;
  struct RSrc { RSrc1 s[NSRC]; };
  typedef typename TL::Acc Acc;

  template <class F>
  static __device__ __forceinline__ void l_rows(LSrc& s, int valid, size_t seg_stride_bytes, F row_base) {
    init_rows(s, valid, seg_stride_bytes, row_base);
  }
  static __device__ __forceinline__ void l_cols(LSrc& s, const T* base, size_t ld, int rows_valid, int k_valid,
                                                const void* = nullptr) {
    init_cols(s, base, ld, rows_valid, k_valid);
  }
  template <class F>
  static __device__ __forceinline__ void r_rows(RSrc& s, int valid, size_t seg_stride_bytes, F row_base) {
    static_assert(NSRC == 1, "one source");
    init_rows(s.s[0], valid, seg_stride_bytes, row_base);
  }
  static __device__ __forceinline__ void r_cols(RSrc& s, const T* const (&base)[NSRC], size_t ld, int rows_valid,
                                                int k_valid, const void* = nullptr) {
#pragma unroll
    for (int b = 0; b < NSRC; ++b) init_cols(s.s[b], base[b], ld, rows_valid, k_valid);
  }
  static __device__ __forceinline__ void zero(Acc& acc) { TL::zero(acc); }
  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc& R, int nkt, int seg_tiles,
                                                  char* smem) {
    TL::mainloop(acc, L, R.s, nkt, seg_tiles, smem);
    __syncthreads();   // the tile may be restaged (or LDS reused) right after
  }
  // f(m, n, v): row m of the tile, first of 4 consecutive columns n (inside a source), v[s][0..3]
  template <class F>
  static __device__ __forceinline__ void for_each_quad(const Acc& acc, F f) {
#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < TL::NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[NSRC][4];
#pragma unroll
          for (int b = 0; b < NSRC; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) v[b][i] = acc[b][nt][mt][4 * g + i];
          f(TL::acc_m(mt), TL::acc_n(nt, g), v);
        }
  }
  static __device__ __forceinline__ int wave_n() { return threadIdx.x >> 7; }
};

// ---- bf16 ----------------------------------------------------------------------------------------
template <int BM_, int BN_, int NSRC_, bool LK, bool RK, bool KTAIL>
struct Gemm<bf16_t, BM_, BN_, NSRC_, LK, RK, KTAIL> {
  typedef bf16_t T;
  typedef Tile3<BM_, BN_ * NSRC_, NSRC_, LK, RK, KTAIL> TL;
  static constexpr int BM = BM_, BN = BN_, NSRC = NSRC_, BK = TL::BK, THREADS = kThreads2, LDS_BYTES = TL::LDS_BYTES;
  static constexpr int WAVES_N = 4;
  typedef typename TL::LSrc LSrc;
  typedef typename TL::RSrc RSrc;
  typedef typename TL::Acc Acc;

  template <class F>
  static __device__ __forceinline__ void l_rows(LSrc& s, int valid, size_t seg_stride_bytes, F row_base) {
    s.init(valid, seg_stride_bytes, row_base);
  }
  static __device__ __forceinline__ void l_cols(LSrc& s, const T* base, size_t ld, int rows_valid, int k_valid,
                                                const void* zeros = nullptr) {
    const T* const b[1] = {base};
    s.init(b, ld, rows_valid, k_valid, zeros);
  }
  template <class F>
  static __device__ __forceinline__ void r_rows(RSrc& s, int valid, size_t seg_stride_bytes, F row_base) {
    static_assert(NSRC == 1, "one source");
    s.init(valid, seg_stride_bytes, row_base);
  }
  static __device__ __forceinline__ void r_cols(RSrc& s, const T* const (&base)[NSRC], size_t ld, int rows_valid,
                                                int k_valid, const void* zeros = nullptr) {
    s.init(base, ld, rows_valid, k_valid, zeros);
  }
  static __device__ __forceinline__ void zero(Acc& acc) { TL::zero(acc); }
  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc& R, int nkt, int seg_tiles,
                                                  char* smem) {
    TL::mainloop(acc, L, R, nkt, seg_tiles, smem);
  }
  template <class F>
  static __device__ __forceinline__ void for_each_quad(const Acc& acc, F f) {
#pragma unroll
    for (int mt = 0; mt < TL::MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < (NSRC == 1 ? TL::NT : 1); ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[NSRC][4];
#pragma unroll
          for (int b = 0; b < NSRC; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) v[b][i] = acc[NSRC == 1 ? nt : b][mt][4 * g + i];
          f(TL::acc_m(mt), TL::acc_n(nt, g), v);
        }
  }
  static __device__ __forceinline__ int wave_n() { return (threadIdx.x >> 6) % 4; }
};

}  // namespace dsmoe
