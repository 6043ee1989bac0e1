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

// LDS of a kernel built on Gemm<...> GM: static stage arrays (bf16 core) or the dynamic buffer (fp32 core)
#define DSMOE_GEMM_STAGES(GM, st)                                                                            \
  extern __shared__ __align__(16) char dsmoe_dyn_smem[];                                                     \
  DSMOE_STAGE_ARRAYS(st, 4, GM::ST_L, GM::ST_R);                                                             \
  (void)st##L4; (void)st##L5; (void)st##R4; (void)st##R5; (void)st##L6; (void)st##L7; (void)st##R6; (void)st##R7;          \
  typename GM::Stages st =                                                                                   \
      GM::make_stages(st##L0, st##L1, st##L2, st##L3, st##R0, st##R1, st##R2, st##R3, dsmoe_dyn_smem)

// W consecutive values to / from memory (W = 4 or 8)
template <int W>
__device__ __forceinline__ void store_chunk(float* p, const float (&v)[W]) {
#pragma unroll
  for (int i = 0; i < W; i += 4) store4(p + i, v[i], v[i + 1], v[i + 2], v[i + 3]);
}
template <int W>
__device__ __forceinline__ void store_chunk(bf16_t* p, const float (&v)[W]) {
  if constexpr (W == 8) {
    const u32x4 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    stg16(p, o);
  } else {
    store4(p, v[0], v[1], v[2], v[3]);
  }
}
// Two-step form of load_chunk for epilogues that request their operands before they need them: load_raw issues
// the 16-byte load of a chunk (4 floats or 8 bf16), unpack_chunk converts it.
__device__ __forceinline__ u32x4 load_raw(const void* p) { return ldg16(p); }
__device__ __forceinline__ void unpack_chunk(const u32x4& q, float (&v)[4], const float*) {
  const f32x4 t = __builtin_bit_cast(f32x4, q);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void unpack_chunk(const u32x4& q, float (&v)[8], const bf16_t*) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(q[i] << 16);
    v[2 * i + 1] = __uint_as_float(q[i] & 0xffff0000u);
  }
}
template <int W>
__device__ __forceinline__ void load_chunk(const float* p, float (&v)[W]) {
#pragma unroll
  for (int i = 0; i < W; i += 4) {
    const f32x4 q = __builtin_bit_cast(f32x4, ldg16(p + i));
    v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
  }
}
template <int W>
__device__ __forceinline__ void load_chunk(const bf16_t* p, float (&v)[W]) {
  if constexpr (W == 8) {
    const u32x4 q = ldg16(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(q[i] << 16);
      v[2 * i + 1] = __uint_as_float(q[i] & 0xffff0000u);
    }
  } else {
    typedef __attribute__((address_space(1))) const u32x2 g_u32x2;
    const u32x2 q = *(g_u32x2*)(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
  }
}

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
  struct Stages { char* smem; };
  static constexpr int ST_L = 16, ST_R = 16, CHUNK = 4;   // stages live in dynamic LDS; 4 columns per lane
  static __device__ __forceinline__ Stages make_stages(char*, char*, char*, char*, char*, char*, char*, char*,
                                                       char* dyn) {
    return Stages{dyn};
  }

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
                                                  const Stages& st) {
    TL::mainloop(acc, L, R.s, nkt, seg_tiles, st.smem);
    __syncthreads();   // the tile may be restaged (or LDS reused) right after
  }
  // two-phase form of the main loop (the bf16 core starts loading the next tile before the epilogue)
  struct Iter {};
  static __device__ __forceinline__ void prefetch(const LSrc&, const RSrc&, Iter&, int, int, const Stages&) {}
  static __device__ __forceinline__ void run(Acc& acc, const LSrc& L, const RSrc& R, Iter&, int nkt, int seg_tiles,
                                             const Stages& st) {
    mainloop(acc, L, R, nkt, seg_tiles, st);
  }
  // f(m, n, v): row m of the tile, first of CHUNK consecutive columns n (inside a source), v[s][0..CHUNK)
  template <class F>
  static __device__ __forceinline__ void for_each_chunk(const Acc& acc, const Stages&, F f) {
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
  // Same walk with the operands of f requested first: load(j, m, n) is called for the chunks of a group, then
  // f(j, m, n, v) for the same chunks; j < NJ numbers the chunks of a group (one chunk per group here).
  static constexpr int NJ = 1;
  template <class LD, class F>
  static __device__ __forceinline__ void for_each_chunk_loaded(const Acc& acc, const Stages& st, LD load, F f) {
    for_each_chunk(acc, st, [&](int m, int n, const float (&v)[NSRC][4]) {
      load(0, m, n);
      f(0, m, n, v);
    });
  }
  static __device__ __forceinline__ int wave_n() { return threadIdx.x >> 7; }
  // sum of p over the lanes that hold the same tile row in one for_each_chunk call; row_leader() is true on one of them
  static __device__ __forceinline__ float row_sum(float p) { return p + __shfl_xor(p, 32, 64); }
  static __device__ __forceinline__ bool row_leader() { return (threadIdx.x & 63) < 32; }
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
  typedef Stages3 Stages;
  static constexpr int ST_L = TL::LDS_L, ST_R = TL::LDS_R, CHUNK = TL::CHUNK;
  static __device__ __forceinline__ Stages make_stages(char* l0, char* l1, char* l2, char* l3, char* r0, char* r1,
                                                       char* r2, char* r3, char*) {
    Stages s;
    s.l[0] = (lds_char*)l0; s.l[1] = (lds_char*)l1; s.l[2] = (lds_char*)l2; s.l[3] = (lds_char*)l3;
    s.r[0] = (lds_char*)r0; s.r[1] = (lds_char*)r1; s.r[2] = (lds_char*)r2; s.r[3] = (lds_char*)r3;
    s.l[4] = s.l[5] = s.r[4] = s.r[5] = s.l[6] = s.l[7] = s.r[6] = s.r[7] = nullptr;
    return s;
  }

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
                                                  const Stages& st) {
    TL::mainloop(acc, L, R, nkt, seg_tiles, st);
  }
  typedef typename TL::Iter Iter;
  static __device__ __forceinline__ void prefetch(const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                                  const Stages& st) {
    TL::prefetch(L, R, it, nkt, seg_tiles, st);
  }
  static __device__ __forceinline__ void run(Acc& acc, const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                             const Stages& st) {
    TL::run(acc, L, R, it, nkt, seg_tiles, st);
  }
  template <class F>
  static __device__ __forceinline__ void for_each_chunk(const Acc& acc, const Stages& st, F f) {
    TL::for_each_chunk(acc, st, [](int, int, int) {}, [&](int, int m, int n, const float (&v)[NSRC][8]) { f(m, n, v); });
  }
  static constexpr int NJ = TL::NJ;
  template <class LD, class F>
  static __device__ __forceinline__ void for_each_chunk_loaded(const Acc& acc, const Stages& st, LD load, F f) {
    TL::template for_each_chunk<true>(acc, st, load, f);
  }
  static __device__ __forceinline__ int wave_n() { return (threadIdx.x >> 6) % 4; }
  static __device__ __forceinline__ float row_sum(float p) {
    constexpr int OPR = NSRC == 1 ? 8 : 4;
#pragma unroll
    for (int o = 1; o < OPR; o <<= 1) p += __shfl_xor(p, o, 64);
    return p;
  }
  static __device__ __forceinline__ bool row_leader() { return (threadIdx.x & (NSRC == 1 ? 7 : 3)) == 0; }
};

}  // namespace dsmoe
