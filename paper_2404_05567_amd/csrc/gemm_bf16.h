// bf16 MFMA contraction for gfx950, 512 threads (8 waves) per block, used by the compute-bound kernels.
//
//   Out[m][n] = sum_k L[m][k] * R[k][n]
//
// Per K step of 64 the block stages
//   * the token-side tile L as [row][k]   (144-byte pitch, fragments read with ds_read_b128), and
//   * the weight-side tile R as [k][n], exactly as it lies in memory (n contiguous).  The MFMA needs
//     8 consecutive k per lane, which the transposing LDS read of gfx950 (ds_read_b64_tr_b16)
//     delivers straight from this layout: inside a group of 16 lanes, lane r addresses element
//     [k0 + r/4][n0 + 4*(r%4)] and receives the column [k0 .. k0+3][n0 + r].
//     So no register transposes and no layout change of the weights are needed.
// LDS holds two stages; a third K step is in flight in registers.  One barrier per K step.
//
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand: a lane of the
// 32x32 accumulator owns one token row and 4 consecutive output columns per register quad.
#pragma once

#include "gemm_core.h"

namespace dsmoe {

constexpr int kThreads2 = 512;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ u32x2 lds_read_tr16(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// Token-side source: rows k-contiguous in memory; thread t stages rows t/8 + 64 i, 16-byte column t%8.
template <int ROWS>
struct LRows2 {
  static constexpr int NV = ROWS / 64;
  const char* p[NV];   // row base + (t%8)*16
  size_t seg_stride;   // bytes between K segments
  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
    const size_t off = (size_t)seg * seg_stride + (size_t)kin * kRowBytes;
#pragma unroll
    for (int i = 0; i < NV; ++i) r[i] = ldg16(p[i] + off);
  }
  static __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) {
    char* q = lds + (threadIdx.x >> 3) * kLdsPitch + (threadIdx.x & 7) * 16;
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<u32x4*>(q + i * 64 * kLdsPitch) = r[i];
  }
};

// Weight-side source: NSRC matrices stored [k][n] (n contiguous), each contributing BN / NSRC columns
// of the tile.  LDS column order interleaves the sources in runs of 32 so that one wave's 64-column
// slice holds 32 columns of source 0 followed by the same 32 columns of source 1 (gate | up).
template <int BN, int NSRC>
struct RCols2 {
  static constexpr int BK = 64;
  static constexpr int CH = BN / 8;                 // 16-byte chunks per k row
  static constexpr int NV = BK * CH / kThreads2;    // chunks per thread
  static constexpr int KSTEP = kThreads2 / CH;      // k rows between a thread's chunks
  static constexpr int PITCH = BN * 2 + 64;
  const char* p;       // this thread's first chunk (k row t / CH) of K segment 0, already at its column
  size_t ld_bytes;     // bytes between consecutive k
  size_t seg_stride;
  int lds_off;         // byte offset of the thread's first chunk inside the R stage
  bool ok;             // the thread's column chunk lies inside the matrix
  int k_valid;         // k >= k_valid are zero-filled (tails of a K that is not a multiple of 64)

  // base[s]: element [k=0][n0] of source s; cols_valid: columns of each source that exist from n0 on
  __device__ __forceinline__ void init(const bf16_t* const (&base)[NSRC], size_t ld_elems, int cols_valid, int kv) {
    const int cc = threadIdx.x % CH, krow = threadIdx.x / CH;
    constexpr int CPS = CH / NSRC;                  // chunks per source
    const int src = cc / CPS, col = (cc % CPS) * 8; // column inside the source
    const int pos = NSRC == 1 ? col : (col / 32) * 64 + src * 32 + (col % 32);
    ld_bytes = ld_elems * 2;
    seg_stride = 0;
    ok = col < cols_valid;
    k_valid = kv;
    p = reinterpret_cast<const char*>(base[src] + (size_t)krow * ld_elems + (ok ? col : 0));
    lds_off = krow * PITCH + pos * 2;
  }
  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
    const char* q = p + (size_t)seg * seg_stride + (size_t)kin * BK * ld_bytes;
    const int k0 = kin * BK + threadIdx.x / CH;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const u32x4 z = {0u, 0u, 0u, 0u};
      r[i] = (ok && k0 + i * KSTEP < k_valid) ? ldg16(q + (size_t)i * KSTEP * ld_bytes) : z;
    }
  }
  __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<u32x4*>(lds + lds_off + i * KSTEP * PITCH) = r[i];
  }
};

template <int BM_, int BN_, int WGM_, int WGN_>
struct Tile2 {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static_assert(WGM * WGN == 8, "8 waves");
  static constexpr int BK = 64;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int MT = WM / 32, NT = WN / 32;
  static constexpr int R_PITCH = BN * 2 + 64;
  static constexpr int LDS_L = BM * kLdsPitch, LDS_R = BK * R_PITCH, STAGE = LDS_L + LDS_R;
  static constexpr int LDS_BYTES = 2 * STAGE;
  typedef f32x16 Acc[NT][MT];

  static __device__ __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][mt][i] = 0.f;
  }

  static __device__ __forceinline__ void compute(Acc& acc, const char* stage) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const char* fL = stage + (wm * WM + (lane & 31)) * kLdsPitch + (lane >> 5) * 16;
    // transposing read: lane r of a 16-lane group addresses [k0 + r/4][n0 + 4*(r%4)]
    const int r = lane & 15;
    const char* fR = stage + LDS_L + ((lane >> 5) * 8 + (r >> 2)) * R_PITCH +
                     (wn * WN + ((lane >> 4) & 1) * 16 + (r & 3) * 4) * 2;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 xf[MT], wf[NT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xf[mt] = *reinterpret_cast<const u32x4*>(fL + mt * 32 * kLdsPitch + ks * 32);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const u32x2 lo = lds_read_tr16(fR + (ks * 16) * R_PITCH + nt * 64);
        const u32x2 hi = lds_read_tr16(fR + (ks * 16 + 4) * R_PITCH + nt * 64);
        wf[nt] = u32x4{lo.x, lo.y, hi.x, hi.y};
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) Mma<bf16_t>::run(acc[nt][mt], wf[nt], xf[mt]);
    }
  }

  template <typename LSrc, typename RSrc>
  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc& R, int nkt, int seg_tiles,
                                                  char* smem) {
    u32x4 lr[LSrc::NV], rr[RSrc::NV];
    int seg = 0, kin = 0;
    L.load(lr, 0, 0);
    R.load(rr, 0, 0);
    __syncthreads();   // the previous tile's last K step has been consumed
    L.store(lr, smem);
    R.store(rr, smem + LDS_L);
    if (nkt > 1) {
      if (++kin == seg_tiles) { kin = 0; ++seg; }
      L.load(lr, seg, kin);
      R.load(rr, seg, kin);
    }
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
      char* cur = smem + (kt & 1) * STAGE;
      char* nxt = smem + ((kt + 1) & 1) * STAGE;
      if (kt + 1 < nkt) {
        L.store(lr, nxt);
        R.store(rr, nxt + LDS_L);
        if (kt + 2 < nkt) {
          if (++kin == seg_tiles) { kin = 0; ++seg; }
          L.load(lr, seg, kin);
          R.load(rr, seg, kin);
        }
      }
      compute(acc, cur);
      __syncthreads();
    }
  }

  static __device__ __forceinline__ int acc_m(int mt) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave % WGM) * WM + mt * 32 + (lane & 31);
  }
  // column inside the wave's WN-wide slice (tile nt, register quad g)
  static __device__ __forceinline__ int acc_n_local(int nt, int g) {
    const int lane = threadIdx.x & 63;
    return nt * 32 + g * 8 + (lane >> 5) * 4;
  }
  static __device__ __forceinline__ int wave_n() { return (threadIdx.x >> 6) / WGM; }
};

}  // namespace dsmoe
