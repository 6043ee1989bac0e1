// bf16 MFMA contraction for gfx950, 512 threads (8 waves) per block, used by the compute-bound kernels.
//
//   Out[m][n] = sum_k L[m][k] * R[k][n]
//
// Per K step of 32 the block stages
//   * the token-side tile L as [row][k]   (64 data bytes per row, 80-byte pitch: the 16-byte fragment
//     reads of 16 consecutive rows then hit 16 disjoint bank quads), and
//   * the weight-side tile R as [k][n], exactly as it lies in memory (n contiguous).  The MFMA needs
//     8 consecutive k per lane, which the transposing LDS read of gfx950 (ds_read_b64_tr_b16)
//     delivers straight from this layout: inside a group of 16 lanes, lane r addresses element
//     [k0 + r/4][n0 + 4*(r%4)] and receives the column [k0 .. k0+3][n0 + r].
//     So no register transposes and no layout change of the weights are needed.
// Memory latency is covered by THREE K steps in flight in registers (global load -> register ->
// LDS three steps later) on top of two LDS stages; one barrier per K step.
//
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand: a lane of the
// 32x32 accumulator owns one token row and 4 consecutive output columns per register quad.
#pragma once

#include "gemm_core.h"

namespace dsmoe {

constexpr int kThreads2 = 512;
constexpr int kBK2 = 32;          // K elements per step
constexpr int kLPitch2 = 80;      // LDS pitch of an L row (64 data bytes)
constexpr int kRegStages = 3;     // K steps held in registers

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ u32x2 lds_read_tr16(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// Operand whose rows are k-contiguous in memory (token activations, or a weight used transposed);
// thread t stages rows t/4 + 128 i, 16-byte column t%4.  Usable on either side of the product.
template <int ROWS>
struct LRows2 {
  static constexpr bool kKMajor = false;             // LDS tile is [row][k]
  static constexpr int LDS = ROWS * kLPitch2;
  static constexpr int NV = ROWS / 128;
  const char* p[NV];   // row base + (t%4)*16, K segment 0
  size_t seg_stride;   // bytes between K segments
  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
    const size_t off = (size_t)seg * seg_stride + (size_t)kin * (kBK2 * 2);
#pragma unroll
    for (int i = 0; i < NV; ++i) r[i] = ldg16(p[i] + off);
  }
  static __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) {
    char* q = lds + (threadIdx.x >> 2) * kLPitch2 + (threadIdx.x & 3) * 16;
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<u32x4*>(q + i * 128 * kLPitch2) = r[i];
  }
};

// Operand stored [k][n] with n contiguous (a weight matrix, or X^T / dY for the weight gradients);
// usable on either side of the product.  NSRC matrices each contribute BN / NSRC columns
// of the tile; source s occupies LDS columns [s * BN / NSRC, (s + 1) * BN / NSRC).  Columns past the
// end of the matrix are read from a clamped (valid) address and never reach a stored output.
// KTAIL: zero-fill k >= k_valid (needed only when K is not a multiple of 32).
template <int BN, int NSRC, bool KTAIL = false>
struct RCols2 {
  static constexpr bool kKMajor = true;               // LDS tile is [k][n]
  static constexpr int LDS = kBK2 * (BN * 2 + 64);
  static constexpr int CH = BN / 8;                   // 16-byte chunks per k row
  static constexpr int NV = kBK2 * CH / kThreads2;    // chunks per thread
  static constexpr int KSTEP = kThreads2 / CH;        // k rows between a thread's chunks
  static constexpr int PITCH = BN * 2 + 64;
  const char* p;       // this thread's first chunk (k row t / CH) of K segment 0, already at its column
  size_t ld_bytes;     // bytes between consecutive k
  size_t seg_stride;
  int lds_off;         // byte offset of the thread's first chunk inside the R stage
  int k_valid;

  // base[s]: element [k=0][n0] of source s; cols_valid: columns of each source that exist from n0 on
  __device__ __forceinline__ void init(const bf16_t* const (&base)[NSRC], size_t ld_elems, int cols_valid, int kv) {
    const int cc = threadIdx.x % CH, krow = threadIdx.x / CH;
    constexpr int CPS = CH / NSRC;                    // chunks per source
    const int src = cc / CPS, col = (cc % CPS) * 8;   // column inside the source
    ld_bytes = ld_elems * 2;
    seg_stride = 0;
    k_valid = kv;
    p = reinterpret_cast<const char*>(base[src] + (size_t)krow * ld_elems + (col < cols_valid ? col : 0));
    lds_off = krow * PITCH + cc * 16;
  }
  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
    const char* q = p + (size_t)seg * seg_stride + (size_t)kin * kBK2 * ld_bytes;
    const int k0 = kin * kBK2 + threadIdx.x / CH;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      if (KTAIL) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        r[i] = (k0 + i * KSTEP < k_valid) ? ldg16(q + (size_t)i * KSTEP * ld_bytes) : z;
      } else {
        r[i] = ldg16(q + (size_t)i * KSTEP * ld_bytes);
      }
    }
  }
  __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<u32x4*>(lds + lds_off + i * KSTEP * PITCH) = r[i];
  }
};

// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
constexpr int kSgMfma = 0x008, kSgVmemRd = 0x020, kSgDsRd = 0x100, kSgDsWr = 0x200;

template <int MASK, int N>
__device__ __forceinline__ void sched_group() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
// NMMA groups of {1 MFMA, a share of NA instructions of kind MASKA}
template <int I, int NMMA, int NA, int MASKA>
struct Interleave {
  static __device__ __forceinline__ void run() {
    if constexpr (I < NMMA) {
      sched_group<kSgMfma, 1>();
      sched_group<MASKA, (NA * (I + 1)) / NMMA - (NA * I) / NMMA>();
      Interleave<I + 1, NMMA, NA, MASKA>::run();
    }
  }
};

// NSRC = 2: the wave's NT = 2 column tiles are the same 32 columns of source 0 (gate) and source 1 (up).
// L_KMAJOR / R_KMAJOR: LDS layout of the token-side / weight-side tile ([k][col] read with the
// transposing load, or [row][k] read with 16-byte loads); they must match the source types used.
template <int BM_, int BN_, int WGM_, int WGN_, int NSRC_ = 1, bool L_KMAJOR = false, bool R_KMAJOR = true>
struct Tile2 {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, NSRC = NSRC_;
  static_assert(WGM * WGN == 8, "8 waves");
  static constexpr int BK = kBK2;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int MT = WM / 32, NT = WN / 32;
  static_assert(NSRC == 1 || NT == NSRC, "one column tile per source");
  static constexpr int L_PITCH = L_KMAJOR ? BM * 2 + 64 : kLPitch2;
  static constexpr int R_PITCH = R_KMAJOR ? BN * 2 + 64 : kLPitch2;
  static constexpr int LDS_L = L_KMAJOR ? BK * L_PITCH : BM * L_PITCH;
  static constexpr int LDS_R = R_KMAJOR ? BK * R_PITCH : BN * R_PITCH;
  static constexpr int STAGE = LDS_L + LDS_R;
  static constexpr int LDS_BYTES = 2 * STAGE;
  // LDS column of the wave's first column, and distance between its column tiles
  static constexpr int WCOL = NSRC == 1 ? WN : 32, NT_COLS = NSRC == 1 ? 32 : BN / NSRC;
  static constexpr int NFR = (L_KMAJOR ? 2 : 1) * MT + (R_KMAJOR ? 2 : 1) * NT;   // LDS reads per 16-wide K slice
  typedef f32x16 Acc[NT][MT];

  static __device__ __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][mt][i] = 0.f;
  }

  // lane base address inside a tile for 32-wide fragment `first` (in rows / columns of the tile)
  template <bool KMAJOR>
  static __device__ __forceinline__ const char* frag_base(const char* tile, int pitch, int first) {
    const int lane = threadIdx.x & 63, r = lane & 15;
    if (KMAJOR)   // transposing read: lane r of a 16-lane group addresses [k0 + r/4][n0 + 4*(r%4)]
      return tile + ((lane >> 5) * 8 + (r >> 2)) * pitch + (first + ((lane >> 4) & 1) * 16 + (r & 3) * 4) * 2;
    return tile + (first + (lane & 31)) * pitch + (lane >> 5) * 16;
  }
  // fragment of 32 rows/columns starting `off` after the lane base, K slice ks (16 wide)
  template <bool KMAJOR>
  static __device__ __forceinline__ u32x4 read_frag(const char* base, int pitch, int off, int ks) {
    if (KMAJOR) {
      const u32x2 lo = lds_read_tr16(base + (ks * 16) * pitch + off * 2);
      const u32x2 hi = lds_read_tr16(base + (ks * 16 + 4) * pitch + off * 2);
      return u32x4{lo.x, lo.y, hi.x, hi.y};
    }
    return *reinterpret_cast<const u32x4*>(base + off * pitch + ks * 32);
  }

  // MFMA work of one K step (two 16-wide slices) on LDS stage `cur`, the fragment reads of the second
  // slice interleaved with the MFMAs of the first.
  static __device__ __forceinline__ void compute(Acc& acc, const char* cur) {
    constexpr int NMMA = MT * NT;
    const int wave = threadIdx.x >> 6;
    const char* fL = frag_base<L_KMAJOR>(cur, L_PITCH, (wave / WGN) * WM);
    const char* fR = frag_base<R_KMAJOR>(cur + LDS_L, R_PITCH, (wave % WGN) * WCOL);
    u32x4 xa[MT], xb[MT], wa[NT], wb[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xa[mt] = read_frag<L_KMAJOR>(fL, L_PITCH, mt * 32, 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wa[nt] = read_frag<R_KMAJOR>(fR, R_PITCH, nt * NT_COLS, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xb[mt] = read_frag<L_KMAJOR>(fL, L_PITCH, mt * 32, 1);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wb[nt] = read_frag<R_KMAJOR>(fR, R_PITCH, nt * NT_COLS, 1);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) Mma<bf16_t>::run(acc[nt][mt], wa[nt], xa[mt]);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) Mma<bf16_t>::run(acc[nt][mt], wb[nt], xb[mt]);
    sched_group<kSgDsRd, NFR>();
    Interleave<0, NMMA, NFR, kSgDsRd>::run();
    sched_group<kSgMfma, NMMA>();
  }

  // acc += L * R over nkt K steps; K may be split in segments of seg_tiles steps (see the sources).
  // Step t is loaded into register slot t % 3 while step t - 4 is computed, written to LDS stage
  // t & 1 while step t - 1 is computed, and consumed one barrier later.
  template <typename LSrc, typename RSrc>
  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc& R, int nkt, int seg_tiles,
                                                  char* smem) {
    static_assert(LSrc::kKMajor == L_KMAJOR && RSrc::kKMajor == R_KMAJOR, "source / tile layout mismatch");
    static_assert(LSrc::LDS == LDS_L && RSrc::LDS == LDS_R, "source / tile size mismatch");
    u32x4 lr[kRegStages][LSrc::NV], rr[kRegStages][RSrc::NV];
    int seg = 0, kin = 0, next = 0;   // K position / index of the next step to load
    // Loads are issued unconditionally (steps past the end re-read the last one): the compiler can
    // then count outstanding loads and wait only for the oldest register stage.
    auto load_next = [&](u32x4 (&a)[LSrc::NV], u32x4 (&b)[RSrc::NV]) {
      L.load(a, seg, kin);
      R.load(b, seg, kin);
      if (++next < nkt && ++kin == seg_tiles) { kin = 0; ++seg; }
    };
    load_next(lr[0], rr[0]);
    load_next(lr[1], rr[1]);
    load_next(lr[2], rr[2]);
    L.store(lr[0], smem);            // the previous tile ended with a barrier after its last LDS read
    R.store(rr[0], smem + LDS_L);
    load_next(lr[0], rr[0]);
    __syncthreads();
    auto step = [&](int kt, u32x4 (&a)[LSrc::NV], u32x4 (&b)[RSrc::NV]) {
      char* nxt = smem + ((kt + 1) & 1) * STAGE;
      L.store(a, nxt);                                  // step kt + 1 (a harmless re-store at the end)
      R.store(b, nxt + LDS_L);
      load_next(a, b);                                  // step kt + 4 into the slot just drained
      compute(acc, smem + (kt & 1) * STAGE);
      __syncthreads();
    };
    // three steps per trip with fixed register slots and no exits inside the loop body
    int kt = 0;
    for (; kt + kRegStages <= nkt; kt += kRegStages) {
      step(kt, lr[1], rr[1]);
      step(kt + 1, lr[2], rr[2]);
      step(kt + 2, lr[0], rr[0]);
    }
    if (kt < nkt) {
      step(kt, lr[1], rr[1]);
      if (kt + 1 < nkt) step(kt + 1, lr[2], rr[2]);
    }
  }

  static __device__ __forceinline__ int acc_m(int mt) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave / WGN) * WM + mt * 32 + (lane & 31);
  }
  // column (inside its source) of register quad g of column tile nt
  static __device__ __forceinline__ int acc_n(int nt, int g) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave % WGN) * WCOL + (NSRC == 1 ? nt * 32 : 0) + g * 8 + (lane >> 5) * 4;
  }
};

}  // namespace dsmoe
