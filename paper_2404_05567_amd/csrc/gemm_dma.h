// bf16 MFMA contraction for gfx950 with direct global -> LDS loads, 512 threads (8 waves, 2 x 4).
//
//   Out[m][n] = sum_k L[m][k] * R[k][n]
//
// Per K step of 32 every wave issues `global_load_lds_dwordx4` instructions: each moves 64 x 16 bytes
// from per-lane global addresses into 1 KB of consecutive LDS, without passing through registers.  Four
// LDS stages of one K step each are kept in flight (three steps of prefetch distance); a step costs one
// barrier, placed between the MFMAs of its two 16-wide K slices so that the fragments of the next slice
// are read while the current one multiplies.
//
// The LDS image of a 1 KB chunk is fixed (lane i writes bytes [16 i, 16 i + 16)), so bank conflicts are
// avoided by choosing WHICH global 16 bytes a lane fetches (an XOR swizzle), not by padding:
//   "rows" operand (rows k-contiguous: activations, or a weight used transposed): tile [row][32 k], 64 bytes
//       per row; the 16-byte piece kc of row r lies at position kc ^ ((r >> 2) & 3).  Read with ds_read_b128.
//   "cols" operand (stored [k][n], n contiguous: a weight, or X^T / dY for weight gradients): tile [32 k][n];
//       the 64-byte unit U of row k lies at unit U ^ (k & 3).  Read with the transposing ds_read_b64_tr_b16,
//       which hands a lane the 4 k-consecutive values of one column.
// Both layouts can serve either side of the product.  Each stage is a separate __shared__ array: the
// compiler then knows which loads a fragment read depends on and waits only for those.
//
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand: a lane of the 32x32
// accumulator owns one token row and 4 consecutive output columns per register quad.
#pragma once

#include <type_traits>

#include "gemm_core.h"

namespace dsmoe {

constexpr int kThreads2 = 512;   // threads per block of the bf16 kernels
constexpr int kBK2 = 32;         // K elements per step

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read (ds_read_b64_tr_b16): inside a group of 16 lanes, lane r addresses element
// [k0 + r/4][n0 + 4*(r%4)] of a [k][n] tile and receives the column [k0 .. k0+3][n0 + r].
__device__ __forceinline__ u32x2 lds_read_tr16(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}

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


constexpr int kMaxStages3 = 8;   // LDS stages a kernel may use (Tile3's NST: 4 for the MFMA-bound kernels, 6 or 8 for streaming)

typedef __attribute__((address_space(1))) const void gvoid_t;
typedef __attribute__((address_space(3))) void lvoid_t;
typedef __attribute__((address_space(3))) char lds_char;           // LDS pointers stay typed as such
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

__device__ __forceinline__ void dma16(const char* g, lds_char* lds) {
  __builtin_amdgcn_global_load_lds((gvoid_t*)g, (lvoid_t*)lds, 16, 0, 0);
}
__device__ __forceinline__ u32x2 lds_read_tr16(const lds_char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}
// LDS accesses of the epilogues, written as assembly so that the compiler's wait-count insertion does not tie them
// to the global -> LDS loads still in flight: it cannot tell which stage a read touches once the address is
// selected at run time, and would put `s_waitcnt vmcnt(0)` before every read, which also waits for every
// global store issued so far (one counter covers loads and stores), i.e. the epilogue would pay a full store
// round trip per row block.  The caller guarantees that no load in flight targets the bytes read (the epilogues
// use the wave's own slices of the last two stages, loads in flight go to the first ones).  LDS operations of a
// wave execute in order, so the reads see the wave's earlier writes.
//
// -DDSMOE_CONSERVATIVE_WAITS builds the same sources with none of these assumptions: every counted wait becomes a
// wait for ALL vector-memory and LDS operations of the wave, and the accessors below first wait for everything in
// flight.  Slower, but independent of how many loads are in flight where.  Every sum in the library has a fixed
// order, so the two builds must agree bit for bit; a GPU test compares them.
#ifdef DSMOE_CONSERVATIVE_WAITS
#define DSMOE_FREE_PREFIX "s_waitcnt vmcnt(0) lgkmcnt(0)\n\t"
constexpr bool kConservativeWaits = true;
#else
#define DSMOE_FREE_PREFIX ""
constexpr bool kConservativeWaits = false;
#endif
__device__ __forceinline__ u32x4 lds_read16_free(const lds_char* p) {
  u32x4 v;
  asm volatile(DSMOE_FREE_PREFIX "ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ void lds_write8_free(lds_char* p, u32x2 v) {
  asm volatile(DSMOE_FREE_PREFIX "ds_write_b64 %0, %1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write16_free(lds_char* p, u32x4 v) {
  asm volatile(DSMOE_FREE_PREFIX "ds_write_b128 %0, %1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_read16x2_free(const lds_char* p0, const lds_char* p1, u32x4& a, u32x4& b) {
  asm volatile(DSMOE_FREE_PREFIX "ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(a), "=&v"(b) : "v"(p0), "v"(p1) : "memory");
}

// s_waitcnt on the vector-memory counter alone (N outstanding loads allowed), optionally also on all LDS reads
template <int N, bool LGKM0>
__device__ __forceinline__ void wait_vm() {
  if constexpr (kConservativeWaits) __builtin_amdgcn_s_waitcnt(7 << 4);   // vmcnt(0) lgkmcnt(0)
  else __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | ((LGKM0 ? 0 : 15) << 8));
}

// The thread index as a value the compiler cannot trace back to threadIdx: what is derived from it is
// computed where it is used instead of being hoisted out of a tile loop and kept (spilled) across the main
// loop.  A spill reload is a vector-memory load, and the wait for it also waits for every global store in
// flight.
__device__ __forceinline__ int opaque_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

// ---- "rows" operand -----------------------------------------------------------------------------------
template <int ROWS>
struct DRows {
  static constexpr bool kKMajor = false;
  static constexpr int LDS = ROWS * 64;
  static constexpr int CPW = ROWS / 128;          // 1 KB chunks (16 rows) per wave and K step
  static constexpr int NI = CPW;
  const char* p[CPW];   // this lane's piece of each of its chunks, K segment 0, step 0
  size_t seg_stride;    // bytes between K segments
  // K segments may continue in another matrix with the same row pitch: from segment brk[i] on, jump[i] bytes
  // are added to every address (uniform values: the switch costs scalar instructions only)
  int brk[2];
  long long jump[2];

  // row_base(r): address of element [row r][k = 0]; rows >= valid re-read row valid - 1
  template <class F>
  __device__ __forceinline__ void init(int valid, size_t seg_stride_bytes, F row_base) {
    seg_stride = seg_stride_bytes;
    brk[0] = brk[1] = 0x7fffffff;
    jump[0] = jump[1] = 0;
    const int tid = opaque_tid();
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
      const int r = 16 * (wave * CPW + i) + (lane >> 2);
      const int kc = (lane & 3) ^ ((r >> 2) & 3);
      p[i] = reinterpret_cast<const char*>(row_base(min(r, valid - 1))) + kc * 16;
    }
  }
  // segments >= at continue at (address of segment `at` in the new matrix) = old address + bytes
  __device__ __forceinline__ void set_jump(int i, int at, long long bytes) {
    brk[i] = at;
    jump[i] = bytes;
  }
  // load instruction i (of NI) of a K step
  __device__ __forceinline__ void issue_one(lds_char* stage, int seg, int kin, int i) const {
    const long long off = (long long)seg * (long long)seg_stride + (long long)kin * 64 +
                          (seg >= brk[0] ? jump[0] : 0ll) + (seg >= brk[1] ? jump[1] : 0ll);
    dma16(p[i] + off, stage + (threadIdx.x >> 6) * (CPW * 1024) + i * 1024);
  }
  __device__ __forceinline__ void issue(lds_char* stage, int seg, int kin) const {
#pragma unroll
    for (int i = 0; i < CPW; ++i) issue_one(stage, seg, kin, i);
  }
  // lane offset of the fragment of 32 rows starting at `first` (a multiple of 32), K slice ks
  static __device__ __forceinline__ int frag_off(int first, int ks) {
    const int lane = threadIdx.x & 63;
    return (first + (lane & 31)) * 64 + (((2 * ks + (lane >> 5)) ^ ((lane >> 2) & 3)) * 16);
  }
  static __device__ __forceinline__ u32x4 read(const lds_char* tile, int off, int group) {
    return *reinterpret_cast<const lds_u32x4*>(tile + off + group * (32 * 64));
  }
};

// ---- "cols" operand -----------------------------------------------------------------------------------
// NSRC matrices each contribute COLS / NSRC columns; source s occupies tile columns [s * COLS / NSRC, ...).
// KTAIL: k >= k_valid is read from `zeros` (at least 16 readable zero bytes).
template <int COLS, int NSRC, bool KTAIL = false>
struct DCols {
  static constexpr bool kKMajor = true;
  static constexpr int RB = COLS * 2;             // bytes per k row
  static constexpr int LDS = kBK2 * RB;
  static constexpr int KPC = 1024 / RB;           // k rows per 1 KB chunk
  static constexpr int PPR = RB / 16;             // 16-byte pieces per k row
  static constexpr int CPW = COLS / 128;          // chunks per wave and K step
  static constexpr int NI = CPW;
  const char* p[CPW];
  size_t step_bytes;    // bytes between K steps (32 * ld)
  size_t seg_stride;
  int k_valid;
  const char* zeros;

  // base[s]: element [k = 0][first column of the tile] of source s; cols_valid: columns of each source that
  // exist from there on (columns past the end are read from column 0 and never reach a stored output)
  __device__ __forceinline__ void init(const bf16_t* const (&base)[NSRC], size_t ld_elems, int cols_valid, int kv,
                                       const void* zero_page = nullptr) {
    const int tid = opaque_tid();
    const int lane = tid & 63, wave = tid >> 6;
    step_bytes = (size_t)kBK2 * ld_elems * 2;
    seg_stride = 0;
    k_valid = kv;
    zeros = static_cast<const char*>(zero_page);
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
      const int k = (wave * CPW + i) * KPC + lane / PPR, q = lane % PPR;
      const int U = (q >> 2) ^ (k & 3), col = U * 32 + (q & 3) * 8;      // tile column of this lane's piece
      constexpr int CPS = COLS / NSRC;
      const int src = col / CPS, cs = col % CPS;
      p[i] = reinterpret_cast<const char*>(base[src] + (size_t)k * ld_elems + (cs < cols_valid ? cs : 0));
    }
  }
  __device__ __forceinline__ void issue_one(lds_char* stage, int seg, int kin, int i) const {
    const size_t off = (size_t)seg * seg_stride + (size_t)kin * step_bytes;
    const char* g = p[i] + off;
    if (KTAIL) {
      const int k = kin * kBK2 + ((threadIdx.x >> 6) * CPW + i) * KPC + (threadIdx.x & 63) / PPR;
      g = k < k_valid ? g : zeros;
    }
    dma16(g, stage + (threadIdx.x >> 6) * (CPW * 1024) + i * 1024);
  }
  __device__ __forceinline__ void issue(lds_char* stage, int seg, int kin) const {
#pragma unroll
    for (int i = 0; i < CPW; ++i) issue_one(stage, seg, kin, i);
  }
  // lane offset (without the column-unit term) of a fragment, K slice ks; unit_off(first) adds the columns
  static __device__ __forceinline__ int frag_off(int first, int ks) {
    const int lane = threadIdx.x & 63, i = lane & 15;
    return (16 * ks + 8 * (lane >> 5) + (i >> 2)) * RB + (((first >> 5) ^ (i >> 2)) * 64) + 32 * ((lane >> 4) & 1) +
           8 * (i & 3);
  }
  static __device__ __forceinline__ u32x4 read(const lds_char* tile, int off) {
    const u32x2 lo = lds_read_tr16(tile + off);
    const u32x2 hi = lds_read_tr16(tile + off + 4 * RB);
    return u32x4{lo.x, lo.y, hi.x, hi.y};
  }
};

// The LDS stages of a kernel: separate __shared__ arrays (so that the compiler can tell the stages apart),
// declared once per kernel with DSMOE_TILE3_STAGES and handed to the main loop and the epilogue.
struct Stages3 { lds_char* l[kMaxStages3]; lds_char* r[kMaxStages3]; };
#define DSMOE_STAGE_ARRAYS(st, NST, LB, RB)                                                                  \
  __shared__ __align__(1024) char st##L0[LB], st##L1[LB], st##L2[LB], st##L3[LB], st##L4[(NST) > 4 ? (LB) : 16],  \
      st##L5[(NST) > 5 ? (LB) : 16], st##L6[(NST) > 6 ? (LB) : 16], st##L7[(NST) > 7 ? (LB) : 16];           \
  __shared__ __align__(1024) char st##R0[RB], st##R1[RB], st##R2[RB], st##R3[RB], st##R4[(NST) > 4 ? (RB) : 16],  \
      st##R5[(NST) > 5 ? (RB) : 16], st##R6[(NST) > 6 ? (RB) : 16], st##R7[(NST) > 7 ? (RB) : 16]
#define DSMOE_TILE3_STAGES(TL, st)                                                                           \
  DSMOE_STAGE_ARRAYS(st, TL::NST, TL::LDS_L, TL::LDS_R);                                                     \
  dsmoe::Stages3 st;                                                                                         \
  st.l[0] = (dsmoe::lds_char*)st##L0; st.l[1] = (dsmoe::lds_char*)st##L1; st.l[2] = (dsmoe::lds_char*)st##L2; \
  st.l[3] = (dsmoe::lds_char*)st##L3; st.l[4] = (dsmoe::lds_char*)st##L4; st.l[5] = (dsmoe::lds_char*)st##L5; \
  st.l[6] = (dsmoe::lds_char*)st##L6; st.l[7] = (dsmoe::lds_char*)st##L7;                                    \
  st.r[0] = (dsmoe::lds_char*)st##R0; st.r[1] = (dsmoe::lds_char*)st##R1; st.r[2] = (dsmoe::lds_char*)st##R2; \
  st.r[3] = (dsmoe::lds_char*)st##R3; st.r[4] = (dsmoe::lds_char*)st##R4; st.r[5] = (dsmoe::lds_char*)st##R5; \
  st.r[6] = (dsmoe::lds_char*)st##R6; st.r[7] = (dsmoe::lds_char*)st##R7

// NSRC = 2: the wave's two column tiles are the same 32 columns of source 0 (gate) and source 1 (up).
// The block's eight waves form a WGM x WGN grid over the tile (WGN_ = 4 or 2).
template <int BM_, int BN_, int NSRC_ = 1, bool L_KMAJOR = false, bool R_KMAJOR = true, bool KTAIL = false, int NST_ = 4,
          int WGN_ = 4>
struct Tile3 {
  static constexpr int BM = BM_, BN = BN_, NSRC = NSRC_, BK = kBK2, WGN = WGN_, WGM = 8 / WGN_, NST = NST_;
  static_assert(NST >= 4 && NST <= kMaxStages3, "four to eight stages");
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int MT = WM / 32, NT = WN / 32;
  static_assert(NSRC == 1 || NT == NSRC, "one column tile per source");
  static_assert(NSRC == 1 || R_KMAJOR, "several sources need the k-major weight layout");
  typedef std::conditional_t<L_KMAJOR, DCols<BM, 1, KTAIL>, DRows<BM>> LSrc;
  typedef std::conditional_t<R_KMAJOR, DCols<BN, NSRC, KTAIL>, DRows<BN>> RSrc;
  static constexpr int LDS_L = LSrc::LDS, LDS_R = RSrc::LDS;
  static constexpr int LDS_BYTES = 0;                                   // stages are static arrays of the kernel
  static constexpr int NI = LSrc::NI + RSrc::NI;                        // loads per wave and K step
  static constexpr int WCOL = NSRC == 1 ? WN : 32, NT_COLS = NSRC == 1 ? 32 : BN / NSRC;
  static constexpr int NFR = (L_KMAJOR ? 2 : 1) * MT + (R_KMAJOR ? 2 : 1) * NT;   // LDS reads per K slice
  static constexpr int NMMA = MT * NT;
  typedef f32x16 Acc[NT][MT];
  struct Frag { u32x4 x[MT], w[NT]; };
  struct Offs { int l[2][L_KMAJOR ? MT : 1], r[2][R_KMAJOR ? NT : 1]; };

  static __device__ __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][mt][i] = 0.f;
  }

  static __device__ __forceinline__ void offsets(Offs& o) {
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      if constexpr (L_KMAJOR) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) o.l[ks][mt] = LSrc::frag_off((wave / WGN) * WM + mt * 32, ks);
      } else {
        o.l[ks][0] = LSrc::frag_off((wave / WGN) * WM, ks);
      }
      if constexpr (R_KMAJOR) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) o.r[ks][nt] = RSrc::frag_off((wave % WGN) * WCOL + nt * NT_COLS, ks);
      } else {
        o.r[ks][0] = RSrc::frag_off((wave % WGN) * WCOL, ks);
      }
    }
  }
  static __device__ __forceinline__ void read_frags(Frag& f, const lds_char* sl, const lds_char* sr, const Offs& o,
                                                    int ks) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if constexpr (L_KMAJOR) f.x[mt] = LSrc::read(sl, o.l[ks][mt]);
      else f.x[mt] = LSrc::read(sl, o.l[ks][0], mt);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      if constexpr (R_KMAJOR) f.w[nt] = RSrc::read(sr, o.r[ks][nt]);
      else f.w[nt] = RSrc::read(sr, o.r[ks][0], nt);
    }
  }
  static __device__ __forceinline__ void mma(Acc& acc, const Frag& f) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) Mma<bf16_t>::run(acc[nt][mt], f.w[nt], f.x[mt]);
  }
  // the MFMAs I0 <= nt * MT + mt < I1 of mma()
  template <int I0, int I1>
  static __device__ __forceinline__ void mma_range(Acc& acc, const Frag& f) {
#pragma unroll
    for (int i = I0; i < I1; ++i) Mma<bf16_t>::run(acc[i / MT][i % MT], f.w[i / MT], f.x[i % MT]);
  }
  // issue order for the scheduler: the LDS reads of the next slice go out two per MFMA, so that the last of
  // them has the remaining MFMAs to arrive
  static __device__ __forceinline__ void interleave() {
    constexpr int NG = (NFR + 1) / 2 < NMMA ? (NFR + 1) / 2 : NMMA;
    Interleave<0, NG, NFR, kSgDsRd>::run();
    sched_group<kSgMfma, NMMA - NG>();
  }

  // Position of the next K step to load.
  struct Iter { int seg, kin, next; };
  static __device__ __forceinline__ void issue_step(const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                                    lds_char* sl, lds_char* sr) {
    L.issue(sl, it.seg, it.kin);
    R.issue(sr, it.seg, it.kin);
    // steps past the end re-read the last one (only the variant for ragged step counts asks for them)
    if (++it.next < nkt && ++it.kin == seg_tiles) { it.kin = 0; ++it.seg; }
  }
  struct Loop {   // what a K step needs besides the stage number
    Acc& acc; Frag& fa; Frag& fb; const LSrc& L; const RSrc& R; Iter& it; int nkt, seg_tiles; const Stages3& st;
    const Offs& o;
  };
  // the same, one load instruction at a time: P = 0 .. NI-1, the position advances after the last one
  template <int P>
  static __device__ __forceinline__ void issue_part(const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                                    lds_char* sl, lds_char* sr) {
    if constexpr (P < LSrc::NI) L.issue_one(sl, it.seg, it.kin, P);
    else R.issue_one(sr, it.seg, it.kin, P - LSrc::NI);
    if constexpr (P == NI - 1)
      if (++it.next < nkt && ++it.kin == seg_tiles) { it.kin = 0; ++it.seg; }
  }
  // second half of a K step when it refills a stage: the next slice's fragment reads ride on the first NG MFMAs,
  // then every load instruction of the refill is followed by one MFMA, so that the matrix pipe works through the
  // address arithmetic and the load issue instead of idling behind the barrier
  template <int P, int M0>
  static __device__ __forceinline__ void refill_and_mma(const Loop& q, lds_char* sl, lds_char* sr) {
    if constexpr (P < NI) {
      issue_part<P>(q.L, q.R, q.it, q.nkt, q.seg_tiles, sl, sr);
      if constexpr (M0 < NMMA) mma_range<M0, M0 + 1>(q.acc, q.fb);
      __builtin_amdgcn_sched_barrier(0);
      refill_and_mma<P + 1, (M0 < NMMA ? M0 + 1 : M0)>(q, sl, sr);
    } else {
      mma_range<M0, NMMA>(q.acc, q.fb);
    }
  }

  // First part of the prologue: K steps 0 .. NST-3 into the stages of the same number.  May be called as soon
  // as every wave has left the previous run() (nobody reads the stages any more), e.g. before the previous
  // tile's epilogue, which only touches the wave's own slices of the last two stages.
  template <int ST = 0>
  static __device__ __forceinline__ void prefetch(const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                                  const Stages3& st) {
    if constexpr (ST == 0) { it.seg = 0; it.kin = 0; it.next = 0; }
    if constexpr (ST < NST - 2) {
      issue_step(L, R, it, nkt, seg_tiles, st.l[ST], st.r[ST]);
      prefetch<ST + 1>(L, R, it, nkt, seg_tiles, st);
    }
  }

  // One K step on stage ST: slice 0 multiplies while slice 1 is read; then, once step + 1 has landed for
  // every wave (and every wave has read this stage to the end), the stage is refilled with step + NST and
  // slice 0 of the next stage is read while slice 1 multiplies.  WAITN: loads that may stay in flight.
  template <int ST, int WAITN, bool ISSUE>
  static __device__ __forceinline__ void step(const Loop& q) {
    constexpr int NX = (ST + 1) % NST;
    read_frags(q.fb, q.st.l[ST], q.st.r[ST], q.o, 1);
    mma(q.acc, q.fa);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<WAITN, true>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (ISSUE) {
      constexpr int NG = (NFR + 1) / 2 < NMMA ? (NFR + 1) / 2 : NMMA;
      read_frags(q.fa, q.st.l[NX], q.st.r[NX], q.o, 0);
      mma_range<0, NG>(q.acc, q.fb);
      Interleave<0, NG, NFR, kSgDsRd>::run();
      __builtin_amdgcn_sched_barrier(0);
      refill_and_mma<0, NG>(q, q.st.l[ST], q.st.r[ST]);
    } else {
      read_frags(q.fa, q.st.l[NX], q.st.r[NX], q.o, 0);
      mma(q.acc, q.fb);
      interleave();
    }
  }
  // N consecutive refilling steps from stage ST
  template <int ST, int N>
  static __device__ __forceinline__ void steps(const Loop& q) {
    if constexpr (N > 0) {
      step<ST, (NST - 2) * NI, true>(q);
      steps<(ST + 1) % NST, N - 1>(q);
    }
  }
  // the last NST steps of an exact run: nothing is refilled, ever fewer loads remain in flight
  template <int ST>
  static __device__ __forceinline__ void tail(const Loop& q) {
    if constexpr (ST < NST - 1) {
      step<ST, (NST - 2 - ST) * NI, false>(q);
      tail<ST + 1>(q);
    } else {
      read_frags(q.fb, q.st.l[ST], q.st.r[ST], q.o, 1);
      mma(q.acc, q.fa);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      wait_vm<0, true>();             // own fragment reads done before the stages may be refilled
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      mma(q.acc, q.fb);
    }
  }
  // up to NST - 1 further refilling steps (ragged step counts)
  template <int ST>
  static __device__ __forceinline__ void rest(const Loop& q, int r) {
    if constexpr (ST < NST - 1) {
      if (r > 0) {
        step<ST, (NST - 2) * NI, true>(q);
        rest<ST + 1>(q, r - 1);
      }
    }
  }

  // acc += L * R over nkt K steps (K may be split in segments of seg_tiles steps, see the sources), after
  // prefetch() with the same arguments.  Must be called by all 512 threads; returns with none of this wave's
  // loads in flight and no wave reading the stages any more.
  // Global stores issued between prefetch() and run() are fine: the counter waits below only rely on loads
  // completing in order among loads, so they can at worst wait for such a store too.
  static __device__ __forceinline__ void run(Acc& acc, const LSrc& L, const RSrc& R, Iter& it, int nkt, int seg_tiles,
                                             const Stages3& st) {
    Offs o;
    offsets(o);
    Frag fa, fb;
    issue_step(L, R, it, nkt, seg_tiles, st.l[NST - 2], st.r[NST - 2]);
    issue_step(L, R, it, nkt, seg_tiles, st.l[NST - 1], st.r[NST - 1]);
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<(NST - 1) * NI, true>();  // step 0 has landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(fa, st.l[0], st.r[0], o, 0);
    const Loop q{acc, fa, fb, L, R, it, nkt, seg_tiles, st, o};
    if (nkt % NST == 0) {
      // exact: every load is a real step; the last NST steps refill nothing
      for (int kt = 0; kt + 2 * NST <= nkt; kt += NST) steps<0, NST>(q);
      tail<0>(q);
    } else {
      // ragged step count: loads are issued unconditionally (re-reading the last step into a stage nobody
      // reads any more), which keeps the loop free of branches and the number of loads in flight constant
      int kt = 0;
      for (; kt + NST <= nkt; kt += NST) steps<0, NST>(q);
      rest<0>(q, nkt - kt);
      __builtin_amdgcn_sched_barrier(0);
      wait_vm<0, true>();             // drain the re-read loads
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc& R, int nkt, int seg_tiles,
                                                  const Stages3& st) {
    Iter it;
    prefetch(L, R, it, nkt, seg_tiles, st);
    run(acc, L, R, it, nkt, seg_tiles, st);
  }

  // ---- chained tiles: the load pipeline keeps running from one tile into the next --------------------------
  // A wave cannot count its loads past stores it has in flight (one counter for both, and stores may
  // complete ahead of older loads), so the first counted wait after an epilogue waits for the epilogue's
  // stores.  In a chain that wait comes late: the last K steps of a tile already request steps 0 .. NST-2 of
  // the next one, they have landed before the epilogue's first store, and the next tile's first NST-2 steps
  // need no wait at all.  The stores then have those steps to complete behind the MFMAs.  The epilogue
  // between two run_chain() calls may use the wave's own slices of stage NST-1 only.
  // Needs nkt % NST == 0 and nkt >= 2 * NST.
  static constexpr bool chainable(int nkt) { return nkt % NST == 0 && nkt >= 2 * NST; }
  static __device__ __forceinline__ void chain_begin(const LSrc& L, const RSrc& R, Iter& it, int nkt, const Stages3& st) {
    it.seg = 0; it.kin = 0; it.next = 0;
    chain_issue<0>(L, R, it, nkt, st);
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<0, true>();
    __builtin_amdgcn_sched_barrier(0);
  }
  template <int ST>
  static __device__ __forceinline__ void chain_issue(const LSrc& L, const RSrc& R, Iter& it, int nkt, const Stages3& st) {
    if constexpr (ST < NST - 1) {
      issue_step(L, R, it, nkt, 1 << 30, st.l[ST], st.r[ST]);
      chain_issue<ST + 1>(L, R, it, nkt, st);
    }
  }
  // N consecutive refilling steps from stage ST whose next step is known to have landed
  template <int ST, int N>
  static __device__ __forceinline__ void steps_landed(const Loop& q) {
    if constexpr (N > 0) {
      step<ST, 63, true>(q);
      steps_landed<(ST + 1) % NST, N - 1>(q);
    }
  }
  // acc += L * R for one tile of a chain.  On entry this tile's steps 0 .. NST-2 have been requested and every
  // wave has seen its own land; (Ln, Rn, itn) is the next tile at step 0, or a copy of (L, R, it) when there is
  // none (the last steps then re-read into stages nobody reads any more).  On return the next tile's steps
  // 0 .. NST-2 have landed as far as this wave requested them, itn stands at step NST-1, and no wave reads
  // stage NST-1 any more.
  static __device__ __forceinline__ void run_chain(Acc& acc, const LSrc& L, const RSrc& R, Iter& it, const LSrc& Ln,
                                                   const RSrc& Rn, Iter& itn, int nkt, const Stages3& st) {
    Offs o;
    offsets(o);
    Frag fa, fb;
    issue_step(L, R, it, nkt, 1 << 30, st.l[NST - 1], st.r[NST - 1]);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();     // every wave's share of steps 0 .. NST-2 has landed
    __builtin_amdgcn_sched_barrier(0);
    read_frags(fa, st.l[0], st.r[0], o, 0);
    const Loop q{acc, fa, fb, L, R, it, nkt, 1 << 30, st, o};
    const Loop qn{acc, fa, fb, Ln, Rn, itn, nkt, 1 << 30, st, o};
    steps_landed<0, NST - 2>(q);
    steps<NST - 2, 2>(q);
    for (int kt = NST; kt + 2 * NST <= nkt; kt += NST) steps<0, NST>(q);
    steps<0, NST - 1>(qn);
    read_frags(fb, st.l[NST - 1], st.r[NST - 1], o, 1);
    mma(acc, fa);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<0, true>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    mma(acc, fb);
  }

  // Transposed walk over the accumulators.  The MFMA leaves a lane with one row and 4 consecutive columns
  // per register quad, which makes 8-byte accesses spread over 32 rows.  Here every 32-row block of the
  // wave goes through the wave's own slices of the last two stages (fp32, XOR-swizzled 16-byte units, no
  // barrier needed: no other wave writes there once this wave's loads have drained; the first stages may
  // already be receiving the next tile, see prefetch()), and comes back with
  // a lane owning 8 consecutive columns of one row: f(m, n, v) gets the tile row m, the first column n
  // (inside its source) and v[s][0..7]; 8 (NSRC = 1) or 4 (NSRC = 2) neighbouring lanes cover a row, so
  // global accesses made from f are whole 128-byte (bf16: 64..128-byte) row segments.
  static constexpr int CHUNK = 8;
  // The thread index as a value the compiler cannot trace back to threadIdx: everything an epilogue derives from
  // it (row and column of a lane, LDS offsets) is then computed inside the epilogue instead of being hoisted out
  // of the tile loop and kept, spilled, across the main loop.  A spill reload is a vector-memory load, and the
  // wait for it would also wait for every global store the epilogue has issued.
  static __device__ __forceinline__ int epilogue_tid() { return opaque_tid(); }
  // load(j, m, n) is called for the NJ chunks of a 32-row block before the block crosses the LDS, f(j, m, n, v)
  // after: global loads an epilogue needs (saved activations ...) are then all in flight together and ahead of
  // the block's stores, instead of each waiting behind the stores of the chunk before.
  // LOADS: `load` really issues global loads.  They are then waited for once per block, before the block's first
  // store: the compiler cannot count a load behind stores in flight (this ISA has one counter for both and lets
  // them complete out of order), so a loaded value first used after a store costs a full drain of the stores.
  static constexpr int NJ = NSRC == 1 ? 4 : 2;
  template <bool LOADS = false, class LD, class F>
  static __device__ __forceinline__ void for_each_chunk(const Acc& acc, const Stages3& st, LD load, F f) {
    static_assert(RSrc::LDS / 8 == 2048 && LSrc::LDS / 8 == 2048, "a wave's slice of a stage holds 8 rows of 64 floats");
    constexpr int OPR = NSRC == 1 ? 8 : 4;        // lanes (column octets) per row and source
    constexpr int RPI = 64 / OPR;                  // rows covered by one read instruction
    static_assert(NJ == 32 / RPI, "chunks of a lane per 32-row block");
    const int tid = epilogue_tid();
    const int lane = tid & 63, wave = tid >> 6;
    const int wslice = wave * 2048;
    const int m = lane & 31, kg = lane >> 5;
    // the stage addresses are link-time constants: keep them as values (a table in memory would be indexed)
    lds_char* const r0 = st.r[NST - 2];
    lds_char* const r1 = st.r[NST - 1];
    lds_char* const r2 = st.l[NST - 2];
    lds_char* const r3 = st.l[NST - 1];
    auto area = [=](int row) -> lds_char* {        // 8 rows of 256 bytes in each of the four stages
      const int piece = row >> 3;
      lds_char* const lo = (piece & 1) ? r1 : r0;
      lds_char* const hi = (piece & 1) ? r3 : r2;
      return ((piece & 2) ? hi : lo) + wslice + (row & 7) * 256;
    };
    lds_char* wrow = area(m);
    const int q = lane % OPR;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        load(j, (wave / WGN) * WM + mt * 32 + RPI * j + lane / OPR, (wave % WGN) * WCOL + 8 * q);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int u = nt * 8 + g * 2 + kg;
          f32x4 v = {acc[nt][mt][4 * g], acc[nt][mt][4 * g + 1], acc[nt][mt][4 * g + 2], acc[nt][mt][4 * g + 3]};
          lds_write16_free(wrow + ((u ^ (m & 15)) * 16), __builtin_bit_cast(u32x4, v));
        }
      if constexpr (LOADS) wait_vm<0, false>();
#pragma unroll
      for (int j = 0; j < 32 / RPI; ++j) {
        const int r = RPI * j + lane / OPR;
        const lds_char* rrow = area(r);
        float v[NSRC][8];
#pragma unroll
        for (int s = 0; s < NSRC; ++s) {
          const int ub = s * 8 + 2 * q;
          u32x4 ua, ub4;
          lds_read16x2_free(rrow + ((ub ^ (r & 15)) * 16), rrow + (((ub + 1) ^ (r & 15)) * 16), ua, ub4);
          const f32x4 a = __builtin_bit_cast(f32x4, ua), b = __builtin_bit_cast(f32x4, ub4);
          v[s][0] = a.x; v[s][1] = a.y; v[s][2] = a.z; v[s][3] = a.w;
          v[s][4] = b.x; v[s][5] = b.y; v[s][6] = b.z; v[s][7] = b.w;
        }
        f(j, (wave / WGN) * WM + mt * 32 + r, (wave % WGN) * WCOL + 8 * q, v);
      }
    }
  }

  // Packed variant for bf16 outputs: pre(mt, m, n, v, out) runs in the accumulator layout (row m, 4 consecutive
  // columns from n, v[s][0..3]) and produces NOUT values per element; they are rounded to bf16, staged (one
  // 2 KB piece of the wave's scratch slices per output and 32-column tile: 32 rows of 64 bytes, XOR-swizzled),
  // and handed to f(m, n, p) with p[o] = 8 consecutive bf16 of output o, 4 lanes covering a 64-byte row
  // segment.  A quarter of the LDS traffic of the fp32 walk when the epilogue has one output.
  // LAST_STAGE: the scratch pieces lie in stage NST-1 alone (at most two; for the epilogues of a chain).
  template <int NOUT, bool LAST_STAGE = false, class P, class F>
  static __device__ __forceinline__ void for_each_chunk_bf16(const Acc& acc, const Stages3& st, P pre, F f) {
    constexpr int NTC = NSRC == 1 ? NT : 1;       // 32-column tiles of an output per wave
    static_assert(NOUT * NTC <= (LAST_STAGE ? 2 : 4), "four scratch pieces per wave, two in one stage");
    // the first two pieces lie in the right operand's stages, the other two in the left operand's
    static_assert(RSrc::LDS / 8 == 2048 && (NOUT * NTC <= (LAST_STAGE ? 1 : 2) || LSrc::LDS / 8 == 2048),
                  "a wave's slice of a stage holds 32 rows of 64 bytes");
    const int tid = epilogue_tid();
    const int lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kg = lane >> 5;
    lds_char* const piece[4] = {st.r[LAST_STAGE ? NST - 1 : NST - 2] + wave * 2048,
                                (LAST_STAGE ? st.l[NST - 1] : st.r[NST - 1]) + wave * 2048,
                                st.l[NST - 2] + wave * 2048, st.l[NST - 1] + wave * 2048};
    const int woff = m * 64 + kg * 8, wsw = (m >> 2) & 3;
    const int rrow = lane >> 2, rq = lane & 3;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int tc = 0; tc < NTC; ++tc)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v[NSRC][4];
          float out[NOUT][4];
#pragma unroll
          for (int s = 0; s < NSRC; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) v[s][i] = acc[NSRC == 1 ? tc : s][mt][4 * g + i];
          pre(mt, acc_m(mt), acc_n(tc, g), v, out);
#pragma unroll
          for (int o = 0; o < NOUT; ++o) {
            const u32x2 pk = {pack_bf16x2(out[o][0], out[o][1]), pack_bf16x2(out[o][2], out[o][3])};
            lds_write8_free(piece[o * NTC + tc] + woff + ((g ^ wsw) * 16), pk);
          }
        }
#pragma unroll
      for (int tc = 0; tc < NTC; ++tc)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int r = 16 * j + rrow;
          u32x4 p[NOUT];
#pragma unroll
          for (int o = 0; o < NOUT; ++o)
            p[o] = lds_read16_free(piece[o * NTC + tc] + r * 64 + ((rq ^ ((r >> 2) & 3)) * 16));
          f((wave / WGN) * WM + mt * 32 + r, (wave % WGN) * WCOL + tc * 32 + 8 * rq, p);
        }
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
