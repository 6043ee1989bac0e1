// Tiled MFMA contraction shared by the expert-FFN and dense-training kernels (gfx950).
//
//   Out[m][n] = sum_k L[m][k] * R[k][n]
//
// "L" is the token-side operand (m indexes tokens / rows of the output), "R" the weight-side
// operand.  A block of 256 threads (2 x 2 waves) owns a BM x BN output tile per R source; up to NR
// R sources share one L tile (gate and up projections).  Each K step stages 128 bytes of every
// operand row (64 bf16 or 32 fp32 values) in LDS as [row][k] with a 144-byte row pitch, which
// makes the 16-byte fragment reads of 32 consecutive rows conflict-free.  Global loads for the next
// K step are issued into registers before the MFMA work of the current one.
//
// The weight fragment is the MFMA "A" operand and the token fragment the "B" operand, so that a
// lane of the 32x32 accumulator owns ONE token and four consecutive output columns per register
// quad: per-token scalars (row weights, router scores) are per-lane values and stores are 8/16 bytes.
#pragma once

#include "common.h"

namespace dsmoe {

constexpr int kThreads = 256;
constexpr int kRowBytes = 128;   // bytes of an operand row staged per K tile
constexpr int kLdsPitch = 144;   // padded LDS row pitch

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
  static constexpr int VEC = 4;   // elements per 16 bytes
  static constexpr int BK = 32;   // elements per K tile
};
template <> struct ElemTraits<bf16_t> {
  static constexpr int VEC = 8;
  static constexpr int BK = 64;
};

// 16-byte load through the GLOBAL address space.  Pointers that reach the loaders through structs or
// selects lose their address space; a generic (flat) load would also tie up the LDS counter and force
// full waits, which serialises the software pipeline.
typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
typedef __attribute__((address_space(1))) u32x4 global_u32x4_w;
typedef __attribute__((address_space(1))) u32x2 global_u32x2_w;
__device__ __forceinline__ u32x4 ldg16(const void* p) { return *(global_u32x4*)(p); }
__device__ __forceinline__ void stg16(void* p, u32x4 v) { *(global_u32x4_w*)(p) = v; }
__device__ __forceinline__ void stg8(void* p, u32x2 v) { *(global_u32x2_w*)(p) = v; }

// ---- operand sources ---------------------------------------------------------------------------

// Rows stored k-contiguous in memory (activations X / H, or a weight used transposed).
// Thread t stages rows (t/8 + 32 i), 16-byte column t%8 of each 128-byte K slice.
template <typename T, int ROWS>
struct SrcRows {
  static constexpr int NV = ROWS / 32;
  const char* p[NV];     // row base + (t%8)*16 bytes, K segment 0
  size_t seg_stride;     // bytes between K segments (0 if K is one contiguous run)

  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
    const size_t off = (size_t)seg * seg_stride + (size_t)kin * kRowBytes;
#pragma unroll
    for (int i = 0; i < NV; ++i) r[i] = ldg16(p[i] + off);
  }
  __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) const {
    char* q = lds + (threadIdx.x >> 3) * kLdsPitch + (threadIdx.x & 7) * 16;
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<u32x4*>(q + i * 32 * kLdsPitch) = r[i];
  }
};

// register transpose of a VEC x VEC block: in[v] holds VEC consecutive rows of K index v,
// out[n] holds VEC consecutive K values of row n.
__device__ __forceinline__ void transpose_block(const u32x4 (&in)[4], u32x4 (&out)[4], float) {
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    out[n][0] = in[0][n]; out[n][1] = in[1][n]; out[n][2] = in[2][n]; out[n][3] = in[3][n];
  }
}
__device__ __forceinline__ void transpose_block(const u32x4 (&in)[8], u32x4 (&out)[8], bf16_t) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {     // dword j of a source vector holds rows 2j (low half) and 2j+1 (high half)
#pragma unroll
    for (int p = 0; p < 4; ++p) {   // K pair (2p, 2p+1)
      const unsigned ev = in[2 * p][j], od = in[2 * p + 1][j];
      out[2 * j][p] = (ev & 0xffffu) | (od << 16);
      out[2 * j + 1][p] = (ev >> 16) | (od & 0xffff0000u);
    }
  }
}

// Operand stored [k][row] with rows contiguous (a weight matrix W[k][n], or X^T / dY for the
// weight gradients).  Threads load VEC x VEC blocks with 16-byte loads and transpose in registers.
template <typename T, int ROWS>
struct SrcCols {
  static constexpr int VEC = ElemTraits<T>::VEC;
  static constexpr int BK = ElemTraits<T>::BK;
  static constexpr int RB = ROWS / VEC;                 // blocks along the row dimension
  static constexpr int NBLK = (BK / VEC) * RB;          // blocks per K tile
  static constexpr int NBT = (NBLK + kThreads - 1) / kThreads;
  static constexpr int NV = NBT * VEC;
  const char* base;    // element [k = 0][first row of the tile], K segment 0
  size_t ld_bytes;     // bytes between consecutive k
  size_t seg_stride;   // bytes between K segments
  int rows_valid;      // rows >= rows_valid are zero-filled (multiple of VEC)
  int k_valid;         // k >= k_valid (within a segment) are zero-filled

  __device__ __forceinline__ void load(u32x4 (&r)[NV], int seg, int kin) const {
#pragma unroll
    for (int j = 0; j < NBT; ++j) {
      const int b = threadIdx.x + j * kThreads;
      const int rb = b % RB, kb = b / RB;
      const int k0 = kin * BK + kb * VEC;
      const char* q = base + (size_t)seg * seg_stride + (size_t)k0 * ld_bytes + rb * 16;
      const bool ok = (NBLK % kThreads == 0 || b < NBLK) && rb * VEC < rows_valid;
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        u32x4 z = {0u, 0u, 0u, 0u};
        r[j * VEC + v] = (ok && k0 + v < k_valid) ? ldg16(q + (size_t)v * ld_bytes) : z;
      }
    }
  }
  __device__ __forceinline__ void store(const u32x4 (&r)[NV], char* lds) const {
#pragma unroll
    for (int j = 0; j < NBT; ++j) {
      const int b = threadIdx.x + j * kThreads;
      if (NBLK % kThreads != 0 && b >= NBLK) continue;
      const int rb = b % RB, kb = b / RB;
      u32x4 in[VEC], out[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) in[v] = r[j * VEC + v];
      transpose_block(in, out, T());
      char* q = lds + (rb * VEC) * kLdsPitch + kb * 16;
#pragma unroll
      for (int n = 0; n < VEC; ++n) *reinterpret_cast<u32x4*>(q + n * kLdsPitch) = out[n];
    }
  }
};

// ---- MFMA step over one 32-byte K slice --------------------------------------------------------
template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
  static __device__ __forceinline__ void run(f32x16& acc, const u32x4& w, const u32x4& x) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x),
                                                  acc, 0, 0, 0);
  }
};
template <> struct Mma<float> {
  static __device__ __forceinline__ void run(f32x16& acc, const u32x4& w, const u32x4& x) {
    const f32x4 wf = __builtin_bit_cast(f32x4, w), xf = __builtin_bit_cast(f32x4, x);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.x, xf.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.y, xf.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.z, xf.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.w, xf.w, acc, 0, 0, 0);
  }
};

template <typename T, int BM_, int BN_, int NR_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, NR = NR_;
  static constexpr int BK = ElemTraits<T>::BK;
  static constexpr int WM = BM / 2, WN = BN / 2;   // 2 x 2 waves
  static constexpr int MT = WM / 32, NT = WN / 32;
  static constexpr int LDS_L = BM * kLdsPitch, LDS_R = BN * kLdsPitch;
  static constexpr int LDS_BYTES = LDS_L + NR * LDS_R;
  typedef f32x16 Acc[NR][NT][MT];

  static __device__ __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int b = 0; b < NR; ++b)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[b][nt][mt][i] = 0.f;
  }

  // acc += L * R over nkt K tiles; K may be split in segments of seg_tiles tiles (see the sources).
  template <typename LSrc, typename RSrc>
  static __device__ __forceinline__ void mainloop(Acc& acc, const LSrc& L, const RSrc (&R)[NR], int nkt,
                                                  int seg_tiles, char* smem) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const char* fL = smem + (wm * WM + (lane & 31)) * kLdsPitch + (lane >> 5) * 16;
    const char* fR = smem + LDS_L + (wn * WN + (lane & 31)) * kLdsPitch + (lane >> 5) * 16;

    u32x4 lr[LSrc::NV];
    u32x4 rr[NR][RSrc::NV];
    int seg = 0, kin = 0;
    L.load(lr, 0, 0);
#pragma unroll
    for (int b = 0; b < NR; ++b) R[b].load(rr[b], 0, 0);

    for (int kt = 0; kt < nkt; ++kt) {
      __syncthreads();   // every wave has finished reading the previous tile
      L.store(lr, smem);
#pragma unroll
      for (int b = 0; b < NR; ++b) R[b].store(rr[b], smem + LDS_L + b * LDS_R);
      __syncthreads();
      if (kt + 1 < nkt) {
        if (++kin == seg_tiles) { kin = 0; ++seg; }
        L.load(lr, seg, kin);
#pragma unroll
        for (int b = 0; b < NR; ++b) R[b].load(rr[b], seg, kin);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        u32x4 xf[MT], wf[NR][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xf[mt] = *reinterpret_cast<const u32x4*>(fL + mt * 32 * kLdsPitch + ks * 32);
#pragma unroll
        for (int b = 0; b < NR; ++b)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            wf[b][nt] = *reinterpret_cast<const u32x4*>(fR + b * LDS_R + nt * 32 * kLdsPitch + ks * 32);
#pragma unroll
        for (int b = 0; b < NR; ++b)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) Mma<T>::run(acc[b][nt][mt], wf[b][nt], xf[mt]);
      }
    }
  }

  // Coordinates of accumulator quad g (0..3) of tile (nt, mt) held by this lane:
  // token row m (local to the block tile) and first of 4 consecutive columns n.
  static __device__ __forceinline__ int acc_m(int mt) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave & 1) * WM + mt * 32 + (lane & 31);
  }
  static __device__ __forceinline__ int acc_n(int nt, int g) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    return (wave >> 1) * WN + nt * 32 + g * 8 + (lane >> 5) * 4;
  }
};

// ---- output helpers ----------------------------------------------------------------------------
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
  f32x4 v = {a, b, c, d};
  stg16(p, __builtin_bit_cast(u32x4, v));
}
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
  u32x2 v = {pack_bf16x2(a, b), pack_bf16x2(c, d)};
  stg8(p, v);
}
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

// Per-block table of row tiles of a grouped (per-expert) problem, built from expert_off.
struct GroupTiles {
  int tile_off[kMaxExperts + 1];   // exclusive prefix sum of ceil(cnt_e / BM)
  int row_off[kMaxExperts + 1];
};
// expert_off == nullptr: every group has uniform_rows rows (dense layer: all tokens in every expert).
__device__ __forceinline__ void build_group_tiles(GroupTiles& g, const int32_t* __restrict__ expert_off, int E, int BM,
                                                  int uniform_rows = 0) {
  if (threadIdx.x < 64) {
    const int e = threadIdx.x;
    int lo = 0, hi = 0;
    if (e < E) {
      lo = expert_off ? expert_off[e] : e * uniform_rows;
      hi = expert_off ? expert_off[e + 1] : (e + 1) * uniform_rows;
    }
    int t = (hi - lo + BM - 1) / BM;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(t, s, 64);
      if (e >= s) t += o;
    }
    g.tile_off[e + 1] = t;
    if (e == 0) g.tile_off[0] = 0;
    if (e < E) g.row_off[e] = lo;
    if (e == E - 1) g.row_off[E] = hi;
  }
  __syncthreads();
}
__device__ __forceinline__ int find_group(const GroupTiles& g, int E, int tile) {
  int lo = 0, hi = E - 1;   // largest e with tile_off[e] <= tile
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (g.tile_off[mid] <= tile) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Maps the block to its next tile: tiles are dealt to the 8 XCDs in 8 contiguous chunks (workgroup
// ids are distributed round-robin over XCDs), so an XCD's L2 sees consecutive tiles of few experts.
struct TileWalker {
  int total, per, slots, xcd, i;
  __device__ __forceinline__ void init(int total_tiles) {
    total = total_tiles;
    per = (total + 7) >> 3;
    slots = gridDim.x >> 3;
    xcd = blockIdx.x & 7;
    i = blockIdx.x >> 3;
  }
  __device__ __forceinline__ bool next(int& idx) {
    if (i >= per) return false;
    idx = xcd * per + i;
    i += slots;
    return idx < total;
  }
};

// Row tiles of a grouped problem in two heights.  An expert's rows are cut into full tiles of 2 * HB rows; a
// remainder of more than HB rows is one more (ragged) full tile, a remainder of 1 .. HB rows is a half tile.
struct SplitTiles {
  int full_off[kMaxExperts + 1];   // exclusive prefix sums of the experts' full tiles ...
  int half_off[kMaxExperts + 1];   // ... and of their half tiles (0 or 1 each)
  int row_off[kMaxExperts + 1];
};
__device__ __forceinline__ void build_split_tiles(SplitTiles& g, const int32_t* __restrict__ expert_off, int E, int HB,
                                                  int uniform_rows = 0) {
  if (threadIdx.x < 64) {
    const int e = threadIdx.x;
    int lo = 0, hi = 0;
    if (e < E) {
      lo = expert_off ? expert_off[e] : e * uniform_rows;
      hi = expert_off ? expert_off[e + 1] : (e + 1) * uniform_rows;
    }
    const int units = (hi - lo + HB - 1) / HB;
    int nf = units >> 1, nh = units & 1;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int of = __shfl_up(nf, s, 64), oh = __shfl_up(nh, s, 64);
      if (e >= s) { nf += of; nh += oh; }
    }
    g.full_off[e + 1] = nf;
    g.half_off[e + 1] = nh;
    if (e == 0) { g.full_off[0] = 0; g.half_off[0] = 0; }
    if (e < E) g.row_off[e] = lo;
    if (e == E - 1) g.row_off[E] = hi;
  }
  __syncthreads();
}
__device__ __forceinline__ int find_in_prefix(const int* off, int E, int i) {
  int lo = 0, hi = E - 1;   // largest e with off[e] <= i
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (off[mid] <= i) lo = mid; else hi = mid - 1;
  }
  return lo;
}

struct RowTile { int e, row0, valid, nt; };   // expert, first row, rows, column tile

// Deals the tiles of a SplitTiles table (times n_tiles column tiles, column tile fastest) to a persistent
// grid.  Full and half tiles are each cut in 8 contiguous chunks, one per XCD, and a chunk's tiles go round
// robin over the XCD's blocks: first the full tiles (next_full), then the half tiles (next_half).  When the
// full tiles do not fill the blocks' last turn evenly and there is room, the ones left over are cut in two
// halves and dealt with the half tiles, so that the last turn costs every block half a tile instead of
// costing few blocks a whole one.
struct SplitWalker {
  int n_tiles, slots, HB;
  int fi, f_end;                    // next full tile of this block, end of the ones dealt as full tiles
  int n_split, h_begin, n_p2, j;    // full tiles dealt as two halves (from f_end on), first half tile, items, next
  __device__ __forceinline__ void init(const SplitTiles& g, int E, int n_tiles_, int HB_) {
    n_tiles = n_tiles_;
    HB = HB_;
    slots = gridDim.x >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int F = g.full_off[E] * n_tiles, H = g.half_off[E] * n_tiles;
    const int per = (F + 7) >> 3, perh = (H + 7) >> 3;
    const int f_begin = min(F, xcd * per), f_stop = min(F, f_begin + per);
    h_begin = min(H, xcd * perh);
    const int h_cnt = min(H, h_begin + perh) - h_begin;
    const int left = (f_stop - f_begin) % slots;
    const bool split = left > 0 && 2 * left + h_cnt <= slots;
    n_split = split ? left : 0;
    f_end = f_stop - n_split;
    n_p2 = 2 * n_split + h_cnt;
    fi = f_begin + slot;
    // the half tiles start at the first block that has no full tile in the last turn
    j = (slot - (split ? 0 : left) + slots) % slots;
  }
  __device__ __forceinline__ void full_tile(const SplitTiles& g, int E, int idx, RowTile& t) const {
    const int mg = idx / n_tiles;
    t.nt = idx - mg * n_tiles;
    t.e = find_in_prefix(g.full_off, E, mg);
    t.row0 = g.row_off[t.e] + (mg - g.full_off[t.e]) * 2 * HB;
    t.valid = min(2 * HB, g.row_off[t.e + 1] - t.row0);
  }
  __device__ __forceinline__ bool next_full(const SplitTiles& g, int E, RowTile& t) {
    if (fi >= f_end) return false;
    full_tile(g, E, fi, t);
    fi += slots;
    return true;
  }
  __device__ __forceinline__ bool next_half(const SplitTiles& g, int E, RowTile& t) {
    if (j >= n_p2) return false;
    if (j < 2 * n_split) {           // a full tile has more than HB rows: both halves hold rows
      full_tile(g, E, f_end + (j >> 1), t);
      t.row0 += (j & 1) * HB;
      t.valid = min(HB, t.valid - (j & 1) * HB);
    } else {
      const int idx = h_begin + j - 2 * n_split, hm = idx / n_tiles;
      t.nt = idx - hm * n_tiles;
      t.e = find_in_prefix(g.half_off, E, hm);
      t.row0 = g.row_off[t.e] + (g.full_off[t.e + 1] - g.full_off[t.e]) * 2 * HB;
      t.valid = g.row_off[t.e + 1] - t.row0;
    }
    j += slots;
    return true;
  }
};

// the reciprocal instruction (1 ulp) instead of a full-precision division: ten instructions fewer per element
__device__ __forceinline__ float silu_f(float g) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)); }
// exact GeLU: g * Phi(g)
__device__ __forceinline__ float gelu_f(float g) { return 0.5f * g * (1.f + erff(g * 0.70710678118654752f)); }
// Phi(g) for results that are rounded to bf16: erf by a degree-5 polynomial in 1 / (1 + p |x|) times the Gaussian
// (Abramowitz & Stegun 7.1.26, absolute error 1.5e-7: three orders below the 2^-9 step of the storage type), about
// a third of the instructions of the library erf, which weigh on the epilogue of a 64-step tile.
__device__ __forceinline__ float gelu_cdf_bf16_f(float g) {
  const float x = fabsf(g) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float half_tail = 0.5f * p * t * __expf(-x * x);     // (1 - erf |x|) / 2
  return g < 0.f ? half_tail : 1.f - half_tail;
}
__device__ __forceinline__ float gelu_bf16_f(float g) { return g * gelu_cdf_bf16_f(g); }

}  // namespace dsmoe
