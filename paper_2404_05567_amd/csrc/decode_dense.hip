// Sparse-inference forward (Eq. 1) for decode-sized batches in which nearly every expert is selected by some
// token: with a few dozen tokens and a handful of experts per token the union of the selected experts is the
// whole layer, so the call is bound by reading ALL expert weights once (paper Sec. 4.4: decoding is I/O-bound)
// and is laid out as one persistent kernel that never stops streaming them:
//
//   * rows are the tokens themselves: every expert is evaluated for all T <= 128 tokens (the MFMA tile has
//     128 rows anyway) and the router weight, or 0 for a token that did not select the expert, is applied
//     to the hidden activations: Ht[t, e f + c] = S[t,e] [e in A(t)] act(x_t W_gate[e])_c (x_t W_up[e])_c.
//     The layer output is then ONE product over the concatenated hidden width, O = Ht [W_down[0]; ..; W_down[E-1]]
//     (W_down[E,f,d] is that [E f, d] matrix as stored).  No dispatch, no gather, no per-expert combine;
//   * the router runs inside the kernel: block t scores token t (all experts), selects, and publishes the
//     token's probabilities and mask with write-through stores while its first weight tiles are in flight;
//     the values are needed only ~20 us later, in the epilogues;
//   * work is dealt by XCD (the eight dies, each with its own L2; a block reads from the hardware which one it
//     runs on): XCD x computes the hidden columns of experts [x E/8, (x+1) E/8)
//     and then the part of the output product whose K range is exactly those columns.  The hidden activations
//     therefore pass from producer to consumer blocks through that XCD's L2 alone: a producer waits until its
//     stores have reached the L2 and bumps a counter, a consumer polls the counter (bounded) before it reads;
//     no device-wide cache write-back or invalidation sits between the two phases, and the weight stream of the
//     second phase can start while the block still waits;
//   * the eight (or 16, 32) K-range partial outputs are added in a fixed order by a small second kernel.
// Results are bitwise reproducible: no floating-point atomics, every sum has a fixed order.
#include <algorithm>

#include "gemm.h"
#include "router_common.h"

namespace dsmoe {

namespace {

constexpr int kDT = kDecodeMaxTokens;

// Development aid (-DDSMOE_TRACE): every block records when it passed each point of the kernel, in 10 ns ticks.
#ifdef DSMOE_TRACE
#define DSMOE_MARK(i) do { if (threadIdx.x == 0) a.trace[blockIdx.x * 16 + (i)] = (long long)__builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define DSMOE_MARK(i) do { } while (0)
#endif

__device__ __forceinline__ int sync_load(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// every store this wave has issued has been acknowledged by the L2 (or by memory, for write-through stores)
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Called by all threads.  Returns once *ctr >= target; gives up after `limit` polls and raises the deferred
// status instead (the caller then goes on with whatever the memory holds: every access stays in bounds).
// first failure of a call: what the block saw, for the message of dsmoe_poll_error
__device__ __forceinline__ void raise_internal(int32_t* sync, int32_t* err_flag, int reason, int counter, int seen,
                                               int wanted) {
  int32_t* diag = sync + kDenseSyncWords;   // kDenseDiagWords words
  if (__hip_atomic_exchange(diag, reason, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
    diag[1] = blockIdx.x; diag[2] = (int)xcc_id(); diag[3] = counter; diag[4] = seen; diag[5] = wanted;
  }
  __hip_atomic_store(err_flag, (int32_t)DSMOE_ERR_INTERNAL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void wait_at_least(int32_t* sync, int counter, int target, int limit, int32_t* err_flag) {
  if (threadIdx.x == 0) {
    bool ok = false;
    int seen = 0;
    for (int i = 0; i < limit && !ok; ++i) {
      seen = sync_load(sync + counter);
      ok = seen >= target;
      if (!ok) __builtin_amdgcn_s_sleep(2);
    }
    if (!ok) raise_internal(sync, err_flag, 2, counter, seen, target);
  }
  __syncthreads();
}

struct DenseDecodeArgs {
  const bf16_t* x; const bf16_t* w_r; const bf16_t* b_r;
  const bf16_t* w_gate; const bf16_t* w_up; const bf16_t* w_down;
  float* probs; unsigned long long* mask; int32_t* cnt_tok;
  bf16_t* ht;          // [T][E f]
  float* part;         // [8 KS][T][d]
  int32_t* sync;       // kDenseSyncWords, zero between calls
  int32_t* err_flag;
  int T, d, f, E, mode, k; float eps;
  long long max_rows;
  int KS;              // partial outputs per XCD (K chunks of its range in the output product)
  int spin_limit;
  long long* trace;    // development aid: [grid][16] time stamps
};

// Called by all threads.  Returns once bits [i0, i1) of the bitmap are all set (bounded like wait_at_least).
__device__ __forceinline__ void wait_bits(int32_t* sync, const int32_t* words, int i0, int i1, int limit, int32_t* err_flag) {
  if (threadIdx.x == 0) {
    for (int w = i0 >> 5; w * 32 < i1; ++w) {
      const int lo = max(i0 - w * 32, 0), hi = min(i1 - w * 32, 32);
      const unsigned want = (hi == 32 ? ~0u : (1u << hi) - 1u) & ~((1u << lo) - 1u);
      bool ok = false;
      unsigned seen = 0;
      for (int i = 0; i < limit && !ok; ++i) {
        seen = (unsigned)sync_load(words + w);
        ok = (seen & want) == want;
        if (!ok) __builtin_amdgcn_s_sleep(2);
      }
      if (!ok) raise_internal(sync, err_flag, 2, (int)(words - sync) + w, (int)seen, (int)want);
    }
  }
  __syncthreads();
}

// Work items of a phase belong to an XCD (their data meets in that XCD's L2) and are claimed in a bitmap of that
// XCD: a block first takes item `slot`, `slot + slots`, .. of the XCD it actually runs on - with the usual
// round-robin placement (block b on XCD b mod 8) every such claim succeeds, and the first one is made at kernel
// start, while the item's first loads are in flight - and then whatever is still unclaimed, e.g. the items of a
// block that the hardware placed on another XCD.  Every item is run exactly once, by a block of the right XCD.
struct ItemClaims {
  int32_t* words;      // this XCD's bitmap of the phase
  int items, slots, next_static;
  int first;           // the item claimed at kernel start (-1: none), handed out first
  bool all_claimed;    // a look at the bitmap, taken when every block had long started, showed no item unclaimed
  int* s_item;         // LDS word for the block-wide answer
  static __device__ __forceinline__ bool claim_bit(int32_t* words, int item) {   // one thread
    const int bit = 1 << (item & 31);
    return !(__hip_atomic_fetch_or(words + (item >> 5), bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit);
  }
  static __device__ __forceinline__ bool none_unclaimed(const int32_t* words, int items) {   // one thread
    bool none = true;
    for (int w = 0; w * 32 < items; ++w) {
      const int n = min(32, items - w * 32);
      const unsigned valid = n == 32 ? ~0u : (1u << n) - 1u;
      none = none && (~(unsigned)sync_load(words + w) & valid) == 0u;
    }
    return none;
  }
  // the next item of this block, or -1 when the XCD has none left unclaimed (all threads)
  __device__ __forceinline__ int next() {
    if (first != -2) {
      const int r = first;
      first = -2;
      if (r >= 0) return r;
    }
    if (next_static >= items && all_claimed) return -1;
    if (threadIdx.x == 0) {
      int got = -1;
      while (next_static < items && got < 0) {
        if (claim_bit(words, next_static)) got = next_static;
        next_static += slots;
      }
      for (int w = 0; w * 32 < items && got < 0; ++w) {
        const int n = min(32, items - w * 32);
        const unsigned valid = n == 32 ? ~0u : (1u << n) - 1u;
        unsigned freeb = ~(unsigned)sync_load(words + w) & valid;
        while (freeb != 0 && got < 0) {
          const int i = __builtin_ctz(freeb);
          if (claim_bit(words, w * 32 + i)) got = w * 32 + i;
          freeb &= ~(1u << i);
        }
      }
      s_item[0] = got;
      s_item[1] = next_static;
    }
    __syncthreads();
    const int item = s_item[0];
    next_static = s_item[1];
    __syncthreads();
    return item;
  }
};

// EP: experts padded to 32 or 64 for the router; with 32 its scratch leaves room for eight LDS stages (six K steps
// of weights in flight per CU) instead of six.
template <bool GELU, int EP>
__global__ void __launch_bounds__(kThreads2) decode_dense_kernel(const DenseDecodeArgs a) {
  constexpr int BNS = GELU ? 128 : 64;   // hidden columns per first-phase item
  constexpr int NST = EP == 32 ? 8 : 6;
  typedef std::conditional_t<GELU, Tile3<kDT, 128, 1, false, true, false, NST, 2>,
                             Tile3<kDT, 128, 2, false, true, false, NST, 2>> T1;
  typedef Tile3<kDT, 128, 1, false, true, false, NST, 2> T2;
  static_assert(T1::LDS_L == T2::LDS_L && T1::LDS_R == T2::LDS_R, "both phases run in the same stages");
  DSMOE_TILE3_STAGES(T1, st);
  constexpr int kRouteTok = 8;
  __shared__ __align__(16) char sRoute[route_bf16_lds<EP, kRouteTok>()];
  __shared__ int sOverflow, sItem[2], sAllClaimed[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int xcd = (int)(xcc_id() & 7u);               // the die whose L2 this block shares, from the hardware
  const int slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
  const int T = a.T, d = a.d, f = a.f, E = a.E;
  const int g = E >> 3;                               // experts per XCD
  const int ns1 = (f + BNS - 1) / BNS, items1 = g * ns1;
  const int ns2 = (d + 127) / 128, items2 = ns2 * a.KS;
  const size_t ef = (size_t)E * f;
  int32_t* const claim1 = a.sync + kDenseSyncClaim1 + xcd * kDenseClaimWords;
  int32_t* const claim2 = a.sync + kDenseSyncClaim2 + xcd * kDenseClaimWords;
  int32_t* const done1 = a.sync + kDenseSyncDone1 + xcd * kDenseClaimWords;
  unsigned* const wpub = reinterpret_cast<unsigned*>(a.sync + kDensePubWeight);
  int32_t* const cpub = a.sync + kDensePubCount;
  DSMOE_MARK(0);

  // ---- phase 1: hidden activations of this XCD's experts -------------------------------------------------
  auto setup1 = [&](int item, typename T1::LSrc& L, typename T1::RSrc& R) {
    const int e = xcd * g + item / ns1, n0 = (item % ns1) * BNS;
    L.init(T, 0, [&](int r) { return a.x + (size_t)r * d; });
    const size_t wo = (size_t)e * d * f + n0;
    if constexpr (GELU) {
      const bf16_t* const base[1] = {a.w_gate + wo};
      R.init(base, f, min(BNS, f - n0), d);
    } else {
      const bf16_t* const base[2] = {a.w_gate + wo, a.w_up + wo};
      R.init(base, f, min(BNS, f - n0), d);
    }
  };
  typename T1::LSrc L1;
  typename T1::RSrc R1;
  typename T1::Iter it1;
  const int nkt1 = d / kBK2;
  int in_flight = -1;                                 // item whose first K steps have been requested
  if (slot < items1) {
    setup1(slot, L1, R1);
    T1::prefetch(L1, R1, it1, nkt1, 1 << 30, st);     // the weight stream starts before anything else
    in_flight = slot;
  }
  // The block's first item of either phase is marked as taken, and run whatever the mark's answer would be: if
  // a block that the hardware placed on this XCD against the round-robin rule shares the slot, both run the item,
  // which is harmless (same inputs, same stores) and costs no round trip at kernel start.
  if (threadIdx.x == 0) {
    if (slot < items1) __hip_atomic_fetch_or(claim1 + (slot >> 5), 1 << (slot & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (slot < items2) __hip_atomic_fetch_or(claim2 + (slot >> 5), 1 << (slot & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sAllClaimed[0] = sAllClaimed[1] = 0;
  }
  // The router: eight tokens per block, by the first blocks (the same code as the stand-alone router kernel, with
  // eight K slices in flight per wave instead of sixteen: its registers must fit beside the tile pipeline's).
  // What the other blocks need is published write-through; nobody waits for it here.
  for (int t0 = blockIdx.x * kRouteTok; t0 < T; t0 += gridDim.x * kRouteTok)
    route_bf16_tile<EP, kRouteTok, true, 8>(a.x, a.w_r, a.b_r, T, d, E, a.probs, a.mode, a.k, a.eps, a.mask, nullptr, t0,
                                            sRoute, wpub, cpub);
  __syncthreads();
  bool routed = false;
  DSMOE_MARK(1);
  ItemClaims q1{claim1, items1, slots, slot + slots, slot < items1 ? slot : -1, false, sItem};
  for (int item = q1.next(); item >= 0; item = q1.next()) {
    const int e = xcd * g + item / ns1, n0 = (item % ns1) * BNS;
    if (item != in_flight) {
      if (in_flight >= 0) {                           // the requested item went to another block: let its tiles land
        wait_vm<0, true>();
        __syncthreads();
      }
      setup1(item, L1, R1);
      T1::prefetch(L1, R1, it1, nkt1, 1 << 30, st);
    }
    in_flight = -1;
    typename T1::Acc acc;
    T1::zero(acc);
    DSMOE_MARK(2);
    T1::run(acc, L1, R1, it1, nkt1, 1 << 30, st);
    DSMOE_MARK(3);
    // Router weight of this lane's token for expert e (0: not selected), from what the routing blocks published
    // long ago (the polls below do not spin in practice).  The capacity rule of the staged path holds here too:
    // more selected pairs than max_rows gives an all-zero output and raises the deferred status.
    const int trow = T1::acc_m(0);
    unsigned wbits = kNotPublished;
    if (trow < T) wbits = __hip_atomic_load(wpub + (size_t)trow * kMaxExperts + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!routed) {
      if (wave == 0) {
        int c0 = 1, c1 = 1;                           // counts of tokens lane and lane + 64 (1: no such token)
        if (lane < T) c0 = __hip_atomic_load(cpub + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane + 64 < T) c1 = __hip_atomic_load(cpub + lane + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // by now every block has long made its first claims: a bitmap without gaps stays without gaps
        bool none1 = false, none2 = false;
        if (lane == 0) {
          none1 = ItemClaims::none_unclaimed(claim1, items1);
          none2 = ItemClaims::none_unclaimed(claim2, items2);
        }
        for (int i = 0; i < a.spin_limit && c0 == 0; ++i)
          c0 = __hip_atomic_load(cpub + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = 0; i < a.spin_limit && c1 == 0; ++i)
          c1 = __hip_atomic_load(cpub + lane + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c0 == 0 || c1 == 0) raise_internal(a.sync, a.err_flag, 2, kDensePubCount, 0, 1);
        int c = (lane < T ? c0 : 0) + (lane + 64 < T ? c1 : 0);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) c += __shfl_xor(c, s, 64);
        if (lane == 0) {
          sOverflow = (long long)c > a.max_rows;
          if (sOverflow && blockIdx.x == 0)
            __hip_atomic_store(a.err_flag, (int32_t)DSMOE_ERR_CAPACITY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          sAllClaimed[0] = none1;
          sAllClaimed[1] = none2;
        }
      }
      __syncthreads();
      q1.all_claimed = sAllClaimed[0] != 0;
      routed = true;
      DSMOE_MARK(4);
    }
    float wte = 0.f;
    if (trow < T) {
      for (int i = 0; i < a.spin_limit && wbits == kNotPublished; ++i)
        wbits = __hip_atomic_load(wpub + (size_t)trow * kMaxExperts + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (wbits == kNotPublished) {
        raise_internal(a.sync, a.err_flag, 2, kDensePubWeight, trow, e);
        wbits = 0u;
      }
      wte = sOverflow ? 0.f : __uint_as_float(wbits);
      bf16_t* hrow = a.ht + (size_t)trow * ef + (size_t)e * f;
      if constexpr (GELU) {
#pragma unroll
        for (int nt = 0; nt < T1::NT; ++nt)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = n0 + T1::acc_n(nt, q);
            if (n >= f) continue;
            const f32x16& G = acc[nt][0];
            float h[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = wte == 0.f ? 0.f : wte * gelu_f(G[4 * q + i]);
            store4(hrow + n, h[0], h[1], h[2], h[3]);
          }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + T1::acc_n(0, q);
          if (n >= f) continue;
          const f32x16& G = acc[0][0];
          const f32x16& U = acc[1][0];
          float h[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) h[i] = wte == 0.f ? 0.f : wte * (silu_f(G[4 * q + i]) * U[4 * q + i]);
          store4(hrow + n, h[0], h[1], h[2], h[3]);
        }
      }
    }
    // hand-off to the second phase through this XCD's L2
    stores_done();
    __syncthreads();
    if (threadIdx.x == 0)
      __hip_atomic_fetch_or(done1 + (item >> 5), 1 << (item & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    DSMOE_MARK(5);
  }
  DSMOE_MARK(6);
  if (in_flight >= 0) {   // the requested item went to another block and nothing else was left
    wait_vm<0, true>();
    __syncthreads();
  }

  // ---- phase 2: this XCD's K range of the output product ------------------------------------------------------
  // item = (output column slice of 128, K chunk h of the range); a chunk waits for the first-phase items that
  // produce its hidden columns
  const int klen = g * f / a.KS;
  ItemClaims q2{claim2, items2, slots, slot + slots, slot < items2 ? slot : -1, routed && sAllClaimed[1] != 0, sItem};
  for (int item = q2.next(); item >= 0; item = q2.next()) {
    const int h = item % a.KS, n0 = (item / a.KS) * 128;
    const int lo = h * klen, hi = lo + klen;
    DSMOE_MARK(7);
    wait_bits(a.sync, done1, lo / f * ns1, ((hi - 1) / f + 1) * ns1, a.spin_limit, a.err_flag);
    DSMOE_MARK(8);
    const size_t kb = (size_t)xcd * g * f + lo;
    typename T2::LSrc L;
    typename T2::RSrc R;
    L.init(T, 0, [&](int r) { return a.ht + (size_t)r * ef + kb; });
    const bf16_t* const base[1] = {a.w_down + kb * d + n0};
    R.init(base, d, min(128, d - n0), klen);
    typename T2::Acc acc;
    T2::zero(acc);
    T2::mainloop(acc, L, R, klen / kBK2, 1 << 30, st);
    DSMOE_MARK(9);
    const int trow = T2::acc_m(0);
    if (trow < T) {
      float* prow = a.part + ((size_t)(xcd * a.KS + h) * T + trow) * d;
#pragma unroll
      for (int nt = 0; nt < T2::NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + T2::acc_n(nt, q);
          if (n >= d) continue;
          const f32x16& A = acc[nt][0];
          store4(prow + n, A[4 * q], A[4 * q + 1], A[4 * q + 2], A[4 * q + 3]);
        }
    }
    if (threadIdx.x == 0)
      __hip_atomic_fetch_or(a.sync + kDenseSyncDone2 + xcd * kDenseClaimWords + (item >> 5), 1 << (item & 31),
                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    DSMOE_MARK(10);
  }
  DSMOE_MARK(11);

}

// out[t, :] = sum of the K-range partial outputs in ascending order (fixed: bitwise reproducible).  The kernel
// also closes the call of the persistent kernel before it: it checks that every XCD ran all its second-phase
// items (an XCD that received no block at all would have run none) and leaves every counter at zero and every
// publication word unset for the next call.
__global__ void __launch_bounds__(256) decode_dense_reduce_kernel(const float* __restrict__ part, int nparts, int T, int d,
                                                                  bf16_t* __restrict__ out, int32_t* __restrict__ sync,
                                                                  int32_t* __restrict__ err_flag, int items2) {
  const int bid = blockIdx.y * gridDim.x + blockIdx.x, nb = gridDim.x * gridDim.y;
  if (bid == 0 && threadIdx.x < 8 &&
      !ItemClaims::none_unclaimed(sync + kDenseSyncDone2 + threadIdx.x * kDenseClaimWords, items2))
    raise_internal(sync, err_flag, 3, kDenseSyncDone2 + threadIdx.x * kDenseClaimWords, 0, items2);
  __syncthreads();
  unsigned* wpub = reinterpret_cast<unsigned*>(sync + kDensePubWeight);
  for (int i = bid * 256 + threadIdx.x; i < kDenseSyncWords; i += nb * 256) sync[i] = 0;
  for (int i = bid * 256 + threadIdx.x; i < T; i += nb * 256) sync[kDensePubCount + i] = 0;
  for (int i = bid * 256 + threadIdx.x; i < T * kMaxExperts; i += nb * 256) wpub[i] = kNotPublished;
  const int t = blockIdx.x, c0 = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (c0 >= d) return;
  const float* p = part + (size_t)t * d + c0;
  const size_t stride = (size_t)T * d;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int i0 = 0; i0 < nparts; i0 += 8) {
    f32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = i0 + u < nparts ? __builtin_bit_cast(f32x4, ldg16(p + (size_t)(i0 + u) * stride)) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + u < nparts) acc += v[u];
  }
  store4(out + (size_t)t * d + c0, acc.x, acc.y, acc.z, acc.w);
}

}  // namespace

// K chunks of an XCD's range in the output product (= partial outputs per XCD): enough items for the XCD's
// blocks, limited by the partial-sum buffer and by the K steps available.
static int dense_ksplit(const dsmoe_ctx* c, int T, int slots) {
  const int d = c->desc.d_model, f = c->desc.d_ff, g = c->desc.n_experts / 8;
  const int ns2 = (d + 127) / 128, row_cap = decode_row_cap(c);
  int ks = 1;
  while (ns2 * ks < slots && (g * f / (2 * ks)) % kBK2 == 0 && g * f / (2 * ks) >= 4 * kBK2 &&
         (long)8 * 2 * ks * T <= row_cap)
    ks *= 2;
  return ks;
}

// Batches of more than 64 tokens stay with the kernels that gather each expert's own rows: with every token a
// row of every tile, the token operand re-read from the L2 per K step weighs as much as the weight stream itself.
constexpr int kDenseMaxTokens = 64;

bool decode_dense_applies(const dsmoe_ctx* c, int T, int mode, int k, float eps) {
  if (c->desc.dtype != DSMOE_BF16 || T < 1 || T > kDenseMaxTokens || c->n_cu < 8) return false;
  const int E = c->desc.n_experts;
  if ((long)8 * T > decode_row_cap(c)) return false;
  const int bns = c->expert_kind == DSMOE_EXPERT_GELU ? 128 : 64;
  const int items1 = E / 8 * ((c->desc.d_ff + bns - 1) / bns);
  const int items2 = (c->desc.d_model + 127) / 128 * dense_ksplit(c, T, c->n_cu / 8);
  if (items1 > 32 * kDenseClaimWords || items2 > 32 * kDenseClaimWords) return false;   // the claim bitmaps hold 1024 items
  if (mode == DSMOE_SEL_TOPK) {
    // share of the experts that T tokens with k uniformly spread choices each leave unselected
    double idle = 1.0;
    for (int t = 0; t < T; ++t) idle *= 1.0 - (double)k / E;
    return idle <= 0.1;
  }
  if (mode == DSMOE_SEL_THRESHOLD) return T >= 8 && eps * E <= 1.f;   // a normalised threshold below 1: many experts per token
  return false;
}

hipError_t launch_decode_dense(const dsmoe_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_gate,
                               const void* w_up, const void* w_down, int T, int mode, int k, float eps, void* out,
                               hipStream_t s) {
  char* w = c->workspace;
  const int grid = c->n_cu / 8 * 8;
  DenseDecodeArgs a;
  a.x = (const bf16_t*)x; a.w_r = (const bf16_t*)w_r; a.b_r = (const bf16_t*)b_r;
  a.w_gate = (const bf16_t*)w_gate; a.w_up = (const bf16_t*)w_up; a.w_down = (const bf16_t*)w_down;
  a.probs = reinterpret_cast<float*>(w + c->ws.probs);
  a.mask = reinterpret_cast<unsigned long long*>(w + c->ws.mask);
  a.cnt_tok = reinterpret_cast<int32_t*>(w + c->ws.cnt_tok);
  a.ht = reinterpret_cast<bf16_t*>(w + c->ws.dec_ht);
  a.part = reinterpret_cast<float*>(w + c->ws.dec_p2);
  a.sync = reinterpret_cast<int32_t*>(w + c->ws.dec_sync);
  a.err_flag = reinterpret_cast<int32_t*>(w + c->ws.err_flag);
  a.T = T; a.d = c->desc.d_model; a.f = c->desc.d_ff; a.E = c->desc.n_experts;
  a.mode = mode; a.k = k; a.eps = eps;
  a.max_rows = c->desc.max_rows;
  a.KS = dense_ksplit(c, T, grid / 8);
  a.spin_limit = c->spin_limit;
  a.trace = reinterpret_cast<long long*>(w + c->ws.dec_p1);   // (development aid; that buffer is idle in this path)
  const bool gelu = c->expert_kind == DSMOE_EXPERT_GELU;
  if (a.E <= 32) {
    if (gelu) decode_dense_kernel<true, 32><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
    else decode_dense_kernel<false, 32><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
  } else {
    if (gelu) decode_dense_kernel<true, 64><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
    else decode_dense_kernel<false, 64><<<dim3(grid), dim3(kThreads2), 0, s>>>(a);
  }
  if (hipError_t e = hipGetLastError()) return e;
  decode_dense_reduce_kernel<<<dim3(T, (a.d + 1023) / 1024), dim3(256), 0, s>>>(
      a.part, 8 * a.KS, T, a.d, (bf16_t*)out, a.sync, a.err_flag, (a.d + 127) / 128 * a.KS);
  return hipGetLastError();
}

}  // namespace dsmoe
