// Softmax and expert selection of one token by one wave, one lane per expert: shared by the router kernels and
// by the decode kernel that routes its own tokens (Eq. 1: scores; Sec. 3.1 / 3.2: top-K and threshold selection).
#pragma once

#include "gemm_dma.h"

namespace dsmoe {

// Wave-wide reductions on the data-parallel-primitive path of the VALU (no LDS round trips): four steps
// leave each 16-lane row's result in all of its lanes, the four row results are combined as scalars.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
constexpr int kDppSwap1 = 0xB1, kDppSwap2 = 0x4E, kDppRor4 = 0x124, kDppRor8 = 0x128;   // quad_perm / row_ror
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<kDppSwap1>(v));
  v = fmaxf(v, dpp_f32<kDppSwap2>(v));
  v = fmaxf(v, dpp_f32<kDppRor4>(v));
  v = fmaxf(v, dpp_f32<kDppRor8>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppSwap1>(v);
  v += dpp_f32<kDppSwap2>(v);
  v += dpp_f32<kDppRor4>(v);
  v += dpp_f32<kDppRor8>(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) {
    const unsigned long long o = __shfl_xor(v, s, 64);
    v = o > v ? o : v;
  }
  return v;
}

// Selection for one token, one lane per expert (p < 0 on lanes that hold no expert).
// mode < 0: no selection.  Ties go to the lower expert index; an empty threshold set keeps the arg-max.
__device__ __forceinline__ unsigned long long select_wave(float p, int lane, int E, int mode, int k, float eps) {
  const bool in = lane < E;
  if (mode == DSMOE_SEL_THRESHOLD) {
    unsigned long long m = __ballot(in && p > eps);
    if (m == 0ull) {
      const unsigned long long key =
          in ? (((unsigned long long)__float_as_uint(p)) << 32) | (unsigned)(63 - lane) : 0ull;
      m = 1ull << (63 - (int)(wave_max_u64(key) & 63ull));
    }
    return m;
  }
  int rank = 0;   // experts that precede this lane's: larger probability, or equal and lower index
  for (int j = 0; j < E; ++j) {
    const float pj = lane_value(p, j);
    rank += (pj > p || (pj == p && j < lane)) ? 1 : 0;
  }
  return __ballot(in && rank < k);
}

// EP: experts padded to 32 or 64.  TOK: tokens per block, 32 (a full MFMA tile) or 8 (decode-sized calls: one
// token per wave in the softmax / selection tail, and four times the blocks).
// PUBLISH: each token's combine weights (the score of a selected expert, 0 for the others: `wpub`, 64 per token) and
// its number of selected experts (`cpub`) are also stored write-through at system scope, for readers on other XCDs
// inside the same kernel; those words hold kNotPublished / 0 until then, so a reader polls the word it needs.
// smem: route_bf16_lds<EP, TOK>() bytes of LDS, 16-byte aligned.  Called by all 512 threads of a block.
template <int EP, int TOK>
constexpr int route_bf16_lds() { return (kThreads2 / 64) * 2 * 16 * (EP * 2 + 16) + (kThreads2 / 64) * TOK * (EP + 1) * 4; }

constexpr unsigned kNotPublished = 0xffffffffu;   // (a NaN pattern no weight takes: NaN weights are stored canonical)

// RING: 16-wide K slices (of X and of W_r) a wave keeps in flight, times EP / 32
template <int EP, int TOK, bool PUBLISH = false, int RING = 16>
__device__ __forceinline__ void route_bf16_tile(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w_r,
                                                const bf16_t* __restrict__ b_r, int T_tokens, int d, int E,
                                                float* __restrict__ probs, int mode, int k, float eps,
                                                unsigned long long* __restrict__ mask, int32_t* __restrict__ cnt_tok,
                                                int t0, char* smem, unsigned* __restrict__ wpub = nullptr,
                                                int32_t* __restrict__ cpub = nullptr) {
  constexpr int ET = EP / 32;            // 32-expert MFMA tiles
  constexpr int kRouteRing2 = RING / ET;   // 16-wide K slices in flight per wave
  constexpr int WP = EP * 2 + 16;        // LDS pitch of a W_r row
  constexpr int CPR = EP / 8;            // 16-byte chunks per W_r row
  constexpr int NW = kThreads2 / 64;
  char* sW = smem;                                                     // [NW][2][16 * WP]
  float (*sPart)[TOK][EP + 1] =
      reinterpret_cast<float (*)[TOK][EP + 1]>(smem + NW * 2 * 16 * WP);             // [NW][TOK][EP + 1]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r16 = lane & 15;
  const int S = d / 16;                                                // 16-wide K slices
  const int s_begin = wave * S / NW, s_end = (wave + 1) * S / NW;

  const int trow = min(t0 + min(lane & 31, TOK - 1), T_tokens - 1);
  const bf16_t* xp = x + (size_t)trow * d + (lane >> 5) * 8;           // + 16 s
  // this lane's chunks of a W_r slice: chunk c = lane + 64 i -> row c / CPR, 8 experts from (c % CPR) * 8
  int w_goff[ET], w_loff[ET];
  bool w_ok[ET];
#pragma unroll
  for (int i = 0; i < ET; ++i) {
    const int c = lane + 64 * i, row = c / CPR, cc = c % CPR;
    w_ok[i] = cc * 8 < E;
    w_goff[i] = row * E + (w_ok[i] ? cc * 8 : 0);
    w_loff[i] = row * WP + cc * 16;
  }
  char* myW = sW + wave * 2 * 16 * WP;
  // transposing read: lane r of a 16-lane group addresses [k0 + r/4][n0 + 4*(r%4)] and receives [k0..k0+3][n0 + r]
  const int f_off = ((lane >> 5) * 8 + (r16 >> 2)) * WP + (((lane >> 4) & 1) * 16 + (r16 & 3) * 4) * 2;

  f32x16 acc[ET];
#pragma unroll
  for (int et = 0; et < ET; ++et)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[et][i] = 0.f;

  u32x4 xr[kRouteRing2], wr[kRouteRing2][ET];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < kRouteRing2; ++j)
    if (s_begin + j < s_end) {
      xr[j] = ldg16(xp + (size_t)(s_begin + j) * 16);
#pragma unroll
      for (int i = 0; i < ET; ++i)
        wr[j][i] = w_ok[i] ? ldg16(w_r + (size_t)(s_begin + j) * 16 * E + w_goff[i]) : zero4;
    }
  for (int s0 = s_begin; s0 < s_end; s0 += kRouteRing2) {
#pragma unroll
    for (int j = 0; j < kRouteRing2; ++j) {
      const int s = s0 + j;
      if (s < s_end) {
        char* tile = myW + (j & 1) * 16 * WP;
#pragma unroll
        for (int i = 0; i < ET; ++i) *reinterpret_cast<u32x4*>(tile + w_loff[i]) = wr[j][i];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int et = 0; et < ET; ++et) {
          const u32x2 lo = lds_read_tr16(tile + f_off + et * 64);
          const u32x2 hi = lds_read_tr16(tile + f_off + et * 64 + 4 * WP);
          const u32x4 wf = {lo.x, lo.y, hi.x, hi.y};
          Mma<bf16_t>::run(acc[et], wf, xr[j]);
        }
        if (s + kRouteRing2 < s_end) {
          xr[j] = ldg16(xp + (size_t)(s + kRouteRing2) * 16);
#pragma unroll
          for (int i = 0; i < ET; ++i)
            wr[j][i] = w_ok[i] ? ldg16(w_r + (size_t)(s + kRouteRing2) * 16 * E + w_goff[i]) : zero4;
        }
      }
    }
  }

  // partial logits of this wave: lane owns token lane%32; register 4q+i <-> expert 8q + 4*(lane/32) + i
#pragma unroll
  for (int et = 0; et < ET; ++et)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (TOK == 32 || (lane & 31) < TOK)
        sPart[wave][lane & 31][et * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3)] = acc[et][i];
  __syncthreads();

  const float bias = (b_r != nullptr && lane < E) ? to_f32(b_r[lane]) : 0.f;
  constexpr int TPW = TOK / NW;
  for (int tt = wave * TPW; tt < wave * TPW + TPW; ++tt) {
    const int t = t0 + tt;
    if (t >= T_tokens) break;
    float z = -INFINITY;
    if (lane < E) {
      z = sPart[0][tt][lane];
#pragma unroll
      for (int w = 1; w < NW; ++w) z += sPart[w][tt][lane];
      z += bias;
    }
    const float zmax = wave_max(z);
    const float ez = lane < E ? expf(z - zmax) : 0.f;
    const float p = ez / wave_sum(ez);
    if (lane < E) probs[(size_t)t * E + lane] = p;
    if (mode >= 0) {
      const unsigned long long m = select_wave(lane < E ? p : -1.f, lane, E, mode, k, eps);
      if (lane == 0) {
        mask[t] = m;
        if (cnt_tok) cnt_tok[t] = __popcll(m);
      }
      if constexpr (PUBLISH) {
        unsigned wbits = ((m >> lane) & 1ull) ? __float_as_uint(p) : 0u;
        if (wbits == kNotPublished) wbits = 0x7fc00000u;
        if (lane < E) __hip_atomic_store(wpub + (size_t)t * kMaxExperts + lane, wbits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (lane == 0) __hip_atomic_store(cpub + t, (int32_t)__popcll(m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
}


}  // namespace dsmoe
