// Softmax and expert selection of one token by one wave, one lane per expert: shared by the router kernels and
// by the decode kernel that routes its own tokens (Eq. 1: scores; Sec. 3.1 / 3.2: top-K and threshold selection).
#pragma once

#include "common.h"

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

}  // namespace dsmoe
