// Mixture-of-Attention-heads layer (paper Sec. 3.2, Eq. 7-8), forward, bf16: C-ABI entry points and the
// attention kernel.  The router is the MLP layer's fused router kernel; the query and output projections are
// the grouped / dense bf16 GEMM kernels of the expert FFN; what is new here is the attention itself.
//
//   Q[e][t]      = x[t] W_q[e]                                  grouped GEMM, every group reads all T rows
//   C[e][t][j]   = softmax_l(scale * Q[e][t][j] . K[j][l]) V[j]  l <= L - T + t     (this file)
//   Cs[t][e][j]  = S[t][e] [e in A(t)] * C[e][t][j]             folded into the attention epilogue
//   out[t]       = Cs[t] W_o  with W_o[E, n_head*d_head, d] read as one [E*n_head*d_head, d] matrix
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <new>

#include "gemm_core.h"
#include "moa_internal.h"

using namespace dsmoe;

namespace {

int32_t moa_fail(dsmoe_moa_ctx* c, int32_t code, const char* fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}
bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define MOA_PTR(c, p)                                                                                   \
  do {                                                                                                  \
    if ((p) == nullptr) return moa_fail((c), DSMOE_ERR_INVALID_ARG, "null pointer: %s", #p);            \
    if (misaligned16(p)) return moa_fail((c), DSMOE_ERR_INVALID_ARG, "pointer not 16-byte aligned: %s", #p); \
  } while (0)
#define MOA_HIP(c, expr)                                                                                \
  do {                                                                                                  \
    hipError_t e_ = (expr);                                                                             \
    if (e_ != hipSuccess) return moa_fail((c), DSMOE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

// One block: 128 queries (4 waves of 32) of one expert e and head j against the keys they may see, 32 keys at
// a time.  Both products run on the 32x32x16 bf16 MFMA with the queries on the lane axis:
//   S^T[key][query]  = K_tile (A operand, keys on the register axis) x Q^T (B operand, kept in registers),
//   O^T[dv][query]  += V_tile^T (A operand) x P^T (B operand).
// The accumulator of the first product leaves a lane (query q, half h) with the keys 8 (r / 4) + 4 h + r % 4,
// r = 0..15.  Registers 8 s .. 8 s + 7 are therefore, in order, the B operand of the second product's MFMA s
// (s = 0, 1) if its k index 8 h + i stands for key 16 s + 8 (i / 4) + 4 h + i % 4; the V operand is read
// from a transposed tile in LDS with the same key order (two 8-byte reads), and the sum over keys does not
// care about their order.  So P never leaves the registers.  Softmax is the running-maximum form; a query's
// two lanes (h = 0, 1) share the maximum and keep separate partial sums until the end.
template <int DH>
__global__ void __launch_bounds__(256, 2)
moa_attention_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                     const float* __restrict__ probs, const unsigned long long* __restrict__ mask,
                     bf16_t* __restrict__ Cs, bf16_t* __restrict__ C_raw, float* __restrict__ lse, int T, int L, int E,
                     int NH, float scale_log2e) {
  constexpr int BQ = 128, BKEY = 32, NS = DH / 16, NDT = DH / 32;
  constexpr int KP = DH * 2 + 16;        // bytes per key row of the K tile (16-byte skew: conflict-free 16-byte reads)
  constexpr int VP = BKEY * 2 + 8;       // bytes per dv row of the transposed V tile (9 x 8 bytes: conflict-free)
  constexpr int KN = DH / 64;            // 16-byte pieces of the K tile per thread (32 keys x DH / 8 pieces)
  constexpr int VITEMS = 2 * DH;         // (key pair, dv octet) items of the V tile
  __shared__ __align__(16) char k_tile[BKEY * KP];
  __shared__ __align__(16) char v_tile[DH * VP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane & 31, h = lane >> 5;
  const int n_qt = (T + BQ - 1) / BQ;
  const int qt = n_qt - 1 - (int)blockIdx.y;             // the tiles with the most keys start first, for every head
  const int j = blockIdx.x % NH, e = blockIdx.x / NH;
  const int pos0 = L - T, hd = NH * DH;
  const int t = qt * BQ + wave * 32 + q, tq = min(t, T - 1);

  u32x4 qf[NS];
  {
    const bf16_t* qrow = Q + ((size_t)e * T + tq) * hd + (size_t)j * DH;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const u32x4*>(qrow + 16 * s + 8 * h);
  }
  f32x16 o[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int t_last = min(T, qt * BQ + BQ) - 1;
  const int n_keys = pos0 + t_last + 1, n_kt = (n_keys + BKEY - 1) / BKEY;
  const bf16_t* Kj = K + (size_t)j * L * DH;
  const bf16_t* Vj = V + (size_t)j * L * DH;

  // staging: registers first (the next tile's loads are in flight while the current tile is multiplied)
  u32x4 kreg[KN], vreg[2];
  const int v_kp = tid % 16, v_oct = tid / 16;           // key pair and dv octet of this thread's V item
  auto load_tile = [&](int kt) {
    const int key0 = kt * BKEY;
#pragma unroll
    for (int i = 0; i < KN; ++i) {
      const int p = tid + 256 * i, key = min(key0 + p / (DH / 8), L - 1), c8 = p % (DH / 8);
      kreg[i] = *reinterpret_cast<const u32x4*>(Kj + (size_t)key * DH + 8 * c8);
    }
    if (tid < VITEMS) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int key = min(key0 + 2 * v_kp + u, L - 1);
        vreg[u] = *reinterpret_cast<const u32x4*>(Vj + (size_t)key * DH + 8 * v_oct);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KN; ++i) {
      const int p = tid + 256 * i, key = p / (DH / 8), c8 = p % (DH / 8);
      *reinterpret_cast<u32x4*>(k_tile + key * KP + c8 * 16) = kreg[i];
    }
    if (tid < VITEMS) {
      // two keys x eight dv -> eight 4-byte (key pair) writes, one per dv row of the transposed tile
      const unsigned a[4] = {vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w};
      const unsigned b[4] = {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned lo = (a[c] & 0xffffu) | (b[c] << 16), hi = (a[c] >> 16) | (b[c] & 0xffff0000u);
        *reinterpret_cast<unsigned*>(v_tile + (8 * v_oct + 2 * c) * VP + v_kp * 4) = lo;
        *reinterpret_cast<unsigned*>(v_tile + (8 * v_oct + 2 * c + 1) * VP + v_kp * 4) = hi;
      }
    }
  };

  const int limit = pos0 + t;                            // last cache position query t sees
  const int wave_limit = pos0 + qt * BQ + wave * 32;     // ... and the wave's first query
  load_tile(0);
  for (int kt = 0; kt < n_kt; ++kt) {
    __syncthreads();                                     // the previous tile has been read by every wave
    store_tile();
    __syncthreads();
    if (kt + 1 < n_kt) load_tile(kt + 1);

    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const u32x4 kf = *reinterpret_cast<const u32x4*>(k_tile + q * KP + (16 * s + 8 * h) * 2);
      Mma<bf16_t>::run(sacc, kf, qf[s]);
    }
    const int key0 = kt * BKEY + 4 * h;
    float mx = -INFINITY;
    if (kt * BKEY + BKEY - 1 <= wave_limit) {            // the whole tile is visible to every query of the wave
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        sacc[r] *= scale_log2e;
        mx = fmaxf(mx, sacc[r]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 8 * (r / 4) + r % 4;
        sacc[r] = key <= limit ? sacc[r] * scale_log2e : -INFINITY;
        mx = fmaxf(mx, sacc[r]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);   // arguments <= 0: the bare instruction will do
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sacc[r] = __builtin_amdgcn_exp2f(sacc[r] - m_safe);
      psum += sacc[r];
    }
    l_run = l_run * alpha + psum;
    if (__any(alpha != 1.f)) {      // most tiles leave every running maximum of the wave as it is
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
    u32x4 pf[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
      pf[s] = u32x4{pack_bf16x2(sacc[8 * s], sacc[8 * s + 1]), pack_bf16x2(sacc[8 * s + 2], sacc[8 * s + 3]),
                    pack_bf16x2(sacc[8 * s + 4], sacc[8 * s + 5]), pack_bf16x2(sacc[8 * s + 6], sacc[8 * s + 7])};
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const char* vrow = v_tile + (32 * dt + q) * VP + (16 * s + 4 * h) * 2;
        const u32x2 lo = *reinterpret_cast<const u32x2*>(vrow), hi = *reinterpret_cast<const u32x2*>(vrow + 16);
        Mma<bf16_t>::run(o[dt], u32x4{lo.x, lo.y, hi.x, hi.y}, pf[s]);
      }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (t >= T) return;
  const bool on = (mask[t] >> e) & 1ull;
  const float wgt = on ? probs[(size_t)t * E + e] / l_tot : 0.f;
  bf16_t* crow = Cs + (size_t)t * E * hd + ((size_t)e * NH + j) * DH + 4 * h;
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      store4(crow + 32 * dt + 8 * g, o[dt][4 * g] * wgt, o[dt][4 * g + 1] * wgt, o[dt][4 * g + 2] * wgt,
             o[dt][4 * g + 3] * wgt);
  if (C_raw == nullptr) return;
  // kept for the backward pass of dense training: the unweighted outputs and, per row, log2 of the softmax
  // denominator in the units of the scaled scores (P = 2^(score - lse))
  const float inv = 1.f / l_tot;
  bf16_t* rrow = C_raw + (size_t)t * E * hd + ((size_t)e * NH + j) * DH + 4 * h;
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      store4(rrow + 32 * dt + 8 * g, o[dt][4 * g] * inv, o[dt][4 * g + 1] * inv, o[dt][4 * g + 2] * inv,
             o[dt][4 * g + 3] * inv);
  if (h == 0) lse[((size_t)e * NH + j) * T + t] = m_run + __builtin_amdgcn_logf(l_tot);
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

extern "C" {

int32_t dsmoe_moa_create(const dsmoe_moa_desc* desc, dsmoe_moa_ctx** out) {
  if (!desc || !out) return DSMOE_ERR_INVALID_ARG;
  *out = nullptr;
  if (desc->d_model <= 0 || desc->n_experts <= 0 || desc->n_head <= 0 || desc->d_head <= 0 || desc->max_tokens < 0)
    return DSMOE_ERR_INVALID_ARG;
  if (desc->dtype != DSMOE_BF16) return DSMOE_ERR_UNSUPPORTED;
  if (desc->n_experts > kMaxExperts || desc->n_experts % 8 != 0 || desc->d_model % 64 != 0) return DSMOE_ERR_UNSUPPORTED;
  if (desc->d_head != 64 && desc->d_head != 128) return DSMOE_ERR_UNSUPPORTED;
  if ((int64_t)desc->n_head * desc->n_experts > 65535) return DSMOE_ERR_UNSUPPORTED;
  dsmoe_moa_ctx* c = new (std::nothrow) dsmoe_moa_ctx();
  if (!c) return DSMOE_ERR_INVALID_ARG;
  c->desc = *desc;
  c->workspace = nullptr;
  c->workspace_bytes = 0;
  c->err[0] = 0;
  const size_t T = (size_t)desc->max_tokens, E = (size_t)desc->n_experts, hd = (size_t)desc->n_head * desc->d_head;
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o = align256(o + bytes); return at; };
  c->o_probs = take(T * E * 4);
  c->o_mask = take(T * 8);
  c->o_cnt = take(T * 4);
  c->o_q = take(E * T * hd * 2);
  c->o_cs = take(T * E * hd * 2);
  c->o_c = take(T * E * hd * 2);
  c->o_lse = take(E * desc->n_head * T * 4);
  c->total = o;
  c->saved_T = c->saved_L = -1;
  c->saved_scale = 0.f;
  // the shared launchers read the shape and the CU count from an MLP-layer context
  dsmoe_ctx& in = c->inner;
  in.desc.d_model = desc->d_model;
  in.desc.d_ff = (int32_t)hd;
  in.desc.n_experts = desc->n_experts;
  in.desc.dtype = DSMOE_BF16;
  in.desc.max_tokens = desc->max_tokens;
  in.desc.max_rows = 0;
  in.esize = 2;
  in.workspace = nullptr;
  in.workspace_bytes = 0;
  in.expert_kind = DSMOE_EXPERT_SWIGLU;
  in.err[0] = 0;
  in.n_cu = 256;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    in.n_cu = prop.multiProcessorCount;
  else
    (void)hipGetLastError();
  *out = c;
  return DSMOE_OK;
}

int32_t dsmoe_moa_destroy(dsmoe_moa_ctx* c) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  delete c;
  return DSMOE_OK;
}

const char* dsmoe_moa_last_error(const dsmoe_moa_ctx* c) { return c ? c->err : "null context"; }

int32_t dsmoe_moa_workspace_bytes(const dsmoe_moa_ctx* c, size_t* bytes) {
  if (!c || !bytes) return DSMOE_ERR_INVALID_ARG;
  *bytes = c->total;
  return DSMOE_OK;
}

int32_t dsmoe_moa_set_workspace(dsmoe_moa_ctx* c, void* workspace, size_t bytes) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return moa_fail(c, DSMOE_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
  if (bytes < c->total) return moa_fail(c, DSMOE_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", bytes, c->total);
  c->workspace = static_cast<char*>(workspace);
  c->workspace_bytes = bytes;
  return DSMOE_OK;
}

int32_t dsmoe_moa_fwd(dsmoe_moa_ctx* c, const void* x, const void* w_r, const void* b_r, const void* w_q,
                      const void* k_cache, const void* v_cache, const void* w_o, int32_t T, int32_t L, int32_t mode,
                      int32_t k, float eps, float scale, void* out, void* stream) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  const int E = c->desc.n_experts, d = c->desc.d_model, NH = c->desc.n_head, DH = c->desc.d_head, hd = NH * DH;
  if (T < 0 || T > c->desc.max_tokens) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "T = %d outside [0, %d]", T, c->desc.max_tokens);
  if (L < T) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "the cache holds the T tokens themselves: L = %d < T = %d", L, T);
  if (mode == (DSMOE_SEL_THRESHOLD | DSMOE_SEL_NORMALISED)) {   // the paper's normalised threshold (Sec. 4.2): N S_i > eps
    if (!(eps >= 0.f) || std::isinf(eps)) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "eps must be finite and >= 0");
    mode = DSMOE_SEL_THRESHOLD;
    eps = eps / static_cast<float>(E);
  }
  if (mode == DSMOE_SEL_TOPK) {
    if (k < 1 || k > E) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "k = %d outside [1, %d]", k, E);
  } else if (mode == DSMOE_SEL_THRESHOLD) {
    if (!(eps >= 0.f) || std::isinf(eps)) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "eps must be finite and >= 0");
  } else if (mode != DSMOE_SEL_ALL) {
    return moa_fail(c, DSMOE_ERR_INVALID_ARG, "unknown selection mode %d", mode);
  }
  if (!std::isfinite(scale)) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "scale must be finite");
  if (!c->workspace) return moa_fail(c, DSMOE_ERR_WORKSPACE, "no workspace set (dsmoe_moa_set_workspace)");
  c->saved_T = c->saved_L = -1;
  if (T == 0) return DSMOE_OK;
  MOA_PTR(c, x); MOA_PTR(c, w_r); MOA_PTR(c, w_q); MOA_PTR(c, k_cache); MOA_PTR(c, v_cache); MOA_PTR(c, w_o); MOA_PTR(c, out);
  if (b_r && misaligned16(b_r)) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "pointer not 16-byte aligned: b_r");
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* probs = reinterpret_cast<float*>(c->workspace + c->o_probs);
  uint64_t* mask = reinterpret_cast<uint64_t*>(c->workspace + c->o_mask);
  int32_t* cnt = reinterpret_cast<int32_t*>(c->workspace + c->o_cnt);
  bf16_t* q = reinterpret_cast<bf16_t*>(c->workspace + c->o_q);
  bf16_t* cs = reinterpret_cast<bf16_t*>(c->workspace + c->o_cs);
  const bool all = mode == DSMOE_SEL_ALL;
  bf16_t* c_raw = all ? reinterpret_cast<bf16_t*>(c->workspace + c->o_c) : nullptr;
  float* lse = reinterpret_cast<float*>(c->workspace + c->o_lse);
  c->saved_T = all ? T : -1;      // what dsmoe_moa_bwd may rely on
  c->saved_L = all ? L : -1;
  c->saved_scale = scale;

  // every expert selected = the E highest scores: the masks are then all ones
  MOA_HIP(c, launch_route(&c->inner, x, w_r, b_r, T, probs, all ? DSMOE_SEL_TOPK : mode, all ? E : k, eps, mask, cnt, s));
  MOA_HIP(c, launch_shared_rows_gemm(&c->inner, x, E, T, d, hd, w_q, q, s));
  const dim3 grid(NH * E, (T + 127) / 128);
  const float sl2e = scale * 1.4426950408889634f;
  const unsigned long long* mk = reinterpret_cast<const unsigned long long*>(mask);
  if (DH == 64)
    moa_attention_kernel<64><<<grid, dim3(256), 0, s>>>(q, (const bf16_t*)k_cache, (const bf16_t*)v_cache, probs, mk, cs,
                                                        c_raw, lse, T, L, E, NH, sl2e);
  else
    moa_attention_kernel<128><<<grid, dim3(256), 0, s>>>(q, (const bf16_t*)k_cache, (const bf16_t*)v_cache, probs, mk, cs,
                                                         c_raw, lse, T, L, E, NH, sl2e);
  MOA_HIP(c, hipGetLastError());
  MOA_HIP(c, launch_down_dense(&c->inner, cs, T, E * hd, w_o, out, s));
  return DSMOE_OK;
}

int32_t dsmoe_moa_routing(dsmoe_moa_ctx* c, int32_t T, float* probs, uint64_t* mask, void* stream) {
  if (!c) return DSMOE_ERR_INVALID_ARG;
  if (T < 0 || T > c->desc.max_tokens) return moa_fail(c, DSMOE_ERR_INVALID_ARG, "T = %d outside [0, %d]", T, c->desc.max_tokens);
  if (!c->workspace) return moa_fail(c, DSMOE_ERR_WORKSPACE, "no workspace set (dsmoe_moa_set_workspace)");
  if (T == 0) return DSMOE_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (probs)
    MOA_HIP(c, hipMemcpyAsync(probs, c->workspace + c->o_probs, (size_t)T * c->desc.n_experts * 4, hipMemcpyDeviceToDevice, s));
  if (mask) MOA_HIP(c, hipMemcpyAsync(mask, c->workspace + c->o_mask, (size_t)T * 8, hipMemcpyDeviceToDevice, s));
  return DSMOE_OK;
}

}  // extern "C"
