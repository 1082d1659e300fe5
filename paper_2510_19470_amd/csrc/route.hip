// Gating: gate projection, top-k selection and gate weights (paper Sec. 2.1: the gate
// network is the router that picks the activated experts of every token).
//
// Selection: one token is handled by a group of W lanes of a 64-wide wavefront (W = power
// of two, >= min(E,64)), so that small expert counts pack several tokens into one
// wavefront.  Each lane keeps ceil(E/W) logits in registers.  The k winners are found by k
// rounds of "local best, then butterfly arg-max across the group"; the order relation is
// total on finite floats: larger logit first, equal logits by lower expert id.  The same
// device function serves moe_route_logits (logits in global memory) and the fused
// moe_route kernel (logits in LDS), so both select identically from identical logits.
#include "moe_internal.h"

namespace {

struct Cand {
  float v;
  int id;  // INT_MAX = no candidate
};

__device__ __forceinline__ bool better(const Cand& b, const Cand& a) {
  // true when b should replace a
  if (b.id == 0x7fffffff) return false;
  if (a.id == 0x7fffffff) return true;
  return (b.v > a.v) || (b.v == a.v && b.id < a.id);
}

// Selection and weights of token t, done by the W lanes [sub*W, sub*W+W) of the wavefront.
// `row` points at the token's E logits (global memory or LDS); every lane of the wavefront
// must call this together (dead groups pass live = false).
template <int W, int VPL>
__device__ __forceinline__ void select_token(const float* row, bool live, int t, int E, int k,
                                             int renormalize, int32_t* __restrict__ topk_idx,
                                             float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int sub = lane / W;  // token slot inside the wavefront
  const int gl = lane % W;   // lane inside the group

  float v[VPL];
  bool taken[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int e = gl + i * W;
    const bool ok = live && e < E;
    v[i] = ok ? row[e] : 0.f;
    taken[i] = !ok;
  }

  float sel_v[MOE_MAX_TOPK];
  int sel_id[MOE_MAX_TOPK];
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    sel_v[j] = 0.f;
    sel_id[j] = 0;
  }

#pragma unroll 1
  for (int j = 0; j < k; ++j) {
    Cand best{0.f, 0x7fffffff};
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      Cand c{v[i], taken[i] ? 0x7fffffff : gl + i * W};
      if (better(c, best)) best = c;
    }
#pragma unroll
    for (int off = W / 2; off >= 1; off >>= 1) {
      Cand o;
      o.v = __shfl_xor(best.v, off, 64);
      o.id = __shfl_xor(best.id, off, 64);
      if (better(o, best)) best = o;
    }
    // all lanes of the group take lane 0's answer (identical for finite inputs)
    best.v = __shfl(best.v, sub * W, 64);
    best.id = __shfl(best.id, sub * W, 64);
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (best.id == gl + i * W) taken[i] = true;
#pragma unroll
    for (int jj = 0; jj < MOE_MAX_TOPK; ++jj)
      if (jj == j) {
        sel_v[jj] = best.v;
        sel_id[jj] = best.id;
      }
  }

  // weights: exp(l - max) over the selection, normalised over the selection or over all E
  const float m = sel_v[0];
  float den = 0.f;
  if (renormalize) {
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j)
      if (j < k) den += expf(sel_v[j] - m);
  } else {
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int e = gl + i * W;
      if (live && e < E) part += expf(v[i] - m);
    }
#pragma unroll
    for (int off = W / 2; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
    den = __shfl(part, sub * W, 64);
  }
  if (live && gl == 0) {
    const float inv = 1.f / den;
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j)
      if (j < k) {
        topk_idx[(size_t)t * k + j] = sel_id[j] == 0x7fffffff ? 0 : sel_id[j];
        topk_w[(size_t)t * k + j] = expf(sel_v[j] - m) * inv;
      }
  }
}

template <int W, int VPL>
__global__ __launch_bounds__(256) void route_select_kernel(const float* __restrict__ logits, int T,
                                                           int E, int k, int renormalize,
                                                           int32_t* __restrict__ topk_idx,
                                                           float* __restrict__ topk_w) {
  constexpr int TOK_PER_WAVE = 64 / W;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int t = wave * TOK_PER_WAVE + lane / W;
  const bool live = t < T;
  select_token<W, VPL>(logits + (size_t)(live ? t : 0) * E, live, t, E, k, renormalize, topk_idx,
                       topk_w);
}

// ---- fused gate projection + selection for bf16 inputs (matrix cores) -----------------
// One block = 32 tokens.  Its 4 wavefronts split d into quarters; each accumulates
// logits[32 tokens][64 experts] with MFMA 32x32x16 (gate rows are the "A" operand, token
// rows the "B" operand, both read straight from global memory: a lane fetches 64
// contiguous bytes of its row per 64-wide k-step, with the same k-to-lane assignment on
// both operands).  The partial sums meet in LDS, the bias is added, the logits are written
// out when the caller wants them, and the block selects the top-k of its 32 tokens from
// LDS.  The token rows are read exactly once: the kernel is bound by HBM.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
constexpr int GATE_TOK = 32;

template <int W, int VPL>
__global__ __launch_bounds__(256) void gate_route_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ Wg,
    const float* __restrict__ bias, int T, int E, int d, int k, int renormalize,
    float* __restrict__ logits_out, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  constexpr int EP = W * VPL < 64 ? 64 : W * VPL;  // expert slots kept in LDS
  __shared__ float part[4][GATE_TOK][64 + 1];
  __shared__ float fin[GATE_TOK][EP + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * GATE_TOK;
  const int kq = d >> 2;  // k range of this wavefront
  const uint4* xp = reinterpret_cast<const uint4*>(x + (size_t)min(t0 + r, T - 1) * d +
                                                   wave * kq + h * 32);
  for (int e0 = 0; e0 < E; e0 += 64) {
    const uint4* wp[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      wp[j] = reinterpret_cast<const uint4*>(Wg + (size_t)min(e0 + j * 32 + r, E - 1) * d +
                                             wave * kq + h * 32);
    f32x16_t acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int ks = 0; ks < kq / 64; ++ks) {
      uint4 xv[4], wv0[4], wv1[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        xv[c] = xp[ks * 8 + c];
        wv0[c] = wp[0][ks * 8 + c];
        wv1[c] = wp[1][ks * 8 + c];
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wv0[c]),
                                                         __builtin_bit_cast(bf16x8_t, xv[c]),
                                                         acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wv1[c]),
                                                         __builtin_bit_cast(bf16x8_t, xv[c]),
                                                         acc[1], 0, 0, 0);
      }
    }
    // the lane holds token r and experts 32j + 8g + 4h + i of this group of 64
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          part[wave][r][32 * j + 8 * g + 4 * h + i] = acc[j][g * 4 + i];
    __syncthreads();
    for (int idx = tid; idx < GATE_TOK * 64; idx += 256) {
      const int tok = idx >> 6, el = idx & 63, e = e0 + el;
      if (e < E) {
        const float v = ((part[0][tok][el] + part[1][tok][el]) +
                         (part[2][tok][el] + part[3][tok][el])) +
                        (bias != nullptr ? bias[e] : 0.f);
        fin[tok][e] = v;
        if (logits_out != nullptr && t0 + tok < T) logits_out[(size_t)(t0 + tok) * E + e] = v;
      }
    }
    __syncthreads();
  }
  constexpr int TOK_PER_WAVE = 64 / W;
  for (int base = 0; base < GATE_TOK; base += 4 * TOK_PER_WAVE) {
    const int tok = base + wave * TOK_PER_WAVE + lane / W;
    const bool live = tok < GATE_TOK && t0 + tok < T;
    select_token<W, VPL>(&fin[live ? tok : 0][0], live, t0 + tok, E, k, renormalize, topk_idx,
                         topk_w);
  }
}

template <int W, int VPL>
int launch_sel(const float* logits, int T, int E, int k, int renorm, int32_t* idx, float* w,
               hipStream_t s) {
  constexpr int TOK_PER_WAVE = 64 / W;
  const int tok_per_block = TOK_PER_WAVE * 4;
  const int grid = (T + tok_per_block - 1) / tok_per_block;
  hipLaunchKernelGGL((route_select_kernel<W, VPL>), dim3(grid), dim3(256), 0, s, logits, T, E, k,
                     renorm, idx, w);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

template <int W, int VPL>
int launch_gate(const moe_ctx* c, const void* x, const void* Wg, const float* bias, int T,
                float* logits, int32_t* idx, float* w, hipStream_t s) {
  const int grid = (T + GATE_TOK - 1) / GATE_TOK;
  hipLaunchKernelGGL((gate_route_mfma_kernel<W, VPL>), dim3(grid), dim3(256), 0, s,
                     (const uint16_t*)x, (const uint16_t*)Wg, bias, T, c->cfg.E, c->cfg.d,
                     c->cfg.k, c->cfg.renormalize, logits, idx, w);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

}  // namespace

int launch_route_select(const moe_ctx* c, const float* logits, int T, int32_t* idx, float* w,
                        hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int E = c->cfg.E, k = c->cfg.k, rn = c->cfg.renormalize;
  if (E <= 2) return launch_sel<2, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 4) return launch_sel<4, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 8) return launch_sel<8, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 16) return launch_sel<16, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 32) return launch_sel<32, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 64) return launch_sel<64, 1>(logits, T, E, k, rn, idx, w, s);
  if (E <= 128) return launch_sel<64, 2>(logits, T, E, k, rn, idx, w, s);
  if (E <= 256) return launch_sel<64, 4>(logits, T, E, k, rn, idx, w, s);
  return MOE_EUNSUPPORTED;
}

bool gate_route_fused_supported(const moe_ctx* c) {
  return c->cfg.dtype == MOE_BF16 && c->cfg.d % 256 == 0;
}

int launch_gate_route_fused(const moe_ctx* c, const void* x, const void* Wg, const float* bias,
                            int T, float* logits, int32_t* idx, float* w, hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int E = c->cfg.E;
  if (E <= 2) return launch_gate<2, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 4) return launch_gate<4, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 8) return launch_gate<8, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 16) return launch_gate<16, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 32) return launch_gate<32, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 64) return launch_gate<64, 1>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 128) return launch_gate<64, 2>(c, x, Wg, bias, T, logits, idx, w, s);
  if (E <= 256) return launch_gate<64, 4>(c, x, Wg, bias, T, logits, idx, w, s);
  return MOE_EUNSUPPORTED;
}
