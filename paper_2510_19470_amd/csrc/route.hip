// Gating: top-k selection and gate weights from fp32 logits (paper Sec. 2.1: the gate
// network is the router that picks the activated experts of every token).
//
// One token is handled by a group of W lanes of a 64-wide wavefront (W = power of two,
// >= min(E,64)), so that small expert counts pack several tokens into one wavefront.
// Each lane keeps ceil(E/W) logits in registers.  The k winners are found by k rounds of
// "local best, then butterfly arg-max across the group"; the order relation is total on
// finite floats: larger logit first, equal logits by lower expert id.
#include "moe_internal.h"

namespace {

constexpr int MAX_VPL = MOE_MAX_EXPERTS / 64;  // logits per lane when E > 64

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

template <int W, int VPL>
__global__ __launch_bounds__(256) void route_select_kernel(const float* __restrict__ logits, int T,
                                                           int E, int k, int renormalize,
                                                           int32_t* __restrict__ topk_idx,
                                                           float* __restrict__ topk_w) {
  constexpr int TOK_PER_WAVE = 64 / W;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int sub = lane / W;       // token slot inside the wavefront
  const int gl = lane % W;        // lane inside the group
  const int t = wave * TOK_PER_WAVE + sub;
  const bool live = t < T;

  float v[VPL];
  bool taken[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int e = gl + i * W;
    const bool ok = live && e < E;
    v[i] = ok ? logits[(size_t)t * E + e] : 0.f;
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
int launch_sel(const float* logits, int T, int E, int k, int renorm, int32_t* idx, float* w,
               hipStream_t s) {
  constexpr int TOK_PER_WAVE = 64 / W;
  const int tok_per_block = TOK_PER_WAVE * 4;
  const int grid = (T + tok_per_block - 1) / tok_per_block;
  hipLaunchKernelGGL((route_select_kernel<W, VPL>), dim3(grid), dim3(256), 0, s, logits, T, E, k,
                     renorm, idx, w);
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
