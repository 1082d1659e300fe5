// Backward of the gate (paper Sec. 2.1: the gate network picks K experts per token; the
// layer's output depends on the gate through the K combine weights).  The Top-k choice is
// piecewise constant, so the gradient flows only through the weights of the selected experts:
//   p = softmax of the logits over the selected experts (renormalize) or over all E,
//   dlogits[t,e] = p_e * ( [e selected] dw_e - sum_j dw_j w_j ),   w_j = p[idx_j] = topk_w,
//   dWg = dlogits^T x,  dbias = sum_t dlogits[t],  dx += dlogits Wg.
// Three HBM-bound kernels: the logit gradients (one wavefront per token), the weight
// gradient as per-chunk partial sums over 128 tokens followed by a fixed-order sum over the
// chunks (deterministic, no floating-point atomics), and the input gradient (one wavefront
// per token, added to the dx the dispatch backward has written).
#include "moe_internal.h"
#include "numeric.h"

namespace {

constexpr int RB_TOK = 128;   // tokens per partial-sum chunk
constexpr int RB_COLS = 256;  // columns per block of the weight-gradient kernel

// One wavefront per token; lane e, e+64, ... own the experts.
__global__ __launch_bounds__(256) void route_bwd_dlogits_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ topk_idx,
    const float* __restrict__ topk_w, const float* __restrict__ dtopk_w, int T, int E, int k,
    int renormalize, float* __restrict__ dlogits) {
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= T) return;
  float inner = 0.f;
  for (int j = 0; j < k; ++j) inner += dtopk_w[(size_t)t * k + j] * topk_w[(size_t)t * k + j];
  float mx = -INFINITY, den = 1.f;
  if (!renormalize) {   // full softmax of the row
    for (int e = lane; e < E; e += 64) mx = fmaxf(mx, logits[(size_t)t * E + e]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float s = 0.f;
    for (int e = lane; e < E; e += 64) s += expf(logits[(size_t)t * E + e] - mx);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    den = s;
  }
  for (int e = lane; e < E; e += 64) {
    float sel_dw = 0.f, w = 0.f;
    bool selected = false;
    for (int j = 0; j < k; ++j)
      if (topk_idx[(size_t)t * k + j] == e) {
        selected = true;
        sel_dw = dtopk_w[(size_t)t * k + j];
        w = topk_w[(size_t)t * k + j];
      }
    float p;
    if (renormalize) p = selected ? w : 0.f;
    else p = expf(logits[(size_t)t * E + e] - mx) / den;
    dlogits[(size_t)t * E + e] = p * ((selected ? sel_dw : 0.f) - inner);
  }
}

// partial[chunk][e][c] = sum over the chunk's tokens of dlogits[t][e] * x[t][c].
// Block = 256 columns x one chunk of 128 tokens x one group of RB_EG experts (the chunk's
// dlogits for those experts staged in LDS); a thread owns one column.  RB_EG = 8 or 16: the
// kernel is bound by its multiply-adds, so 32 accumulators per thread (x read once up to 32
// experts, but half as many blocks) are slower than two groups of 16.
template <typename T, int RB_EG>
__global__ __launch_bounds__(RB_COLS) void route_bwd_dwg_partial_kernel(
    const T* __restrict__ x, const float* __restrict__ dlogits, int Tn, int d, int E,
    float* __restrict__ partial) {
  __shared__ float dl[RB_TOK][RB_EG];
  const int c = blockIdx.x * RB_COLS + threadIdx.x;
  const int chunk = blockIdx.y;
  const int e0 = blockIdx.z * RB_EG;
  const int t0 = chunk * RB_TOK, nt = min(RB_TOK, Tn - t0);
  const int ne = min(RB_EG, E - e0);
  for (int i = threadIdx.x; i < RB_TOK * RB_EG; i += RB_COLS) {
    const int tt = i / RB_EG, ee = i % RB_EG;
    dl[tt][ee] = (tt < nt && ee < ne) ? dlogits[(size_t)(t0 + tt) * E + e0 + ee] : 0.f;
  }
  __syncthreads();
  if (c >= d) return;
  float acc[RB_EG];
#pragma unroll
  for (int ee = 0; ee < RB_EG; ++ee) acc[ee] = 0.f;
  const T* xp = x + (size_t)t0 * d + c;
  int tt = 0;
  for (; tt + 8 <= nt; tt += 8) {   // 8 loads in flight
    float xv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) xv[u] = to_f32(xp[(size_t)(tt + u) * d]);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int ee = 0; ee < RB_EG; ++ee) acc[ee] = fmaf(dl[tt + u][ee], xv[u], acc[ee]);
  }
  for (; tt < nt; ++tt) {
    const float xv = to_f32(xp[(size_t)tt * d]);
#pragma unroll
    for (int ee = 0; ee < RB_EG; ++ee) acc[ee] = fmaf(dl[tt][ee], xv, acc[ee]);
  }
#pragma unroll
  for (int ee = 0; ee < RB_EG; ++ee)
    if (ee < ne) partial[((size_t)chunk * E + e0 + ee) * d + c] = acc[ee];
}

// dWg[e][c] = sum over the chunks in ascending order (8 loads in flight, added in order).
__global__ __launch_bounds__(256) void route_bwd_dwg_reduce_kernel(const float* __restrict__ partial,
                                                                   int n_chunks, size_t ed,
                                                                   float* __restrict__ dWg) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= ed) return;
  float s = 0.f;
  int ch = 0;
  for (; ch + 8 <= n_chunks; ch += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(ch + u) * ed + i];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; ch < n_chunks; ++ch) s += partial[(size_t)ch * ed + i];
  dWg[i] = s;
}

// dbias[e] = sum_t dlogits[t][e]: one block per expert, fixed reduction tree.
__global__ __launch_bounds__(256) void route_bwd_dbias_kernel(const float* __restrict__ dlogits,
                                                              int T, int E,
                                                              float* __restrict__ dbias) {
  __shared__ float red[256];
  const int e = blockIdx.x;
  float s = 0.f;
  for (int t = threadIdx.x; t < T; t += 256) s += dlogits[(size_t)t * E + e];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off >= 1; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) dbias[e] = red[0];
}

// dx[t] += sum_e dlogits[t][e] * Wg[e]: one wavefront per token, 16 bytes per lane.  With
// renormalisation only the k selected experts have a non-zero logit gradient.
template <typename T>
__global__ __launch_bounds__(256) void route_bwd_dx_kernel(
    const T* __restrict__ Wg, const float* __restrict__ dlogits,
    const int32_t* __restrict__ topk_idx, int Tn, int d, int E, int k, int renormalize,
    T* __restrict__ dx) {
  constexpr int V = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= Tn) return;
  const int n_terms = renormalize ? k : E;
  for (int c = lane * V; c < d; c += 64 * V) {
    float acc[V];
    Vec16<T>::load(dx + (size_t)t * d + c, acc);
    for (int j = 0; j < n_terms; ++j) {
      const int e = renormalize ? topk_idx[(size_t)t * k + j] : j;
      if ((unsigned)e >= (unsigned)E) continue;   // the routing is the caller's: stay inside Wg
      const float g = dlogits[(size_t)t * E + e];
      float w[V];
      Vec16<T>::load(Wg + (size_t)e * d + c, w);
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = fmaf(g, w[v], acc[v]);
    }
    Vec16<T>::store(dx + (size_t)t * d + c, acc);
  }
}

// T == 0: the sums are empty.  (A fill kernel rather than a memset call, so that the launch
// can be part of a captured graph.)
__global__ void route_bwd_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

}  // namespace

size_t route_bwd_workspace_floats(const moe_ctx* c) {
  const size_t chunks = ((size_t)c->cfg.T_max + RB_TOK - 1) / RB_TOK;
  return chunks * (size_t)c->cfg.E * c->cfg.d;
}

int launch_route_bwd(moe_ctx* c, const void* x, const void* Wg, const float* logits,
                     const int32_t* topk_idx, const float* topk_w, const float* dtopk_w, int T,
                     float* dlogits, float* dWg, float* dbias, void* dx, hipStream_t s) {
  const int E = c->cfg.E, d = c->cfg.d, k = c->cfg.k, rn = c->cfg.renormalize;
  if (T == 0) {
    if (dWg != nullptr)
      hipLaunchKernelGGL(route_bwd_zero_kernel, dim3(256), dim3(256), 0, s, dWg, (size_t)E * d);
    if (dbias != nullptr)
      hipLaunchKernelGGL(route_bwd_zero_kernel, dim3(1), dim3(256), 0, s, dbias, (size_t)E);
    if (hipGetLastError() != hipSuccess) return MOE_EHIP;
    return MOE_OK;
  }
  const int wave_grid = (T + 3) / 4;
  hipLaunchKernelGGL(route_bwd_dlogits_kernel, dim3(wave_grid), dim3(256), 0, s, logits, topk_idx,
                     topk_w, dtopk_w, T, E, k, rn, dlogits);
  if (dWg != nullptr) {
    const int chunks = (T + RB_TOK - 1) / RB_TOK;
    const int eg = E <= 8 ? 8 : 16;
    const dim3 g((d + RB_COLS - 1) / RB_COLS, chunks, (E + eg - 1) / eg);
#define DWG_PARTIAL(T_, EG_)                                                                  \
  hipLaunchKernelGGL((route_bwd_dwg_partial_kernel<T_, EG_>), g, dim3(RB_COLS), 0, s,         \
                     (const T_*)x, dlogits, T, d, E, c->d_rbwd_ws)
    if (c->cfg.dtype == MOE_BF16) {
      if (eg == 8) DWG_PARTIAL(uint16_t, 8);
      else DWG_PARTIAL(uint16_t, 16);
    } else {
      if (eg == 8) DWG_PARTIAL(float, 8);
      else DWG_PARTIAL(float, 16);
    }
#undef DWG_PARTIAL
    const size_t ed = (size_t)E * d;
    hipLaunchKernelGGL(route_bwd_dwg_reduce_kernel, dim3((unsigned)((ed + 255) / 256)), dim3(256), 0,
                       s, c->d_rbwd_ws, chunks, ed, dWg);
  }
  if (dbias != nullptr)
    hipLaunchKernelGGL(route_bwd_dbias_kernel, dim3(E), dim3(256), 0, s, dlogits, T, E, dbias);
  if (dx != nullptr) {
    if (c->cfg.dtype == MOE_BF16)
      hipLaunchKernelGGL((route_bwd_dx_kernel<uint16_t>), dim3(wave_grid), dim3(256), 0, s,
                         (const uint16_t*)Wg, dlogits, topk_idx, T, d, E, k, rn, (uint16_t*)dx);
    else
      hipLaunchKernelGGL((route_bwd_dx_kernel<float>), dim3(wave_grid), dim3(256), 0, s,
                         (const float*)Wg, dlogits, topk_idx, T, d, E, k, rn, (float*)dx);
  }
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
