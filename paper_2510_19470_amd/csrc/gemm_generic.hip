// Grouped GEMMs on the vector ALU with fp32 accumulation: the fp32 storage path of the
// expert FFN and its backward, the gate projection, and the fallback for shapes the MFMA
// kernels do not tile.  Plain 64x64x16 LDS tiling, 4x4 outputs per thread, arbitrary
// strides and full bounds checks.  (Paper Sec. 2.1: experts are FFNs; Sec. 3.1: the
// experts of a GPU run one after another on their own tokens -- here one launch walks a
// device-built list of (expert, row block) tiles instead.)
#include "moe_internal.h"
#include "numeric.h"

namespace {

constexpr int BM = GENERIC_BM, BN = 64, BK = 16;

struct Smem {
  float a[BK][BM + 4];
  float b[BK][BN + 4];
};

// acc += A[m0.., 0..K) * B[0..K), n0..) for this thread's 4x4 outputs:
// rows m0 + ty + 16*i (i<4), columns n0 + tx + 16*j (j<4).
template <typename TA, typename TB>
__device__ __forceinline__ void tile_mac(float (&acc)[4][4], const TA* __restrict__ A, long sAm,
                                         long sAk, int m_valid, const TB* __restrict__ B, long sBk,
                                         long sBn, int n_valid, int K, Smem& sm) {
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const bool a_kfast = (sAk == 1);
  const bool b_kfast = (sBk == 1);
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      int mm, kk;
      if (a_kfast) { kk = idx & 15; mm = idx >> 4; } else { mm = idx & 63; kk = idx >> 6; }
      float v = 0.f;
      if (mm < m_valid && k0 + kk < K) v = to_f32(A[mm * sAm + (long)(k0 + kk) * sAk]);
      sm.a[kk][mm] = v;
      int nn;
      if (b_kfast) { kk = idx & 15; nn = idx >> 4; } else { nn = idx & 63; kk = idx >> 6; }
      v = 0.f;
      if (nn < n_valid && k0 + kk < K) v = to_f32(B[(long)(k0 + kk) * sBk + nn * sBn]);
      sm.b[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sm.a[kk][ty + 16 * i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = sm.b[kk][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
}

__device__ __forceinline__ void zero(float (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
}

// ---- gate projection: logits = x Wg^T + bias -------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gate_logits_kernel(const T* __restrict__ x,
                                                          const T* __restrict__ Wg,
                                                          const float* __restrict__ bias, int Tn,
                                                          int E, int d, float* __restrict__ logits) {
  __shared__ Smem sm;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;   // row blocks on grid.x (no 65535 limit)
  float acc[4][4];
  zero(acc);
  tile_mac(acc, x + (size_t)m0 * d, d, 1, Tn - m0, Wg + (size_t)n0 * d, 1, d, E - n0, d, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty + 16 * i;
    if (m >= Tn) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n < E) logits[(size_t)m * E + n] = acc[i][j] + (bias ? bias[n] : 0.f);
    }
  }
}

// ---- forward ------------------------------------------------------------------------
// H = silu(X W1^T) * (X W3^T) for one (expert, row block) x 64 columns of f; with
// W3t == nullptr the two-matrix expert: H = max(X W1^T, 0).
template <typename T>
__global__ __launch_bounds__(256) void ffn_gate_up_kernel(
    const T* __restrict__ xp, const TileSched* __restrict__ sched, const MTile* __restrict__ mt,
    const void* const* __restrict__ W1t, const void* const* __restrict__ W3t, int d, int f,
    T* __restrict__ H, T* __restrict__ Gs, T* __restrict__ Us) {
  __shared__ Smem sm;
  if ((int)blockIdx.x >= sched->n_mtiles) return;
  const MTile tl = mt[blockIdx.x];
  const T* W1 = (const T*)W1t[tl.expert];
  const bool gated = W3t != nullptr;
  const T* W3 = gated ? (const T*)W3t[tl.expert] : nullptr;
  const int n0 = blockIdx.y * BN;
  float g[4][4], u[4][4];
  zero(g);
  zero(u);
  const T* A = xp + (size_t)tl.row0 * d;
  tile_mac(g, A, d, 1, tl.rows, W1 + (size_t)n0 * d, 1, d, f - n0, d, sm);
  if (gated) tile_mac(u, A, d, 1, tl.rows, W3 + (size_t)n0 * d, 1, d, f - n0, d, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ty + 16 * i;
    if (r >= tl.rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n >= f) continue;
      const size_t o = (size_t)(tl.row0 + r) * f + n;
      const float gv = g[i][j], uv = u[i][j];
      H[o] = from_f32<T>(gated ? gv / (1.f + expf(-gv)) * uv : fmaxf(gv, 0.f));
      if (Gs) {
        Gs[o] = from_f32<T>(gv);
        if (gated) Us[o] = from_f32<T>(uv);
      }
    }
  }
}

// Y = H W2^T
template <typename T>
__global__ __launch_bounds__(256) void ffn_down_kernel(const T* __restrict__ H,
                                                       const TileSched* __restrict__ sched,
                                                       const MTile* __restrict__ mt,
                                                       const void* const* __restrict__ W2t, int d,
                                                       int f, T* __restrict__ y) {
  __shared__ Smem sm;
  if ((int)blockIdx.x >= sched->n_mtiles) return;
  const MTile tl = mt[blockIdx.x];
  const T* W2 = (const T*)W2t[tl.expert];
  const int n0 = blockIdx.y * BN;
  float acc[4][4];
  zero(acc);
  tile_mac(acc, H + (size_t)tl.row0 * f, f, 1, tl.rows, W2 + (size_t)n0 * f, 1, f, d - n0, f, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ty + 16 * i;
    if (r >= tl.rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n < d) y[(size_t)(tl.row0 + r) * d + n] = from_f32<T>(acc[i][j]);
    }
  }
}

// ---- backward -----------------------------------------------------------------------
// dH = dY W2, then dG = dH*u*silu'(g), dU = dH*silu(g), H = silu(g)*u (kept for dW2).
// Two-matrix expert (Us == nullptr): dG = dH where g > 0, else 0; H = max(g, 0).
template <typename T>
__global__ __launch_bounds__(256) void ffn_bwd_dh_kernel(
    const T* __restrict__ dy, const T* __restrict__ Gs, const T* __restrict__ Us,
    const TileSched* __restrict__ sched, const MTile* __restrict__ mt,
    const void* const* __restrict__ W2t, int d, int f, T* __restrict__ dG, T* __restrict__ dU,
    T* __restrict__ H) {
  __shared__ Smem sm;
  if ((int)blockIdx.x >= sched->n_mtiles) return;
  const MTile tl = mt[blockIdx.x];
  const T* W2 = (const T*)W2t[tl.expert];  // [d,f]: B(k=c, n) = W2[c*f + n]
  const int n0 = blockIdx.y * BN;
  float acc[4][4];
  zero(acc);
  tile_mac(acc, dy + (size_t)tl.row0 * d, d, 1, tl.rows, W2 + n0, f, 1, f - n0, d, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ty + 16 * i;
    if (r >= tl.rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n >= f) continue;
      const size_t o = (size_t)(tl.row0 + r) * f + n;
      const float g = to_f32(Gs[o]), dh = acc[i][j];
      if (Us == nullptr) {
        dG[o] = from_f32<T>(g > 0.f ? dh : 0.f);
        H[o] = from_f32<T>(fmaxf(g, 0.f));
        continue;
      }
      const float u = to_f32(Us[o]);
      const float sg = 1.f / (1.f + expf(-g));
      dG[o] = from_f32<T>(dh * u * sg * (1.f + g * (1.f - sg)));
      dU[o] = from_f32<T>(dh * g * sg);
      H[o] = from_f32<T>(g * sg * u);
    }
  }
}

// dX = dG W1 + dU W3   (two-matrix expert, W3t == nullptr: dX = dG W1)
template <typename T>
__global__ __launch_bounds__(256) void ffn_bwd_dx_kernel(
    const T* __restrict__ dG, const T* __restrict__ dU, const TileSched* __restrict__ sched,
    const MTile* __restrict__ mt, const void* const* __restrict__ W1t,
    const void* const* __restrict__ W3t, int d, int f, T* __restrict__ dx) {
  __shared__ Smem sm;
  if ((int)blockIdx.x >= sched->n_mtiles) return;
  const MTile tl = mt[blockIdx.x];
  const T* W1 = (const T*)W1t[tl.expert];  // [f,d]: B(k=n_f, n=c) = W1[n_f*d + c]
  const bool gated = W3t != nullptr;
  const T* W3 = gated ? (const T*)W3t[tl.expert] : nullptr;
  const int n0 = blockIdx.y * BN;
  float acc[4][4];
  zero(acc);
  tile_mac(acc, dG + (size_t)tl.row0 * f, f, 1, tl.rows, W1 + n0, d, 1, d - n0, f, sm);
  if (gated) tile_mac(acc, dU + (size_t)tl.row0 * f, f, 1, tl.rows, W3 + n0, d, 1, d - n0, f, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ty + 16 * i;
    if (r >= tl.rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n < d) dx[(size_t)(tl.row0 + r) * d + n] = from_f32<T>(acc[i][j]);
    }
  }
}

// dW[e] [Mo,No] = P_e^T Q_e over the rows of expert e:  P [S,Mo], Q [S,No].
// dW2 = dY^T H (Mo=d, No=f); dW1 = dG^T X (Mo=f, No=d); dW3 = dU^T X.
template <typename T>
__global__ __launch_bounds__(256) void ffn_bwd_dw_kernel(
    const T* __restrict__ P, const T* __restrict__ Q, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ offsets, const void* const* __restrict__ present,
    const void* const* __restrict__ dWt, const TileSched* __restrict__ sched, int Mo, int No) {
  __shared__ Smem sm;
  const int e = blockIdx.z;
  float* dW = (float*)dWt[e];
  if (dW == nullptr || present[e] == nullptr) return;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  // the schedule kernel of this call has checked the caller's counts and offsets against
  // the buffer size: no tiles at all (and zeros here) if any segment does not fit
  const int row0 = offsets[e], rows = sched->n_mtiles > 0 ? counts[e] : 0;
  float acc[4][4];
  zero(acc);
  // A(m, k=r) = P[(row0+r)*Mo + m0+m]; B(k=r, n) = Q[(row0+r)*No + n0+n]
  tile_mac(acc, P + (size_t)row0 * Mo + m0, 1, Mo, Mo - m0, Q + (size_t)row0 * No + n0, No, 1,
           No - n0, rows, sm);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty + 16 * i;
    if (m >= Mo) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx + 16 * j;
      if (n < No) dW[(size_t)m * No + n] = acc[i][j];
    }
  }
}

// ---- tile schedule --------------------------------------------------------------------
// One block: experts with weights present, in id order, cut into row blocks of bm rows.
__global__ __launch_bounds__(256) void build_sched_kernel(const int32_t* __restrict__ counts,
                                                          const int32_t* __restrict__ offsets,
                                                          const void* const* __restrict__ present,
                                                          int E, int S, int bm, int max_mtiles,
                                                          TileSched* __restrict__ sched,
                                                          MTile* __restrict__ mt) {
  __shared__ int32_t start[MOE_MAX_EXPERTS + 1];
  if (threadIdx.x == 0) {
    int run = 0;
    bool bad = false;   // a segment that does not lie inside the S rows of the call's buffers
    for (int e = 0; e < E; ++e) {
      start[e] = run;
      if (present[e] != nullptr) {
        const int n = counts[e], o = offsets[e];
        if (n < 0 || o < 0 || (long)o + n > (long)S) bad = true;
        else run += (n + bm - 1) / bm;
      }
    }
    if (bad) {   // the caller's arrays are inconsistent: no tiles, nothing is computed
      run = 0;
      for (int e = 0; e <= E; ++e) start[e] = 0;
    }
    start[E] = run;
    sched->n_mtiles = run < max_mtiles ? run : max_mtiles;
  }
  __syncthreads();
  for (int e = 0; e < E; ++e) {
    const int n = start[e + 1] - start[e];
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      const int idx = start[e] + i;
      if (idx < max_mtiles) {
        MTile t;
        t.expert = e;
        t.row0 = offsets[e] + i * bm;
        t.rows = min(bm, counts[e] - i * bm);
        t.pad = 0;
        mt[idx] = t;
      }
    }
  }
}

template <typename T>
int ffn_generic_t(moe_ctx* c, bool gated, const void* xp, void* y, void* G, void* U, void* H,
                  hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f;
  const int mtiles = c->max_mtiles[0];
  const void* const* W1 = c->d_wtab + 0 * MOE_MAX_EXPERTS;
  const void* const* W3 = gated ? c->d_wtab + 1 * MOE_MAX_EXPERTS : nullptr;
  const void* const* W2 = c->d_wtab + 2 * MOE_MAX_EXPERTS;
  hipLaunchKernelGGL((ffn_gate_up_kernel<T>), dim3(mtiles, (f + BN - 1) / BN), dim3(256), 0, s,
                     (const T*)xp, c->d_sched[0], c->d_mtiles[0], W1, W3, d, f, (T*)H, (T*)G,
                     (T*)U);
  prof_mark(c, 2, s);
  hipLaunchKernelGGL((ffn_down_kernel<T>), dim3(mtiles, (d + BN - 1) / BN), dim3(256), 0, s,
                     (const T*)H, c->d_sched[0], c->d_mtiles[0], W2, d, f, (T*)y);
  prof_mark(c, 3, s);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

template <typename T>
int ffn_bwd_generic_t(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* G,
                      const void* U, const int32_t* counts, const int32_t* offsets, void* dxp,
                      void* dG, void* dU, void* H, hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f, E = c->cfg.E;
  const int mtiles = c->max_mtiles[0];
  const void* const* W1 = c->d_wtab + 0 * MOE_MAX_EXPERTS;
  const void* const* W3 = gated ? c->d_wtab + 1 * MOE_MAX_EXPERTS : nullptr;
  const void* const* W2 = c->d_wtab + 2 * MOE_MAX_EXPERTS;
  const void* const* dW1 = c->d_wtab + 3 * MOE_MAX_EXPERTS;
  const void* const* dW3 = c->d_wtab + 4 * MOE_MAX_EXPERTS;
  const void* const* dW2 = c->d_wtab + 5 * MOE_MAX_EXPERTS;
  hipLaunchKernelGGL((ffn_bwd_dh_kernel<T>), dim3(mtiles, (f + BN - 1) / BN), dim3(256), 0, s,
                     (const T*)dy, (const T*)G, gated ? (const T*)U : nullptr, c->d_sched[0],
                     c->d_mtiles[0], W2, d, f, (T*)dG, (T*)dU, (T*)H);
  hipLaunchKernelGGL((ffn_bwd_dx_kernel<T>), dim3(mtiles, (d + BN - 1) / BN), dim3(256), 0, s,
                     (const T*)dG, (const T*)dU, c->d_sched[0], c->d_mtiles[0], W1, W3, d, f,
                     (T*)dxp);
  const dim3 g_df((f + BN - 1) / BN, (d + BM - 1) / BM, E);  // output [d,f]
  const dim3 g_fd((d + BN - 1) / BN, (f + BM - 1) / BM, E);  // output [f,d]
  hipLaunchKernelGGL((ffn_bwd_dw_kernel<T>), g_df, dim3(256), 0, s, (const T*)dy, (const T*)H,
                     counts, offsets, W2, dW2, c->d_sched[0], d, f);
  hipLaunchKernelGGL((ffn_bwd_dw_kernel<T>), g_fd, dim3(256), 0, s, (const T*)dG, (const T*)xp,
                     counts, offsets, W1, dW1, c->d_sched[0], f, d);
  if (gated)
    hipLaunchKernelGGL((ffn_bwd_dw_kernel<T>), g_fd, dim3(256), 0, s, (const T*)dU, (const T*)xp,
                       counts, offsets, W3, dW3, c->d_sched[0], f, d);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

}  // namespace

int launch_gate_logits(const moe_ctx* c, const void* x, const void* Wg, const float* bias, int T,
                       float* logits, hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int E = c->cfg.E, d = c->cfg.d;
  const dim3 grid((T + BM - 1) / BM, (E + BN - 1) / BN);
  if (c->cfg.dtype == MOE_BF16)
    hipLaunchKernelGGL((gate_logits_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t*)x,
                       (const uint16_t*)Wg, bias, T, E, d, logits);
  else
    hipLaunchKernelGGL((gate_logits_kernel<float>), grid, dim3(256), 0, s, (const float*)x,
                       (const float*)Wg, bias, T, E, d, logits);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_build_sched(moe_ctx* c, const int32_t* counts, const int32_t* offsets, int which,
                       hipStream_t s) {
  const int bm = which == 0 ? GENERIC_BM : MFMA_BM;
  hipLaunchKernelGGL(build_sched_kernel, dim3(1), dim3(256), 0, s, counts, offsets,
                     c->d_wtab + 0 * MOE_MAX_EXPERTS, c->cfg.E, c->S_call, bm, c->max_mtiles[which],
                     c->d_sched[which], c->d_mtiles[which]);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_ffn_generic(moe_ctx* c, bool gated, const void* x_packed, void* y_packed, void* G,
                       void* U, void* H_tmp, hipStream_t s) {
  return c->cfg.dtype == MOE_BF16
             ? ffn_generic_t<uint16_t>(c, gated, x_packed, y_packed, G, U, H_tmp, s)
             : ffn_generic_t<float>(c, gated, x_packed, y_packed, G, U, H_tmp, s);
}

int launch_ffn_bwd_generic(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* G,
                           const void* U, const int32_t* counts, const int32_t* offsets, void* dxp,
                           void* dG_tmp, void* dU_tmp, void* H_tmp, hipStream_t s) {
  return c->cfg.dtype == MOE_BF16
             ? ffn_bwd_generic_t<uint16_t>(c, gated, dy, xp, G, U, counts, offsets, dxp, dG_tmp,
                                           dU_tmp, H_tmp, s)
             : ffn_bwd_generic_t<float>(c, gated, dy, xp, G, U, counts, offsets, dxp, dG_tmp,
                                        dU_tmp, H_tmp, s);
}
