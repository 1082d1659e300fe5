// Combine / un-permute and the row-wise backward kernels (paper Sec. 2.1: after the
// experts the results are moved back and merged per token).  All three are gathers of k
// packed rows per token: one wavefront per token, 16 bytes per lane, fp32 arithmetic,
// a single rounding to the storage type at the end.
#include "moe_internal.h"
#include "numeric.h"
#include <type_traits>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename T, int K_MAX>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y_packed,
                                                      const int32_t* __restrict__ slot_to_row,
                                                      const float* __restrict__ topk_w, int Tn,
                                                      int k, int S, int d, T* __restrict__ out,
                                                      int stream) {
  constexpr int N = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= Tn) return;
  // Rows are wave-uniform.  Missing slots (j >= k, unmapped) read row 0 and are masked out
  // with a select, so the loads stay unconditional and can all be in flight together.
  const T* rowp[K_MAX];
  float w[K_MAX];
  bool ok[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) {
    const int r = j < k ? slot_to_row[(size_t)t * k + j] : -1;
    ok[j] = (unsigned)r < (unsigned)S;
    rowp[j] = y_packed + (size_t)(ok[j] ? r : 0) * d;
    w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
  }
  // stream != 0 (packed rows larger than the last-level cache): the rows are read once, with
  // non-temporal loads (measured 94 -> 81 us on 403 MB of packed rows; no gain when they fit)
  auto body = [&](auto NT) {
#pragma unroll(K_MAX <= 4 ? 2 : 1)
    for (int c = lane * N; c < d; c += 64 * N) {
      uint4 raw[K_MAX];
#pragma unroll
      for (int j = 0; j < K_MAX; ++j) {
        if constexpr (decltype(NT)::value) {
          const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rowp[j] + c));
          raw[j] = make_uint4(r.x, r.y, r.z, r.w);
        } else {
          raw[j] = Vec16<T>::load_raw(rowp[j] + c);
        }
      }
      float acc[N];
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = 0.f;
#pragma unroll
      for (int j = 0; j < K_MAX; ++j) {
        float v[N];
        Vec16<T>::unpack(raw[j], v);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = ok[j] ? fmaf(w[j], v[i], acc[i]) : acc[i];
      }
      Vec16<T>::store(out + (size_t)t * d + c, acc);
    }
  };
  if (stream) body(std::true_type{}); else body(std::false_type{});
}

template <typename T, int K_MAX>
__global__ __launch_bounds__(256) void combine_bwd_kernel(
    const T* __restrict__ dout, const T* __restrict__ y_packed,
    const int32_t* __restrict__ slot_to_row, const float* __restrict__ topk_w, int Tn, int k,
    int S, int d, T* __restrict__ dy_packed, float* __restrict__ dtopk_w) {
  constexpr int N = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= Tn) return;
  int rows[K_MAX];
  float w[K_MAX], dot[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) {
    int r = j < k ? slot_to_row[(size_t)t * k + j] : -1;
    r = ((unsigned)r < (unsigned)S) ? r : -1;
    rows[j] = __builtin_amdgcn_readfirstlane(r);  // wave-uniform: scalar branches below
    w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
    dot[j] = 0.f;
  }
#pragma unroll(K_MAX <= 4 ? 2 : 1)
  for (int c = lane * N; c < d; c += 64 * N) {
    float g[N];
    Vec16<T>::load(dout + (size_t)t * d + c, g);
    uint4 raw[K_MAX];
#pragma unroll
    for (int j = 0; j < K_MAX; ++j)  // unconditional (row 0 for a missing slot), masked below
      raw[j] = Vec16<T>::load_raw(y_packed + (size_t)(rows[j] >= 0 ? rows[j] : 0) * d + c);
#pragma unroll
    for (int j = 0; j < K_MAX; ++j) {
      float v[N], o[N];
      Vec16<T>::unpack(raw[j], v);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        dot[j] = rows[j] >= 0 ? fmaf(g[i], v[i], dot[j]) : dot[j];
        o[i] = w[j] * g[i];
      }
      if (rows[j] >= 0) Vec16<T>::store(dy_packed + (size_t)rows[j] * d + c, o);
    }
  }
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) {
    float s = dot[j];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0 && j < k) dtopk_w[(size_t)t * k + j] = s;
  }
}

template <typename T, int K_MAX>
__global__ __launch_bounds__(256) void dispatch_bwd_kernel(const T* __restrict__ dx_packed,
                                                           const int32_t* __restrict__ slot_to_row,
                                                           int Tn, int k, int S, int d,
                                                           T* __restrict__ dx) {
  constexpr int N = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= Tn) return;
  const T* rowp[K_MAX];
  bool ok[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) {
    const int r = j < k ? slot_to_row[(size_t)t * k + j] : -1;
    ok[j] = (unsigned)r < (unsigned)S;
    rowp[j] = dx_packed + (size_t)(ok[j] ? r : 0) * d;
  }
#pragma unroll(K_MAX <= 4 ? 2 : 1)
  for (int c = lane * N; c < d; c += 64 * N) {
    uint4 raw[K_MAX];
#pragma unroll
    for (int j = 0; j < K_MAX; ++j) raw[j] = Vec16<T>::load_raw(rowp[j] + c);
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
#pragma unroll
    for (int j = 0; j < K_MAX; ++j) {
      float v[N];
      Vec16<T>::unpack(raw[j], v);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = ok[j] ? acc[i] + v[i] : acc[i];
    }
    Vec16<T>::store(dx + (size_t)t * d + c, acc);
  }
}

#define DISPATCH_K(KERNEL, TYPE, ...)                                                         \
  do {                                                                                        \
    if (k <= 2)                                                                               \
      hipLaunchKernelGGL((KERNEL<TYPE, 2>), dim3(grid), dim3(256), 0, s, __VA_ARGS__);        \
    else if (k <= 4)                                                                          \
      hipLaunchKernelGGL((KERNEL<TYPE, 4>), dim3(grid), dim3(256), 0, s, __VA_ARGS__);        \
    else if (k <= 8)                                                                          \
      hipLaunchKernelGGL((KERNEL<TYPE, 8>), dim3(grid), dim3(256), 0, s, __VA_ARGS__);        \
    else                                                                                      \
      hipLaunchKernelGGL((KERNEL<TYPE, MOE_MAX_TOPK>), dim3(grid), dim3(256), 0, s,           \
                         __VA_ARGS__);                                                        \
  } while (0)

}  // namespace

int launch_combine(const moe_ctx* c, const void* y_packed, const int32_t* slot_to_row,
                   const float* w, int T, void* out, hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int k = c->cfg.k, d = c->cfg.d, S = T * k;
  const int grid = (T + 3) / 4;
  const int stream = (size_t)S * d * c->elem > ((size_t)192 << 20);   // 256 MB last-level cache
  if (c->cfg.dtype == MOE_BF16)
    DISPATCH_K(combine_kernel, uint16_t, (const uint16_t*)y_packed, slot_to_row, w, T, k, S, d,
               (uint16_t*)out, stream);
  else
    DISPATCH_K(combine_kernel, float, (const float*)y_packed, slot_to_row, w, T, k, S, d,
               (float*)out, stream);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_combine_bwd(const moe_ctx* c, const void* dout, const void* y_packed,
                       const int32_t* slot_to_row, const float* w, int T, void* dy_packed,
                       float* dw, hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int k = c->cfg.k, d = c->cfg.d, S = T * k;
  const int grid = (T + 3) / 4;
  if (c->cfg.dtype == MOE_BF16)
    DISPATCH_K(combine_bwd_kernel, uint16_t, (const uint16_t*)dout, (const uint16_t*)y_packed,
               slot_to_row, w, T, k, S, d, (uint16_t*)dy_packed, dw);
  else
    DISPATCH_K(combine_bwd_kernel, float, (const float*)dout, (const float*)y_packed, slot_to_row,
               w, T, k, S, d, (float*)dy_packed, dw);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_dispatch_bwd(const moe_ctx* c, const void* dx_packed, const int32_t* slot_to_row, int T,
                        void* dx, hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int k = c->cfg.k, d = c->cfg.d, S = T * k;
  const int grid = (T + 3) / 4;
  if (c->cfg.dtype == MOE_BF16)
    DISPATCH_K(dispatch_bwd_kernel, uint16_t, (const uint16_t*)dx_packed, slot_to_row, T, k, S, d,
               (uint16_t*)dx);
  else
    DISPATCH_K(dispatch_bwd_kernel, float, (const float*)dx_packed, slot_to_row, T, k, S, d,
               (float*)dx);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
