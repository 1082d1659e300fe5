// Measured ceilings of the part, for the benchmark's roofline: what a plain copy kernel and a
// bare MFMA issue loop reach on the same device, in the same process, as the kernels they are
// compared with.  Measurement aids, not steps of the path.
#include "moe_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// One 16-byte piece per thread, one contiguous 4 KB run per block: read once, written to
// `fanout` destinations `stride_vec` pieces apart (fanout 1 = plain copy, 2 = the read:write
// mix of a top-2 dispatch).
__global__ __launch_bounds__(256) void ceiling_copy_kernel(const u32x4* __restrict__ src,
                                                           u32x4* __restrict__ dst, size_t n_vec,
                                                           int fanout, size_t stride_vec) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_vec) return;
  const u32x4 v = src[i];
  for (int c = 0; c < fanout; ++c) dst[(size_t)c * stride_vec + i] = v;
}

// 8 wavefronts per block (two per SIMD), each with the 8 independent 32x32 accumulators of
// the grouped GEMM's wavefront tile, issuing v_mfma_f32_32x32x16_bf16 back to back from
// registers: no LDS, no memory.  `random` fills the operands with bf16 values of varied
// sign, exponent and mantissa (the power drawn by the matrix cores depends on the data);
// otherwise they are zero.
__global__ __launch_bounds__(512) void ceiling_mfma_kernel(float* __restrict__ sink, int iters,
                                                           int random) {
  const int tid = threadIdx.x;
  bf16x8 a[4], b[2];
  uint32_t h = (uint32_t)(blockIdx.x * 512 + tid) * 2654435761u + 12345u;
  auto next_bf16 = [&]() -> __bf16 {
    h = h * 1664525u + 1013904223u;
    // sign, exponent in [124, 128) (|value| in [0.125, 2)), 7 mantissa bits
    const uint16_t bits = (uint16_t)(((h >> 31) << 15) | ((124u + ((h >> 20) & 3u)) << 7) | ((h >> 8) & 127u));
    return random ? __builtin_bit_cast(__bf16, bits) : __builtin_bit_cast(__bf16, (uint16_t)0);
  };
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[i][e] = next_bf16();
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[j][e] = next_bf16();
  f32x16 acc[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[(i + kk) & 3], acc[j][i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[j][i][r];
  sink[(size_t)blockIdx.x * 512 + tid] = s;
}

}  // namespace

extern "C" int moe_measure_copy(const void* src, void* dst, int64_t bytes, int32_t fanout,
                                void* stream) {
  if (src == nullptr || dst == nullptr || bytes < 16 || bytes % 16 != 0 || fanout < 1 || fanout > 16)
    return MOE_EINVAL;
  if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) != 0)
    return MOE_EINVAL;
  const size_t n_vec = (size_t)bytes / 16;
  const size_t blocks = (n_vec + 255) / 256;
  if (blocks > 0x7fffffffull) return MOE_EUNSUPPORTED;
  hipLaunchKernelGGL(ceiling_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (const u32x4*)src, (u32x4*)dst, n_vec, fanout, n_vec);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

extern "C" int moe_measure_mfma(float* sink, int32_t blocks, int32_t iters, int32_t random_operands,
                                double* flops_out, void* stream) {
  if (sink == nullptr || blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24))
    return MOE_EINVAL;
  hipLaunchKernelGGL(ceiling_mfma_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)stream, sink,
                     iters, random_operands != 0);
  if (flops_out != nullptr)   // 8 wavefronts x 32 MFMAs per iteration x 2*32*32*16 flop
    *flops_out = (double)blocks * 8.0 * iters * 32.0 * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
