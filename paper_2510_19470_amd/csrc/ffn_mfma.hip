// Grouped SwiGLU expert FFN on the matrix cores (bf16 in, fp32 accumulate) for gfx950.
// (Paper Sec. 2.1: experts are replicated FFNs; Sec. 3.1: computation latency is
// dominated by the expert GEMMs and the experts of one GPU run on their own tokens.)
//
// Two launches walk a device-built tile list (no host sync on the token counts):
//   gate/up : H[r, n] = silu(x_r . W1[e][n,:]) * (x_r . W3[e][n,:])   (SwiGLU fused)
//   down    : Y[r, c] = H[r,:] . W2[e][c,:]
// Every operand is contiguous along the contraction dimension, so each lane feeds the
// MFMA with one 16-byte LDS read per operand fragment.
//
// Tiling: 512 threads = 8 wavefronts (2 along rows x 4 along columns), block tile
// 256 rows x 256 weight rows x 64 (k), wavefront tile 128 x 64 = 4 x 2 MFMA 32x32x16
// accumulators (128 fp32 registers).  For gate/up the 256 weight rows are 128 rows of W1
// and the matching 128 rows of W3, laid out so that a wavefront owns gate and up of the
// same columns and applies silu(g)*u in registers.  The weight rows are the MFMA "A"
// operand and the token rows the "B" operand: a lane then holds 4 consecutive output
// columns of one token row and stores them as one 8-byte write.
// LDS: 2 stages x (32 KB tokens + 32 KB weights) = 128 KB, 16-byte chunks XOR-swizzled by
// row so that the 16-byte fragment reads of 16 consecutive rows fall on distinct banks.
// Global loads of stage t+1 are issued before the MFMAs of stage t and written to LDS
// after them: one barrier per k-step.
// Tile order: tiles of one expert that share a weight panel (same column block) are
// consecutive, and the block index is remapped so that each of the 8 XCDs (private L2)
// works on a contiguous range of that order.
#include "moe_internal.h"
#include "numeric.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = MFMA_BM;       // token rows per block tile
constexpr int BNW = 256;          // weight rows per block tile
constexpr int BK = 64;            // k per stage
constexpr int NT = 512;           // threads
constexpr int STAGE_VEC = 2048;   // uint4 per operand per stage (256 rows x 8 chunks)

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

// tile list entry: (mtile index << 12) | column block
__global__ __launch_bounds__(256) void mfma_sched_kernel(
    const int32_t* __restrict__ counts, const int32_t* __restrict__ offsets,
    const void* const* __restrict__ present, int E, int S, int max_mtiles, int nt_up, int nt_down,
    TileSched* __restrict__ sched, MTile* __restrict__ mt, uint32_t* __restrict__ order_up,
    uint32_t* __restrict__ order_down) {
  __shared__ int32_t start[MOE_MAX_EXPERTS + 1];
  __shared__ int bad;
  const int tid = threadIdx.x;
  if (tid == 0) {
    start[0] = 0;
    bad = 0;
  }
  __syncthreads();
  // per-expert tile counts (E <= 256: one expert per thread), then an inclusive scan
  int mine = 0;
  if (tid < E && present[tid] != nullptr) {
    const int n = counts[tid], o = offsets[tid];
    if (n < 0 || o < 0 || (long)o + n > (long)S) bad = 1;  // caller's arrays are inconsistent
    else mine = (n + BM - 1) / BM;
  }
  start[tid + 1] = mine;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    int v = 0;
    if (tid >= off) v = start[tid + 1 - off];
    __syncthreads();
    if (tid >= off) start[tid + 1] += v;
    __syncthreads();
  }
  const int total_m = (bad || start[E] > max_mtiles) ? 0 : start[E];
  if (blockIdx.x == 0 && tid == 0) sched->n_mtiles = total_m;
  const int gsz = gridDim.x * blockDim.x;
  const int gid = blockIdx.x * blockDim.x + tid;
  for (int i = gid; i < total_m; i += gsz) {
    int lo = 0, hi = E;  // largest e with start[e] <= i
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (start[mid] <= i) lo = mid; else hi = mid;
    }
    const int m = i - start[lo];
    MTile t;
    t.expert = lo;
    t.row0 = offsets[lo] + m * BM;
    t.rows = min(BM, counts[lo] - m * BM);
    t.pad = 0;
    mt[i] = t;
  }
  // tile order: expert by expert; inside an expert column block by column block, and for
  // one column block all of the expert's row blocks in a row (they share a weight panel)
  for (int pass = 0; pass < 2; ++pass) {
    const int nt = pass == 0 ? nt_up : nt_down;
    uint32_t* order = pass == 0 ? order_up : order_down;
    const int total = total_m * nt;
    for (int L = gid; L < total; L += gsz) {
      int lo = 0, hi = E;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (start[mid] * nt <= L) lo = mid; else hi = mid;
      }
      const int me = start[lo + 1] - start[lo];
      const int rel = L - start[lo] * nt;
      const int n = rel / me, m = rel % me;
      order[L] = ((uint32_t)(start[lo] + m) << 12) | (uint32_t)n;
    }
  }
}

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// One k-step of the wavefront tile: 4 k-slices of 16, each 6 fragment reads + 8 MFMAs.
// The reads of slice kk+1 are issued before the MFMAs of slice kk (two fragment sets in
// registers), and the wavefront raises its priority while it feeds the matrix core so
// that the other wavefront of the SIMD does its LDS reads in the shadow.
__device__ __forceinline__ void mma_stage(f32x16 (&acc)[2][4], const uint4* __restrict__ As,
                                          const uint4* __restrict__ Bs, const int (&fr_a)[4],
                                          const int (&fr_b)[2], int fr_half, int fr_swz) {
  bf16x8 xa[2][4], wb[2][2];
  {
    const int ch = fr_half ^ fr_swz;
#pragma unroll
    for (int i = 0; i < 4; ++i) xa[0][i] = __builtin_bit_cast(bf16x8, As[fr_a[i] + ch]);
#pragma unroll
    for (int j = 0; j < 2; ++j) wb[0][j] = __builtin_bit_cast(bf16x8, Bs[fr_b[j] + ch]);
  }
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    if (kk < 3) {
      const int ch = ((kk + 1) * 2 + fr_half) ^ fr_swz;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        xa[(kk + 1) & 1][i] = __builtin_bit_cast(bf16x8, As[fr_a[i] + ch]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        wb[(kk + 1) & 1][j] = __builtin_bit_cast(bf16x8, Bs[fr_b[j] + ch]);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[kk & 1][j], xa[kk & 1][i],
                                                            acc[j][i], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Asynchronous global -> LDS copy of one k-step (no registers in between): each wavefront
// fills 4 blocks of 8 rows x 128 B per operand; a lane's 16 bytes land at lane*16 inside
// the block, so the swizzle is applied by choosing which global chunk the lane fetches.
__device__ __forceinline__ void issue_stage(const uint4* const (&a_src)[4],
                                            const uint4* const (&b_src)[4], int kofs,
                                            uint4* As, uint4* Bs, int wave) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + kofs), (lptr_t)(As + (wave * 4 + i) * 64),
                                     16, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr_t)(b_src[i] + kofs), (lptr_t)(Bs + (wave * 4 + i) * 64),
                                     16, 0, 0);
  }
  // keep the copies at the top of the step: the scheduler would otherwise sink them
  // below the MFMAs and expose their whole latency at the barrier
  __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ void wait_stage_and_sync() {
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): my copies landed, my reads are done
  __syncthreads();
}

template <bool GATED>
__global__ __launch_bounds__(NT) void ffn_mfma_kernel(
    const uint16_t* __restrict__ A, const TileSched* __restrict__ sched,
    const MTile* __restrict__ mt, const uint32_t* __restrict__ order, int n_tiles_n,
    const void* const* __restrict__ Bt0, const void* const* __restrict__ Bt1, int K, int N,
    uint16_t* __restrict__ C, uint16_t* __restrict__ Gs, uint16_t* __restrict__ Us) {
  // two stages, each 256 token rows + 256 weight rows of 64 bf16 (separate arrays so that
  // reads of one stage are known not to alias the copy in flight into the other)
  __shared__ uint4 ldsA0[STAGE_VEC];
  __shared__ uint4 ldsB0[STAGE_VEC];
  __shared__ uint4 ldsA1[STAGE_VEC];
  __shared__ uint4 ldsB1[STAGE_VEC];

  const int total = sched->n_mtiles * n_tiles_n;
  const int per_xcd = (total + 7) >> 3;
  const int slot = blockIdx.x >> 3;
  const int L = (blockIdx.x & 7) * per_xcd + slot;
  if (slot >= per_xcd || L >= total) return;
  const uint32_t ent = order[L];
  const MTile tl = mt[ent >> 12];
  const int nblk = ent & 0xfff;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- global -> LDS assignment: lane (lane>>3, lane&7) of block b = wave*4+i fills LDS
  // row 8b + (lane>>3), chunk slot (lane&7), which must hold global chunk slot ^ swz(row)
  const uint4* a_src[4];
  const uint4* b_src[4];
  const uint16_t* B0 = (const uint16_t*)Bt0[tl.expert];
  const uint16_t* B1 = GATED ? (const uint16_t*)Bt1[tl.expert] : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (wave * 4 + i) * 8 + (lane >> 3);
    const int ch = (lane & 7) ^ swz(row);
    const int arow = min(row, tl.rows - 1);
    a_src[i] = (const uint4*)(A + (size_t)(tl.row0 + arow) * K) + ch;
    const uint16_t* bp;
    if (GATED)
      bp = (row < 128 ? B0 : B1) + (size_t)(nblk * 128 + (row & 127)) * K;
    else
      bp = B0 + (size_t)(nblk * 256 + row) * K;
    b_src[i] = (const uint4*)bp + ch;
  }

  // ---- fragment read offsets (uint4 units inside one operand stage)
  const int fr_row = lane & 31, fr_half = lane >> 5;
  const int fr_swz = swz(fr_row);
  int fr_a[4], fr_b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) fr_a[i] = (wm * 128 + i * 32 + fr_row) * 8;
#pragma unroll
  for (int j = 0; j < 2; ++j) fr_b[j] = (j * 128 + wn * 32 + fr_row) * 8;

  f32x16 acc[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  // K is a multiple of 128, so the number of k-steps is even and the loop can alternate
  // the two stages without a conditional exit (keeps the accumulators in registers).
  const int KT = K / BK;
  issue_stage(a_src, b_src, 0, ldsA0, ldsB0, wave);
  wait_stage_and_sync();
  for (int kt = 0; kt < KT; kt += 2) {
    issue_stage(a_src, b_src, (kt + 1) * 8, ldsA1, ldsB1, wave);
    mma_stage(acc, ldsA0, ldsB0, fr_a, fr_b, fr_half, fr_swz);
    wait_stage_and_sync();
    // the copy after the last step re-reads that step into the idle stage: in bounds,
    // unconditional, and nobody reads it
    const int kn = kt + 2 < KT ? kt + 2 : kt;
    issue_stage(a_src, b_src, kn * 8, ldsA0, ldsB0, wave);
    mma_stage(acc, ldsA1, ldsB1, fr_a, fr_b, fr_half, fr_swz);
    wait_stage_and_sync();
  }

  // ---- epilogue: lane holds, per 32x32 accumulator, token row (lane&31) and the weight
  // rows 8*g + 4*(lane>>5) + {0..3}, g = 0..3
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m_local = wm * 128 + i * 32 + fr_row;
    if (m_local >= tl.rows) continue;
    const size_t rbase = (size_t)(tl.row0 + m_local) * N;
    if (GATED) {
      const int col0 = nblk * 128 + wn * 32 + 4 * fr_half;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float h[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float gv = acc[0][i][g * 4 + r], uv = acc[1][i][g * 4 + r];
          h[r] = silu_f(gv) * uv;
        }
        const size_t o = rbase + col0 + 8 * g;
        *reinterpret_cast<uint2*>(C + o) = make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3]));
        if (Gs != nullptr) {
          *reinterpret_cast<uint2*>(Gs + o) =
              make_uint2(pack_bf16x2(acc[0][i][g * 4], acc[0][i][g * 4 + 1]),
                         pack_bf16x2(acc[0][i][g * 4 + 2], acc[0][i][g * 4 + 3]));
          *reinterpret_cast<uint2*>(Us + o) =
              make_uint2(pack_bf16x2(acc[1][i][g * 4], acc[1][i][g * 4 + 1]),
                         pack_bf16x2(acc[1][i][g * 4 + 2], acc[1][i][g * 4 + 3]));
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col0 = nblk * 256 + j * 128 + wn * 32 + 4 * fr_half;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const size_t o = rbase + col0 + 8 * g;
          *reinterpret_cast<uint2*>(C + o) =
              make_uint2(pack_bf16x2(acc[j][i][g * 4], acc[j][i][g * 4 + 1]),
                         pack_bf16x2(acc[j][i][g * 4 + 2], acc[j][i][g * 4 + 3]));
        }
      }
    }
  }
}

}  // namespace

bool ffn_mfma_supported(const moe_ctx* c) {
  const int d = c->cfg.d, f = c->cfg.f;
  return c->cfg.dtype == MOE_BF16 && d % 256 == 0 && f % 128 == 0 &&  // K % 128 == 0 too
         f / 128 < 4096 &&
         d / 256 < 4096;
}

size_t ffn_mfma_order_entries(const moe_ctx* c) {
  const int nt_up = c->cfg.f / 128, nt_down = c->cfg.d / 256;
  return (size_t)c->max_mtiles[1] * (nt_up > nt_down ? nt_up : nt_down);
}

int launch_ffn_mfma(moe_ctx* c, const int32_t* counts, const int32_t* offsets, const void* x_packed,
                    void* y_packed, void* G, void* U, hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f, E = c->cfg.E;
  const int nt_up = f / 128, nt_down = d / 256;
  const void* const* W1 = c->d_wtab + 0 * MOE_MAX_EXPERTS;
  const void* const* W3 = c->d_wtab + 1 * MOE_MAX_EXPERTS;
  const void* const* W2 = c->d_wtab + 2 * MOE_MAX_EXPERTS;
  const int max_mt = c->max_mtiles[1];
  prof_mark(c, 0, s);
  hipLaunchKernelGGL(mfma_sched_kernel, dim3(32), dim3(256), 0, s, counts, offsets, W1, E,
                     c->S_max, max_mt, nt_up, nt_down, c->d_sched[1], c->d_mtiles[1], c->d_order_up, c->d_order_down);
  const int grid_up = ((max_mt * nt_up + 7) / 8) * 8;
  const int grid_down = ((max_mt * nt_down + 7) / 8) * 8;
  prof_mark(c, 1, s);
  hipLaunchKernelGGL((ffn_mfma_kernel<true>), dim3(grid_up), dim3(NT), 0, s,
                     (const uint16_t*)x_packed, c->d_sched[1], c->d_mtiles[1], c->d_order_up, nt_up,
                     W1, W3, d, f, (uint16_t*)c->d_H, (uint16_t*)G, (uint16_t*)U);
  prof_mark(c, 2, s);
  hipLaunchKernelGGL((ffn_mfma_kernel<false>), dim3(grid_down), dim3(NT), 0, s,
                     (const uint16_t*)c->d_H, c->d_sched[1], c->d_mtiles[1], c->d_order_down,
                     nt_down, W2, (const void* const*)nullptr, f, d, (uint16_t*)y_packed,
                     (uint16_t*)nullptr, (uint16_t*)nullptr);
  prof_mark(c, 3, s);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
