// Weight gradients of the expert FFN on the matrix cores without transposed copies of the
// activations: the chain rule of the expert FFN of Sec. 2.1 taken with respect to its
// weights (the paper itself only notes, in Sec. 6, that the backward pass adds a constant
// all-reduce term to its model).
//
//   dW[e][m, n] = sum over the rows r of expert e of  P[r, m] * Q[r, n]      (fp32 out)
//
// Both operands are stored with the contraction index (the token row) OUTERMOST: an MFMA
// fragment (one output row or column, 8 consecutive k) is a column of 8 rows in memory.  The
// tiles are copied to LDS as they are (32 token rows x 256 columns, 512 bytes per row, direct
// global -> LDS copies) and read with the LDS transpose read of gfx950,
// ds_read_b64_tr_b16: inside a group of 16 lanes, lane s supplies the address of 4 elements
// of row (s >> 2) -- column group (s & 3) -- and lane i receives element (i & 3) of the four
// addresses of lanes (i >> 2) + {0, 4, 8, 12}.  With lane s pointing at row k0 + (s >> 2),
// columns c0 + 4 * (s & 3) .. + 3, lane i ends up with column c0 + i, rows k0 .. k0 + 3: two
// such reads give the 8 consecutive k of one MFMA operand register pair.
//
// Block tile 256 (m) x 256 (n), 8 wavefronts (2 along m x 4 along n), wavefront tile 128 x 64
// = 4 x 2 accumulators of v_mfma_f32_32x32x16_bf16, as in the forward kernels.  The k-loop
// runs in half-steps of 32 token rows through 4 LDS stages of 32 KB (P tile 16 KB + Q tile
// 16 KB); the copies of half-step h+3 are issued when half-step h starts.  16-byte chunks of
// a row are XOR-swizzled (tr_swz below), which puts the rows x 32 bytes that the groups of 16
// lanes sharing an LDS cycle read on distinct banks.  Rows past the end of the expert's segment are fetched
// from a row of zeros, so a ragged segment needs no padded copy.
#include "moe_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int NT = 512;
constexpr int HK = 32;                 // token rows per half-step
constexpr int STAGES = 4;
constexpr int TILE_BYTES = HK * 512;   // one operand tile of a stage
constexpr int STAGE_BYTES = 2 * TILE_BYTES;

struct WgradArgs {
  struct Job {
    const uint16_t* P;   // [S, p_pitch]; the tile's columns start at p_col0 + 256 * (row block)
    const uint16_t* Q;   // [S, q_pitch]
    const void* const* dWt;   // [E] fp32 outputs [Mo, No]
    int p_pitch, p_col0, q_pitch, Mo, No;
  } job[3];
  int n_jobs, E;
  int n_list;                         // experts that get weight gradients
  uint8_t list[MOE_MAX_EXPERTS];      // ... their ids, ascending
  const int32_t* counts;
  const int32_t* offsets;
  const TileSched* sched;     // of the data-gradient GEMMs of the same call: n_mtiles == 0 when
                              // the caller's counts and offsets do not fit the buffers
  const uint16_t* zero_row;   // 512 bytes of zeros
};

// Swizzle of the 16-byte chunks of a 512-byte tile row.  A transpose read takes, per group of
// 16 lanes, 4 rows (j4 = row & 3) x 32 bytes; the four groups of a wavefront are (hh = bit 3
// of the row, cb = the 32-byte column half).  LDS has 64 banks of 4 bytes and serves 32 lanes
// per cycle, and the row pitch is a multiple of 256 bytes, so the 16 chunks of any two
// groups that can share a cycle -- (hh, cb = 0 | 1) or (hh = 0 | 1, cb) -- must differ
// modulo 16: bits 2-3 of the chunk take j4, bit 1 takes hh (cb sits in bit 1 already).
__device__ __forceinline__ int tr_swz(int row) { return ((row & 3) << 2) ^ (((row >> 3) & 1) << 1); }

// 16 bytes per lane global -> LDS, per-lane 64-bit address; the wavefront's 1 KB lands at
// lds_addr (wave-uniform, via M0) + lane * 16.
__device__ __forceinline__ void dma16v(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr)
               : "memory", "m0");
}

__global__ __launch_bounds__(NT) void wgrad_tr_kernel(const WgradArgs p) {
  __shared__ uint4 lds[STAGES * STAGE_BYTES / 16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  // block -> tile.  The tiles are ordered (expert, job, groups of 4 row blocks of dW, column
  // block, row block inside the group): 32 consecutive tiles are a 4 x 8 patch of one matrix,
  // 12 operand panels for 32 tiles.  The hardware deals blocks round-robin to the 8 XCDs, each
  // with an L2 of its own, so XCD x (= blockIdx & 7) takes the chunks of 32 consecutive tiles
  // x, x + 8, ...: the 32 blocks resident on an XCD share their panels in its L2.  (Every job
  // has the same number of tiles per expert.)
  const int tiles = (p.job[0].Mo >> 8) * (p.job[0].No >> 8);
  const int total = p.n_list * p.n_jobs * tiles;
  const int slot = (int)(blockIdx.x >> 3), xcd = (int)(blockIdx.x & 7);
  const int L = ((slot >> 5) * 8 + xcd) * 32 + (slot & 31);
  if (L >= total) return;
  const int ej = L / tiles, rel = L % tiles;
  const int e = p.list[ej / p.n_jobs];
  const WgradArgs::Job& J = p.job[ej % p.n_jobs];
  const int NoT = J.No >> 8, MoT = J.Mo >> 8;
  const int mg = rel / (4 * NoT), r2 = rel % (4 * NoT);
  const int gm = min(4, MoT - 4 * mg);
  const int nblk = r2 / gm, mblk = 4 * mg + r2 % gm;
  float* dW = (float*)J.dWt[e];
  if (dW == nullptr) return;   // this gradient is not wanted
  // counts and offsets are the caller's; the schedule kernel of this call has checked them
  // against the buffer size (no tiles at all if any segment does not fit: zeros come out)
  const int n_e = p.sched->n_mtiles > 0 ? p.counts[e] : 0;
  const int row0 = p.offsets[e];
  const int NH = (n_e + HK - 1) / HK;

  f32x16 acc[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;

  // ---- copies: instruction c (0..15) of a tile fills rows 2c (lanes 0-31) and 2c+1 (lanes
  // 32-63), 32 chunk slots each; slot s of row r holds global chunk s ^ tr_swz(r).
  // Wavefront w issues instructions w and w + 8 of the P tile and of the Q tile.
  const int c_row = lane >> 5, c_slot = lane & 31;
  const char* p_col = (const char*)(J.P + J.p_col0 + mblk * 256);
  const char* q_col = (const char*)(J.Q + nblk * 256);
  auto issue = [&](int h) {   // all copies of half-step h (rows past the segment: zeros)
    const uint32_t sb = lds_base + (uint32_t)(h & (STAGES - 1)) * STAGE_BYTES;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = wave + 8 * u;
      const int r = 2 * c + c_row;                     // row inside the stage
      const int rg = h * HK + r;                       // row inside the expert's segment
      const int gch = c_slot ^ tr_swz(r);              // global chunk this lane fetches
      const bool ok = rg < n_e;
      const size_t rr = (size_t)(row0 + min(rg, n_e - 1));   // in bounds also when not used
      const char* zp = (const char*)p.zero_row + gch * 16;
      const char* pa = p_col + rr * J.p_pitch * 2 + gch * 16;
      const char* qa = q_col + rr * J.q_pitch * 2 + gch * 16;
      dma16v(ok ? pa : zp, sb + c * 1024);
      dma16v(ok ? qa : zp, sb + TILE_BYTES + c * 1024);
    }
  };

  // ---- transpose reads: per-lane byte offsets inside an operand tile
  const int g16 = lane >> 4, hh = g16 >> 1, cb = g16 & 1;
  const int s16 = lane & 15, j4 = s16 >> 2, q4 = s16 & 3;
  const int rd_row = 8 * hh + j4;                 // + 16 * kk + 4 * t
  const int rd_swz = tr_swz(rd_row);              // + 16 * kk + 4 * t leaves the swizzle unchanged
  const int rd_half = (q4 & 1) * 8;
  int x_chunk[4], w_chunk[2];                     // chunk of the lane's 4 columns, before the swizzle
#pragma unroll
  for (int i = 0; i < 4; ++i) x_chunk[i] = (wm * 128 + i * 32 + cb * 16) / 8 + (q4 >> 1);
#pragma unroll
  for (int j = 0; j < 2; ++j) w_chunk[j] = (j * 128 + wn * 32 + cb * 16) / 8 + (q4 >> 1);
  auto frag = [&](uint32_t tile_base, int kk, int chunk) -> bf16x8 {
    const uint32_t a0 = tile_base + (uint32_t)(rd_row + 16 * kk) * 512 +
                        (uint32_t)((chunk ^ rd_swz) << 4) + rd_half;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)a0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(a0 + 4 * 512));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  if (NH > 0) {
    issue(0);
    issue(1);
    issue(2);
    for (int h = 0; h < NH; ++h) {
      // half-step h has landed for this wavefront (the copies of h+1 and h+2, 8 instructions,
      // may still be in flight) and, after the barrier, for everybody; everybody has also
      // finished reading half-step h-1, whose stage takes half-step h+3
      asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
      issue(h + 3);
      const uint32_t sb = (uint32_t)(h & (STAGES - 1)) * STAGE_BYTES;   // LDS offsets from 0: generic
      const uint32_t pt = lds_base + sb, qt = lds_base + sb + TILE_BYTES;
      // all 12 fragments of the half-step first (24 transpose reads in flight), then the 16
      // MFMAs: the other wavefront of the SIMD computes meanwhile (one barrier per half-step
      // lets the wavefronts drift apart; a strict two-group ping-pong with two barriers per
      // half-step measured 13 % slower)
      bf16x8 xa[2][4], wb[2][2];
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int j = 0; j < 2; ++j) wb[kk][j] = frag(qt, kk, w_chunk[j]);
#pragma unroll
        for (int i = 0; i < 4; ++i) xa[kk][i] = frag(pt, kk, x_chunk[i]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[kk][j], xa[kk][i], acc[j][i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy in flight into LDS at exit
  }

  // ---- epilogue: lane holds row (lane & 31) of each 32-row block and the columns
  // 8g + 4(lane >> 5) + {0..3} of each 32-column block
  const int fr_row = lane & 31, fr_half = lane >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float* orow = dW + (size_t)(mblk * 256 + wm * 128 + i * 32 + fr_row) * J.No;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col0 = nblk * 256 + j * 128 + wn * 32 + 4 * fr_half;
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<float4*>(orow + col0 + 8 * g) =
            make_float4(acc[j][i][g * 4], acc[j][i][g * 4 + 1], acc[j][i][g * 4 + 2],
                        acc[j][i][g * 4 + 3]);
    }
  }
}

}  // namespace

// dy, xp: [S,d]; H: [S,f]; dGU: [S,gw] (dG | dU, or dG alone for the two-matrix expert).
int launch_wgrad_tr(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* H,
                    const void* dGU, const int32_t* counts, const int32_t* offsets,
                    hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f, E = c->cfg.E;
  const int gw = gated ? 2 * f : f;
  WgradArgs a{};
  a.n_jobs = gated ? 3 : 2;
  a.E = E;
  a.counts = counts;
  a.offsets = offsets;
  a.sched = c->d_sched[1];
  for (int e = 0; e < E; ++e)   // host copy of the pointer tables: resident, some dW wanted
    if (c->h_wtab[0][e] != nullptr &&
        (c->h_wtab[3][e] != nullptr || c->h_wtab[4][e] != nullptr || c->h_wtab[5][e] != nullptr))
      a.list[a.n_list++] = (uint8_t)e;
  if (a.n_list == 0) return MOE_OK;
  a.zero_row = (const uint16_t*)c->d_zero;
  const void* const* dW1 = c->d_wtab + 3 * MOE_MAX_EXPERTS;
  const void* const* dW3 = c->d_wtab + 4 * MOE_MAX_EXPERTS;
  const void* const* dW2 = c->d_wtab + 5 * MOE_MAX_EXPERTS;
  // dW2 [d,f] = dY^T H;  dW1 [f,d] = dG^T X;  dW3 [f,d] = dU^T X
  a.job[0] = {(const uint16_t*)dy, (const uint16_t*)H, dW2, d, 0, f, d, f};
  a.job[1] = {(const uint16_t*)dGU, (const uint16_t*)xp, dW1, gw, 0, d, f, d};
  a.job[2] = {(const uint16_t*)dGU, (const uint16_t*)xp, dW3, gw, f, d, f, d};
  const int tiles = (d / 256) * (f / 256);
  const int total = a.n_jobs * a.n_list * tiles;
  hipLaunchKernelGGL(wgrad_tr_kernel, dim3((total + 255) / 256 * 256), dim3(NT), 0, s, a);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
