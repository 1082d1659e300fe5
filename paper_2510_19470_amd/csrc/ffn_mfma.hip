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
// LDS: 2 stages x (32 KB tokens + 32 KB weights) = 128 KB, filled by asynchronous
// global->LDS copies (no registers in between); 16-byte chunks are XOR-swizzled by row so
// that the 16-byte fragment reads of 16 consecutive rows fall on distinct banks.
// Main loop ("ping-pong"): the wavefronts of the upper 128 token rows and those of the
// lower 128 rows alternate between a memory cluster (fragment reads of one 32-row token
// block, two copy instructions) and a compute cluster (8 MFMAs), the second group one
// cluster behind the first, so every SIMD always has one wavefront on the matrix core
// and one on memory.  A token block is refilled as soon as its group has read it, the
// weight rows as soon as both groups have read them (first cluster of a step), each with
// the data of two steps ahead: copies are spread evenly over the step and have more
// than one step to land.
// Tile order: an expert's row blocks in groups of 8; inside a group the tiles that share a
// weight panel (same column block) are consecutive, and the block index is remapped so that
// each of the 8 XCDs (private L2) works on a contiguous range of that order: the 32 tiles an
// XCD has in flight are 8 row blocks x 4 column blocks.
#include "moe_internal.h"
#include "numeric.h"

#include <algorithm>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int BM = MFMA_BM;       // token rows per block tile
constexpr int BK = 64;            // k per stage
constexpr int NT = 512;           // threads
constexpr int STAGE_VEC = 2048;   // uint4 per operand per stage (256 rows x 8 chunks)
constexpr int ORDER_GROUP_M = 8;  // row blocks per group of the tile order

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }
// ... of a k-major stage (512-byte rows, transpose reads): the groups of 16 lanes that can
// share an LDS cycle read 4 rows (row & 3) x 32 bytes each, from the two halves of bit 3 of
// the row or the two 32-byte column halves; their 16 chunks must differ modulo 16
__device__ __forceinline__ int tr_swz(int row) { return ((row & 3) << 2) ^ (((row >> 3) & 1) << 1); }

// tile list entry: (mtile index << 12) | column block
__global__ __launch_bounds__(256) void mfma_sched_kernel(
    const int32_t* __restrict__ counts, const int32_t* __restrict__ offsets,
    const void* const* __restrict__ present, int E, int S, int max_mtiles, int nt_up, int nt_down,
    int n_cu, int kt_down, TileSched* __restrict__ sched, const void* const* __restrict__ up_b0,
    const void* const* __restrict__ up_b1, const void* const* __restrict__ down_b0,
    const void* const* __restrict__ down_b1, TileDesc* __restrict__ order_up,
    TileDesc* __restrict__ order_down) {
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
  if (blockIdx.x == 0 && tid == 0) {
    sched->n_mtiles = total_m;
    // Down GEMM: when the last round of tiles fills at most half of the compute units, its
    // tiles are cut along the contraction into `split` parts (2 .. 8; every part a whole
    // number >= 4 of k-step pairs, the first parts one pair longer when the pairs do not
    // divide evenly; all parts together still one round), summed afterwards.
    const int total = total_m * nt_down;
    const int tail = total % n_cu;
    const int pairs = kt_down / 2;
    int split = 1;
    while (tail > 0 && split < 8 && tail * (split + 1) <= n_cu && pairs / (split + 1) >= 4)
      ++split;
    sched->down_split = split;
    sched->down_split_tiles = split > 1 ? tail : 0;
    sched->down_full = split > 1 ? total - tail : total;
  }
  const int gsz = gridDim.x * blockDim.x;
  const int gid = blockIdx.x * blockDim.x + tid;
  // tile order: expert by expert; inside an expert in groups of 8 row blocks; inside a group
  // column block by column block, the group's row blocks in a row (they share a weight panel)
  for (int pass = 0; pass < 2; ++pass) {
    const int nt = pass == 0 ? nt_up : nt_down;
    TileDesc* order = pass == 0 ? order_up : order_down;
    const int total = total_m * nt;
    for (int L = gid; L < total; L += gsz) {
      int lo = 0, hi = E;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (start[mid] * nt <= L) lo = mid; else hi = mid;
      }
      const int me = start[lo + 1] - start[lo];
      const int rel = L - start[lo] * nt;
      // groups of up to 8 row blocks: inside a group column block by column block, so that 32
      // consecutive tiles are 8 row blocks x 4 column blocks (12 panels for 32 tiles)
      const int per_group = ORDER_GROUP_M * nt;
      const int mg = rel / per_group, r2 = rel % per_group;
      const int gm = min(ORDER_GROUP_M, me - mg * ORDER_GROUP_M);
      const int n = r2 / gm, m = mg * ORDER_GROUP_M + r2 % gm;
      TileDesc t;
      t.row0 = offsets[lo] + m * BM;
      t.rows = min(BM, counts[lo] - m * BM);
      t.nblk = n;
      t.expert = lo;
      t.b0 = pass == 0 ? up_b0[lo] : down_b0[lo];
      const void* const* tab1 = pass == 0 ? up_b1 : down_b1;
      t.b1 = tab1 != nullptr ? tab1[lo] : nullptr;
      order[L] = t;
    }
  }
}

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Asynchronous 16 bytes per lane global -> LDS: lane reads base + off (wave-uniform 64-bit
// base in scalar registers, 32-bit per-lane byte offset), the wavefront's 1 KB lands at
// lds_addr (wave-uniform byte address, via M0) + lane * 16.  Written as assembly so that
// the compiler does not serialise later LDS reads behind it; completion is tracked by hand
// (vmcnt) in the main loop.
__device__ __forceinline__ void dma16(uint32_t off, const char* base, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_addr)
               : "memory", "m0");
}

// Epilogue stores.  A lane holds, per accumulator, 4 consecutive output columns 8g + 4h + {0..3}
// (h = lane >> 5) of one token row for g = 0..3: 8-byte pieces.  Swapping between the two
// half-wavefronts turns the pieces of g and g+1 into one 16-byte piece per lane -- lanes 0-31
// get columns 8g .. 8g+7, lanes 32-63 columns 8(g+1) .. 8(g+1)+7 of their row -- so that a
// wavefront stores 32 contiguous bytes per row with one instruction instead of 16 with two.
__device__ __forceinline__ uint4 pair16(uint2 a /* piece g */, uint2 b /* piece g+1 */) {
  // v_permlane32_swap: lanes 32-63 of the first operand <-> lanes 0-31 of the second
  const auto x = __builtin_amdgcn_permlane32_swap(a.x, b.x, false, false);
  const auto y = __builtin_amdgcn_permlane32_swap(a.y, b.y, false, false);
  return make_uint4(x[0], y[0], x[1], y[1]);
}
__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}
// The inverse, for epilogue loads: every lane loads the 16 bytes pair16 would store (lanes
// 0-31 columns 8g .. 8g+7, lanes 32-63 columns 8(g+1) .. 8(g+1)+7 of their row); the swaps
// give each lane its own 8-byte pieces of g (a) and g+1 (b).
__device__ __forceinline__ void unpair16(const uint4& v, uint2& a, uint2& b) {
  const auto x = __builtin_amdgcn_permlane32_swap(v.x, v.z, false, false);
  const auto y = __builtin_amdgcn_permlane32_swap(v.y, v.w, false, false);
  a = make_uint2(x[0], y[0]);
  b = make_uint2(x[1], y[1]);
}

enum { MODE_UP = 0, MODE_DOWN = 1, MODE_DH = 2, MODE_UP1 = 4, MODE_DH1 = 5 };

struct GemmArgs {
  const uint16_t* A;    // token-role operand: [rows, lda]
  int lda;              // elements per row of A
  const TileSched* sched;
  const TileDesc* order;
  int n_tiles_n;
  int K;                   // contraction length
  int N;                   // elements per output row
  uint16_t* C;             // UP: H; DOWN: Y / dX; DH: [dG|dU] with row pitch 2N
  uint16_t* C2;            // DH: H
  float* split_ws;         // DOWN: fp32 partial tiles of the K-split tail
  uint16_t* Gs;            // UP: optional save (out); DH: saved G (in)
  uint16_t* Us;
  // k-major weight-role operand (BKM kernels): B[k][n] with ldb elements per k-row; the first
  // kseg k-steps come from the tile's first matrix, the rest from its second one
  int ldb, kseg;
};

// One unit of work of a block: a whole tile, or one K-split part of a tile (all fields are
// wave-uniform and live in scalar registers).
struct Unit {
  int valid;
  int row0, rows, nblk;     // tile: first packed row, valid rows, column block
  const char* abase;        // token-role operand: first row of the tile, first k of the range
  const char* bbase0;       // weight-role operand: first row of the column block (gate/up: W1)
  const char* bbase1;       // gate/up: the same rows of W3; else bbase0 + 128 rows
  int KT;                   // k-steps of 64 (even)
  int kstart;               // first k-step of the unit (K-split parts; 0 otherwise)
  int ws_unit;              // >= 0: K-split part, index of its partial tile in the workspace
};

// The idx-th unit of this block.  The hardware deals blocks round-robin to the XCDs: XCD x
// (= blockIdx & 7) holds the blocks x, x + 8, ...  The tile order is walked in rounds of
// gridDim tiles; a round is cut into 8 chunks of consecutive tiles (32 in a full round: 8 row
// blocks x 4 column blocks that share 12 panels), chunk x goes to XCD x, one tile per block:
// at any time an XCD works on one chunk.  The last, partial round is cut into 8 equal chunks as
// well, so that every XCD stays in use.  Going round by round (rather than giving an XCD a
// contiguous eighth of the whole order) spreads the cheap tiles of short row blocks -- which
// come in runs -- over all XCDs.  After its whole tiles a block takes its share of the
// K-split units of the tail (a contiguous range per XCD).  The sequence of a block is dense:
// once a unit is invalid, all later ones are.
template <int MODE, bool BKM>
__device__ __forceinline__ Unit fetch_unit(const GemmArgs& p, int idx) {
  Unit u;
  u.valid = 0;
  u.ws_unit = -1;
  const int total = p.sched->n_mtiles * p.n_tiles_n;
  const int n_full = MODE == MODE_DOWN ? p.sched->down_full : total;
  const int split = MODE == MODE_DOWN ? p.sched->down_split : 1;
  const int n_units = MODE == MODE_DOWN ? p.sched->down_split_tiles * split : 0;
  const int per_xcd_s = (n_units + 7) >> 3;
  const int x = blockIdx.x & 7, slot = (int)(blockIdx.x >> 3);
  const int G = (int)gridDim.x, gsz = G >> 3;
  const int rfull = n_full / G, m_last = n_full - rfull * G;   // full rounds, tiles of the last one
  const int per_last = (m_last + 7) >> 3;
  const bool in_last = slot < per_last && x * per_last + slot < m_last;
  const int nfu = rfull + (in_last ? 1 : 0);
  const int ns = max(0, min(per_xcd_s, n_units - x * per_xcd_s));
  int L, part = 0, kstart = 0;   // kstart: first k-step of a K-split part
  if (idx < nfu) {
    L = idx < rfull ? idx * G + x * gsz + slot : rfull * G + x * per_last + slot;
    u.KT = p.K / BK;
  } else {
    const int qs = slot + (idx - nfu) * gsz;   // among the XCD's split units
    if (qs >= ns) return u;
    const int su = x * per_xcd_s + qs;
    L = n_full + su / split;
    part = su % split;
    // pairs of k-steps of this part: the first `rem` parts take one pair more
    const int pairs = p.K / BK / 2, base = pairs / split, rem = pairs % split;
    u.KT = 2 * (base + (part < rem ? 1 : 0));
    kstart = 2 * (part * base + min(part, rem));
    u.ws_unit = su;
  }
  const TileDesc td = p.order[L];
  u.valid = 1;
  u.row0 = td.row0;
  u.rows = td.rows;
  u.nblk = td.nblk;
  u.kstart = kstart;
  const size_t kbeg = (size_t)kstart * (BK * 2);  // bytes into a row
  u.abase = (const char*)p.A + (size_t)td.row0 * p.lda * 2 + kbeg;
  if (BKM) {   // column block of the k-major matrices; the k-step is applied per copy
    u.bbase0 = (const char*)td.b0 + (size_t)td.nblk * 512;
    u.bbase1 = (const char*)td.b1 + (size_t)td.nblk * 512;
  } else if (MODE == MODE_UP) {
    u.bbase0 = (const char*)td.b0 + (size_t)td.nblk * 128 * p.K * 2 + kbeg;
    u.bbase1 = (const char*)td.b1 + (size_t)td.nblk * 128 * p.K * 2 + kbeg;
  } else {
    u.bbase0 = (const char*)td.b0 + (size_t)td.nblk * 256 * p.K * 2 + kbeg;
    u.bbase1 = u.bbase0 + (size_t)128 * p.K * 2;
  }
  return u;
}

// One cluster pair of the main loop: memory cluster of token block I in stage S (fragment
// reads; two copies, base + offset each, into the rows read one cluster ago), then the
// compute cluster.
template <int S, int I, bool BKM>
__device__ __forceinline__ void pp_cluster(f32x16 (&acc)[2][4], bf16x8 (&wb)[2][4],
                                           const uint4* lds, const int (&fr_a)[4],
                                           const int (&fr_b)[2], int fr_half, int fr_swz,
                                           uint32_t offa, const char* basea, uint32_t offb,
                                           const char* baseb, uint32_t a_dst, uint32_t b_dst,
                                           int nact) {
  const uint4* As = lds + (2 * S) * STAGE_VEC;
  const uint4* Bs = lds + (2 * S + 1) * STAGE_VEC;
  bf16x8 xa[4];
  if (I == 0) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (BKM) {
          // k-major stage (64 k-rows x 512 bytes): fr_b[j] is the lane's LDS byte address for
          // k-rows 0..3 of its 16-row group; two transpose reads make the 8 k of the fragment
          const uint32_t a0 = (uint32_t)fr_b[j] + (2 * S + 1) * 32768 + kk * 8192;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)a0);
          const s16x4 hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(a0 + 4 * 512));
          const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          wb[j][kk] = __builtin_bit_cast(bf16x8, v);
        } else {
          wb[j][kk] = __builtin_bit_cast(bf16x8, Bs[fr_b[j] + ((kk * 2 + fr_half) ^ fr_swz)]);
        }
      }
  }
  // nact (wave-uniform): 32-row blocks of this wavefront's half of the tile that hold rows;
  // the others are neither read nor multiplied (their accumulators stay zero and are not
  // stored), the copies and barriers go on as ever
  const bool act = I < nact;
  if (act) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      xa[kk] = __builtin_bit_cast(bf16x8, As[fr_a[I] + ((kk * 2 + fr_half) ^ fr_swz)]);
  }
  constexpr int blk = (I + 3) & 3;
  constexpr int st = I == 0 ? (S ^ 1) : S;
  dma16(offa, basea, a_dst + st * 65536 + blk * 4096);
  dma16(offb, baseb, b_dst + st * 65536 + blk * 8192);
  // My fragment reads are done (the rows may be refilled after the next barrier) and all
  // but my last 6 vector-memory operations have completed: the data read in cluster n
  // was copied in clusters <= n-4, and every wavefront passes this point in cluster n-1
  // before anybody reads in cluster n.  (Stores of an epilogue count as well and only
  // make the wait stricter: copies complete in issue order among themselves.)
  asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_setprio(1);
  if (act) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[j][I] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[j][kk], xa[kk], acc[j][I], 0, 0, 0);
  }
  __builtin_amdgcn_s_setprio(0);
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_barrier" ::: "memory");
}

// MODE_UP   : H = silu(A W1^T) * (A W3^T)            (gate/up, SwiGLU fused)
// MODE_UP1  : H = max(A W1^T, 0)                      (first GEMM of the two-matrix expert)
// MODE_DOWN : C = A B^T                               (down projection; also dX = [dG|dU][W1^T|W3^T]^T)
// MODE_DH   : dH = A B^T, then dG = dH*u*silu'(g), dU = dH*silu(g), H = silu(g)*u
// MODE_DH1  : dH = A B^T, then dG = dH where g > 0 (else 0), H = max(g, 0)   (two-matrix expert)
//
// Tiled modes run persistent blocks (one per compute unit) over a static share of the tile
// order, and the copy stream does not stop at a tile boundary: during the last two k-steps
// of a tile the rows that become free are refilled with the first two k-steps of the
// block's next tile, so that only the very first tile of a block pays a load latency.
//
// BKM: the weight-role operand is stored k-major, B[k][n] (the data gradients contract over
// the other index of the weights).  A stage then holds 64 k-rows x 256 columns (512 bytes
// per row, 16-byte chunks XOR-swizzled by tr_swz(row)), copied as it is -- one copy
// instruction fills two k-rows -- and the fragments come out of LDS through the transpose
// read ds_read_b64_tr_b16 (the layout and the lane arithmetic of wgrad_tr.hip).
template <int MODE, bool BKM = false>
__global__ __launch_bounds__(NT) void ffn_mfma_kernel(const GemmArgs p) {
  // stage s: token rows at (2s) * STAGE_VEC, weight rows at (2s+1) * STAGE_VEC
  __shared__ uint4 lds[4 * STAGE_VEC];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = __builtin_amdgcn_readfirstlane(wave >> 2), wn = wave & 3;
  Unit cur;
  // global -> LDS assignment: one copy instruction fills 8 rows (lane>>3) x 8 chunk slots
  // (lane&7); slot c of row r must hold global chunk c ^ swz(r).  Token rows: copy i of a
  // wavefront fills 8 rows of block i of its own group's half; weight rows: copy i fills
  // row block 8i + wave (gate/up: blocks 0..15 are rows of W1, 16..31 the same rows of W3;
  // otherwise bbase1 is bbase0 + 128 rows).  Per-lane byte offsets from the unit's bases:
  uint32_t a_off[4], b_off[4];
  const int a_pitch = p.lda * 2;                                   // bytes per token-role row
  const int b_pitch = p.K * 2;                                     // ... per weight-role row
  auto token_off = [&](int rows, int i) -> uint32_t {
    const int ra = (16 * wm + 4 * i + wn) * 8 + (lane >> 3);
    return (uint32_t)min(ra, rows - 1) * a_pitch + (((lane & 7) ^ swz(ra)) << 4);
  };
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (BKM) {   // copy i of the wavefront: k-rows 2c and 2c+1 of the step, c = 8i + wave
      const int r = 2 * (8 * i + wave) + (lane >> 5);
      b_off[i] = (uint32_t)r * (uint32_t)(p.ldb * 2) + (((lane & 31) ^ tr_swz(r)) << 4);
    } else {
      const int rb = (8 * i + wave) * 8 + (lane >> 3);
      b_off[i] = (uint32_t)(rb & 127) * b_pitch + (((lane & 7) ^ swz(rb)) << 4);
    }
  }
  // weight-role source of k-step `step` of unit u (half: 0 = first, 1 = second 128 rows of the
  // column block when the operand is row-major)
  const size_t bstep = (size_t)BK * p.ldb * 2;
  auto bsrc = [&](const Unit& u, int step, int half) -> const char* {
    if (BKM) {
      const int kg = u.kstart + step;
      return kg < p.kseg ? u.bbase0 + (size_t)kg * bstep : u.bbase1 + (size_t)(kg - p.kseg) * bstep;
    }
    return (half ? u.bbase1 : u.bbase0) + step * 128;
  };
  cur = fetch_unit<MODE, BKM>(p, 0);
  if (!cur.valid) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) a_off[i] = token_off(cur.rows, i);

  // ---- fragment read offsets (uint4 units inside one operand stage)
  const int fr_row = lane & 31, fr_half = lane >> 5;
  const int fr_swz = swz(fr_row);
  int fr_a[4], fr_b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) fr_a[i] = (wm * 128 + i * 32 + fr_row) * 8;
#pragma unroll
  for (int j = 0; j < 2; ++j) fr_b[j] = (j * 128 + wn * 32 + fr_row) * 8;
  if (BKM) {
    // transpose reads: groups of 16 lanes; lane (j4 = (lane & 15) >> 2, q4 = lane & 3) of group
    // g16 = lane >> 4 points at k-row 8 * (g16 >> 1) + j4 and the 4 columns 16 * (g16 & 1) +
    // 4 * q4 .. + 3 of the fragment's 32 columns
    const int g16 = lane >> 4, j4 = (lane & 15) >> 2, q4 = lane & 3;
    const uint32_t lb = (uint32_t)(uintptr_t)(lptr_t)lds;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int chunk = (j * 128 + wn * 32 + (g16 & 1) * 16) / 8 + (q4 >> 1);
      const int row = 8 * (g16 >> 1) + j4;
      fr_b[j] = (int)(lb + row * 512 + ((chunk ^ tr_swz(row)) << 4) + (q4 & 1) * 8);
    }
  }

  f32x16 acc[2][4];

  // ---- epilogue of one unit: lane holds, per 32x32 accumulator, token row (lane&31) and
  // the weight rows 8*g + 4*(lane>>5) + {0..3}, g = 0..3
  auto epilogue = [&](const Unit& u) {
    if (MODE == MODE_DOWN && u.ws_unit >= 0) {
      // partial sums of one K-split part, in accumulator order: [unit][j][i][quad][thread]
      float4* ws = reinterpret_cast<float4*>(p.split_ws) + (size_t)u.ws_unit * (32 * NT) + tid;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            ws[((j * 4 + i) * 4 + q) * NT] = make_float4(acc[j][i][q * 4], acc[j][i][q * 4 + 1],
                                                         acc[j][i][q * 4 + 2], acc[j][i][q * 4 + 3]);
      return;
    }
    // bf16 outputs: every lane takes part in the half-wavefront swaps, only the stores are
    // predicated on the row being inside the tile; gp = 0, 1 are the column pairs g = (0,1), (2,3)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m_local = wm * 128 + i * 32 + fr_row;
      const bool live = m_local < u.rows;
      const size_t row = (size_t)(u.row0 + m_local);
      // MODE_DH, MODE_DH1: the saved G (and U) of the whole row block, 16 bytes per lane at the
      // addresses the outputs are stored to, all requested before the first is used
      uint4 gsv[2][2], usv[2][2];
      if (MODE == MODE_DH || MODE == MODE_DH1) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const size_t col = (size_t)u.nblk * 256 + j * 128 + wn * 32 + 8 * fr_half + 16 * gp;
            gsv[j][gp] = usv[j][gp] = make_uint4(0, 0, 0, 0);
            if (live) {
              gsv[j][gp] = *reinterpret_cast<const uint4*>(p.Gs + row * p.N + col);
              if (MODE == MODE_DH) usv[j][gp] = *reinterpret_cast<const uint4*>(p.Us + row * p.N + col);
            }
          }
      }
      if (MODE == MODE_UP) {
        const int colb = u.nblk * 128 + wn * 32 + 8 * fr_half;
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
          uint2 hp[2];
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const int g = 2 * gp + t;
            float h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) h[r] = silu_f(acc[0][i][g * 4 + r]) * acc[1][i][g * 4 + r];
            hp[t] = pack4(h[0], h[1], h[2], h[3]);
          }
          const size_t o = row * p.N + colb + 16 * gp;
          const uint4 hv = pair16(hp[0], hp[1]);
          if (live) *reinterpret_cast<uint4*>(p.C + o) = hv;
          if (p.Gs != nullptr) {
            const int g = 2 * gp;
            const uint4 gv = pair16(pack4(acc[0][i][g * 4], acc[0][i][g * 4 + 1], acc[0][i][g * 4 + 2], acc[0][i][g * 4 + 3]),
                                    pack4(acc[0][i][g * 4 + 4], acc[0][i][g * 4 + 5], acc[0][i][g * 4 + 6], acc[0][i][g * 4 + 7]));
            const uint4 uv = pair16(pack4(acc[1][i][g * 4], acc[1][i][g * 4 + 1], acc[1][i][g * 4 + 2], acc[1][i][g * 4 + 3]),
                                    pack4(acc[1][i][g * 4 + 4], acc[1][i][g * 4 + 5], acc[1][i][g * 4 + 6], acc[1][i][g * 4 + 7]));
            if (live) {
              *reinterpret_cast<uint4*>(p.Gs + o) = gv;
              *reinterpret_cast<uint4*>(p.Us + o) = uv;
            }
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int colb = u.nblk * 256 + j * 128 + wn * 32 + 8 * fr_half;
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const int g0 = 2 * gp;
            const size_t col = colb + 16 * gp;
            if (MODE == MODE_DOWN) {
              const uint4 v = pair16(pack4(acc[j][i][g0 * 4], acc[j][i][g0 * 4 + 1], acc[j][i][g0 * 4 + 2], acc[j][i][g0 * 4 + 3]),
                                     pack4(acc[j][i][g0 * 4 + 4], acc[j][i][g0 * 4 + 5], acc[j][i][g0 * 4 + 6], acc[j][i][g0 * 4 + 7]));
              if (live) *reinterpret_cast<uint4*>(p.C + row * p.N + col) = v;
            } else if (MODE == MODE_UP1) {
              float r[8];
#pragma unroll
              for (int q = 0; q < 8; ++q) r[q] = fmaxf(acc[j][i][g0 * 4 + q], 0.f);
              const uint4 v = pair16(pack4(r[0], r[1], r[2], r[3]), pack4(r[4], r[5], r[6], r[7]));
              if (live) *reinterpret_cast<uint4*>(p.C + row * p.N + col) = v;
              if (p.Gs != nullptr) {
                const uint4 gv = pair16(pack4(acc[j][i][g0 * 4], acc[j][i][g0 * 4 + 1], acc[j][i][g0 * 4 + 2], acc[j][i][g0 * 4 + 3]),
                                        pack4(acc[j][i][g0 * 4 + 4], acc[j][i][g0 * 4 + 5], acc[j][i][g0 * 4 + 6], acc[j][i][g0 * 4 + 7]));
                if (live) *reinterpret_cast<uint4*>(p.Gs + row * p.N + col) = gv;
              }
            } else {  // MODE_DH, MODE_DH1
              uint2 dgp[2], dup[2], hhp[2];
              uint2 gqs[2], uqs[2];
              unpair16(gsv[j][gp], gqs[0], gqs[1]);
              unpair16(usv[j][gp], uqs[0], uqs[1]);
#pragma unroll
              for (int t = 0; t < 2; ++t) {
                const int g = g0 + t;
                const uint2 gq = gqs[t], uq = uqs[t];
                const uint32_t gw[2] = {gq.x, gq.y}, uw[2] = {uq.x, uq.y};
                float dg[4], du[4], hh[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  const float gv = __uint_as_float((r & 1) ? (gw[r >> 1] & 0xffff0000u) : (gw[r >> 1] << 16));
                  const float dh = acc[j][i][g * 4 + r];
                  if (MODE == MODE_DH1) {   // two-matrix expert: dG = dH where g > 0, H = max(g, 0)
                    dg[r] = gv > 0.f ? dh : 0.f;
                    du[r] = 0.f;
                    hh[r] = fmaxf(gv, 0.f);
                  } else {
                    const float uv = __uint_as_float((r & 1) ? (uw[r >> 1] & 0xffff0000u) : (uw[r >> 1] << 16));
                    const float sg = sigmoid_f(gv);
                    dg[r] = dh * uv * sg * (1.f + gv * (1.f - sg));
                    du[r] = dh * gv * sg;
                    hh[r] = gv * sg * uv;
                  }
                }
                dgp[t] = pack4(dg[0], dg[1], dg[2], dg[3]);
                dup[t] = pack4(du[0], du[1], du[2], du[3]);
                hhp[t] = pack4(hh[0], hh[1], hh[2], hh[3]);
              }
              const uint4 dgv = pair16(dgp[0], dgp[1]), hhv = pair16(hhp[0], hhp[1]);
              if (MODE == MODE_DH) {
                const uint4 duv = pair16(dup[0], dup[1]);
                if (live) {
                  *reinterpret_cast<uint4*>(p.C + row * (2 * (size_t)p.N) + col) = dgv;
                  *reinterpret_cast<uint4*>(p.C + row * (2 * (size_t)p.N) + p.N + col) = duv;
                }
              } else if (live) {
                *reinterpret_cast<uint4*>(p.C + row * p.N + col) = dgv;
              }
              if (live) *reinterpret_cast<uint4*>(p.C2 + row * p.N + col) = hhv;
            }
          }
        }
      }
    }
  };

  auto zero_acc = [&]() {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;
  };

  // Every unit has an even number of k-steps (K is a multiple of 128 and the K-split keeps
  // its parts even).  KT == 0 cannot come out of the schedule (K >= 128); should it ever,
  // nothing is loaded and zeros are stored.
  if (cur.KT == 0) {
    zero_acc();
    epilogue(cur);
    return;
  }

  const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;
  // wave-uniform LDS byte addresses: + stage * 65536 + block * 4096 (tokens) / 8192 (weights)
  const uint32_t a_dst = __builtin_amdgcn_readfirstlane(lds_base + (16 * wm + wn) * 1024);
  const uint32_t b_dst = __builtin_amdgcn_readfirstlane(lds_base + 32768 + wave * 1024);
  // first unit: both stages in full (stage 0 first), then the second group falls one
  // cluster behind
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dma16(a_off[i], cur.abase + st * 128, a_dst + st * 65536 + i * 4096);
      dma16(b_off[i], bsrc(cur, st, i >= 2), b_dst + st * 65536 + i * 8192);
    }
  // stage 0 has landed (stage 1 is first read four clusters on, after the vmcnt(6) waits)
  asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
  if (wm == 1) asm volatile("s_barrier" ::: "memory");

  bf16x8 wb[2][4];
  for (int idx = 0;; ++idx) {
    const Unit nxt = fetch_unit<MODE, BKM>(p, idx + 1);
    zero_acc();
    const int KT = cur.KT;
    const int nact = __builtin_amdgcn_readfirstlane(min(4, max(0, (cur.rows - wm * 128 + 31) >> 5)));
    // steady part: steps 0 .. KT-3; what was read one cluster ago is refilled with the data
    // of its next use (token block i-1 and weight row blocks 8(i-1)+wave of this stage with
    // step k+2; at i == 0 block 3 of the other stage with step k+1)
    for (int kt = 0; kt < KT - 2; kt += 2) {
      const char* a1 = cur.abase + (kt + 1) * 128;  // step kt+1 (+128: kt+2, +256: kt+3)
#define PP(S, I, OA, BA, OB, BB) \
  pp_cluster<S, I, BKM>(acc, wb, lds, fr_a, fr_b, fr_half, fr_swz, OA, BA, OB, BB, a_dst, b_dst, nact)
      PP(0, 0, a_off[3], a1, b_off[3], bsrc(cur, kt + 1, 1));
      PP(0, 1, a_off[0], a1 + 128, b_off[0], bsrc(cur, kt + 2, 0));
      PP(0, 2, a_off[1], a1 + 128, b_off[1], bsrc(cur, kt + 2, 0));
      PP(0, 3, a_off[2], a1 + 128, b_off[2], bsrc(cur, kt + 2, 1));
      PP(1, 0, a_off[3], a1 + 128, b_off[3], bsrc(cur, kt + 2, 1));
      PP(1, 1, a_off[0], a1 + 256, b_off[0], bsrc(cur, kt + 3, 0));
      PP(1, 2, a_off[1], a1 + 256, b_off[1], bsrc(cur, kt + 3, 0));
      PP(1, 3, a_off[2], a1 + 256, b_off[2], bsrc(cur, kt + 3, 1));
    }
    // last two steps: the refills fetch steps 0 and 1 of the next unit (the token offsets
    // are switched block by block, each right after its last use for this unit).  Without a
    // next unit the last step is fetched again (in bounds, never read): the copy count per
    // cluster stays fixed, which the vmcnt arithmetic relies on.
    {
      const int last = (KT - 1) * 128;
      const char* na = nxt.valid ? nxt.abase : cur.abase + last;      // next unit's step 0
      const char* nb0 = nxt.valid ? bsrc(nxt, 0, 0) : bsrc(cur, KT - 1, 0);
      const char* nb1 = nxt.valid ? bsrc(nxt, 0, 1) : bsrc(cur, KT - 1, 1);
      const int o1 = nxt.valid ? 128 : 0;                             // ... its step 1
      const char* nc0 = nxt.valid ? bsrc(nxt, 1, 0) : nb0;
      const char* nc1 = nxt.valid ? bsrc(nxt, 1, 1) : nb1;
      PP(0, 0, a_off[3], cur.abase + last, b_off[3], bsrc(cur, KT - 1, 1));
      if (nxt.valid) {
#pragma unroll
        for (int i = 0; i < 3; ++i) a_off[i] = token_off(nxt.rows, i);
      }
      PP(0, 1, a_off[0], na, b_off[0], nb0);
      PP(0, 2, a_off[1], na, b_off[1], nb0);
      PP(0, 3, a_off[2], na, b_off[2], nb1);
      if (nxt.valid) a_off[3] = token_off(nxt.rows, 3);
      PP(1, 0, a_off[3], na, b_off[3], nb1);
      PP(1, 1, a_off[0], na + o1, b_off[0], nc0);
      PP(1, 2, a_off[1], na + o1, b_off[1], nc0);
      PP(1, 3, a_off[2], na + o1, b_off[2], nc1);
#undef PP
    }
    epilogue(cur);
    if (!nxt.valid) break;
    cur = nxt;
  }
  if (wm == 0) asm volatile("s_barrier" ::: "memory");  // as many barriers as the other group
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // no copy in flight into LDS at exit
}

// Sums the parts of every K-split tile of the down GEMM in a fixed order (part 0, 1, ...:
// deterministic) and stores the tile like the GEMM's own epilogue.  Eight blocks per split
// tile, one per accumulator (j, i) of the GEMM's wavefront tile; thread and accumulator
// indices mean what they mean in ffn_mfma_kernel.  All parts of a quad are loaded before
// they are added.
__global__ __launch_bounds__(NT) void ffn_split_reduce_kernel(const GemmArgs p) {
  const int n_tiles = p.sched->down_split_tiles;
  const int tile = blockIdx.x >> 3, ji = blockIdx.x & 7;
  if (tile >= n_tiles) return;
  const int split = p.sched->down_split;
  const TileDesc tl = p.order[p.sched->down_full + tile];
  const int j = ji >> 2, i = ji & 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int fr_row = lane & 31, fr_half = lane >> 5;
  const float4* ws = reinterpret_cast<const float4*>(p.split_ws) +
                     (size_t)tile * split * (32 * NT) + (size_t)(ji * 4) * NT + tid;
  const int m_local = wm * 128 + i * 32 + fr_row;
  const bool live = m_local < tl.rows;
  const size_t row = (size_t)(tl.row0 + m_local);
  const int col0 = tl.nblk * 256 + j * 128 + wn * 32 + 4 * fr_half;
  // every part of all four quads is requested before anything is added (up to 32 loads of
  // 16 bytes in flight per thread: with one quad at a time the kernel was bound by four
  // memory latencies in a row)
  float4 part[4][8];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int pt = 0; pt < 8; ++pt)
      part[q][pt] = pt < split ? ws[(size_t)pt * (32 * NT) + q * NT] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float4 v = part[q][0];
#pragma unroll
    for (int pt = 1; pt < 8; ++pt) {
      v.x += part[q][pt].x; v.y += part[q][pt].y; v.z += part[q][pt].z; v.w += part[q][pt].w;
    }
    if (live)
      *reinterpret_cast<uint2*>(p.C + row * p.N + col0 + 8 * q) =
          make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
  }
}

}  // namespace

// two-matrix expert: the first GEMM has 256-column blocks of one matrix
bool ffn_mfma_supported_2mat(const moe_ctx* c) {
  return c->cfg.dtype == MOE_BF16 && c->cfg.d % 256 == 0 && c->cfg.f % 256 == 0;
}

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

static int run_sched(moe_ctx* c, const int32_t* counts, const int32_t* offsets, int nt_a, int nt_b,
                     int kt_b, const void* const* up_b0, const void* const* up_b1,
                     const void* const* down_b0, const void* const* down_b1, hipStream_t s) {
  hipLaunchKernelGGL(mfma_sched_kernel, dim3(32), dim3(256), 0, s, counts, offsets,
                     c->d_wtab + 0 * MOE_MAX_EXPERTS, c->cfg.E, c->S_call, c->max_mtiles[1], nt_a,
                     nt_b, c->n_cu, kt_b, c->d_sched[1], up_b0, up_b1, down_b0, down_b1,
                     c->d_order_up, c->d_order_down);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

// One block per compute unit (a block takes all of a unit's LDS), a multiple of 8 so that
// every XCD gets the same number of blocks.
static int persistent_grid(const moe_ctx* c) { return std::max(8, (c->n_cu / 8) * 8); }

// Down-type GEMM (plain epilogue) with the K-split tail: the GEMM, then the sum of the parts.
static void launch_down(moe_ctx* c, GemmArgs& a, hipStream_t s) {
  a.split_ws = c->d_split_ws;
  hipLaunchKernelGGL((ffn_mfma_kernel<MODE_DOWN>), dim3(persistent_grid(c)), dim3(NT), 0, s, a);
  hipLaunchKernelGGL(ffn_split_reduce_kernel, dim3((c->n_cu / 2) * 8), dim3(NT), 0, s, a);
}

static GemmArgs tiled_args(moe_ctx* c, const void* A, int lda, const TileDesc* order, int nt,
                           int K, int N, void* C) {
  GemmArgs a{};
  a.A = (const uint16_t*)A;
  a.lda = lda;
  a.sched = c->d_sched[1];
  a.order = order;
  a.n_tiles_n = nt;
  a.K = K;
  a.N = N;
  a.C = (uint16_t*)C;
  return a;
}

int launch_ffn_mfma(moe_ctx* c, bool gated, const int32_t* counts, const int32_t* offsets,
                    const void* x_packed, void* y_packed, void* G, void* U, hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f;
  const int nt_up = gated ? f / 128 : f / 256, nt_down = d / 256;
  const void* const* W1 = c->d_wtab + 0 * MOE_MAX_EXPERTS;
  const void* const* W3 = c->d_wtab + 1 * MOE_MAX_EXPERTS;
  const void* const* W2 = c->d_wtab + 2 * MOE_MAX_EXPERTS;
  prof_mark(c, 0, s);
  int st = run_sched(c, counts, offsets, nt_up, nt_down, f / BK, W1, gated ? W3 : nullptr, W2,
                     nullptr, s);
  if (st != MOE_OK) return st;
  prof_mark(c, 1, s);
  GemmArgs up = tiled_args(c, x_packed, d, c->d_order_up, nt_up, d, f, c->d_H);
  up.Gs = (uint16_t*)G;
  up.Us = (uint16_t*)U;
  if (gated)
    hipLaunchKernelGGL((ffn_mfma_kernel<MODE_UP>), dim3(persistent_grid(c)), dim3(NT), 0, s, up);
  else
    hipLaunchKernelGGL((ffn_mfma_kernel<MODE_UP1>), dim3(persistent_grid(c)), dim3(NT), 0, s, up);
  prof_mark(c, 2, s);
  GemmArgs dn = tiled_args(c, c->d_H, f, c->d_order_down, nt_down, f, d, y_packed);
  launch_down(c, dn, s);
  prof_mark(c, 3, s);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

bool ffn_bwd_mfma_supported(const moe_ctx* c) {
  return ffn_mfma_supported(c) && c->cfg.f % 256 == 0;
}

// dy, xp: [S,d]; G, U: [S,f] (forward saves); dxp out.  Workspace (context): d_H [S,f],
// d_dGU [S,2f].  Two-matrix expert (!gated): no U, no W3: d_dGU holds dG [S,f], two weight
// gradients.  The weights are read as they are stored: W2 [d,f] is k-major for dH = dY W2,
// W1 and W3 [f,d] are k-major for dX = dG W1 + dU W3 (one GEMM over the concatenated k).
int launch_ffn_bwd_mfma(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* G,
                        const void* U, const int32_t* counts, const int32_t* offsets, void* dxp,
                        hipStream_t s) {
  const int d = c->cfg.d, f = c->cfg.f;
  const void* const* W1 = c->d_wtab + 0 * MOE_MAX_EXPERTS;
  const void* const* W3 = c->d_wtab + 1 * MOE_MAX_EXPERTS;
  const void* const* W2 = c->d_wtab + 2 * MOE_MAX_EXPERTS;
  const int nt_f = f / 256, nt_d = d / 256;
  const int gw = gated ? 2 * f : f;   // elements per row of [dG|dU]
  int st = run_sched(c, counts, offsets, nt_f, nt_d, gw / BK, W2, nullptr, W1,
                     gated ? W3 : nullptr, s);
  if (st != MOE_OK) return st;
  // dH = dY W2 with the activation's derivative in the epilogue -> [dG|dU], H
  GemmArgs dh = tiled_args(c, dy, d, c->d_order_up, nt_f, d, f, c->d_dGU);
  dh.C2 = (uint16_t*)c->d_H;
  dh.Gs = (uint16_t*)const_cast<void*>(G);
  dh.Us = (uint16_t*)const_cast<void*>(U);
  dh.ldb = f;
  dh.kseg = d / BK;
  if (gated)
    hipLaunchKernelGGL((ffn_mfma_kernel<MODE_DH, true>), dim3(persistent_grid(c)), dim3(NT), 0, s, dh);
  else
    hipLaunchKernelGGL((ffn_mfma_kernel<MODE_DH1, true>), dim3(persistent_grid(c)), dim3(NT), 0, s, dh);
  // weight gradients straight from dY, X, H and [dG|dU] (transpose reads from LDS), right
  // after the kernel that wrote H and [dG|dU]; dX last, so that the caller's next kernel
  // (the backward of dispatch) finds it in the last-level cache
  st = launch_wgrad_tr(c, gated, dy, xp, c->d_H, c->d_dGU, counts, offsets, s);
  if (st != MOE_OK) return st;
  // dX = [dG|dU] [W1; W3]  (one GEMM with contraction length 2f; f without U)
  GemmArgs dx = tiled_args(c, c->d_dGU, gw, c->d_order_down, nt_d, gw, d, dxp);
  dx.ldb = d;
  dx.kseg = f / BK;
  dx.split_ws = c->d_split_ws;
  hipLaunchKernelGGL((ffn_mfma_kernel<MODE_DOWN, true>), dim3(persistent_grid(c)), dim3(NT), 0, s, dx);
  hipLaunchKernelGGL(ffn_split_reduce_kernel, dim3((c->n_cu / 2) * 8), dim3(NT), 0, s, dx);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
