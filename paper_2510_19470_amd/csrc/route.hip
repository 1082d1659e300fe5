// Gating: gate projection, top-k selection and gate weights (paper Sec. 2.1: the gate
// network is the router that picks the activated experts of every token).
//
// Selection: one token is handled by a group of W lanes of a 64-wide wavefront (W = power
// of two, >= min(E,64)), so that small expert counts pack several tokens into one
// wavefront.  Each lane keeps ceil(E/W) logits in registers.  The k winners are found by k
// rounds of "local best, then butterfly arg-max across the group" on 64-bit keys (logit,
// id); the order relation is total on finite floats: larger logit first, equal logits by
// lower expert id.  The same
// device function serves moe_route_logits (logits in global memory) and the fused
// moe_route kernel (logits in LDS), so both select identically from identical logits.
#include "moe_internal.h"

namespace {

// A logit and its expert id as one 64-bit key whose unsigned order is the selection order:
// high word = the float's bits mapped monotonically to unsigned (-0 is folded into +0 first,
// the two compare equal), low word = INT_MAX - id, so that of two equal logits the lower id
// has the larger key.  0 = no candidate (smaller than every key of a finite logit).
typedef unsigned long long key_t;

__device__ __forceinline__ key_t make_key(float v, int id) {
  const uint32_t u = __float_as_uint(v + 0.f);
  const uint32_t ord = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((key_t)ord << 32) | (uint32_t)(0x7fffffff - id);
}
__device__ __forceinline__ float key_value(key_t k) {
  const uint32_t ord = (uint32_t)(k >> 32);
  return __uint_as_float((ord & 0x80000000u) ? (ord ^ 0x80000000u) : ~ord);
}
__device__ __forceinline__ int key_id(key_t k) { return 0x7fffffff - (int)(uint32_t)k; }

// Exchange inside a group of W lanes for a reduction whose operator is commutative and
// associative on the values at hand (max of keys; the sum's rounding is the same on every
// lane of a pair, since both add the same two numbers).  Levels 1, 2 swap inside quads, level
// 4 mirrors 8 lanes and level 8 mirrors 16 (after the lower levels every lane of a half holds
// the half's result, so any lane of the other half will do): data-parallel-primitive moves
// instead of LDS permutes; above that, LDS permutes.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
template <int OFF>
__device__ __forceinline__ uint32_t partner32(uint32_t x) {
  if (OFF == 1) return dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
  if (OFF == 2) return dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
  if (OFF == 4) return dpp_mov<0x141>(x);   // row_half_mirror
  if (OFF == 8) return dpp_mov<0x140>(x);   // row_mirror
  return (uint32_t)__shfl_xor((int)x, OFF, 64);
}
template <int OFF>
__device__ __forceinline__ key_t partner(key_t k) {
  return ((key_t)partner32<OFF>((uint32_t)(k >> 32)) << 32) | partner32<OFF>((uint32_t)k);
}
template <int W, int OFF = 1>
__device__ __forceinline__ key_t group_max(key_t best) {
  if constexpr (OFF < W) {
    const key_t o = partner<OFF>(best);
    return group_max<W, OFF * 2>(o > best ? o : best);
  } else {
    return best;
  }
}
template <int W, int OFF = 1>
__device__ __forceinline__ float group_sum(float x) {
  if constexpr (OFF < W) {
    return group_sum<W, OFF * 2>(x + __uint_as_float(partner32<OFF>(__float_as_uint(x))));
  } else {
    return x;
  }
}

// Selection and weights of token t, done by the W lanes [sub*W, sub*W+W) of the wavefront.
// `row` points at the token's E logits (global memory or LDS); every lane of the wavefront
// must call this together (dead groups pass live = false).  Round j finds the largest key
// left (local scan, then a butterfly over the group); the winner is kept by lane j mod W of
// the group (slot j / W), which later computes and writes that slot's weight.
// lds_ids (optional): the token's k ids are also stored there (the fused kernel ranks them).
template <int W, int VPL>
__device__ __forceinline__ void select_token(const float* row, bool live, int t, int E, int k,
                                             int renormalize, int32_t* __restrict__ topk_idx,
                                             float* __restrict__ topk_w,
                                             int32_t* lds_ids = nullptr) {
  const int lane = threadIdx.x & 63;
  const int gl = lane % W;   // lane inside the group
  constexpr int SLOTS = (MOE_MAX_TOPK + W - 1) / W;

  float v[VPL];
  key_t key[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) {
    const int e = gl + i * W;
    const bool ok = live && e < E;
    v[i] = ok ? row[e] : 0.f;
    key[i] = ok ? make_key(v[i], e) : 0;
  }

  key_t mine[SLOTS];
#pragma unroll
  for (int q = 0; q < SLOTS; ++q) mine[q] = 0;
  key_t first = 0;   // the winner of round 0: the largest logit

#pragma unroll 1
  for (int j = 0; j < k; ++j) {
    key_t best = 0;
#pragma unroll
    for (int i = 0; i < VPL; ++i) best = key[i] > best ? key[i] : best;
    best = group_max<W>(best);
#pragma unroll
    for (int i = 0; i < VPL; ++i) key[i] = key[i] == best ? 0 : key[i];
    if (j == 0) first = best;
#pragma unroll
    for (int q = 0; q < SLOTS; ++q)
      if (j == q * W + gl) mine[q] = best;
  }

  // weights: exp(l - max) over the selection, normalised over the selection or over all E
  const float m = key_value(first);
  float part = 0.f;
  if (renormalize) {
#pragma unroll
    for (int q = 0; q < SLOTS; ++q)
      if (q * W + gl < k) part += expf(key_value(mine[q]) - m);
  } else {
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int e = gl + i * W;
      if (live && e < E) part += expf(v[i] - m);
    }
  }
  part = group_sum<W>(part);
  const float inv = 1.f / part;
  if (live) {
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
      const int j = q * W + gl;
      if (j < k) {
        const int id = mine[q] == 0 ? 0 : key_id(mine[q]);
        topk_idx[(size_t)t * k + j] = id;
        topk_w[(size_t)t * k + j] = expf(key_value(mine[q]) - m) * inv;
        if (lds_ids != nullptr) lds_ids[j] = id;
      }
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
// One block = 32 tokens.  Its 8 wavefronts split d into eighths; each accumulates
// logits[32 tokens][16*NEB experts] with MFMA 16x16x32 (gate rows are the "A" operand, token
// rows the "B" operand, both read straight from global memory with the same k-to-lane
// assignment: lane (n = lane & 15, q = lane >> 4) fetches the 16 bytes at k = 32*ks + 8*q of
// row n, so one load instruction covers 16 rows x 64 contiguous bytes).  A gate fragment is
// used for both token groups of the wavefront; the gate matrix is re-read once per 32
// tokens (from L2).  The partial sums meet in LDS, the bias is added, the logits are
// written out when the caller wants them, and the block selects the top-k of its 32 tokens
// from LDS.  The token rows are read exactly once: the kernel is bound by HBM.
// HIST: the block also does the counting step of the dispatch for its 32 * k slots, which it
// holds anyway: the stable rank of every slot among the block's slots of the same expert
// (ballots inside a wavefront, an LDS table across the 8 wavefronts), the block's expert
// histogram, and that histogram added (integer atomics: order-independent) to the sums of
// the block's super-block of 16 and to the grand totals; the blocks also clear the other
// buffer for the next call: all of its super-block rows that the host knows may be non-zero
// (clear_rows, dealt over the blocks), block 0 its totals.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
constexpr int GATE_TOK = GATE_BLOCK_TOKENS;    // tokens per block
constexpr int GATE_WAVES = 8;   // wavefronts per block, each with an eighth of d
constexpr int GATE_TB = GATE_TOK / 16;

// STAGED (d a multiple of 512, E <= 16 * NEB): the token rows do not go from global memory to
// the MFMA operand registers directly (16 rows x 64 bytes per load instruction) but through
// LDS, copied there asynchronously in full-row pieces: a stage is the block's 32 rows x 256
// elements (512 contiguous bytes per row, one copy instruction = 2 rows), four stages of which
// three are in flight, 16-byte chunks XOR-swizzled by the row so that the fragment reads of 16
// rows fall on distinct banks.  Wavefront w multiplies k-slice w (32 elements) of every stage;
// the gate rows still come straight from global memory (L2), two stages ahead, in registers.
// Their loads are issued by hand as well (gate_load16): a load that the compiler tracks makes
// it wait for "all but the NEB newest memory operations" before the first MFMA, and since it
// does not count the copies, that wait would also cover the copies of the stages ahead.
constexpr int GATE_STAGE_K = 256;                      // elements of a row per stage
constexpr int GATE_STAGE_BYTES = GATE_TOK * GATE_STAGE_K * 2;
constexpr int GATE_STAGES = 4;

// s_waitcnt vmcnt(N) followed by a barrier, N a compile-time constant
template <int N>
__device__ __forceinline__ void gate_wait_barrier() {
  static_assert(N >= 0 && N <= 8, "wait counts of the staged gate loop");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 3) asm volatile("s_waitcnt vmcnt(3)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 5) asm volatile("s_waitcnt vmcnt(5)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 6) asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 7) asm volatile("s_waitcnt vmcnt(7)\n\ts_barrier" ::: "memory");
  else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
  else static_assert(N == 0, "unused wait count");
}

// 16 bytes per lane global -> registers, outside the compiler's bookkeeping of outstanding
// loads: the value is valid only behind a gate_wait_barrier that covers it and the
// gate_arrived() that follows.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t gate_load16(const void* src) {
  u32x4_t r;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(src) : "memory");
  return r;
}
// Ties a register filled by gate_load16 to this point of the program: no use of it can be
// scheduled above the wait that precedes.
__device__ __forceinline__ void gate_arrived(u32x4_t& r) { asm volatile("" : "+v"(r)); }

// 16 bytes per lane global -> LDS; the wavefront's 1 KB lands at lds_addr (wave-uniform, via
// M0) + lane * 16.
__device__ __forceinline__ void gate_dma16(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr)
               : "memory", "m0");
}

template <int W, int VPL, int NEB, bool HIST, bool STAGED>
__global__ __launch_bounds__(64 * GATE_WAVES) void gate_route_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ Wg,
    const float* __restrict__ bias, int T, int E, int d, int k, int renormalize,
    float* __restrict__ logits_out, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int ebits, int32_t* __restrict__ rt_rank, int32_t* __restrict__ rt_hist,
    int32_t* __restrict__ super_acc, int32_t* __restrict__ super_clear, int tot_off,
    int clear_rows) {
  constexpr int EG = 16 * NEB;                     // experts per pass over the token rows
  constexpr int EP = W * VPL < 64 ? 64 : W * VPL;  // expert slots kept in LDS
  // the partial sums [wavefront][token][expert]; the stages of the token rows use the same LDS
  // before them
  constexpr int PART_BYTES = GATE_WAVES * GATE_TOK * (EG + 1) * 4;
  constexpr int SMEM_BYTES = STAGED && GATE_STAGES * GATE_STAGE_BYTES > PART_BYTES
                                 ? GATE_STAGES * GATE_STAGE_BYTES : PART_BYTES;
  __shared__ __align__(16) char smem[SMEM_BYTES];
  float (*part)[GATE_TOK][EG + 1] = reinterpret_cast<float (*)[GATE_TOK][EG + 1]>(smem);
  __shared__ float fin[GATE_TOK][EP + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int t0 = blockIdx.x * GATE_TOK;
  const int kq = d / GATE_WAVES;  // k range of this wavefront
  const uint4* xp[GATE_TB];
#pragma unroll
  for (int tb = 0; tb < GATE_TB; ++tb)
    xp[tb] = reinterpret_cast<const uint4*>(x + (size_t)min(t0 + 16 * tb + n, T - 1) * d +
                                            wave * kq + q * 8);
  for (int e0 = 0; e0 < E; e0 += EG) {
    const uint4* wp[NEB];
#pragma unroll
    for (int eb = 0; eb < NEB; ++eb)
      wp[eb] = reinterpret_cast<const uint4*>(Wg + (size_t)min(e0 + 16 * eb + n, E - 1) * d +
                                              (STAGED ? wave * 32 : wave * kq) + q * 8);
    f32x4_t acc[NEB][GATE_TB];
#pragma unroll
    for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
      for (int tb = 0; tb < GATE_TB; ++tb) acc[eb][tb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if constexpr (STAGED) {
      const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
      const int nit = d / GATE_STAGE_K;   // even: d is a multiple of 512
      // copies: instruction c (0..15) of a stage fills rows 2c, 2c+1 (lane >> 5), 32 chunk slots
      // each; slot s of row r holds global chunk s ^ (r & 15).  This wavefront issues c = wave
      // and c = wave + 8.
      const char* src[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int r = 2 * (wave + 8 * u) + (lane >> 5);
        src[u] = reinterpret_cast<const char*>(x + (size_t)min(t0 + r, T - 1) * d) +
                 (((lane & 31) ^ (r & 15)) << 4);
      }
      auto copy = [&](int it) {
        const uint32_t sb = lds0 + (uint32_t)(it % GATE_STAGES) * GATE_STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < 2; ++u)
          gate_dma16(src[u] + (size_t)it * (GATE_STAGE_K * 2),
                     __builtin_amdgcn_readfirstlane(sb + (wave + 8 * u) * 1024));
      };
      // fragment of token block tb, k-slice `wave` of the stage: row 16 tb + n, chunk 4 wave + q
      int frag[GATE_TB];
#pragma unroll
      for (int tb = 0; tb < GATE_TB; ++tb)
        frag[tb] = (16 * tb + n) * (GATE_STAGE_K * 2) + (((4 * wave + q) ^ n) << 4);
      u32x4_t wq[2][NEB];
      auto gate_rows = [&](int buf, int it) {
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb) wq[buf][eb] = gate_load16(wp[eb] + it * (GATE_STAGE_K / 8));
      };
      auto mac = [&](int buf, int it) {
        const char* st = smem + (it % GATE_STAGES) * GATE_STAGE_BYTES;
        uint4 xv[GATE_TB];
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb) gate_arrived(wq[buf][eb]);
#pragma unroll
        for (int tb = 0; tb < GATE_TB; ++tb) xv[tb] = *reinterpret_cast<const uint4*>(st + frag[tb]);
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int tb = 0; tb < GATE_TB; ++tb)
            acc[eb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8_t, wq[buf][eb]), __builtin_bit_cast(bf16x8_t, xv[tb]),
                acc[eb][tb], 0, 0, 0);
      };
      // Iteration j issues the gate rows of stage j + 2 (NEB loads) and then the copies of stage
      // j + 3 (2 instructions); the prologue does the same for j = -3, -2, -1 (no gate rows for
      // j = -3).  Memory operations complete in issue order and nothing else is outstanding in
      // this loop, so at the top of iteration `it` "at most NEB + 4 outstanding" (the copies of
      // it + 1, the gate rows of it + 1, the copies of it + 2) means that the gate rows and the
      // copies of stage `it` have arrived; the barrier extends that to the copies of the other
      // wavefronts and says that everybody is done with stage it - 1, which the copies of it + 3
      // refill.  The last two iterations have fewer operations behind them.  nit >= 4 and even
      // (the launcher checks d).
      copy(0);
      gate_rows(0, 0);
      copy(1);
      gate_rows(1, 1);
      copy(2);
      for (int it = 0; it < nit - 2; it += 2) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          gate_wait_barrier<NEB + 4>();
          mac(b, it + b);
          gate_rows(b, it + b + 2);
          if (it + b + 3 < nit) copy(it + b + 3);
        }
      }
      gate_wait_barrier<NEB + 2>();   // behind stage nit - 2: the copies and gate rows of nit - 1
      mac(0, nit - 2);
      gate_wait_barrier<0>();
      mac(1, nit - 1);
      __syncthreads();   // every fragment read is done before the partial sums overwrite the stages
    } else {
#pragma unroll 4
    for (int ks = 0; ks < kq / 32; ++ks) {   // a k-slice of 32 = 4 chunks of 16 bytes per row
      uint4 xv[GATE_TB], wv[NEB];
#pragma unroll
      for (int tb = 0; tb < GATE_TB; ++tb) xv[tb] = xp[tb][ks * 4];
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb) wv[eb] = wp[eb][ks * 4];
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
        for (int tb = 0; tb < GATE_TB; ++tb)
          acc[eb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8_t, wv[eb]), __builtin_bit_cast(bf16x8_t, xv[tb]),
              acc[eb][tb], 0, 0, 0);
    }
    }
    // the lane holds token 16*tb + n and experts 16*eb + 4*q + i of this group
#pragma unroll
    for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
      for (int tb = 0; tb < GATE_TB; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wave][16 * tb + n][16 * eb + 4 * q + i] = acc[eb][tb][i];
    __syncthreads();
    for (int idx = tid; idx < GATE_TOK * EG; idx += 64 * GATE_WAVES) {
      const int tok = idx / EG, el = idx % EG, e = e0 + el;
      if (e < E) {
        float v = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < GATE_WAVES; ++w8) v += part[w8][tok][el];   // fixed order
        if (bias != nullptr) v += bias[e];
        fin[tok][e] = v;
        if (logits_out != nullptr && t0 + tok < T) logits_out[(size_t)(t0 + tok) * E + e] = v;
      }
    }
    __syncthreads();
  }
  // the partial sums are not needed any more (the barrier that ends the loop above): their
  // LDS holds the block's selected ids [32][k] and the per-wavefront expert counts [8][256]
  int32_t* ids = reinterpret_cast<int32_t*>(smem);
  int32_t* wcnt = ids + GATE_TOK * MOE_MAX_TOPK;
  static_assert(PART_BYTES >= (int)sizeof(int32_t) * (GATE_TOK * MOE_MAX_TOPK + GATE_WAVES * MOE_MAX_EXPERTS),
                "the ids and counts of the ranking step live in the partial sums' LDS");
  if (HIST) {
    for (int i = tid; i < GATE_TOK * MOE_MAX_TOPK; i += 64 * GATE_WAVES) ids[i] = -1;
    for (int i = tid; i < GATE_WAVES * MOE_MAX_EXPERTS; i += 64 * GATE_WAVES) wcnt[i] = 0;
    __syncthreads();
  }
  constexpr int TOK_PER_WAVE = 64 / W;
  for (int base = 0; base < GATE_TOK; base += GATE_WAVES * TOK_PER_WAVE) {
    const int tok = base + wave * TOK_PER_WAVE + lane / W;
    const bool live = tok < GATE_TOK && t0 + tok < T;
    select_token<W, VPL>(&fin[live ? tok : 0][0], live, t0 + tok, E, k, renormalize, topk_idx,
                         topk_w, HIST ? ids + (live ? tok : 0) * k : nullptr);
  }
  if (HIST) {
    __syncthreads();
    // slot s = tok * k + j of the block, one per thread (32 * k <= 512)
    const int s = tid;
    const int e = s < GATE_TOK * k ? ids[s] : -1;   // -1: no slot, or a token past T
    const unsigned long long same = match_same(e, ebits);
    const int in_wave = __popcll(same & ((1ull << lane) - 1ull));
    if (e >= 0 && in_wave == 0) wcnt[wave * MOE_MAX_EXPERTS + e] = __popcll(same);
    __syncthreads();
    if (e >= 0) {
      int rank = in_wave;
      for (int w8 = 0; w8 < wave; ++w8) rank += wcnt[w8 * MOE_MAX_EXPERTS + e];
      rt_rank[(size_t)blockIdx.x * (GATE_TOK * k) + s] = rank;
    }
    if (tid < E) {
      int n = 0;
#pragma unroll
      for (int w8 = 0; w8 < GATE_WAVES; ++w8) n += wcnt[w8 * MOE_MAX_EXPERTS + tid];
      rt_hist[(size_t)blockIdx.x * E + tid] = n;
      const size_t sup = (size_t)(blockIdx.x / RT_SUPER) * E + tid;
      // grand totals: after the super-block rows, one 128-byte line per expert so that the
      // atomics of all blocks spread over the memory channels
      const size_t tot = (size_t)tot_off + (size_t)tid * RT_TOT_STRIDE;
      if (n != 0) {
        atomicAdd(&super_acc[sup], n);
        atomicAdd(&super_acc[tot], n);
      }
      // the other buffer, for the next call: every super-block row that may hold sums (the
      // call that filled it may have had more tokens than this one), dealt over the blocks
      for (int r = blockIdx.x; r < clear_rows; r += gridDim.x) super_clear[(size_t)r * E + tid] = 0;
      if (blockIdx.x == 0) super_clear[tot] = 0;
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

template <int W, int VPL, int NEB>
int launch_gate(const moe_ctx* c, const void* x, const void* Wg, const float* bias, int T,
                float* logits, int32_t* idx, float* w, bool keep_hist, hipStream_t s) {
  const int grid = (T + GATE_TOK - 1) / GATE_TOK;
  // token rows through LDS when a stage divides the row and one pass covers all experts
  if (c->cfg.d % (2 * GATE_STAGE_K) == 0 && c->cfg.d >= 4 * GATE_STAGE_K && c->cfg.E <= 16 * NEB) {
    int ebits = 0;
    while ((1 << ebits) < c->cfg.E) ++ebits;
    const size_t half = (size_t)c->rt_super_max * c->cfg.E + (size_t)c->cfg.E * RT_TOT_STRIDE;
    if (keep_hist)
      hipLaunchKernelGGL((gate_route_mfma_kernel<W, VPL, NEB, true, true>), dim3(grid),
                         dim3(64 * GATE_WAVES), 0, s, (const uint16_t*)x, (const uint16_t*)Wg, bias,
                         T, c->cfg.E, c->cfg.d, c->cfg.k, c->cfg.renormalize, logits, idx, w, ebits,
                         c->d_rt_rank, c->d_rt_hist, c->d_rt_super + (size_t)c->rt_parity * half,
                         c->d_rt_super + (size_t)(c->rt_parity ^ 1) * half,
                         c->rt_super_max * c->cfg.E, c->rt_dirty[c->rt_parity ^ 1]);
    else
      hipLaunchKernelGGL((gate_route_mfma_kernel<W, VPL, NEB, false, true>), dim3(grid),
                         dim3(64 * GATE_WAVES), 0, s, (const uint16_t*)x, (const uint16_t*)Wg, bias,
                         T, c->cfg.E, c->cfg.d, c->cfg.k, c->cfg.renormalize, logits, idx, w, 0,
                         nullptr, nullptr, nullptr, nullptr, 0, 0);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
  }
  if (keep_hist) {
    int ebits = 0;
    while ((1 << ebits) < c->cfg.E) ++ebits;
    const size_t half = (size_t)c->rt_super_max * c->cfg.E + (size_t)c->cfg.E * RT_TOT_STRIDE;
    hipLaunchKernelGGL((gate_route_mfma_kernel<W, VPL, NEB, true, false>), dim3(grid),
                       dim3(64 * GATE_WAVES), 0, s, (const uint16_t*)x, (const uint16_t*)Wg, bias, T,
                       c->cfg.E, c->cfg.d, c->cfg.k, c->cfg.renormalize, logits, idx, w, ebits,
                       c->d_rt_rank, c->d_rt_hist, c->d_rt_super + (size_t)c->rt_parity * half,
                       c->d_rt_super + (size_t)(c->rt_parity ^ 1) * half,
                       c->rt_super_max * c->cfg.E, c->rt_dirty[c->rt_parity ^ 1]);
  } else {
    hipLaunchKernelGGL((gate_route_mfma_kernel<W, VPL, NEB, false, false>), dim3(grid),
                       dim3(64 * GATE_WAVES), 0, s, (const uint16_t*)x, (const uint16_t*)Wg, bias, T,
                       c->cfg.E, c->cfg.d, c->cfg.k, c->cfg.renormalize, logits, idx, w, 0, nullptr,
                       nullptr, nullptr, nullptr, 0, 0);
  }
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
                            int T, float* logits, int32_t* idx, float* w, bool keep_hist,
                            hipStream_t s) {
  if (T == 0) return MOE_OK;
  const int E = c->cfg.E;
  // a group of 8 lanes per token (8 tokens per wavefront) up to 64 experts: the selection
  // costs (experts per lane + 3 butterfly levels) per round instead of 6 butterfly levels,
  // and the block's 32 tokens are selected in one pass by four wavefronts
#define GATE(W_, VPL_, NEB_) launch_gate<W_, VPL_, NEB_>(c, x, Wg, bias, T, logits, idx, w, keep_hist, s)
  if (E <= 2) return GATE(2, 1, 1);
  if (E <= 4) return GATE(4, 1, 1);
  if (E <= 8) return GATE(8, 1, 1);
  if (E <= 16) return GATE(8, 2, 1);
  if (E <= 32) return GATE(8, 4, 2);
  if (E <= 48) return GATE(8, 6, 3);
  if (E <= 64) return GATE(8, 8, 4);
  if (E <= 128) return GATE(64, 2, 4);
  if (E <= 256) return GATE(64, 4, 4);
#undef GATE
  return MOE_EUNSUPPORTED;
}
