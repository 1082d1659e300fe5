// Dispatch: counts, (dest_rank, expert)-ordered offsets, the stable slot->row permutation
// and the row copy into the packed buffer (paper Sec. 2.1: data is rearranged to the
// activated experts; Sec. 3.2: one contiguous chunk per peer, and the chunk of an expert
// that was fetched by all-gather stays local).
//
// Two launches, no host synchronisation, no waiting between blocks:
//   1. dispatch_count: every chunk of 1024 slots ranks its slots per expert (one ballot per
//      bit of the expert id gives the lanes with the same expert, popcount below the lane
//      gives the rank inside the wavefront; LDS prefix over the 16 wavefronts), stores the
//      in-chunk rank of each slot and the chunk's expert histogram, and adds the histogram
//      to the per-expert totals with integer atomics (their order cannot change the sums).
//   2. dispatch_scatter: every block first turns the totals into expert offsets (scan in
//      segment order, in LDS); one wavefront per token then sums the histograms of the
//      chunks before its own (the prefix that makes the ranking stable across chunks),
//      forms the final rows, writes both maps, reads the token row once (16 B per lane)
//      and writes it to its k packed rows.  Block 0 also writes counts / offsets / rank
//      chunks.
// The permutation is deterministic: no atomic decides a row number.
// The totals are double-buffered: call n accumulates into buffer n&1 and clears the other
// one for call n+1.  The call number lives on the device, in two words so that no block reads
// a word that another block of the same launch writes: the count kernel reads ctr[0] and
// writes ctr[1] = ctr[0] + 1, the scatter kernel reads ctr[1] and writes ctr[0] = ctr[1].
// Nothing on the host changes from call to call, so a captured graph of the two launches can
// be replayed.  (A ticket per scatter block with the last block clearing the totals doubled
// the kernel's time: 4096 returning atomics on one address.)
#include <mutex>

#include "moe_internal.h"

namespace {

constexpr int COUNT_THREADS = DISPATCH_CHUNK;  // one slot per thread, 16 wavefronts
constexpr int COUNT_WAVES = COUNT_THREADS / 64;

__global__ __launch_bounds__(COUNT_THREADS) void dispatch_count_kernel(
    const int32_t* __restrict__ topk_idx, int S, int E, int ebits,
    int32_t* __restrict__ chunk_hist, int32_t* __restrict__ totals2,
    int32_t* __restrict__ slot_rank) {
  __shared__ int32_t wcnt[COUNT_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int s = b * DISPATCH_CHUNK + tid;
  int e = -1;
  if (s < S) {
    e = topk_idx[s];
    if ((unsigned)e >= (unsigned)E) e = -1;
  }
  for (int i = tid; i < COUNT_WAVES * MOE_MAX_EXPERTS; i += COUNT_THREADS) (&wcnt[0][0])[i] = 0;
  int32_t* ctr = totals2 + 2 * MOE_MAX_EXPERTS;
  const int call = ctr[0];
  int32_t* totals = totals2 + (call & 1) * MOE_MAX_EXPERTS;
  if (b == 0) {
    if (tid < MOE_MAX_EXPERTS) totals2[((call + 1) & 1) * MOE_MAX_EXPERTS + tid] = 0;
    if (tid == 0) ctr[1] = call + 1;
  }
  __syncthreads();
  const unsigned long long same = match_same(e, ebits);
  const int in_wave = __popcll(same & ((1ull << lane) - 1ull));
  if (e >= 0 && in_wave == 0) wcnt[wave][e] = __popcll(same);  // the lowest lane of each value
  __syncthreads();
  if (s < S) {
    int rank = -1;
    if (e >= 0) {
      rank = in_wave;
      for (int w = 0; w < wave; ++w) rank += wcnt[w][e];
    }
    slot_rank[s] = rank;  // rank of the slot among its expert's slots of this chunk
  }
  if (tid < E) {
    int n = 0;
#pragma unroll
    for (int w = 0; w < COUNT_WAVES; ++w) n += wcnt[w][tid];
    chunk_hist[(size_t)b * E + tid] = n;
    if (n != 0) atomicAdd(&totals[tid], n);
  }
}

// S == 0: no chunk exists, still the outputs must be defined.
__global__ void dispatch_empty_kernel(int E, int R, int32_t* expert_counts, int32_t* expert_offsets,
                                      int32_t* rank_counts, int32_t* rank_offsets) {
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    expert_counts[e] = 0;
    expert_offsets[e] = 0;
  }
  for (int r = threadIdx.x; r <= R; r += blockDim.x) {
    if (r < R) rank_counts[r] = 0;
    rank_offsets[r] = 0;
  }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Barrier that orders LDS traffic only: __syncthreads() would also wait for the global loads
// in flight (the token row fetched ahead of the preamble).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

constexpr int SCATTER_PF = 8;   // 16-byte pieces of its token row a lane fetches up front

// One wavefront per token: final rows of its k slots, both maps, and the row copy.
// slot_to_row holds the in-chunk ranks on entry and the final rows on exit.
// STREAM (packed buffer larger than the last-level cache): the wavefront requests the first
// SCATTER_PF * 1 KB of its token row before anything else, computes the row numbers while
// those loads are in flight, and writes the packed rows with non-temporal stores, one burst
// of writes that bypasses the cache; measured 104 -> 89 us on a 403 MB packed buffer, but
// 42 -> 58 us on one of 134 MB, which the cache absorbs when it is written normally.
// ROUTED: the counting was done by the fused gate kernel of moe_route.  chunk_hist is then the
// histogram of every gate block of 32 tokens, totals2 the sums of every super-block of 16 gate
// blocks, rt_tot the grand totals (one 128-byte line per expert: the gate blocks add to them
// with atomics), slot_rank the rank of a slot inside its gate block.  A slot's row = its expert's offset + the slots of that expert in the super-blocks
// before its own + those in the gate blocks before its own inside its super-block + its rank.
template <int K_MAX, bool STREAM, bool ROUTED>
__global__ __launch_bounds__(256) void dispatch_scatter_kernel(
    const u32x4* __restrict__ x, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ chunk_hist, int32_t* __restrict__ totals2,
    const int32_t* __restrict__ seg_pos, const int32_t* __restrict__ dest_rank, int T, int k,
    int E, int R, int row_vec, int32_t* __restrict__ slot_to_row,
    int32_t* __restrict__ row_to_slot, u32x4* __restrict__ x_packed,
    int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ rank_counts, int32_t* __restrict__ rank_offsets,
    const int32_t* __restrict__ slot_rank, const int32_t* __restrict__ rt_tot) {
  __shared__ int32_t scan[MOE_MAX_EXPERTS + 1];   // by position in segment order
  __shared__ int32_t offs[MOE_MAX_EXPERTS];       // expert id -> first row of its segment
  __shared__ int32_t rcnt[MOE_MAX_RANKS + 1];
  const int tid = threadIdx.x, lane = tid & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + tid) >> 6);   // wave-uniform
  const bool live = t < T;
  // ---- small loads nothing else depends on, then the token row
  int32_t* ctr = totals2 + 2 * MOE_MAX_EXPERTS;
  const int call = ROUTED ? 0 : ctr[1] - 1;   // the number the count kernel of this call saw
  int pos = 0;
  if (tid < E) pos = seg_pos[tid];
  int e = -1, rk = -1;
  if (live && lane < k) {
    e = topk_idx[t * k + lane];
    rk = ROUTED ? slot_rank[t * k + lane] : slot_to_row[t * k + lane];
  }
  const u32x4* src = x + (size_t)(live ? t : 0) * row_vec;
  u32x4 pre[SCATTER_PF];
#pragma unroll
  for (int u = 0; u < SCATTER_PF; ++u) {
    pre[u] = u32x4{0, 0, 0, 0};
    if (STREAM && live && lane + 64 * u < row_vec)
      pre[u] = __builtin_nontemporal_load(src + lane + 64 * u);
  }
  int mine = 0;
  if (ROUTED) {
    if (tid < E) mine = rt_tot[tid * RT_TOT_STRIDE];
  } else {
    if (tid < E) mine = totals2[(call & 1) * MOE_MAX_EXPERTS + tid];
    if (blockIdx.x == 0 && tid == 0) ctr[0] = call + 1;
  }
  // ---- expert offsets: inclusive scan of the totals taken in segment order
  if (tid < E) scan[pos + 1] = mine;
  if (tid == 0) scan[0] = 0;
  if (blockIdx.x == 0)
    for (int r = tid; r <= R; r += 256) rcnt[r] = 0;
  lds_barrier();
  for (int off = 1; off < E; off <<= 1) {
    int v = 0;
    if (tid >= off && tid < E) v = scan[tid + 1 - off];
    lds_barrier();
    if (tid >= off && tid < E) scan[tid + 1] += v;
    lds_barrier();
  }
  if (tid < E) offs[tid] = scan[pos];
  if (blockIdx.x == 0) {  // the integer outputs of the call
    if (tid < E) {
      expert_offsets[tid] = scan[pos];
      expert_counts[tid] = mine;
      atomicAdd(&rcnt[dest_rank[tid] + 1], mine);  // integer adds: order does not matter
    }
    lds_barrier();
    if (tid == 0) {
      int acc = 0;
      for (int r = 0; r < R; ++r) {
        rank_counts[r] = rcnt[r + 1];
        rank_offsets[r] = acc;
        acc += rcnt[r + 1];
      }
      rank_offsets[R] = acc;
    }
  }
  lds_barrier();
  if (!live) return;
  // ---- rows of this token's k slots (lane j < k owns slot t*k + j)
  if ((unsigned)e >= (unsigned)E || rk < 0) e = -1;
  // the histograms of the chunks before the slot's own, summed for all k slots at once:
  // lane = (slot j, part p) with 64 / K_MAX parts per slot
  constexpr int PARTS = 64 / K_MAX;
  const int j_of = lane / PARTS, p_of = lane % PARTS;
  const int ej = __shfl(e, j_of, 64);
  int part = 0;
  if (ROUTED) {
    const int gb = t / GATE_BLOCK_TOKENS, sc = gb / RT_SUPER;
    if (j_of < k && ej >= 0) {
      for (int r = p_of; r < sc; r += PARTS) part += totals2[(size_t)r * E + ej];
      for (int g = sc * RT_SUPER + p_of; g < gb; g += PARTS) part += chunk_hist[(size_t)g * E + ej];
    }
  } else {
    const int cj = (t * k + j_of) / DISPATCH_CHUNK;
    if (j_of < k && ej >= 0)
      for (int c = p_of; c < cj; c += PARTS) part += chunk_hist[(size_t)c * E + ej];
  }
#pragma unroll
  for (int off = PARTS / 2; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
  const int base = __shfl(part, lane * PARTS, 64);   // lane j < K_MAX: the sum of slot j
  int row = -1;
  if (lane < k) {
    const int s = t * k + lane;
    if (e >= 0) {
      row = offs[e] + base + rk;
      // ranks and histograms that do not belong to this topk_idx (a caller that changed the
      // routing in place after moe_route) must not turn into a write outside the buffers
      if ((unsigned)row >= (unsigned)(T * k)) row = -1;
      else row_to_slot[row] = s;
    }
    slot_to_row[s] = row;
  }
  if (row_vec == 0) return;
  int rows[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) rows[j] = __shfl(row, j, 64);  // lanes >= k hold -1
  if (STREAM) {
#pragma unroll
    for (int u = 0; u < SCATTER_PF; ++u) {
      const int c = lane + 64 * u;
      if (c < row_vec) {
#pragma unroll
        for (int j = 0; j < K_MAX; ++j)
          if (rows[j] >= 0)
            __builtin_nontemporal_store(pre[u], x_packed + (size_t)rows[j] * row_vec + c);
      }
    }
#pragma unroll 4
    for (int c = lane + 64 * SCATTER_PF; c < row_vec; c += 64) {
      const u32x4 v = __builtin_nontemporal_load(src + c);
#pragma unroll
      for (int j = 0; j < K_MAX; ++j)
        if (rows[j] >= 0) __builtin_nontemporal_store(v, x_packed + (size_t)rows[j] * row_vec + c);
    }
  } else {
#pragma unroll 4
    for (int c = lane; c < row_vec; c += 64) {
      const u32x4 v = src[c];
#pragma unroll
      for (int j = 0; j < K_MAX; ++j)
        if (rows[j] >= 0) x_packed[(size_t)rows[j] * row_vec + c] = v;
    }
  }
}

// The two launches, on explicit workspace pointers (a context's, or the static scratch of
// moe_dispatch_noalloc).  chunk_hist holds at least ceil(S / DISPATCH_CHUNK) * E integers.
int launch_dispatch_on(const int32_t* seg_pos, const int32_t* dest_rank, int32_t* chunk_hist,
                       int32_t* totals, int E, int R, int k, int d, int elem, const void* x,
                       const int32_t* topk_idx, int T, void* x_packed, int32_t* slot_to_row,
                       int32_t* row_to_slot, int32_t* expert_counts, int32_t* expert_offsets,
                       int32_t* rank_counts, int32_t* rank_offsets, hipStream_t s) {
  const int S = T * k;
  const int n_chunks = (S + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  int ebits = 0;
  while ((1 << ebits) < E) ++ebits;
  hipLaunchKernelGGL(dispatch_count_kernel, dim3(n_chunks), dim3(COUNT_THREADS), 0, s, topk_idx, S,
                     E, ebits, chunk_hist, totals, slot_to_row);
  const int row_vec = x != nullptr ? d * elem / 16 : 0;
  const int grid = (T + 3) / 4;
  // stream past the cache when the packed rows do not fit it (256 MB on this part)
  const bool stream = (size_t)S * row_vec * 16 > ((size_t)192 << 20);
#define LAUNCH_SCATTER(KM)                                                                       \
  if (stream) LAUNCH_SCATTER2(KM, true); else LAUNCH_SCATTER2(KM, false)
#define LAUNCH_SCATTER2(KM, ST)                                                                  \
  hipLaunchKernelGGL((dispatch_scatter_kernel<KM, ST, false>), dim3(grid), dim3(256), 0, s,       \
                     (const u32x4*)x, topk_idx, chunk_hist, totals, seg_pos, dest_rank, T, k, E, \
                     R, row_vec, slot_to_row, row_to_slot, (u32x4*)x_packed, expert_counts,      \
                     expert_offsets, rank_counts, rank_offsets, nullptr, nullptr)
  if (k <= 2) LAUNCH_SCATTER(2);
  else if (k <= 4) LAUNCH_SCATTER(4);
  else if (k <= 8) LAUNCH_SCATTER(8);
  else LAUNCH_SCATTER(MOE_MAX_TOPK);
#undef LAUNCH_SCATTER
#undef LAUNCH_SCATTER2
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_dispatch_empty(int E, int R, int32_t* expert_counts, int32_t* expert_offsets,
                          int32_t* rank_counts, int32_t* rank_offsets, hipStream_t s) {
  hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, E, R, expert_counts,
                     expert_offsets, rank_counts, rank_offsets);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

}  // namespace

// One launch: the scatter kernel on the side products that the fused gate kernel of the last
// moe_route left in the context (the caller has checked that they describe topk_idx and T).
int launch_dispatch_routed(moe_ctx* c, const void* x, const int32_t* topk_idx, int T,
                           void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                           int32_t* expert_counts, int32_t* expert_offsets, int32_t* rank_counts,
                           int32_t* rank_offsets, hipStream_t s) {
  const int E = c->cfg.E, R = c->cfg.R, k = c->cfg.k;
  const int S = T * k;
  const int row_vec = x != nullptr ? c->cfg.d * c->elem / 16 : 0;
  const int grid = (T + 3) / 4;
  // buffer of the last moe_route: [rt_super_max][E] super-block sums, then the grand totals
  const size_t half = (size_t)c->rt_super_max * E + (size_t)E * RT_TOT_STRIDE;
  int32_t* super = c->d_rt_super + (size_t)c->rt_parity * half;
  const int32_t* rt_tot = super + (size_t)c->rt_super_max * E;
  const bool stream = (size_t)S * row_vec * 16 > ((size_t)192 << 20);
#define LAUNCH_ROUTED(KM)                                                                        \
  if (stream) LAUNCH_ROUTED2(KM, true); else LAUNCH_ROUTED2(KM, false)
#define LAUNCH_ROUTED2(KM, ST)                                                                   \
  hipLaunchKernelGGL((dispatch_scatter_kernel<KM, ST, true>), dim3(grid), dim3(256), 0, s,        \
                     (const u32x4*)x, topk_idx, c->d_rt_hist, super, c->d_seg_pos,               \
                     c->d_dest_rank, T, k, E, R, row_vec, slot_to_row, row_to_slot,              \
                     (u32x4*)x_packed, expert_counts, expert_offsets, rank_counts, rank_offsets, \
                     c->d_rt_rank, rt_tot)
  if (k <= 2) LAUNCH_ROUTED(2);
  else if (k <= 4) LAUNCH_ROUTED(4);
  else if (k <= 8) LAUNCH_ROUTED(8);
  else LAUNCH_ROUTED(MOE_MAX_TOPK);
#undef LAUNCH_ROUTED
#undef LAUNCH_ROUTED2
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

int launch_dispatch(moe_ctx* c, const void* x, const int32_t* topk_idx, int T, void* x_packed,
                    int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                    int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                    hipStream_t s) {
  const int E = c->cfg.E, R = c->cfg.R, k = c->cfg.k;
  const int S = T * k;
  if (S == 0) return launch_dispatch_empty(E, R, expert_counts, expert_offsets, rank_counts, rank_offsets, s);
  const int n_chunks = (S + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  if (n_chunks > c->n_chunks_max) return MOE_EINVAL;
  // d_totals: [2][MOE_MAX_EXPERTS] totals, then the two call counters
  return launch_dispatch_on(c->d_seg_pos, c->d_dest_rank, c->d_chunk_hist, c->d_totals, E, R, k,
                            c->cfg.d, c->elem, x, topk_idx, T, x_packed, slot_to_row, row_to_slot,
                            expert_counts, expert_offsets, rank_counts, rank_offsets, s);
}

// ---- moe_dispatch_noalloc: the same two kernels on a workspace that is part of the loaded
// code object instead of a context's allocations.
namespace {

constexpr int NA_TOTALS = 0;                                    // [2][256] totals + 2 counters
constexpr int NA_SEG_POS = 576;                                 // [256]
constexpr int NA_DEST = NA_SEG_POS + MOE_MAX_EXPERTS;           // [256] sanitised placement
constexpr int NA_HIST = NA_DEST + MOE_MAX_EXPERTS;              // [chunks][E]
constexpr int NA_INTS = NA_HIST + MOE_NOALLOC_MAX_HIST;

// Every GPU the library runs on holds its own copy of this array until the process ends.
static __device__ __align__(256) int32_t scratch[NA_INTS];

// Device addresses of `scratch`, one per device, resolved on first use.  In host code the
// array's name is only a handle for hipGetSymbolAddress: host code uses these pointers.
constexpr int NA_MAX_DEVICES = 64;
int32_t* g_scratch_ptr[NA_MAX_DEVICES];
std::mutex g_scratch_mutex;

int scratch_for_current_device(int32_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MOE_EHIP;
  if (dev < 0 || dev >= NA_MAX_DEVICES) return MOE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return MOE_EHIP;
    }
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_scratch_ptr[dev];
  return MOE_OK;
}

// One block: clears the totals and the call counters (the array keeps what the last call left),
// copies the placement with every entry forced into [0, R), and ranks the experts by
// (destination rank, id): seg_pos[e] = number of experts ordered before e.
__global__ __launch_bounds__(MOE_MAX_EXPERTS) void dispatch_noalloc_prep_kernel(
    const int32_t* __restrict__ dest_in, int E, int R, int32_t* __restrict__ ws) {
  __shared__ int32_t dest[MOE_MAX_EXPERTS];
  const int tid = threadIdx.x;
  for (int i = tid; i < 2 * MOE_MAX_EXPERTS + 2; i += MOE_MAX_EXPERTS) ws[NA_TOTALS + i] = 0;
  int mine = 0;
  if (tid < E) {
    mine = min(max(dest_in[tid], 0), R - 1);
    dest[tid] = mine;
    ws[NA_DEST + tid] = mine;
  }
  __syncthreads();
  if (tid < E) {
    int pos = 0;
    for (int e = 0; e < E; ++e) pos += (dest[e] < mine || (dest[e] == mine && e < tid)) ? 1 : 0;
    ws[NA_SEG_POS + tid] = pos;
  }
}

}  // namespace

// Resolves the static workspace of the current device (moe_create calls it so that the
// address is known before a caller starts capturing).
int dispatch_noalloc_init() {
  int32_t* ws = nullptr;
  return scratch_for_current_device(&ws);
}

extern "C" int moe_dispatch_noalloc(const moe_config* cfg, const int32_t* expert_dest_rank,
                                    const void* x, const int32_t* topk_idx, int32_t T,
                                    void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                                    int32_t* expert_counts, int32_t* expert_offsets,
                                    int32_t* rank_counts, int32_t* rank_offsets, void* stream) {
  if (cfg == nullptr || expert_dest_rank == nullptr) return MOE_EINVAL;
  if (cfg->dtype != MOE_F32 && cfg->dtype != MOE_BF16) return MOE_EINVAL;
  if (cfg->E < 1 || cfg->E > MOE_MAX_EXPERTS) return MOE_EINVAL;
  if (cfg->k < 1 || cfg->k > cfg->E || cfg->k > MOE_MAX_TOPK) return MOE_EINVAL;
  if (cfg->R < 1 || cfg->R > MOE_MAX_RANKS) return MOE_EINVAL;
  if (cfg->d < 8 || cfg->d % 8 != 0 || T < 0) return MOE_EINVAL;
  if (expert_counts == nullptr || expert_offsets == nullptr || rank_counts == nullptr ||
      rank_offsets == nullptr)
    return MOE_EINVAL;
  if ((x == nullptr) != (x_packed == nullptr)) return MOE_EINVAL;
  if (T > 0 && (topk_idx == nullptr || slot_to_row == nullptr || row_to_slot == nullptr))
    return MOE_EINVAL;
  auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (!aligned16(x) || !aligned16(x_packed) || !aligned16(topk_idx) || !aligned16(slot_to_row) ||
      !aligned16(row_to_slot))
    return MOE_EINVAL;
  const long long S = (long long)T * cfg->k;
  if (S > (1ll << 22)) return MOE_EUNSUPPORTED;
  const long long n_chunks = (S + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  if (n_chunks * cfg->E > MOE_NOALLOC_MAX_HIST) return MOE_EUNSUPPORTED;   // beyond the static workspace
  hipStream_t s = (hipStream_t)stream;
  if (S == 0)
    return launch_dispatch_empty(cfg->E, cfg->R, expert_counts, expert_offsets, rank_counts,
                                 rank_offsets, s);
  int32_t* ws = nullptr;
  const int st = scratch_for_current_device(&ws);
  if (st != MOE_OK) return st;
  hipLaunchKernelGGL(dispatch_noalloc_prep_kernel, dim3(1), dim3(MOE_MAX_EXPERTS), 0, s,
                     expert_dest_rank, cfg->E, cfg->R, ws);
  if (hipGetLastError() != hipSuccess) return MOE_EHIP;
  return launch_dispatch_on(ws + NA_SEG_POS, ws + NA_DEST, ws + NA_HIST, ws + NA_TOTALS, cfg->E,
                            cfg->R, cfg->k, cfg->d, cfg->dtype == MOE_BF16 ? 2 : 4, x, topk_idx,
                            (int)T, x_packed, slot_to_row, row_to_slot, expert_counts,
                            expert_offsets, rank_counts, rank_offsets, s);
}
