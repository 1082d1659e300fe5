// Dispatch: counts, (dest_rank, expert)-ordered offsets, the stable slot->row permutation
// and the row copy into the packed buffer (paper Sec. 2.1: data is rearranged to the
// activated experts; Sec. 3.2: one contiguous chunk per peer, and the chunk of an expert
// that was fetched by all-gather stays local).
//
// Two launches, no host synchronisation:
//   1. dispatch_count: every chunk of 1024 slots ranks its slots per expert (ballot +
//      popcount per expert value inside a wavefront, LDS prefix over wavefronts), stores
//      the in-chunk rank of each slot and the chunk's expert histogram; the last block to
//      arrive (atomic ticket, no spinning) turns the histograms into exclusive prefixes
//      over chunks and writes counts / offsets / rank chunks.
//   2. dispatch_scatter: one wavefront per token turns the in-chunk ranks of its k slots
//      into final rows (expert offset + chunk prefix + rank), writes both maps, reads the
//      token row once (16 B per lane) and writes it to its k packed rows.
// The permutation is deterministic: no atomic decides a row number.
#include "moe_internal.h"

namespace {

__device__ __forceinline__ int32_t load_agent(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void dispatch_count_kernel(
    const int32_t* __restrict__ topk_idx, int S, int E, int R, int n_chunks,
    const int32_t* __restrict__ dest_rank, const int32_t* __restrict__ seg_order,
    int32_t* __restrict__ chunk_hist, int32_t* __restrict__ ticket,
    int32_t* __restrict__ slot_rank, int32_t* __restrict__ expert_counts,
    int32_t* __restrict__ expert_offsets, int32_t* __restrict__ rank_counts,
    int32_t* __restrict__ rank_offsets) {
  __shared__ int32_t wcnt[4][MOE_MAX_EXPERTS];
  __shared__ int32_t tot[MOE_MAX_EXPERTS];
  __shared__ int32_t s_order[MOE_MAX_EXPERTS];
  __shared__ int32_t s_dest[MOE_MAX_EXPERTS];
  __shared__ int32_t rcnt[MOE_MAX_RANKS];
  __shared__ int is_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  for (int i = tid; i < 4 * MOE_MAX_EXPERTS; i += 256) (&wcnt[0][0])[i] = 0;
  for (int e = tid; e < E; e += 256) {  // placement, needed only by the last block
    s_order[e] = seg_order[e];
    s_dest[e] = dest_rank[e];
  }
  __syncthreads();
  constexpr int ROUNDS = DISPATCH_CHUNK / 256;
  int my_e[ROUNDS], my_rank[ROUNDS];
  const int wbase = b * DISPATCH_CHUNK + wave * (DISPATCH_CHUNK / 4);
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int s = wbase + r * 64 + lane;
    int e = -1;
    if (s < S) {
      e = topk_idx[s];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
    my_e[r] = e;
    my_rank[r] = 0;
  }
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int e = my_e[r];
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int e0 = __shfl(e, leader, 64);
      const unsigned long long m = __ballot(e == e0);
      if (e == e0) {
        const int before = wcnt[wave][e0];
        my_rank[r] = before + __popcll(m & ((1ull << lane) - 1ull));
        if (lane == leader) wcnt[wave][e0] = before + __popcll(m);
      }
      todo &= ~m;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int s = wbase + r * 64 + lane;
    const int e = my_e[r];
    if (s < S) {
      int rank = -1;
      if (e >= 0) {
        rank = my_rank[r];
        for (int w = 0; w < wave; ++w) rank += wcnt[w][e];
      }
      slot_rank[s] = rank;  // rank of the slot among its expert's slots of this chunk
    }
  }
  for (int e = tid; e < E; e += 256)
    chunk_hist[(size_t)b * E + e] = wcnt[0][e] + wcnt[1][e] + wcnt[2][e] + wcnt[3][e];
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const int prev = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    is_last = (prev == n_chunks - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();

  // exclusive prefix over chunks, one wavefront per expert at a time
  for (int e = wave; e < E; e += 4) {
    int carry = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += 64) {
      const int c = c0 + lane;
      const int v = c < n_chunks ? load_agent(&chunk_hist[(size_t)c * E + e]) : 0;
      int incl = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
      }
      if (c < n_chunks) chunk_hist[(size_t)c * E + e] = carry + incl - v;
      carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) tot[e] = carry;  // total count of expert e
  }
  for (int r = tid; r < R; r += 256) rcnt[r] = 0;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) {
      const int e = s_order[i];
      const int n = tot[e];
      expert_offsets[e] = run;
      expert_counts[e] = n;
      rcnt[s_dest[e]] += n;
      run += n;
    }
    int acc = 0;
    for (int r = 0; r < R; ++r) {
      rank_counts[r] = rcnt[r];
      rank_offsets[r] = acc;
      acc += rcnt[r];
    }
    rank_offsets[R] = acc;
    __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

// One wavefront per token: final rows of its k slots, both maps, and the row copy.
// slot_to_row holds the in-chunk ranks on entry and the final rows on exit.
template <int K_MAX>
__global__ __launch_bounds__(256) void dispatch_scatter_kernel(
    const uint4* __restrict__ x, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ chunk_base, const int32_t* __restrict__ expert_offsets, int T,
    int k, int E, int row_vec, int32_t* __restrict__ slot_to_row,
    int32_t* __restrict__ row_to_slot, uint4* __restrict__ x_packed) {
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= T) return;
  int row = -1;
  if (lane < k) {
    const int s = t * k + lane;
    const int e = topk_idx[s];
    const int rk = slot_to_row[s];
    if ((unsigned)e < (unsigned)E && rk >= 0) {
      row = expert_offsets[e] + chunk_base[(size_t)(s / DISPATCH_CHUNK) * E + e] + rk;
      row_to_slot[row] = s;
    }
    slot_to_row[s] = row;
  }
  if (row_vec == 0) return;
  int rows[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) rows[j] = __shfl(row, j, 64);  // lanes >= k hold -1
  const uint4* src = x + (size_t)t * row_vec;
#pragma unroll 4
  for (int c = lane; c < row_vec; c += 64) {
    const uint4 v = src[c];
#pragma unroll
    for (int j = 0; j < K_MAX; ++j)
      if (rows[j] >= 0) x_packed[(size_t)rows[j] * row_vec + c] = v;
  }
}

}  // namespace

int launch_dispatch(moe_ctx* c, const void* x, const int32_t* topk_idx, int T, void* x_packed,
                    int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                    int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                    hipStream_t s) {
  const int E = c->cfg.E, R = c->cfg.R, k = c->cfg.k;
  const int S = T * k;
  if (S == 0) {
    hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, E, R, expert_counts,
                       expert_offsets, rank_counts, rank_offsets);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
  }
  const int n_chunks = (S + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  if (n_chunks > c->n_chunks_max) return MOE_EINVAL;
  hipLaunchKernelGGL(dispatch_count_kernel, dim3(n_chunks), dim3(256), 0, s, topk_idx, S, E, R,
                     n_chunks, c->d_dest_rank, c->d_seg_order, c->d_chunk_hist, c->d_ticket,
                     slot_to_row, expert_counts, expert_offsets, rank_counts, rank_offsets);
  const int elem = c->cfg.dtype == MOE_BF16 ? 2 : 4;
  const int row_vec = x != nullptr ? c->cfg.d * elem / 16 : 0;
  const int grid = (T + 3) / 4;
#define LAUNCH_SCATTER(KM)                                                                      \
  hipLaunchKernelGGL((dispatch_scatter_kernel<KM>), dim3(grid), dim3(256), 0, s, (const uint4*)x, \
                     topk_idx, c->d_chunk_hist, expert_offsets, T, k, E, row_vec, slot_to_row,  \
                     row_to_slot, (uint4*)x_packed)
  if (k <= 2) LAUNCH_SCATTER(2);
  else if (k <= 4) LAUNCH_SCATTER(4);
  else if (k <= 8) LAUNCH_SCATTER(8);
  else LAUNCH_SCATTER(MOE_MAX_TOPK);
#undef LAUNCH_SCATTER
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
