// Dispatch: counts, (dest_rank, expert)-ordered offsets, the stable slot->row permutation
// and the row copy into the packed buffer (paper Sec. 2.1: data is rearranged to the
// activated experts; Sec. 3.2: one contiguous chunk per peer, and the chunk of an expert
// that was fetched by all-gather stays local).
//
// Three launches, no host synchronisation:
//   1. dispatch_hist_scan: per-chunk expert histograms in LDS; the last block to arrive
//      (atomic ticket, no spinning) turns them into exclusive prefixes over chunks and
//      writes counts / offsets / rank chunks.
//   2. dispatch_rank: every chunk recomputes the stable rank of its slots (ballot + popcount
//      per expert value inside a wavefront, LDS prefix over wavefronts) and writes both maps.
//   3. dispatch_copy: one wavefront per token reads the row once (16 B per lane) and writes
//      it to its k packed rows.
// The permutation is deterministic: no atomics decide a row number.
#include "moe_internal.h"

namespace {

__device__ __forceinline__ int32_t load_agent(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void dispatch_hist_scan_kernel(
    const int32_t* __restrict__ topk_idx, int S, int E, int R, int n_chunks,
    const int32_t* __restrict__ dest_rank, const int32_t* __restrict__ seg_order,
    int32_t* __restrict__ chunk_hist, int32_t* __restrict__ ticket,
    int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ rank_counts, int32_t* __restrict__ rank_offsets) {
  __shared__ int32_t hist[MOE_MAX_EXPERTS];
  __shared__ int32_t rcnt[MOE_MAX_RANKS];
  __shared__ int is_last;
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  for (int e = tid; e < E; e += 256) hist[e] = 0;
  __syncthreads();
  const int base = b * DISPATCH_CHUNK;
#pragma unroll
  for (int i = 0; i < DISPATCH_CHUNK / 256; ++i) {
    const int s = base + i * 256 + tid;
    if (s < S) {
      const int e = topk_idx[s];
      if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = tid; e < E; e += 256) chunk_hist[(size_t)b * E + e] = hist[e];
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
  const int lane = tid & 63, wave = tid >> 6;
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
    if (lane == 0) hist[e] = carry;  // total count of expert e
  }
  for (int r = tid; r < R; r += 256) rcnt[r] = 0;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) {
      const int e = seg_order[i];
      const int n = hist[e];
      expert_offsets[e] = run;
      expert_counts[e] = n;
      rcnt[dest_rank[e]] += n;
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

__global__ __launch_bounds__(256) void dispatch_rank_kernel(
    const int32_t* __restrict__ topk_idx, int S, int E, const int32_t* __restrict__ chunk_base,
    const int32_t* __restrict__ expert_offsets, int32_t* __restrict__ slot_to_row,
    int32_t* __restrict__ row_to_slot) {
  __shared__ int32_t wcnt[4][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  for (int i = tid; i < 4 * MOE_MAX_EXPERTS; i += 256) (&wcnt[0][0])[i] = 0;
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
      int row = -1;
      if (e >= 0) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wcnt[w][e];
        row = expert_offsets[e] + chunk_base[(size_t)b * E + e] + before + my_rank[r];
        row_to_slot[row] = s;
      }
      slot_to_row[s] = row;
    }
  }
}

// One wavefront per token: read the row once, write it k times.
template <int K_MAX>
__global__ __launch_bounds__(256) void dispatch_copy_kernel(const uint4* __restrict__ x,
                                                            const int32_t* __restrict__ slot_to_row,
                                                            int T, int k, int S, int row_vec,
                                                            uint4* __restrict__ x_packed) {
  const int lane = threadIdx.x & 63;
  const int t = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) >> 6);
  if (t >= T) return;
  int rows[K_MAX];
#pragma unroll
  for (int j = 0; j < K_MAX; ++j) {
    int r = j < k ? slot_to_row[(size_t)t * k + j] : -1;
    rows[j] = ((unsigned)r < (unsigned)S) ? r : -1;
  }
  const uint4* src = x + (size_t)t * row_vec;
  for (int c = lane; c < row_vec; c += 256) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (c + u * 64 < row_vec) v[u] = src[c + u * 64];
#pragma unroll
    for (int j = 0; j < K_MAX; ++j) {
      if (rows[j] >= 0) {
        uint4* dst = x_packed + (size_t)rows[j] * row_vec;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (c + u * 64 < row_vec) dst[c + u * 64] = v[u];
      }
    }
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
  hipLaunchKernelGGL(dispatch_hist_scan_kernel, dim3(n_chunks), dim3(256), 0, s, topk_idx, S, E, R,
                     n_chunks, c->d_dest_rank, c->d_seg_order, c->d_chunk_hist, c->d_ticket,
                     expert_counts, expert_offsets, rank_counts, rank_offsets);
  hipLaunchKernelGGL(dispatch_rank_kernel, dim3(n_chunks), dim3(256), 0, s, topk_idx, S, E,
                     c->d_chunk_hist, expert_offsets, slot_to_row, row_to_slot);
  if (x != nullptr) {
    const int elem = c->cfg.dtype == MOE_BF16 ? 2 : 4;
    const int row_vec = c->cfg.d * elem / 16;
    const int grid = (T + 3) / 4;
    if (k <= 2)
      hipLaunchKernelGGL((dispatch_copy_kernel<2>), dim3(grid), dim3(256), 0, s, (const uint4*)x,
                         slot_to_row, T, k, S, row_vec, (uint4*)x_packed);
    else if (k <= 4)
      hipLaunchKernelGGL((dispatch_copy_kernel<4>), dim3(grid), dim3(256), 0, s, (const uint4*)x,
                         slot_to_row, T, k, S, row_vec, (uint4*)x_packed);
    else if (k <= 8)
      hipLaunchKernelGGL((dispatch_copy_kernel<8>), dim3(grid), dim3(256), 0, s, (const uint4*)x,
                         slot_to_row, T, k, S, row_vec, (uint4*)x_packed);
    else
      hipLaunchKernelGGL((dispatch_copy_kernel<MOE_MAX_TOPK>), dim3(grid), dim3(256), 0, s,
                         (const uint4*)x, slot_to_row, T, k, S, row_vec, (uint4*)x_packed);
  }
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
