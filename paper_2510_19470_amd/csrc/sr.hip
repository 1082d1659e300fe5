// Shared/residual expert compression (paper Sec. 4.2 "SR-Based Expert Compression",
// Fig. "SRexpert"(b); compression ratio: Sec. 5.4).
//
//   encode: residual = expert - shared expert (float32); keep the k entries of largest
//           magnitude (equal magnitudes: lower index first) as a value-index list in
//           ascending index order, values rounded to the storage type;
//   decode: expert' = shared + scattered residual, one pass.
//
// The selection is exact.  The magnitude of a float32 is monotone in its low 31 bits, so the
// k-th largest magnitude is found by a radix select over that 31-bit key (12 + 12 + 7 bits;
// LDS-private histograms added to 16 global copies with integer atomics, so the result does
// not depend on the order; after each level a one-block kernel picks the bin holding the
// k-th largest).  Expert and shared are streamed TWICE:
//   1. histogram of the top 12 key bits -> the bin b0 of the k-th largest;
//   2. every element whose top bits are >= b0 (the entries certainly kept plus the candidates
//      of bin b0: a few per cent of the matrix) is appended, as (residual bits, index), to a
//      list in the workspace: one contiguous run per chunk of 8192 elements, in index order
//      inside the run; every block of that pass owns a fixed region of the list and appends
//      the runs of its chunks there (no atomics; every later step goes through the per-chunk
//      table of runs).
// The two lower radix levels, the per-chunk counts of entries above / equal to the threshold,
// and the emit of the value-index list then read only that list (a few MB).  A one-block scan
// turns the counts into output positions (of the equal keys the first k - #above in index
// order are taken), so the output is deterministic.
// When a block's runs do not fit its region (the list has room for 1/16 of the elements: many
// equal magnitudes, or k a large fraction of n) the second pass says so in a flag, and the
// later kernels stream expert and shared again instead of reading the list (three more
// streams + emit): every kernel after the second pass has both sources.
#include "moe_internal.h"
#include "numeric.h"

#include <algorithm>

namespace {

constexpr int SR_THREADS = 512;
constexpr int SR_PER_THREAD = 16;
constexpr int SR_CHUNK = SR_THREADS * SR_PER_THREAD;  // 8192 elements per block iteration
constexpr int SR_BINS = 4096;
constexpr int SR_REPL = 16;   // copies of the global histogram (fewer same-address atomics)

struct SrState {          // device-side selection state (first 8 ints of the workspace)
  uint32_t prefix;        // key bits fixed so far (right-aligned)
  int32_t k_rem;          // entries still to take among the keys that match the prefix
  int32_t pad[2];
  uint32_t unused;
  int32_t overflow;       // 1: the list did not fit, the later passes stream the matrices
  int32_t pad2[2];
};
constexpr int SR_STATE_INTS = 8;

// capacity of the candidate list, in entries of 8 bytes
__host__ __device__ inline int64_t sr_list_cap(int64_t n) {
  const int64_t c = n / 16;
  return c < 65536 ? 65536 : c;
}

template <typename T>
__device__ __forceinline__ uint32_t sr_key(T w, T s, float* r) {
  *r = to_f32(w) - to_f32(s);
  return __float_as_uint(*r) & 0x7fffffffu;
}

// The 16 consecutive elements of one thread: element base + j for j < 16, or fewer at the
// end of the array (keys of missing elements are never used: `cnt` says how many exist).
template <typename T>
struct SrLane {
  float r[SR_PER_THREAD];
  uint32_t key[SR_PER_THREAD];
  int cnt;
  __device__ __forceinline__ void load(const T* __restrict__ W, const T* __restrict__ S,
                                       int64_t base, int64_t n) {
    cnt = (int)max((int64_t)0, min((int64_t)SR_PER_THREAD, n - base));
    if (cnt == SR_PER_THREAD) {
      constexpr int V = 16 / sizeof(T);           // elements per 16-byte vector
      constexpr int NV = SR_PER_THREAD / V;
      uint4 wq[NV], sq[NV];
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        wq[v] = reinterpret_cast<const uint4*>(W + base)[v];
        sq[v] = reinterpret_cast<const uint4*>(S + base)[v];
      }
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        float wf[V], sf[V];
        Vec16<T>::unpack(wq[v], wf);
        Vec16<T>::unpack(sq[v], sf);
#pragma unroll
        for (int e = 0; e < V; ++e) {
          r[v * V + e] = wf[e] - sf[e];
          key[v * V + e] = __float_as_uint(r[v * V + e]) & 0x7fffffffu;
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < SR_PER_THREAD; ++j) {
        r[j] = 0.f;
        key[j] = 0;
        if (j < cnt) key[j] = sr_key(W[base + j], S[base + j], &r[j]);
      }
    }
  }
};

// PASS 0: bin = key[30:19];  PASS 1: keys with key[30:19] == prefix, bin = key[18:7];
// PASS 2: keys with key[30:7] == prefix, bin = key[6:0].  Passes 1 and 2 read the candidate
// list (a wavefront per run) unless it overflowed.
template <typename T, int PASS>
__global__ __launch_bounds__(SR_THREADS) void sr_hist_kernel(
    const T* __restrict__ W, const T* __restrict__ S, int64_t n, const SrState* __restrict__ st,
    int32_t* __restrict__ hist, const uint2* __restrict__ list,
    const int32_t* __restrict__ run_start, const int32_t* __restrict__ run_cnt) {
  __shared__ int32_t h[SR_BINS];
  constexpr int NB = PASS == 2 ? 128 : SR_BINS;
  for (int i = threadIdx.x; i < NB; i += SR_THREADS) h[i] = 0;
  __syncthreads();
  const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  auto add = [&](uint32_t key, bool hit) {
    int bin;
    if (PASS == 0) bin = key >> 19;
    else if (PASS == 1) { hit = hit && (key >> 19) == prefix; bin = (key >> 7) & 0xfffu; }
    else { hit = hit && (key >> 7) == prefix; bin = key & 0x7fu; }
    if (hit) atomicAdd(&h[bin], 1);
  };
  if (PASS != 0 && !st->overflow) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int WPB = SR_THREADS / 64;
    for (int64_t c = (int64_t)blockIdx.x * WPB + wave; c < n_chunks; c += (int64_t)gridDim.x * WPB) {
      const uint2* run = list + run_start[c];
      const int cnt = run_cnt[c];
      for (int i = lane; i < cnt; i += 64) add(run[i].x & 0x7fffffffu, true);
    }
  } else {
    for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
      SrLane<T> L;
      L.load(W, S, c * SR_CHUNK + (int64_t)threadIdx.x * SR_PER_THREAD, n);
#pragma unroll
      for (int j = 0; j < SR_PER_THREAD; ++j) add(L.key[j], j < L.cnt);
    }
  }
  __syncthreads();
  int32_t* mine = hist + (blockIdx.x % SR_REPL) * SR_BINS;
  for (int i = threadIdx.x; i < NB; i += SR_THREADS)
    if (h[i] != 0) atomicAdd(&mine[i], h[i]);
}

// One block: the bin b with  #(keys in bins > b) < k_rem <= #(keys in bins >= b)  is the one
// that holds the k_rem-th largest key; it is appended to the prefix, k_rem loses the keys
// above it, and the histogram is cleared for the next pass.  A thread owns 4 consecutive bins
// (16-byte loads of the 16 copies); the suffix sums over the 1024 threads are a reversed scan
// inside each wavefront (shuffles) plus the 16 wavefront totals through LDS: one barrier.
template <int PASS>
__global__ __launch_bounds__(1024) void sr_pick_kernel(SrState* __restrict__ st,
                                                       int32_t* __restrict__ hist, int32_t k) {
  constexpr int NB = PASS == 2 ? 128 : SR_BINS;
  constexpr int BITS = PASS == 2 ? 7 : 12;
  __shared__ int32_t wtot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int4 loc = make_int4(0, 0, 0, 0);
  if (tid * 4 < NB) {
    int4 v[SR_REPL];
#pragma unroll
    for (int rp = 0; rp < SR_REPL; ++rp)
      v[rp] = *reinterpret_cast<const int4*>(hist + rp * SR_BINS + tid * 4);
#pragma unroll
    for (int rp = 0; rp < SR_REPL; ++rp) {
      loc.x += v[rp].x; loc.y += v[rp].y; loc.z += v[rp].z; loc.w += v[rp].w;
    }
  }
  const int s4 = loc.x + loc.y + loc.z + loc.w;
  // inclusive suffix sum over the lanes of the wavefront: lane l gets the sum of lanes l..63
  int incl = s4;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_down(incl, off, 64);
    if (lane + off < 64) incl += t;
  }
  if (lane == 0) wtot[wave] = incl;
  const int32_t k_rem = PASS == 0 ? k : st->k_rem;
  const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
  __syncthreads();
  int above = incl - s4;   // keys in the bins above this thread's four
#pragma unroll
  for (int w = 0; w < 16; ++w) above += w > wave ? wtot[w] : 0;
  // suf[b] for the thread's bins b = 4 tid + j: keys in bins >= b
  const int suf3 = above + loc.w, suf2 = suf3 + loc.z, suf1 = suf2 + loc.y, suf0 = suf1 + loc.x;
  const int sufs[5] = {suf0, suf1, suf2, suf3, above};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = tid * 4 + j;
    if (b < NB && sufs[j + 1] < k_rem && k_rem <= sufs[j]) {   // exactly one b satisfies this
      st->prefix = (prefix << BITS) | (uint32_t)b;
      st->k_rem = k_rem - sufs[j + 1];
    }
  }
  if (PASS == 0 && tid == 0) st->overflow = 0;   // the second stream sets it when the list is full
  int4* h4 = reinterpret_cast<int4*>(hist);
  for (int b = tid; b < SR_REPL * SR_BINS / 4; b += 1024) h4[b] = make_int4(0, 0, 0, 0);
}

// Per chunk: keys above the threshold, keys equal to it; from the chunk's run of the list (a
// wavefront per run) or, after an overflow, from the matrices (a block per chunk).
template <typename T>
__global__ __launch_bounds__(SR_THREADS) void sr_count_kernel(
    const T* __restrict__ W, const T* __restrict__ S, int64_t n, const SrState* __restrict__ st,
    int32_t* __restrict__ cnt_gt, int32_t* __restrict__ cnt_eq, const uint2* __restrict__ list,
    const int32_t* __restrict__ run_start, const int32_t* __restrict__ run_cnt) {
  __shared__ int32_t red[2][SR_THREADS / 64];
  const uint32_t thr = st->prefix;
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (!st->overflow) {
    constexpr int WPB = SR_THREADS / 64;
    for (int64_t c = (int64_t)blockIdx.x * WPB + wave; c < n_chunks; c += (int64_t)gridDim.x * WPB) {
      const uint2* run = list + run_start[c];
      const int cnt = run_cnt[c];
      int gt = 0, eq = 0;
      for (int i = lane; i < cnt; i += 64) {
        const uint32_t key = run[i].x & 0x7fffffffu;
        gt += key > thr;
        eq += key == thr;
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        gt += __shfl_xor(gt, off, 64);
        eq += __shfl_xor(eq, off, 64);
      }
      if (lane == 0) {
        cnt_gt[c] = gt;
        cnt_eq[c] = eq;
      }
    }
    return;
  }
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    SrLane<T> L;
    L.load(W, S, c * SR_CHUNK + (int64_t)threadIdx.x * SR_PER_THREAD, n);
    int gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < SR_PER_THREAD; ++j) {
      if (j < L.cnt) {
        gt += L.key[j] > thr;
        eq += L.key[j] == thr;
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      gt += __shfl_xor(gt, off, 64);
      eq += __shfl_xor(eq, off, 64);
    }
    if (lane == 0) {
      red[0][wave] = gt;
      red[1][wave] = eq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int g = 0, e = 0;
      for (int w = 0; w < SR_THREADS / 64; ++w) {
        g += red[0][w];
        e += red[1][w];
      }
      cnt_gt[c] = g;
      cnt_eq[c] = e;
    }
    __syncthreads();
  }
}

// One block: exclusive prefix of the equal-key counts, entries each chunk emits (all of its
// keys above the threshold plus its share of the first k_rem equal keys), exclusive prefix
// of those.  Rounds of 8192 consecutive chunks, 8 per thread (two 16-byte loads per array);
// per quantity and round one block-wide exclusive scan of the threads' sums (shuffles inside a
// wavefront, the 16 wavefront totals through LDS), the totals carried from round to round.
__global__ __launch_bounds__(1024) void sr_scan_kernel(const SrState* __restrict__ st,
                                                       const int32_t* __restrict__ cnt_gt,
                                                       const int32_t* __restrict__ cnt_eq,
                                                       int64_t n_chunks,
                                                       int32_t* __restrict__ eq_prefix,
                                                       int32_t* __restrict__ out_prefix) {
  constexpr int PER = 8;
  __shared__ int32_t wtot[2][16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t need_eq = st->k_rem;
  int slot = 0;   // the two LDS rows alternate, so one barrier per scan is enough
  auto excl_scan = [&](int v, int* total) -> int {   // exclusive prefix of v over the block
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off, 64);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wtot[slot][wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int t = wtot[slot][w];
      before += w < wave ? t : 0;
      all += t;
    }
    slot ^= 1;
    *total = all;
    return before + incl - v;
  };
  int eq_carry = 0, out_carry = 0;
  for (int64_t c0 = 0; c0 < n_chunks; c0 += 1024 * PER) {
    const int64_t c = c0 + (int64_t)tid * PER;
    int eq[PER], gt[PER];
    if (c + PER <= n_chunks) {   // the arrays start 16-byte aligned and c is a multiple of 8
      const int4 a0 = *reinterpret_cast<const int4*>(cnt_eq + c), a1 = *reinterpret_cast<const int4*>(cnt_eq + c + 4);
      const int4 b0 = *reinterpret_cast<const int4*>(cnt_gt + c), b1 = *reinterpret_cast<const int4*>(cnt_gt + c + 4);
      eq[0] = a0.x; eq[1] = a0.y; eq[2] = a0.z; eq[3] = a0.w; eq[4] = a1.x; eq[5] = a1.y; eq[6] = a1.z; eq[7] = a1.w;
      gt[0] = b0.x; gt[1] = b0.y; gt[2] = b0.z; gt[3] = b0.w; gt[4] = b1.x; gt[5] = b1.y; gt[6] = b1.z; gt[7] = b1.w;
    } else {
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        eq[j] = c + j < n_chunks ? cnt_eq[c + j] : 0;
        gt[j] = c + j < n_chunks ? cnt_gt[c + j] : 0;
      }
    }
    int eq_sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) eq_sum += eq[j];
    int eq_all, take_all;
    int eq_before = eq_carry + excl_scan(eq_sum, &eq_all);
    int take[PER], eqp[PER], take_sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      eqp[j] = eq_before;
      take[j] = gt[j] + max(0, min(eq[j], need_eq - eq_before));
      take_sum += take[j];
      eq_before += eq[j];
    }
    int out_before = out_carry + excl_scan(take_sum, &take_all);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (c + j < n_chunks) {
        eq_prefix[c + j] = eqp[j];
        out_prefix[c + j] = out_before;
      }
      out_before += take[j];
    }
    eq_carry += eq_all;
    out_carry += take_all;
  }
}

// Writes the value-index list: a chunk's entries go to out_prefix[chunk] + rank inside the
// chunk (thread order = index order: a thread owns 16 consecutive elements).
template <typename T>
__global__ __launch_bounds__(SR_THREADS) void sr_emit_kernel(
    const T* __restrict__ W, const T* __restrict__ S, int64_t n, const SrState* __restrict__ st,
    const int32_t* __restrict__ eq_prefix, const int32_t* __restrict__ out_prefix, int64_t k,
    T* __restrict__ values, int32_t* __restrict__ indices, const uint2* __restrict__ list,
    const int32_t* __restrict__ run_start, const int32_t* __restrict__ run_cnt) {
  __shared__ int32_t wsum[2][SR_THREADS / 64];
  const uint32_t thr = st->prefix;
  const int32_t need_eq = st->k_rem;
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (!st->overflow) {
    // from the list: a wavefront per run, 64 entries per round, ranks by ballot (lane order
    // = index order)
    constexpr int WPB = SR_THREADS / 64;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int64_t c = (int64_t)blockIdx.x * WPB + wave; c < n_chunks; c += (int64_t)gridDim.x * WPB) {
      const uint2* run = list + run_start[c];
      const int cnt = run_cnt[c];
      int eq_rank = eq_prefix[c];
      int64_t pos = out_prefix[c];
      for (int i0 = 0; i0 < cnt; i0 += 64) {
        const bool valid = i0 + lane < cnt;
        const uint2 en = valid ? run[i0 + lane] : make_uint2(0u, 0u);
        const uint32_t key = en.x & 0x7fffffffu;
        const bool iseq = valid && key == thr;
        const unsigned long long eqm = __ballot(iseq);
        const bool sel = valid && (key > thr || (iseq && eq_rank + __popcll(eqm & below) < need_eq));
        const unsigned long long sm = __ballot(sel);
        const int64_t p = pos + __popcll(sm & below);
        if (sel && p < k) {   // p < k always holds when the counts are consistent
          values[p] = from_f32<T>(__uint_as_float(en.x));
          indices[p] = (int32_t)en.y;
        }
        eq_rank += __popcll(eqm);
        pos += __popcll(sm);
      }
    }
    return;
  }
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t base = c * SR_CHUNK + (int64_t)threadIdx.x * SR_PER_THREAD;
    SrLane<T> L;
    L.load(W, S, base, n);
    // rank of this thread's first equal key among the chunk's equal keys
    int eq = 0;
#pragma unroll
    for (int j = 0; j < SR_PER_THREAD; ++j)
      if (j < L.cnt) eq += L.key[j] == thr;
    int incl = eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[0][wave] = incl;
    __syncthreads();
    int eq_rank = eq_prefix[c] + incl - eq;
    for (int w = 0; w < wave; ++w) eq_rank += wsum[0][w];
    // selection flags and this thread's count
    uint32_t sel = 0;
    int taken = 0;
#pragma unroll
    for (int j = 0; j < SR_PER_THREAD; ++j) {
      if (j < L.cnt) {
        bool s = L.key[j] > thr;
        if (L.key[j] == thr) {
          s = eq_rank < need_eq;
          ++eq_rank;
        }
        if (s) {
          sel |= 1u << j;
          ++taken;
        }
      }
    }
    int incl2 = taken;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl2, off, 64);
      if (lane >= off) incl2 += v;
    }
    if (lane == 63) wsum[1][wave] = incl2;
    __syncthreads();
    int64_t pos = (int64_t)out_prefix[c] + incl2 - taken;
    for (int w = 0; w < wave; ++w) pos += wsum[1][w];
#pragma unroll
    for (int j = 0; j < SR_PER_THREAD; ++j)
      if ((sel >> j) & 1u) {
        if (pos < k) {   // always true when the counts are consistent
          values[pos] = from_f32<T>(L.r[j]);
          indices[pos] = (int32_t)(base + j);
        }
        ++pos;
      }
    __syncthreads();
  }
}

// ---- second stream: the entries whose top 12 key bits reach the bin of the k-th largest go
// to the list, one run per chunk (index order inside the run).  Block b appends the runs of
// its chunks to its own region [b * region, (b + 1) * region) of the list.
template <typename T>
__global__ __launch_bounds__(SR_THREADS) void sr_compact_kernel(
    const T* __restrict__ W, const T* __restrict__ S, int64_t n, SrState* __restrict__ st,
    int64_t region, uint2* __restrict__ list, int32_t* __restrict__ run_start,
    int32_t* __restrict__ run_cnt) {
  __shared__ int32_t wsum[SR_THREADS / 64];
  const uint32_t b0 = st->prefix;
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t used = 0;   // entries of this block's region in use (the same in every thread)
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t base = c * SR_CHUNK + (int64_t)threadIdx.x * SR_PER_THREAD;
    SrLane<T> L;
    L.load(W, S, base, n);
    uint32_t sel = 0;
#pragma unroll
    for (int j = 0; j < SR_PER_THREAD; ++j)
      if (j < L.cnt && (L.key[j] >> 19) >= b0) sel |= 1u << j;
    const int mine = __popc(sel);
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int before = incl - mine, total = 0;
#pragma unroll
    for (int w = 0; w < SR_THREADS / 64; ++w) {
      before += w < wave ? wsum[w] : 0;
      total += wsum[w];
    }
    const bool fits = used + total <= region;
    const int64_t run0 = (int64_t)blockIdx.x * region + used;
    if (threadIdx.x == 0) {
      run_start[c] = fits ? (int32_t)run0 : 0;
      run_cnt[c] = fits ? total : 0;
      if (!fits) st->overflow = 1;
    }
    if (fits) {
      uint2* p = list + run0 + before;
#pragma unroll
      for (int j = 0; j < SR_PER_THREAD; ++j)
        if ((sel >> j) & 1u) *p++ = make_uint2(__float_as_uint(L.r[j]), (uint32_t)(base + j));
      used += total;
    }
    __syncthreads();
  }
}

// Decode: out = shared, plus the residual where the list has an entry.  A block stages the
// entries of its chunk (a contiguous piece of the ascending list, found by binary search)
// in LDS as float32 plus a presence flag, so that untouched elements keep the shared
// expert's exact bits.
template <typename T>
__global__ __launch_bounds__(SR_THREADS) void sr_decode_kernel(
    const T* __restrict__ S, const T* __restrict__ values, const int32_t* __restrict__ indices,
    int64_t n, int64_t k, T* __restrict__ out) {
  __shared__ float res[SR_CHUNK];
  __shared__ uint8_t has[SR_CHUNK];
  __shared__ int64_t range[2];
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t start = c * SR_CHUNK, end = min(n, start + SR_CHUNK);
    if (threadIdx.x < 128) {   // lower_bound of start (wavefront 0) / end (wavefront 1) in
      // the ascending index list, 64 probes per round (4 rounds for a million entries)
      const int lane = threadIdx.x & 63;
      const int64_t target = threadIdx.x < 64 ? start : end;
      int64_t lo = 0, hi = k;
      while (hi > lo) {
        const int64_t stride = (hi - lo + 63) / 64;
        const int64_t pos = lo + lane * stride;
        const bool below = pos < hi && (int64_t)indices[pos] < target;
        const int m = __popcll(__ballot(below));   // probes 0..m-1 are below the target
        if (m == 0) {
          hi = lo;
        } else {
          hi = min(hi, lo + m * stride);           // probe m (if any) is not below
          lo = lo + (m - 1) * stride + 1;
        }
      }
      if (lane == 0) range[threadIdx.x >> 6] = lo;
    }
    for (int i = threadIdx.x; i < SR_CHUNK / 4; i += SR_THREADS)
      reinterpret_cast<uint32_t*>(has)[i] = 0;
    __syncthreads();
    for (int64_t e = range[0] + threadIdx.x; e < range[1]; e += SR_THREADS) {
      const int64_t i = (int64_t)indices[e] - start;
      if (i >= 0 && i < SR_CHUNK) {   // the list is the caller's: stay inside the chunk
        res[i] = to_f32(values[e]);
        has[i] = 1;
      }
    }
    __syncthreads();
    const int64_t base = start + (int64_t)threadIdx.x * SR_PER_THREAD;
    const int cnt = (int)max((int64_t)0, min((int64_t)SR_PER_THREAD, n - base));
    const int l0 = threadIdx.x * SR_PER_THREAD;
    if (cnt == SR_PER_THREAD) {
      constexpr int V = 16 / sizeof(T);
      constexpr int NV = SR_PER_THREAD / V;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        uint4 q = reinterpret_cast<const uint4*>(S + base)[v];
        bool any = false;
#pragma unroll
        for (int e = 0; e < V; ++e) any |= has[l0 + v * V + e] != 0;
        if (any) {
          float f[V];
          Vec16<T>::unpack(q, f);
          T o[V];
          const T* raw = reinterpret_cast<const T*>(&q);
#pragma unroll
          for (int e = 0; e < V; ++e)
            o[e] = has[l0 + v * V + e] ? from_f32<T>(f[e] + res[l0 + v * V + e]) : raw[e];
          __builtin_memcpy(&q, o, 16);
        }
        reinterpret_cast<uint4*>(out + base)[v] = q;
      }
    } else {
      for (int j = 0; j < cnt; ++j) {
        const T s = S[base + j];
        out[base + j] = has[l0 + j] ? from_f32<T>(to_f32(s) + res[l0 + j]) : s;
      }
    }
    __syncthreads();
  }
}

template <typename T>
int encode_t(moe_ctx* c, const T* W, const T* S, int64_t n, int64_t k, T* values, int32_t* indices,
             hipStream_t s) {
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int64_t nc2 = (n_chunks + 3) & ~(int64_t)3;   // keeps the per-chunk arrays 16-byte aligned
  const int grid = (int)std::min<int64_t>(n_chunks, (int64_t)c->n_cu * 8);
  SrState* st = reinterpret_cast<SrState*>(c->d_sr_ws);
  int32_t* hist = c->d_sr_ws + SR_STATE_INTS;
  int32_t* cnt_gt = hist + SR_REPL * SR_BINS;
  int32_t* cnt_eq = cnt_gt + nc2;
  int32_t* eq_prefix = cnt_eq + nc2;
  int32_t* out_prefix = eq_prefix + nc2;
  int32_t* run_start = out_prefix + nc2;
  int32_t* run_cnt = run_start + nc2;
  uint2* list = reinterpret_cast<uint2*>(run_cnt + nc2);
  // the histogram is zero on entry: cleared at allocation and by every pick kernel
  const int hgrid = (int)std::min<int64_t>(n_chunks, (int64_t)c->n_cu * 2);
  const int64_t region = sr_list_cap(n) / hgrid;   // list entries per block of the second stream
#define SR_LAUNCH(kern, g, b, ...) hipLaunchKernelGGL(kern, dim3(g), dim3(b), 0, s, __VA_ARGS__)
  SR_LAUNCH((sr_hist_kernel<T, 0>), hgrid, SR_THREADS, W, S, n, st, hist, list, run_start, run_cnt);
  SR_LAUNCH((sr_pick_kernel<0>), 1, 1024, st, hist, (int32_t)k);
  SR_LAUNCH((sr_compact_kernel<T>), hgrid, SR_THREADS, W, S, n, st, region, list, run_start, run_cnt);
  SR_LAUNCH((sr_hist_kernel<T, 1>), hgrid, SR_THREADS, W, S, n, st, hist, list, run_start, run_cnt);
  SR_LAUNCH((sr_pick_kernel<1>), 1, 1024, st, hist, (int32_t)k);
  SR_LAUNCH((sr_hist_kernel<T, 2>), hgrid, SR_THREADS, W, S, n, st, hist, list, run_start, run_cnt);
  SR_LAUNCH((sr_pick_kernel<2>), 1, 1024, st, hist, (int32_t)k);
  SR_LAUNCH((sr_count_kernel<T>), grid, SR_THREADS, W, S, n, st, cnt_gt, cnt_eq, list, run_start,
            run_cnt);
  SR_LAUNCH(sr_scan_kernel, 1, 1024, st, cnt_gt, cnt_eq, n_chunks, eq_prefix, out_prefix);
  SR_LAUNCH((sr_emit_kernel<T>), grid, SR_THREADS, W, S, n, st, eq_prefix, out_prefix, k, values,
            indices, list, run_start, run_cnt);
#undef SR_LAUNCH
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}

}  // namespace

size_t sr_workspace_ints(int64_t n) {
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int64_t nc2 = (n_chunks + 3) & ~(int64_t)3;
  // state, histograms, six per-chunk arrays, the candidate list (8 bytes per entry)
  return (size_t)(SR_STATE_INTS + SR_REPL * SR_BINS + 6 * nc2 + 2 * sr_list_cap(n));
}

int launch_sr_encode(moe_ctx* c, const void* W, const void* S, int64_t n, int64_t k, void* values,
                     int32_t* indices, hipStream_t s) {
  if (c->cfg.dtype == MOE_BF16)
    return encode_t<uint16_t>(c, (const uint16_t*)W, (const uint16_t*)S, n, k, (uint16_t*)values,
                              indices, s);
  return encode_t<float>(c, (const float*)W, (const float*)S, n, k, (float*)values, indices, s);
}

int launch_sr_decode(moe_ctx* c, const void* S, const void* values, const int32_t* indices,
                     int64_t n, int64_t k, void* out, hipStream_t s) {
  const int64_t n_chunks = (n + SR_CHUNK - 1) / SR_CHUNK;
  const int grid = (int)std::min<int64_t>(n_chunks, (int64_t)c->n_cu * 8);
  if (c->cfg.dtype == MOE_BF16)
    hipLaunchKernelGGL((sr_decode_kernel<uint16_t>), dim3(grid), dim3(SR_THREADS), 0, s,
                       (const uint16_t*)S, (const uint16_t*)values, indices, n, k, (uint16_t*)out);
  else
    hipLaunchKernelGGL((sr_decode_kernel<float>), dim3(grid), dim3(SR_THREADS), 0, s,
                       (const float*)S, (const float*)values, indices, n, k, (float*)out);
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_EHIP;
}
