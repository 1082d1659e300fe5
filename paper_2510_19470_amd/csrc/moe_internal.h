// Internal declarations shared by the HIP translation units of libmoe_hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

typedef uint16_t bf16_t;  // raw bf16 bit pattern in memory

// One row block of one expert segment, as the grouped GEMMs see it.
struct MTile {
  int32_t expert;
  int32_t row0;   // first packed row
  int32_t rows;   // valid rows (1..BM)
  int32_t pad;
};

// One tile of an MFMA grouped GEMM, complete: a block needs one 32-byte read to start.
struct TileDesc {
  int32_t row0;    // first packed row
  int32_t rows;    // valid rows (1..256)
  int32_t nblk;    // column block
  int32_t expert;
  const void* b0;  // weight-role operand of this expert (gate/up: W1)
  const void* b1;  // gate/up: W3
};

// Tile schedule built on the device from expert_counts/offsets (no host sync).
struct TileSched {
  int32_t n_mtiles;     // number of valid MTile entries
  // K-split of the last, partly filled round of the down GEMM (MFMA path): the first
  // down_full tiles of the order run whole, the remaining down_split_tiles are cut into
  // down_split parts along the contraction (down_split == 1: nothing is cut)
  int32_t down_full;
  int32_t down_split_tiles;
  int32_t down_split;
};

// pointer-table rows: W1, W3, W2, dW1, dW3, dW2
#define MOE_WTAB_ROWS 6

struct moe_ctx {
  moe_config cfg;
  int device;
  int elem;               // bytes per stored element
  int ffn_path;           // MOE_FFN_AUTO / MOE_FFN_VALU
  // placement
  int32_t* d_dest_rank;   // [E]
  int32_t* d_seg_pos;     // [E] position of every expert in (dest_rank, id) order
  // dispatch workspace
  int32_t n_chunks_max;   // slot chunks of DISPATCH_CHUNK
  int32_t* d_chunk_hist;  // [n_chunks_max][E] per-chunk expert histograms
  int32_t* d_totals;      // [2][MOE_MAX_EXPERTS] per-expert totals, double-buffered per call, then
                          // [2] the call number as the device keeps it
  float* d_logits;        // [T_max][E] when the caller does not want the logits
  // side products of the fused gate kernel for moe_dispatch_routed (nullptr: not kept):
  // per 32-token gate block the rank of every slot among the block's slots of the same
  // expert and the block's expert histogram; per super-block of 16 gate blocks the histogram
  // sums, accumulated with integer atomics into buffer rt_parity (the launch clears the other)
  int32_t* d_rt_rank;     // [S_max]
  int32_t* d_rt_hist;     // [ceil(T_max/32)][E]
  int32_t* d_rt_super;    // [2] x ([rt_super_max][E] super-block sums, [E][RT_TOT_STRIDE] totals)
  int32_t rt_super_max;
  int rt_parity;          // buffer the last moe_route accumulated into
  int32_t rt_dirty[2];    // super-block rows of each buffer that may be non-zero (rows at and
                          // above it are zero); the next launch clears them in the other buffer
  int rt_valid;           // the side products describe rt_idx / rt_T
  const int32_t* rt_idx;
  int32_t rt_T;
  // expert weight pointer tables: device copy [6][MOE_MAX_EXPERTS] (W1, W3, W2, dW1, dW3,
  // dW2), refreshed only when the host tables change
  const void** d_wtab;
  const void* h_wtab[MOE_WTAB_ROWS][MOE_MAX_EXPERTS];
  int wtab_valid;
  // grouped GEMM schedules: [0] 64-row tiles (vector ALU path), [1] 256-row tiles (MFMA)
  TileSched* d_sched[2];
  MTile* d_mtiles[2];
  int32_t max_mtiles[2];
  // activations between the two GEMMs, and the backward's temporaries (allocated on the
  // first backward call)
  TileDesc* d_order_up;   // MFMA tile order of the gate/up GEMM
  TileDesc* d_order_down; // ... and of the down GEMM
  int n_cu;               // compute units of the device
  float* d_split_ws;      // fp32 partial tiles of the K-split tail: [n_cu][256*256]
  int32_t S_max;          // T_max*k
  int32_t S_call;         // T*k of the expert-FFN call being launched: the rows its buffers hold
  void* d_H;              // [T_max*k][f]
  void* d_dG;             // [T_max*k][f]   (vector-ALU backward)
  void* d_dU;             // [T_max*k][f]
  void* d_dGU;            // [T_max*k][2f]  (MFMA backward: dG | dU)
  void* d_zero;           // 512 bytes of zeros (rows past a segment's end in the weight gradients)
  // gate backward: per-chunk partial sums of dWg, [T_max/128][E][d] (first call allocates)
  float* d_rbwd_ws;
  // shared/residual compression: selection state, histogram, per-chunk counts
  int32_t* d_sr_ws;
  size_t sr_ws_ints;      // capacity of d_sr_ws
  // optional HIP-event timing of the internal launches of moe_expert_ffn
  int prof_calls;         // capacity in calls (0 = off)
  int prof_n;             // calls recorded so far
  int prof_mask;          // bit i: launch i is timed (events i and i+1 are recorded)
  hipEvent_t* prof_ev;    // [prof_calls][MOE_PROF_SLOTS + 1]
};

// Records event `slot` of the current profiled call (no-op when profiling is off).
inline void prof_mark(moe_ctx* c, int slot, hipStream_t s) {
  const int need = c->prof_mask | (c->prof_mask << 1);   // event i brackets launches i-1 and i
  if (c->prof_calls > 0 && c->prof_n < c->prof_calls && ((need >> slot) & 1))
    (void)hipEventRecord(c->prof_ev[(size_t)c->prof_n * (MOE_PROF_SLOTS + 1) + slot], s);
}

#define DISPATCH_CHUNK 1024      // slots per histogram / ranking block
#define GATE_BLOCK_TOKENS 32     // tokens per block of the fused gate kernel
#define RT_SUPER 16              // gate blocks per super-block of the routed dispatch
#define RT_TOT_STRIDE 32         // ints between the grand totals of two experts (one line each)

// Lanes of the wavefront holding the same value as this lane (value in [0,256) or -1 for
// "none"): one ballot per bit of the value, no loop over the distinct values.
__device__ __forceinline__ unsigned long long match_same(int e, int nbits) {
  unsigned long long m = __ballot(e >= 0);
  for (int b = 0; b < nbits; ++b) {
    const unsigned long long bal = __ballot((e >> b) & 1);
    m &= ((e >> b) & 1) ? bal : ~bal;
  }
  return m;
}
#define GENERIC_BM 64
#define MFMA_BM 256

// ---- launchers (defined in the .hip files); all return a moe_status ----
int launch_route_select(const moe_ctx* c, const float* logits, int T, int32_t* idx, float* w,
                        hipStream_t s);
bool gate_route_fused_supported(const moe_ctx* c);
// keep_hist: also write the side products of moe_dispatch_routed (c->d_rt_*, buffer c->rt_parity)
int launch_gate_route_fused(const moe_ctx* c, const void* x, const void* Wg, const float* bias,
                            int T, float* logits, int32_t* idx, float* w, bool keep_hist,
                            hipStream_t s);
int launch_dispatch_routed(moe_ctx* c, const void* x, const int32_t* topk_idx, int T,
                           void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                           int32_t* expert_counts, int32_t* expert_offsets, int32_t* rank_counts,
                           int32_t* rank_offsets, hipStream_t s);
int launch_gate_logits(const moe_ctx* c, const void* x, const void* Wg, const float* bias, int T,
                       float* logits, hipStream_t s);
int launch_dispatch(moe_ctx* c, const void* x, const int32_t* topk_idx, int T, void* x_packed,
                    int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                    int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                    hipStream_t s);
int dispatch_noalloc_init();   // resolves the static dispatch workspace of the current device
int launch_combine(const moe_ctx* c, const void* y_packed, const int32_t* slot_to_row,
                   const float* w, int T, void* out, hipStream_t s);
int launch_combine_bwd(const moe_ctx* c, const void* dout, const void* y_packed,
                       const int32_t* slot_to_row, const float* w, int T, void* dy_packed,
                       float* dw, hipStream_t s);
int launch_dispatch_bwd(const moe_ctx* c, const void* dx_packed, const int32_t* slot_to_row, int T,
                        void* dx, hipStream_t s);
int launch_build_sched(moe_ctx* c, const int32_t* counts, const int32_t* offsets, int which,
                       hipStream_t s);
int launch_ffn_generic(moe_ctx* c, bool gated, const void* x_packed, void* y_packed, void* G,
                       void* U, void* H_tmp, hipStream_t s);
bool ffn_mfma_supported(const moe_ctx* c);
size_t ffn_mfma_order_entries(const moe_ctx* c);
bool ffn_mfma_supported_2mat(const moe_ctx* c);
int launch_ffn_mfma(moe_ctx* c, bool gated, const int32_t* counts, const int32_t* offsets,
                    const void* x_packed, void* y_packed, void* G, void* U, hipStream_t s);
bool ffn_bwd_mfma_supported(const moe_ctx* c);
int launch_ffn_bwd_mfma(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* G,
                        const void* U, const int32_t* counts, const int32_t* offsets, void* dxp,
                        hipStream_t s);
int launch_wgrad_tr(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* H,
                    const void* dGU, const int32_t* counts, const int32_t* offsets,
                    hipStream_t s);
size_t route_bwd_workspace_floats(const moe_ctx* c);
int launch_route_bwd(moe_ctx* c, const void* x, const void* Wg, const float* logits,
                     const int32_t* topk_idx, const float* topk_w, const float* dtopk_w, int T,
                     float* dlogits, float* dWg, float* dbias, void* dx, hipStream_t s);
size_t sr_workspace_ints(int64_t n);
int launch_sr_encode(moe_ctx* c, const void* W, const void* S, int64_t n, int64_t k, void* values,
                     int32_t* indices, hipStream_t s);
int launch_sr_decode(moe_ctx* c, const void* S, const void* values, const int32_t* indices,
                     int64_t n, int64_t k, void* out, hipStream_t s);
int launch_ffn_bwd_generic(moe_ctx* c, bool gated, const void* dy, const void* xp, const void* G,
                           const void* U, const int32_t* counts, const int32_t* offsets, void* dxp,
                           void* dG_tmp, void* dU_tmp, void* H_tmp, hipStream_t s);
