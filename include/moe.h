/*
 * moe.h -- C ABI of the one-GPU MoE hot path (gfx950 / MI355X).
 *
 * One GPU's share of an expert-parallel Mixture-of-Experts layer under a given
 * expert-placement map: top-k gating, dispatch into contiguous per-(destination
 * rank, expert) buffers, grouped SwiGLU expert FFN on the resident experts,
 * weighted combine, and the backward of the last three.
 *
 * Structure of the layer: paper Sec. 2.1 "Expert Parallelism" and Fig.
 * "MoE-structure" (gate network as router, data moved to the activated experts,
 * experts are replicated FFNs, results merged back).  Placement semantics: paper
 * Sec. 3.2 "Relationships between Two Communications" (an expert obtained by
 * all-gather is computed locally, its data chunk is not sent) and the domain rule
 * of Sec. 4.1 / Algorithm 1 (which rank the tokens of a non-resident expert go
 * to).  Per-peer contiguous chunks: Sec. 3.2 "All-to-All Communication Modeling".
 *
 * Conventions
 *   - Every function returns 0 (MOE_OK) or a negative moe_status.  Nothing throws
 *     or aborts across this boundary.  moe_strerror() names a status.
 *   - Pointers marked [dev] are device pointers the CALLER owns (allocated with
 *     any HIP allocator), 16-byte aligned, row-major, dense.  Pointers marked
 *     [host] are host memory, read during the call only.
 *   - The library owns only the opaque moe_ctx and its small device workspace.
 *   - All compute calls are asynchronous on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream), do no host synchronisation and copy
 *     nothing back to the host: counts and offsets stay on the device.
 *   - Arguments are validated on the host before anything is launched; on error
 *     nothing is launched.
 *   - Slot s = t*k + j is token t's j-th selected expert; S = T*k; rows of the
 *     packed buffers are numbered 0..S-1.
 *   - Storage type `dtype` applies to x, Wg, expert weights, packed buffers and
 *     outputs.  Accumulation is always fp32.  Indices are int32.
 *   - Calls on one moe_ctx must not overlap in time (they share its workspace).
 */
#ifndef MOE_HOTPATH_MOE_H
#define MOE_HOTPATH_MOE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef enum {
  MOE_OK = 0,
  MOE_EINVAL = -1,       /* bad argument (range, NULL, alignment, size) */
  MOE_EUNSUPPORTED = -2, /* valid but outside what the kernels cover */
  MOE_ENOMEM = -3,       /* workspace allocation failed */
  MOE_EHIP = -4          /* a HIP runtime call failed */
} moe_status;

/* Limits of the kernels. */
#define MOE_MAX_EXPERTS 256
#define MOE_MAX_TOPK 16
#define MOE_MAX_RANKS 256

typedef struct {
  int32_t T_max;       /* largest T any call will pass (sizes the workspace)        */
  int32_t d;           /* d_model; multiple of 8                                      */
  int32_t E;           /* experts, 1..MOE_MAX_EXPERTS                                 */
  int32_t k;           /* top-k, 1..min(E, MOE_MAX_TOPK)                              */
  int32_t f;           /* ffn_dim; multiple of 8                                      */
  int32_t R;           /* virtual ranks, 1..MOE_MAX_RANKS                             */
  int32_t local_rank;  /* this GPU's rank, 0..R-1                                     */
  int32_t dtype;       /* moe_dtype                                                   */
  int32_t renormalize; /* 1: gate weights = softmax over the selected k; 0: over all E */
} moe_config;

const char* moe_strerror(int status);

/* Create / destroy a context.  moe_create validates cfg, allocates the device
 * workspace on the current device and installs the default placement
 * dest_rank[e] = e / ceil(E/R).  *out is NULL on error.  The workspace, with S = T_max*k:
 * H [S, f] in dtype between the two GEMMs of the FFN (the largest part: 470 MB at T_max =
 * 8192, k = 2, f = 14336, bf16); 64 MB of fp32 partial tiles for contraction-split GEMM
 * tiles; the tile lists (32 bytes per 256-row block and column block); [T_max, E] fp32 logits;
 * S/1024 * E + O(E) integers for the dispatch.  The first moe_expert_ffn_bwd adds [S, 2f] in
 * dtype, the first moe_route_bwd that wants dWg ceil(T_max/128) * E * d floats.
 * MOE_EUNSUPPORTED: S > 2^22. */
int moe_create(moe_ctx** out, const moe_config* cfg);
int moe_destroy(moe_ctx* ctx);

/* Expert-placement map (paper Sec. 3.2, Sec. 4.1): expert_dest_rank [host][E],
 * each in [0,R).  dest_rank[e] == local_rank  <=>  expert e is resident (home or
 * migrated here): its tokens are packed into the local compute region.  Any other
 * value: its tokens are packed into that rank's send buffer.  Copies the map to
 * the device with a synchronous copy. */
int moe_set_placement(moe_ctx* ctx, const int32_t* expert_dest_rank);

/* Which kernels moe_expert_ffn uses.  MOE_FFN_AUTO (default): the bf16 MFMA kernels when
 * dtype is bf16, d % 256 == 0 and f % 128 == 0, else the vector-ALU kernels.  MOE_FFN_VALU:
 * always the vector-ALU kernels (any shape and both dtypes; a slow cross-check). */
#define MOE_FFN_AUTO 0
#define MOE_FFN_VALU 1
int moe_set_ffn_path(moe_ctx* ctx, int path);

/* Gating (Sec. 2.1 "Expert Parallelism": the gate network routes every token to K experts).
 *   logits[t,e] = sum_c x[t,c]*Wg[e,c] (+ bias[e]);  the k largest per token in
 *   descending order, equal logits ordered by ascending expert id;  weights =
 *   softmax over the selected k (renormalize) or over all E, computed in fp32.
 * x [dev][T,d] dtype; Wg [dev][E,d] dtype; bias [dev][E] fp32 or NULL;
 * logits [dev][T,E] fp32 out, or NULL (then the workspace holds them);
 * topk_idx [dev][T,k] int32 out; topk_w [dev][T,k] fp32 out.  0 <= T <= T_max. */
int moe_route(moe_ctx* ctx, const void* x, const void* Wg, const float* bias, int32_t T,
              float* logits, int32_t* topk_idx, float* topk_w, void* stream);

/* The selection and weights alone, from given fp32 logits [dev][T,E]: pure
 * comparisons, so topk_idx is reproducible bit for bit from the same logits. */
int moe_route_logits(moe_ctx* ctx, const float* logits, int32_t T, int32_t* topk_idx,
                     float* topk_w, void* stream);

/* Dispatch (Sec. 2.1 data rearrangement; Sec. 3.2 per-peer chunks and the rule
 * that a fetched expert keeps its chunk local).  Segments are ordered by
 * (dest_rank[e], e); inside a segment rows follow ascending slot id (stable), so
 * exactly one permutation is correct.
 *   expert_counts[e]  = number of slots routed to e
 *   expert_offsets[e] = first packed row of e's segment
 *   rank_counts[r], rank_offsets[r] (R+1 entries, last = S): rank r's chunk
 *   slot_to_row[s], row_to_slot[row]: the permutation and its inverse
 *   x_packed[slot_to_row[t*k+j]] = x[t]   (bit copy)
 * Rows [rank_offsets[local_rank], rank_offsets[local_rank+1]) are the compute
 * region; every other rank's range is that rank's send buffer.
 * x [dev][T,d]; topk_idx [dev][T,k] with every entry in [0,E) (entries outside
 * are not detected on the host; they are skipped on the device and leave their
 * slot unmapped); all outputs [dev], int32 except x_packed [dev][T*k,d] dtype.
 * x and x_packed may be NULL together to compute the maps only. */
int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* topk_idx, int32_t T,
                 void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                 int32_t* expert_counts, int32_t* expert_offsets, int32_t* rank_counts,
                 int32_t* rank_offsets, void* stream);

/* moe_dispatch of the routing that the last moe_route on this context wrote: same arguments,
 * same outputs bit for bit, one kernel launch instead of two.  moe_route's gate kernel holds
 * the k expert ids of its tokens anyway and leaves the counting step of the dispatch in the
 * context (per 32 tokens: the rank of every slot among the slots of its expert, the expert
 * histogram; sums of 16 such histograms); this call turns them into offsets and rows inside
 * the kernel that copies the token rows.
 * CONTRACT: topk_idx must be the array the last moe_route on ctx wrote, UNCHANGED since (same
 * pointer, same T); a caller that edits the routing in between (drops or remaps experts) must
 * call moe_dispatch (with an edited routing the maps come out wrong, but every write stays
 * inside the output buffers: rows outside [0, T*k) are refused on the device).  When the
 * context holds no such side products -- pointer or T differ,
 * the gate of this configuration is not the fused kernel (fp32 storage, d % 256 != 0),
 * T_max > 131072, or moe_route ran on a stream that was being captured -- the call is
 * moe_dispatch.  May be repeated; the side products stay valid until the next moe_route. */
int moe_dispatch_routed(moe_ctx* ctx, const void* x, const int32_t* topk_idx, int32_t T,
                        void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                        int32_t* expert_counts, int32_t* expert_offsets, int32_t* rank_counts,
                        int32_t* rank_offsets, void* stream);

/* moe_dispatch for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  It needs no moe_ctx (creating
 * one allocates) and calls no allocator: the per-chunk expert histograms, the per-expert
 * totals and the segment positions live in a static device array inside the library, of
 * MOE_NOALLOC_MAX_HIST + 1088 int32 (just over 1 MiB) per GPU, which every GPU the library
 * runs on holds until the process ends.  The first call on a device (or moe_create on that
 * device) looks its address up; make that call outside a capture.
 *   cfg [host]: d, E, k, R, dtype are used as in moe_create; the other fields are ignored.
 *   expert_dest_rank [dev][E]: the placement map on the DEVICE (read by a kernel: nothing is
 *   copied from the host); an entry outside [0,R) is taken as the nearest valid rank.
 *   All other arguments as in moe_dispatch; same outputs, bit for bit.
 * Limits: T*k <= 2^22 and ceil(T*k / 1024) * E <= MOE_NOALLOC_MAX_HIST, else
 * MOE_EUNSUPPORTED and nothing is launched; MOE_EUNSUPPORTED also for a device ordinal >= 64.
 * Every call on a GPU uses that GPU's one array (each call clears what it needs at its start):
 * calls that overlap in time on one GPU, on different streams or from different threads,
 * race.  Calls on one stream are ordered and safe. */
#define MOE_NOALLOC_MAX_HIST (256 * 1024)
int moe_dispatch_noalloc(const moe_config* cfg, const int32_t* expert_dest_rank, const void* x,
                         const int32_t* topk_idx, int32_t T, void* x_packed,
                         int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                         int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                         void* stream);

/* Grouped SwiGLU expert FFN (Sec. 2.1: experts are replicated FFNs; Sec. 3.1: the
 * experts of one GPU are computed one after another on their own tokens).  For
 * every expert e whose three table entries are non-NULL and every row r of its
 * segment [expert_offsets[e], +expert_counts[e]):
 *   g = x_r W1[e]^T, u = x_r W3[e]^T, h = silu(g)*u, y_r = h W2[e]^T
 * W1,W3,W2: [host][E] tables of device pointers; W1[e],W3[e] [dev][f,d],
 * W2[e] [dev][d,f], dtype; an expert with NULL entries is not computed and its
 * rows of y_packed are left untouched.  In production the non-NULL set is the
 * resident set; loopback tests pass every expert.
 * y_packed [dev][S,d] dtype out.  G_save,U_save [dev][S,f] dtype out or both NULL:
 * the pre-activation projections kept for the backward.  bf16: h (and g,u when
 * saved) are rounded to bf16 between the two GEMMs.
 * W3 == NULL (the table pointer itself) selects the paper's own expert, a two-matrix FFN
 * (Sec. 2.1; Table 2 counts 2*H*M parameters per expert):
 *   g = x_r W1[e]^T, y_r = max(g, 0) W2[e]^T
 * (the paper does not name the activation; ReLU, as in the Transformer FFN it cites).
 * U_save must then be NULL, G_save may receive g.
 * expert_counts, expert_offsets [dev][E] are read on the device (no host copy).  If the segment
 * of any computed expert does not lie inside the T*k rows of the buffers (negative count or
 * offset, offset + count > T*k), the call computes nothing: y_packed and the saves are left
 * untouched; moe_expert_ffn_bwd then leaves dx_packed untouched and writes zeros to the wanted
 * weight gradients.  No error is reported (the host never sees the arrays). */
int moe_expert_ffn(moe_ctx* ctx, const void* x_packed, const int32_t* expert_counts,
                   const int32_t* expert_offsets, const void* const* W1, const void* const* W3,
                   const void* const* W2, int32_t T, void* y_packed, void* G_save, void* U_save,
                   void* stream);

/* Combine / un-permute (Sec. 2.1: the second rearrangement, after the experts).
 *   out[t] = sum_{j<k} topk_w[t,j] * y_packed[slot_to_row[t*k+j]], j ascending, fp32.
 * y_packed [dev][S,d] must hold every row (remote rows are what came back from the
 * other ranks; the caller supplies them).  out [dev][T,d] dtype. */
int moe_combine(moe_ctx* ctx, const void* y_packed, const int32_t* slot_to_row,
                const float* topk_w, int32_t T, void* out, void* stream);

/* Backward of combine (the chain rule of the second rearrangement of Sec. 2.1; the paper
 * models the backward pass only as the forward plus a constant all-reduce term, Sec. 6):
 *                       dy_packed[row(t,j)] = topk_w[t,j]*dout[t];
 *                       dtopk_w[t,j] = <dout[t], y_packed[row(t,j)]>.
 * dout [dev][T,d]; dy_packed [dev][S,d] out; dtopk_w [dev][T,k] fp32 out. */
int moe_combine_bwd(moe_ctx* ctx, const void* dout, const void* y_packed,
                    const int32_t* slot_to_row, const float* topk_w, int32_t T,
                    void* dy_packed, float* dtopk_w, void* stream);

/* Backward of the expert FFN (chain rule of the replicated FFN of Sec. 2.1; Sec. 3.1's GeMM
 * cost model applies to these products as to the forward ones; the cross-rank reduction of
 * the gradients of migrated experts, the all-reduce of Sec. 6, is not part of this call),
 * for every expert with non-NULL table entries:
 *   dH = dY W2; dG = dH*u*silu'(g); dU = dH*silu(g); dX = dG W1 + dU W3;
 *   dW2 = dY^T H; dW1 = dG^T X; dW3 = dU^T X        (H = silu(G)*U recomputed)
 * dy_packed,x_packed [dev][S,d]; G_save,U_save [dev][S,f] from the forward;
 * dx_packed [dev][S,d] out (rows of experts not computed are left untouched);
 * dW1,dW3,dW2: [host][E] tables of device pointers to fp32 [f,d],[f,d],[d,f],
 * overwritten (not accumulated); NULL entry = that gradient is not wanted.
 * W3 == NULL (the table pointer) is the backward of the two-matrix expert:
 *   dH = dY W2; dG = dH where g > 0, else 0; dX = dG W1; dW2 = dY^T max(G,0); dW1 = dG^T X
 * (g > 0 is decided on the stored G_save); U_save and dW3 must then be NULL as well.
 * Errors: MOE_EINVAL for a NULL or misaligned pointer, tables that disagree about which
 * experts are present, or U_save/dW3 not matching W3; MOE_ENOMEM when the first call
 * cannot allocate the backward workspace. */
int moe_expert_ffn_bwd(moe_ctx* ctx, const void* dy_packed, const void* x_packed,
                       const void* G_save, const void* U_save, const int32_t* expert_counts,
                       const int32_t* expert_offsets, const void* const* W1,
                       const void* const* W3, const void* const* W2, int32_t T, void* dx_packed,
                       float* const* dW1, float* const* dW3, float* const* dW2, void* stream);

/* Backward of dispatch (chain rule of the first rearrangement of Sec. 2.1, the transpose of
 * the pack): dx[t] = sum_j dx_packed[slot_to_row[t*k+j]], j ascending, fp32.
 * dx_packed [dev][S,d] must hold every row (rows of other ranks' experts are what came back
 * from them); dx [dev][T,d] dtype out. */
int moe_dispatch_bwd(moe_ctx* ctx, const void* dx_packed, const int32_t* slot_to_row, int32_t T,
                     void* dx, void* stream);

/* ---- Placement planning (host only; no GPU is touched) --------------------------------
 * The multilevel description of Sec. 4.1: L levels, SF[l] = workers a level-(l-1) worker
 * expands into (SF[0] = workers at level 0), S_ED[l] = expert-domain size at level l
 * (1 <= S_ED[l], S_ED[l] divides SF[l]); G = prod SF[l] GPUs, global rank as in PyTorch.
 * All arrays are [host]. */
#define MOE_PLAN_MAX_LEVELS 8
#define MOE_COMM_NONE 0
#define MOE_COMM_AG 1
#define MOE_COMM_A2A 2
#define MOE_PLAN_CASE_MIX 1     /* 2D - G*P_E <  0: both A2A and AG (Case 1 + 2.1) */
#define MOE_PLAN_CASE_AG_ONLY 2 /* 2D - G*P_E >= 0: p = 0 (Case 2.2)               */

/* Location renumbering (Sec. 4.1): loc[i] = floor(rank / prod_{j>i} SF[j]) mod SF[i]. */
int moe_plan_location(int32_t rank, int32_t L, const int32_t* SF, int32_t* loc /*[L]*/);

/* Communication topology of Sec. 4.1 (Algorithm 1) for the pair (m, n) at one level:
 * MOE_COMM_AG inside a domain (different offsets), MOE_COMM_A2A across domains (same
 * offset), else MOE_COMM_NONE.  Which pairs may talk at level l is where this library departs
 * from the algorithm as printed.  MOE_PLAN_RULE_ALL_OTHER (what moe_plan_comm_type,
 * moe_plan_comm_frequency and moe_plan_expert_dest_rank use): every OTHER coordinate of the
 * two locations must agree, so a pair differs in exactly one level's worker number.
 * MOE_PLAN_RULE_PRINTED: only the deeper coordinates must agree, as the listing and the
 * sentence before it say; at the innermost level that pairs GPUs of different DCs.  With one
 * level the two rules coincide (all that Table 7 covers).  On the paper's example of 4 DCs x
 * 4 GPUs, SF = [4,4], S_ED = [2,4]: 64 AG + 16 A2A ordered pairs under ALL_OTHER, 208 AG +
 * 16 A2A under PRINTED.  MOE_EINVAL for an unknown rule. */
#define MOE_PLAN_RULE_ALL_OTHER 0
#define MOE_PLAN_RULE_PRINTED 1
int moe_plan_comm_type(int32_t m, int32_t n, int32_t level, int32_t L, const int32_t* SF,
                       const int32_t* S_ED, int32_t* type_out);
int moe_plan_comm_type_rule(int32_t m, int32_t n, int32_t level, int32_t L, const int32_t* SF,
                            const int32_t* S_ED, int32_t rule, int32_t* type_out);

/* Communication frequency (Sec. 5.6, Table 7): number of GPU-to-GPU communications of
 * each type over all ordered pairs and levels.  G <= 4096.  Closed forms: ALL_OTHER
 * n_ag = G sum_l (S_ED[l]-1), n_a2a = G sum_l (SF[l]/S_ED[l]-1); PRINTED: term l times
 * prod_{j<l} SF[j]. */
int moe_plan_comm_frequency(int32_t L, const int32_t* SF, const int32_t* S_ED, int64_t* n_ag,
                            int64_t* n_a2a);
int moe_plan_comm_frequency_rule(int32_t L, const int32_t* SF, const int32_t* S_ED, int32_t rule,
                                 int64_t* n_ag, int64_t* n_a2a);

/* The map moe_set_placement takes, for E experts spread evenly over the G GPUs (expert e at
 * home rank e / (E/G)): dest[e] = local_rank when the home is reachable by all-gather at
 * every level (the expert is resident), else the rank of the home's domain with the local
 * offsets (domain rule), level by level: the destination is one all-to-all hop away per level
 * whose domains differ, and the home reaches it by all-gather hops only.
 * dest [E] out; E must be a multiple of G. */
int moe_plan_expert_dest_rank(int32_t local_rank, int32_t E, int32_t L, const int32_t* SF,
                              const int32_t* S_ED, int32_t* dest);

/* Stream model (Sec. 3): D = data bytes leaving a GPU per A2A, P_E = expert bytes per GPU,
 * B = bandwidth (bytes/s), lat_pe = pre-expert compute time (s), G GPUs.  *p_star = the
 * closed-form optimal A2A proportion (Sec. 3.4), *case_id = MOE_PLAN_CASE_*, *best_S = the
 * divisor S of G whose exact proportion (G-S)/(G-1) has the lowest modelled latency. */
int moe_plan_model(double D, double P_E, double B, double lat_pe, int32_t G, double* p_star,
                   int32_t* case_id, int32_t* best_S);

/* Backward of the gate (Sec. 2.1: the gate network picks the K experts of a token; the
 * output depends on it through the K combine weights).  The Top-k choice itself is
 * piecewise constant and carries no gradient.  With p = softmax of the logits over the
 * selected experts (renormalize = 1) or over all E (renormalize = 0), w_j = p[idx_j]:
 *   dlogits[t,e] = p_e * ( [e selected] dtopk_w[t,j(e)] - sum_j dtopk_w[t,j] topk_w[t,j] )
 *   dWg = dlogits^T x      dbias[e] = sum_t dlogits[t,e]      dx[t] += dlogits[t] Wg
 * x [dev][T,d] dtype (needed for dWg); Wg [dev][E,d] dtype (needed for dx); logits
 * [dev][T,E] fp32 as moe_route returned them (needed when renormalize = 0, else may be
 * NULL); topk_idx, topk_w from moe_route; dtopk_w [dev][T,k] fp32 from moe_combine_bwd.
 * dlogits [dev][T,E] fp32 out (required); dWg [dev][E,d] fp32 out or NULL; dbias [dev][E]
 * fp32 out or NULL; dx [dev][T,d] dtype IN/OUT or NULL: the gate's contribution is ADDED to
 * what moe_dispatch_bwd wrote there (fp32 add, rounded once to dtype).  Deterministic
 * (fixed-order partial sums).  The first call that asks for dWg allocates a workspace
 * of ceil(T_max/128) * E * d floats. */
int moe_route_bwd(moe_ctx* ctx, const void* x, const void* Wg, const float* logits,
                  const int32_t* topk_idx, const float* topk_w, const float* dtopk_w, int32_t T,
                  float* dlogits, float* dWg, float* dbias, void* dx, void* stream);

/* ---- Shared/residual expert compression (Sec. 4.2 "SR-Based Expert Compression";
 * compression ratio CR: Sec. 5.4).  An expert weight matrix is sent to the other GPUs of
 * its domain as the k largest-magnitude entries of (expert - shared expert) in value-index
 * form and rebuilt there as shared + scattered residual.  n = elements of the matrix (any
 * shape, taken flat), 1 <= n < 2^31; storage type = the context's dtype.
 *
 * moe_sr_keep_count: k = max(1, floor(n / cr)); 0 if n < 1 or cr < 1.  Host only.
 *
 * moe_sr_encode: expert, shared [dev][n] dtype in (16-byte aligned); values [dev][k] dtype
 * and indices [dev][k] int32 out: the k entries with the largest |expert - shared| (float32
 * difference of the stored values; equal magnitudes: lower index first), ordered by
 * ascending index; values = that difference rounded to dtype.  1 <= k <= n.  Exact
 * (radix select), deterministic.  Uses a workspace in the context that grows with the
 * largest n seen (the growing call allocates and synchronises the device).
 *
 * moe_sr_decode: shared [dev][n] in, values/indices [dev][k] in (indices ascending, in
 * [0, n)), expert_out [dev][n] out (16-byte aligned, must not alias shared):
 * expert_out[i] = shared[i], except expert_out[indices[j]] = shared[indices[j]] + values[j]
 * (float32 add, rounded once to dtype).  Entries with an index outside [0, n) or out of
 * order may be ignored; nothing outside expert_out[0..n) is written. */
int64_t moe_sr_keep_count(int64_t n, int32_t cr);
int moe_sr_encode(moe_ctx* ctx, const void* expert, const void* shared, int64_t n, int64_t k,
                  void* values, int32_t* indices, void* stream);
int moe_sr_decode(moe_ctx* ctx, const void* shared, const void* values, const int32_t* indices,
                  int64_t n, int64_t k, void* expert_out, void* stream);

/* ---- Chunked overlap schedule of the forward path --------------------------------------
 * (Sec. 3.2, stream model: the computation stream and the communication streams work on
 * different chunks of a layer's data at the same time; Fig. "overlap".)  The T tokens of a
 * call are cut into n_chunks contiguous chunks of chunk_tokens = the next multiple of 4 of
 * ceil(T / n_chunks) tokens (the last chunk takes the rest, possibly none); chunk c runs
 * moe_route -> moe_dispatch -> moe_expert_ffn -> moe_combine on internal stream
 * c mod n_streams, which has a context of its own.  On one GPU there are no transfers: what
 * overlaps is the HBM-bound work of one chunk with the expert GEMMs of another.  The result
 * is that of the four calls made per chunk: every chunk has its own packed layout.
 *
 * moe_pipeline_create: cfg as for moe_create with cfg->T_max = most tokens of one call;
 * 1 <= n_chunks <= 64, 1 <= n_streams <= 8 (streams of default priority, created here).
 * moe_pipeline_chunk_range: [host] the token range [*t_begin, *t_end) of a chunk for a call
 * with T tokens.
 * moe_pipeline_forward: x [dev][T,d], Wg, bias, W1/W3/W2 as in moe_route / moe_expert_ffn
 * (W3 == NULL: two-matrix expert).  Outputs, all [dev], caller-owned, chunk c at token
 * offset t_begin(c) (slot / packed-row offset t_begin(c)*k), row numbers relative to the
 * chunk: topk_idx, topk_w [T,k]; x_packed, y_packed [T*k,d]; slot_to_row, row_to_slot [T*k];
 * expert_counts, expert_offsets [n_chunks][E]; rank_counts [n_chunks][R]; rank_offsets
 * [n_chunks][R+1]; out [T,d].  y_packed rows of experts without weights are left as the
 * caller filled them (rows "received back").  The work is ordered after everything queued
 * on `stream` before the call, and `stream` waits for it: no host synchronisation.  Calls
 * on one pipeline must not overlap each other.  Errors as for the four calls; after an
 * error the streams are still joined. */
typedef struct moe_pipeline moe_pipeline;
int moe_pipeline_create(moe_pipeline** out, const moe_config* cfg, int32_t n_chunks,
                        int32_t n_streams);
int moe_pipeline_destroy(moe_pipeline* pipe);
int moe_pipeline_set_placement(moe_pipeline* pipe, const int32_t* expert_dest_rank /*[host][E]*/);
int moe_pipeline_chunk_range(const moe_pipeline* pipe, int32_t T, int32_t chunk,
                             int32_t* t_begin, int32_t* t_end);
int moe_pipeline_forward(moe_pipeline* pipe, const void* x, const void* Wg, const float* bias,
                         int32_t T, const void* const* W1, const void* const* W3,
                         const void* const* W2, int32_t* topk_idx, float* topk_w, void* x_packed,
                         int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                         int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                         void* y_packed, void* out, void* stream);

/* Measurement aid.  moe_profile_ffn(ctx, n_calls) makes the next n_calls calls of
 * moe_expert_ffn record HIP events on their stream around each internal launch
 * (n_calls = 0 switches it off and frees the events; creates events, so not for use
 * under graph capture).  moe_profile_ffn_read synchronises with those events and returns
 * the average duration in milliseconds of each launch over the recorded calls:
 * ms[0] tile schedule, ms[1] gate/up GEMM (+SwiGLU), ms[2] down GEMM; *n_recorded = calls
 * averaged.  ms [host][MOE_PROF_SLOTS].
 * moe_profile_ffn_launches(ctx, mask) restricts the timing to the launches whose bit is set
 * (bit 0 schedule, 1 gate/up, 2 down; default all): an event record costs a few microseconds
 * of idle GPU, so a caller that times a whole step wants only the launch it reports; the
 * others read as 0.  MOE_EINVAL for an empty mask or while calls are recorded and not read. */
#define MOE_PROF_SLOTS 3
int moe_profile_ffn(moe_ctx* ctx, int32_t n_calls);
int moe_profile_ffn_launches(moe_ctx* ctx, int32_t mask);
int moe_profile_ffn_read(moe_ctx* ctx, float* ms, int32_t* n_recorded);

/* Measured ceilings for the roofline report (Sec. 3.1 prices a GeMM with the compute
 * efficiency C of the device: these two kernels measure what the device gives a kernel that
 * does nothing but copy, or nothing but issue matrix instructions).
 * moe_measure_copy: one launch that reads `bytes` (a multiple of 16) from src once and writes
 * them to `fanout` (1..16) consecutive copies in dst (fanout * bytes, no overlap with src);
 * both [dev], 16-byte aligned.
 * moe_measure_mfma: one launch of `blocks` blocks of 8 wavefronts that each issue
 * iters * 32 v_mfma_f32_32x32x16_bf16 from registers (operands zero, or varied bf16 values
 * with random_operands != 0); sink [dev][blocks * 512] floats receives a checksum;
 * *flops_out [host] (may be NULL) = the floating-point operations of the launch. */
int moe_measure_copy(const void* src, void* dst, int64_t bytes, int32_t fanout, void* stream);
int moe_measure_mfma(float* sink, int32_t blocks, int32_t iters, int32_t random_operands,
                     double* flops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HOTPATH_MOE_H */
