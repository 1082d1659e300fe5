// Host side of the C ABI: argument validation, the context and its device workspace,
// and the launches.  No entry point synchronises with the device except moe_create,
// moe_destroy and moe_set_placement.
#include <algorithm>
#include <cstring>
#include <new>

#include "moe_internal.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename T>
hipError_t dev_alloc(T** p, size_t n) {
  return hipMalloc(reinterpret_cast<void**>(p), std::max<size_t>(n, 1) * sizeof(T));
}

void free_all(moe_ctx* c) {
  (void)hipFree(c->d_dest_rank);
  (void)hipFree(c->d_seg_pos);
  (void)hipFree(c->d_chunk_hist);
  (void)hipFree(c->d_totals);
  (void)hipFree(c->d_logits);
  (void)hipFree(c->d_rt_rank);
  (void)hipFree(c->d_rt_hist);
  (void)hipFree(c->d_rt_super);
  (void)hipFree(c->d_wtab);
  for (int i = 0; i < 2; ++i) {
    (void)hipFree(c->d_sched[i]);
    (void)hipFree(c->d_mtiles[i]);
  }
  (void)hipFree(c->d_order_up);
  (void)hipFree(c->d_order_down);
  (void)hipFree(c->d_split_ws);
  (void)hipFree(c->d_sr_ws);
  (void)hipFree(c->d_rbwd_ws);
  (void)hipFree(c->d_H);
  (void)hipFree(c->d_dG);
  (void)hipFree(c->d_dU);
  (void)hipFree(c->d_dGU);
  (void)hipFree(c->d_zero);
}

int check_ctx_T(const moe_ctx* c, int32_t T) {
  if (c == nullptr) return MOE_EINVAL;
  if (T < 0 || T > c->cfg.T_max) return MOE_EINVAL;
  return MOE_OK;
}

// Refresh the device copy of the pointer tables when the host tables changed.
// rows: 0 W1, 1 W3, 2 W2, 3 dW1, 4 dW3, 5 dW2; a NULL table leaves its row as it is.
int sync_tables(moe_ctx* c, const void* const* const tabs[MOE_WTAB_ROWS], hipStream_t s) {
  const int E = c->cfg.E;
  bool changed = !c->wtab_valid;
  for (int r = 0; r < MOE_WTAB_ROWS; ++r) {
    if (tabs[r] == nullptr) continue;
    if (std::memcmp(c->h_wtab[r], tabs[r], sizeof(void*) * E) != 0) {
      std::memcpy(c->h_wtab[r], tabs[r], sizeof(void*) * E);
      changed = true;
    }
  }
  if (changed) {
    if (hipMemcpyAsync(c->d_wtab, c->h_wtab, sizeof(c->h_wtab), hipMemcpyHostToDevice, s) !=
        hipSuccess)
      return MOE_EHIP;
    c->wtab_valid = 1;
  }
  return MOE_OK;
}

// W3 == nullptr (the whole table): two-matrix experts, present with both matrices or none.
int check_weight_tables(const moe_ctx* c, const void* const* W1, const void* const* W3,
                        const void* const* W2, bool allow_two_matrix = false) {
  if (W1 == nullptr || W2 == nullptr) return MOE_EINVAL;
  if (W3 == nullptr && !allow_two_matrix) return MOE_EINVAL;
  const int want = W3 != nullptr ? 3 : 2;
  for (int e = 0; e < c->cfg.E; ++e) {
    const void* w3 = W3 != nullptr ? W3[e] : nullptr;
    const int n = (W1[e] != nullptr) + (w3 != nullptr) + (W2[e] != nullptr);
    if (n != 0 && n != want) return MOE_EINVAL;  // an expert is present with all or none
    if (!aligned16(W1[e]) || !aligned16(w3) || !aligned16(W2[e])) return MOE_EINVAL;
  }
  return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_strerror(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_EINVAL: return "invalid argument";
    case MOE_EUNSUPPORTED: return "unsupported configuration";
    case MOE_ENOMEM: return "out of device memory";
    case MOE_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int moe_create(moe_ctx** out, const moe_config* cfg) {
  if (out == nullptr) return MOE_EINVAL;
  *out = nullptr;
  if (cfg == nullptr) return MOE_EINVAL;
  if (cfg->dtype != MOE_F32 && cfg->dtype != MOE_BF16) return MOE_EINVAL;
  if (cfg->E < 1 || cfg->E > MOE_MAX_EXPERTS) return MOE_EINVAL;
  if (cfg->k < 1 || cfg->k > cfg->E || cfg->k > MOE_MAX_TOPK) return MOE_EINVAL;
  if (cfg->R < 1 || cfg->R > MOE_MAX_RANKS) return MOE_EINVAL;
  if (cfg->local_rank < 0 || cfg->local_rank >= cfg->R) return MOE_EINVAL;
  if (cfg->T_max < 0 || cfg->d < 8 || cfg->f < 8) return MOE_EINVAL;
  if (cfg->d % 8 != 0 || cfg->f % 8 != 0) return MOE_EINVAL;
  if (cfg->renormalize != 0 && cfg->renormalize != 1) return MOE_EINVAL;
  const long long S = (long long)cfg->T_max * cfg->k;
  if (S > (1ll << 22)) return MOE_EUNSUPPORTED;                           // grid / int32 headroom
  if (S * std::max(cfg->d, cfg->f) > (1ll << 40)) return MOE_EUNSUPPORTED;

  moe_ctx* c = new (std::nothrow) moe_ctx();
  if (c == nullptr) return MOE_ENOMEM;
  std::memset(c, 0, sizeof(*c));
  c->cfg = *cfg;
  c->elem = cfg->dtype == MOE_BF16 ? 2 : 4;
  c->ffn_path = MOE_FFN_AUTO;
  c->S_max = (int32_t)S;
  if (hipGetDevice(&c->device) != hipSuccess ||
      hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device) !=
          hipSuccess) {
    delete c;
    return MOE_EHIP;
  }
  (void)dispatch_noalloc_init();   // so that moe_dispatch_noalloc need not do it under a capture
  const int E = cfg->E;
  c->n_chunks_max = std::max<int>(1, (int)((S + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK));
  c->max_mtiles[0] = (int)(S / GENERIC_BM) + E;
  c->max_mtiles[1] = (int)(S / MFMA_BM) + E;
  bool ok = true;
  ok = ok && dev_alloc(&c->d_dest_rank, E) == hipSuccess;
  ok = ok && dev_alloc(&c->d_seg_pos, E) == hipSuccess;
  ok = ok && dev_alloc(&c->d_chunk_hist, (size_t)c->n_chunks_max * E) == hipSuccess;
  ok = ok && dev_alloc(&c->d_totals, 2 * MOE_MAX_EXPERTS + 2) == hipSuccess;
  ok = ok && dev_alloc(&c->d_logits, (size_t)cfg->T_max * E) == hipSuccess;
  ok = ok && dev_alloc(&c->d_wtab, MOE_WTAB_ROWS * MOE_MAX_EXPERTS) == hipSuccess;
  for (int i = 0; i < 2 && ok; ++i) {
    ok = ok && dev_alloc(&c->d_sched[i], 1) == hipSuccess;
    ok = ok && dev_alloc(&c->d_mtiles[i], c->max_mtiles[i]) == hipSuccess;
  }
  if (ok && ffn_mfma_supported(c)) {
    const size_t n = ffn_mfma_order_entries(c);
    ok = ok && dev_alloc(&c->d_order_up, n) == hipSuccess;
    ok = ok && dev_alloc(&c->d_order_down, n) == hipSuccess;
    ok = ok && dev_alloc(&c->d_split_ws, (size_t)c->n_cu * MFMA_BM * 256) == hipSuccess;
  }
  // side products of the fused gate kernel (moe_dispatch_routed); left out when the gate is
  // not fused for this configuration or the histograms would be large
  const long long n_blk = ((long long)cfg->T_max + GATE_BLOCK_TOKENS - 1) / GATE_BLOCK_TOKENS;
  if (ok && gate_route_fused_supported(c) && cfg->T_max <= (1 << 17) && n_blk * E <= (1 << 22)) {
    c->rt_super_max = (int32_t)((n_blk + RT_SUPER - 1) / RT_SUPER);
    const size_t n_sup = (size_t)2 * ((size_t)c->rt_super_max * E + (size_t)E * RT_TOT_STRIDE);
    ok = ok && dev_alloc(&c->d_rt_rank, (size_t)S) == hipSuccess;
    ok = ok && dev_alloc(&c->d_rt_hist, (size_t)n_blk * E) == hipSuccess;
    ok = ok && dev_alloc(&c->d_rt_super, n_sup) == hipSuccess;
    ok = ok && hipMemset(c->d_rt_super, 0, n_sup * sizeof(int32_t)) == hipSuccess;
  }
  ok = ok && hipMalloc(&c->d_H, std::max<size_t>((size_t)S * cfg->f * c->elem, 16)) == hipSuccess;
  ok = ok && hipMemset(c->d_totals, 0, sizeof(int32_t) * (2 * MOE_MAX_EXPERTS + 2)) == hipSuccess;
  ok = ok && hipMemset(c->d_wtab, 0, sizeof(void*) * MOE_WTAB_ROWS * MOE_MAX_EXPERTS) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    free_all(c);
    delete c;
    return MOE_ENOMEM;
  }
  int32_t dest[MOE_MAX_EXPERTS];
  const int per = (E + cfg->R - 1) / cfg->R;
  for (int e = 0; e < E; ++e) dest[e] = e / per;
  const int st = moe_set_placement(c, dest);
  if (st != MOE_OK) {
    free_all(c);
    delete c;
    return st;
  }
  *out = c;
  return MOE_OK;
}

int moe_profile_ffn(moe_ctx* c, int32_t n_calls) {
  if (c == nullptr || n_calls < 0 || n_calls > 4096) return MOE_EINVAL;
  if (c->prof_ev != nullptr) {
    (void)hipDeviceSynchronize();
    for (size_t i = 0; i < (size_t)c->prof_calls * (MOE_PROF_SLOTS + 1); ++i)
      (void)hipEventDestroy(c->prof_ev[i]);
    delete[] c->prof_ev;
    c->prof_ev = nullptr;
  }
  c->prof_calls = 0;
  c->prof_n = 0;
  if (n_calls == 0) return MOE_OK;
  const size_t n = (size_t)n_calls * (MOE_PROF_SLOTS + 1);
  c->prof_ev = new (std::nothrow) hipEvent_t[n];
  if (c->prof_ev == nullptr) return MOE_ENOMEM;
  for (size_t i = 0; i < n; ++i)
    if (hipEventCreate(&c->prof_ev[i]) != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(c->prof_ev[j]);
      delete[] c->prof_ev;
      c->prof_ev = nullptr;
      return MOE_EHIP;
    }
  c->prof_calls = n_calls;
  if (c->prof_mask == 0) c->prof_mask = (1 << MOE_PROF_SLOTS) - 1;
  return MOE_OK;
}

int moe_profile_ffn_launches(moe_ctx* c, int32_t mask) {
  if (c == nullptr || mask < 1 || mask >= (1 << MOE_PROF_SLOTS) || c->prof_n != 0) return MOE_EINVAL;
  c->prof_mask = mask;
  return MOE_OK;
}

int moe_profile_ffn_read(moe_ctx* c, float* ms, int32_t* n_recorded) {
  if (c == nullptr || ms == nullptr || n_recorded == nullptr) return MOE_EINVAL;
  for (int i = 0; i < MOE_PROF_SLOTS; ++i) ms[i] = 0.f;
  *n_recorded = c->prof_n;
  if (c->prof_n == 0) return MOE_OK;
  int last = 0;   // last event recorded in a call
  for (int i = 0; i < MOE_PROF_SLOTS; ++i)
    if ((c->prof_mask >> i) & 1) last = i + 1;
  for (int call = 0; call < c->prof_n; ++call) {
    hipEvent_t* ev = c->prof_ev + (size_t)call * (MOE_PROF_SLOTS + 1);
    if (hipEventSynchronize(ev[last]) != hipSuccess) return MOE_EHIP;
    for (int i = 0; i < MOE_PROF_SLOTS; ++i) {
      if (!((c->prof_mask >> i) & 1)) continue;
      float t = 0.f;
      if (hipEventElapsedTime(&t, ev[i], ev[i + 1]) != hipSuccess) return MOE_EHIP;
      ms[i] += t;
    }
  }
  for (int i = 0; i < MOE_PROF_SLOTS; ++i) ms[i] /= (float)c->prof_n;
  c->prof_n = 0;
  return MOE_OK;
}

int64_t moe_sr_keep_count(int64_t n, int32_t cr) {
  if (n < 1 || cr < 1) return 0;
  const int64_t k = n / cr;
  return k < 1 ? 1 : k;
}

int moe_sr_encode(moe_ctx* c, const void* expert, const void* shared, int64_t n, int64_t k,
                  void* values, int32_t* indices, void* stream) {
  if (c == nullptr || expert == nullptr || shared == nullptr || values == nullptr ||
      indices == nullptr)
    return MOE_EINVAL;
  if (n < 1 || n > 0x7fffffffLL || k < 1 || k > n) return MOE_EINVAL;
  if (!aligned16(expert) || !aligned16(shared)) return MOE_EINVAL;
  const size_t need = sr_workspace_ints(n);
  if (need > c->sr_ws_ints) {   // grow the workspace (synchronises: earlier calls may use it)
    (void)hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(c->d_sr_ws);
    c->d_sr_ws = nullptr;
    c->sr_ws_ints = 0;
    if (hipMalloc(reinterpret_cast<void**>(&c->d_sr_ws), need * sizeof(int32_t)) != hipSuccess) {
      (void)hipGetLastError();
      return MOE_ENOMEM;
    }
    if (hipMemset(c->d_sr_ws, 0, need * sizeof(int32_t)) != hipSuccess) return MOE_EHIP;
    c->sr_ws_ints = need;
  }
  return launch_sr_encode(c, expert, shared, n, k, values, indices, (hipStream_t)stream);
}

int moe_sr_decode(moe_ctx* c, const void* shared, const void* values, const int32_t* indices,
                  int64_t n, int64_t k, void* expert_out, void* stream) {
  if (c == nullptr || shared == nullptr || values == nullptr || indices == nullptr ||
      expert_out == nullptr)
    return MOE_EINVAL;
  if (n < 1 || n > 0x7fffffffLL || k < 1 || k > n) return MOE_EINVAL;
  if (!aligned16(shared) || !aligned16(expert_out) || shared == expert_out) return MOE_EINVAL;
  return launch_sr_decode(c, shared, values, indices, n, k, expert_out, (hipStream_t)stream);
}

int moe_destroy(moe_ctx* c) {
  if (c == nullptr) return MOE_OK;
  (void)hipDeviceSynchronize();
  (void)moe_profile_ffn(c, 0);
  free_all(c);
  delete c;
  return MOE_OK;
}

int moe_set_placement(moe_ctx* c, const int32_t* expert_dest_rank) {
  if (c == nullptr || expert_dest_rank == nullptr) return MOE_EINVAL;
  const int E = c->cfg.E;
  for (int e = 0; e < E; ++e)
    if (expert_dest_rank[e] < 0 || expert_dest_rank[e] >= c->cfg.R) return MOE_EINVAL;
  int32_t order[MOE_MAX_EXPERTS];
  for (int e = 0; e < E; ++e) order[e] = e;
  std::stable_sort(order, order + E, [&](int a, int b) {
    return expert_dest_rank[a] < expert_dest_rank[b];
  });
  int32_t pos[MOE_MAX_EXPERTS];   // expert id -> position in (dest_rank, id) order
  for (int i = 0; i < E; ++i) pos[order[i]] = i;
  if (hipMemcpy(c->d_dest_rank, expert_dest_rank, sizeof(int32_t) * E, hipMemcpyHostToDevice) !=
          hipSuccess ||
      hipMemcpy(c->d_seg_pos, pos, sizeof(int32_t) * E, hipMemcpyHostToDevice) != hipSuccess)
    return MOE_EHIP;
  return MOE_OK;
}

int moe_set_ffn_path(moe_ctx* c, int path) {
  if (c == nullptr || (path != MOE_FFN_AUTO && path != MOE_FFN_VALU)) return MOE_EINVAL;
  c->ffn_path = path;
  return MOE_OK;
}

int moe_route_logits(moe_ctx* c, const float* logits, int32_t T, int32_t* topk_idx, float* topk_w,
                     void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (logits == nullptr || topk_idx == nullptr || topk_w == nullptr) return MOE_EINVAL;
  if (!aligned16(logits) || !aligned16(topk_idx) || !aligned16(topk_w)) return MOE_EINVAL;
  return launch_route_select(c, logits, T, topk_idx, topk_w, (hipStream_t)stream);
}

int moe_route(moe_ctx* c, const void* x, const void* Wg, const float* bias, int32_t T,
              float* logits, int32_t* topk_idx, float* topk_w, void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (x == nullptr || Wg == nullptr || topk_idx == nullptr || topk_w == nullptr) return MOE_EINVAL;
  if (!aligned16(x) || !aligned16(Wg) || !aligned16(bias) || !aligned16(logits) ||
      !aligned16(topk_idx) || !aligned16(topk_w))
    return MOE_EINVAL;
  c->rt_valid = 0;
  if (gate_route_fused_supported(c)) {  // one launch, logits only written when asked for
    // The counting step of the dispatch rides along unless the stream is being captured: the
    // buffer the sums go to alternates from call to call on the host, and a replayed graph
    // would add into the same buffer every time.
    bool keep = c->d_rt_rank != nullptr;
    if (keep) {
      hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing((hipStream_t)stream, &cs) != hipSuccess) {
        (void)hipGetLastError();
        keep = false;
      } else if (cs != hipStreamCaptureStatusNone) {
        keep = false;
      }
    }
    if (keep) c->rt_parity ^= 1;
    st = launch_gate_route_fused(c, x, Wg, bias, T, logits, topk_idx, topk_w, keep,
                                 (hipStream_t)stream);
    if (keep) {
      // the launch adds into rows [0, n_sup) of buffer rt_parity and has cleared every row of
      // the other buffer that could hold sums
      const int n_blk = (T + GATE_BLOCK_TOKENS - 1) / GATE_BLOCK_TOKENS;
      c->rt_dirty[c->rt_parity] = std::max(c->rt_dirty[c->rt_parity], (n_blk + RT_SUPER - 1) / RT_SUPER);
      if (st == MOE_OK) c->rt_dirty[c->rt_parity ^ 1] = 0;
    }
    if (st == MOE_OK && keep) {
      c->rt_valid = 1;
      c->rt_idx = topk_idx;
      c->rt_T = T;
    }
    return st;
  }
  float* L = logits != nullptr ? logits : c->d_logits;
  st = launch_gate_logits(c, x, Wg, bias, T, L, (hipStream_t)stream);
  if (st != MOE_OK) return st;
  return launch_route_select(c, L, T, topk_idx, topk_w, (hipStream_t)stream);
}

int moe_dispatch(moe_ctx* c, const void* x, const int32_t* topk_idx, int32_t T, void* x_packed,
                 int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                 int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                 void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (expert_counts == nullptr || expert_offsets == nullptr || rank_counts == nullptr ||
      rank_offsets == nullptr)
    return MOE_EINVAL;
  if ((x == nullptr) != (x_packed == nullptr)) return MOE_EINVAL;
  if (T > 0 && (topk_idx == nullptr || slot_to_row == nullptr || row_to_slot == nullptr))
    return MOE_EINVAL;
  if (!aligned16(x) || !aligned16(x_packed) || !aligned16(topk_idx) || !aligned16(slot_to_row) ||
      !aligned16(row_to_slot))
    return MOE_EINVAL;
  return launch_dispatch(c, x, topk_idx, T, x_packed, slot_to_row, row_to_slot, expert_counts,
                         expert_offsets, rank_counts, rank_offsets, (hipStream_t)stream);
}

int moe_dispatch_routed(moe_ctx* c, const void* x, const int32_t* topk_idx, int32_t T,
                        void* x_packed, int32_t* slot_to_row, int32_t* row_to_slot,
                        int32_t* expert_counts, int32_t* expert_offsets, int32_t* rank_counts,
                        int32_t* rank_offsets, void* stream) {
  if (c == nullptr) return MOE_EINVAL;
  const bool routed = c->rt_valid && T > 0 && c->rt_idx == topk_idx && c->rt_T == T;
  if (!routed)
    return moe_dispatch(c, x, topk_idx, T, x_packed, slot_to_row, row_to_slot, expert_counts,
                        expert_offsets, rank_counts, rank_offsets, stream);
  if (expert_counts == nullptr || expert_offsets == nullptr || rank_counts == nullptr ||
      rank_offsets == nullptr || slot_to_row == nullptr || row_to_slot == nullptr)
    return MOE_EINVAL;
  if ((x == nullptr) != (x_packed == nullptr)) return MOE_EINVAL;
  if (!aligned16(x) || !aligned16(x_packed) || !aligned16(slot_to_row) || !aligned16(row_to_slot))
    return MOE_EINVAL;
  return launch_dispatch_routed(c, x, topk_idx, T, x_packed, slot_to_row, row_to_slot,
                                expert_counts, expert_offsets, rank_counts, rank_offsets,
                                (hipStream_t)stream);
}

int moe_expert_ffn(moe_ctx* c, const void* x_packed, const int32_t* expert_counts,
                   const int32_t* expert_offsets, const void* const* W1, const void* const* W3,
                   const void* const* W2, int32_t T, void* y_packed, void* G_save, void* U_save,
                   void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  const bool gated = W3 != nullptr;
  st = check_weight_tables(c, W1, W3, W2, /*allow_two_matrix=*/true);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (x_packed == nullptr || y_packed == nullptr || expert_counts == nullptr ||
      expert_offsets == nullptr)
    return MOE_EINVAL;
  if (gated && (G_save == nullptr) != (U_save == nullptr)) return MOE_EINVAL;
  if (!gated && U_save != nullptr) return MOE_EINVAL;
  if (!aligned16(x_packed) || !aligned16(y_packed) || !aligned16(G_save) || !aligned16(U_save))
    return MOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  c->S_call = T * c->cfg.k;   // the schedule kernel checks counts and offsets against it
  const void* const* tabs[MOE_WTAB_ROWS] = {W1, W3, W2, nullptr, nullptr, nullptr};
  st = sync_tables(c, tabs, s);
  if (st != MOE_OK) return st;
  if (c->ffn_path == MOE_FFN_AUTO && (gated ? ffn_mfma_supported(c) : ffn_mfma_supported_2mat(c))) {
    st = launch_ffn_mfma(c, gated, expert_counts, expert_offsets, x_packed, y_packed, G_save, U_save,
                         s);
  } else {
    prof_mark(c, 0, s);
    st = launch_build_sched(c, expert_counts, expert_offsets, 0, s);
    if (st != MOE_OK) return st;
    prof_mark(c, 1, s);
    st = launch_ffn_generic(c, gated, x_packed, y_packed, G_save, U_save, c->d_H, s);
  }
  if (c->prof_calls > 0 && c->prof_n < c->prof_calls) c->prof_n++;
  return st;
}

int moe_combine(moe_ctx* c, const void* y_packed, const int32_t* slot_to_row, const float* topk_w,
                int32_t T, void* out, void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (y_packed == nullptr || slot_to_row == nullptr || topk_w == nullptr || out == nullptr)
    return MOE_EINVAL;
  if (!aligned16(y_packed) || !aligned16(out)) return MOE_EINVAL;
  return launch_combine(c, y_packed, slot_to_row, topk_w, T, out, (hipStream_t)stream);
}

int moe_combine_bwd(moe_ctx* c, const void* dout, const void* y_packed, const int32_t* slot_to_row,
                    const float* topk_w, int32_t T, void* dy_packed, float* dtopk_w,
                    void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (dout == nullptr || y_packed == nullptr || slot_to_row == nullptr || topk_w == nullptr ||
      dy_packed == nullptr || dtopk_w == nullptr)
    return MOE_EINVAL;
  if (!aligned16(dout) || !aligned16(y_packed) || !aligned16(dy_packed)) return MOE_EINVAL;
  return launch_combine_bwd(c, dout, y_packed, slot_to_row, topk_w, T, dy_packed, dtopk_w,
                            (hipStream_t)stream);
}

int moe_expert_ffn_bwd(moe_ctx* c, const void* dy_packed, const void* x_packed, const void* G_save,
                       const void* U_save, const int32_t* expert_counts,
                       const int32_t* expert_offsets, const void* const* W1, const void* const* W3,
                       const void* const* W2, int32_t T, void* dx_packed, float* const* dW1,
                       float* const* dW3, float* const* dW2, void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  const bool gated = W3 != nullptr;   // no W3 table: the two-matrix expert
  st = check_weight_tables(c, W1, W3, W2, /*allow_two_matrix=*/true);
  if (st != MOE_OK) return st;
  if (dW1 == nullptr || dW2 == nullptr || (dW3 == nullptr) == gated) return MOE_EINVAL;
  if ((U_save == nullptr) == gated && T > 0) return MOE_EINVAL;
  for (int e = 0; e < c->cfg.E; ++e)
    if (!aligned16(dW1[e]) || (gated && !aligned16(dW3[e])) || !aligned16(dW2[e]))
      return MOE_EINVAL;
  if (T == 0) return MOE_OK;
  if (dy_packed == nullptr || x_packed == nullptr || G_save == nullptr ||
      expert_counts == nullptr || expert_offsets == nullptr || dx_packed == nullptr)
    return MOE_EINVAL;
  if (!aligned16(dy_packed) || !aligned16(x_packed) || !aligned16(G_save) || !aligned16(U_save) ||
      !aligned16(dx_packed))
    return MOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  c->S_call = T * c->cfg.k;   // the schedule kernel checks counts and offsets against it
  const size_t sf_bytes = std::max<size_t>((size_t)c->S_max * c->cfg.f * c->elem, 16);
  if (c->ffn_path == MOE_FFN_AUTO && ffn_bwd_mfma_supported(c)) {
    // first call: allocate the backward workspace
    if (c->d_dGU == nullptr) {
      bool ok = hipMalloc(&c->d_dGU, 2 * sf_bytes) == hipSuccess;
      // the fill runs on the null stream: wait for it, the caller's stream may not
      ok = ok && hipMalloc(&c->d_zero, 512) == hipSuccess &&
           hipMemset(c->d_zero, 0, 512) == hipSuccess && hipStreamSynchronize(nullptr) == hipSuccess;
      if (!ok) {
        (void)hipGetLastError();
        (void)hipFree(c->d_dGU);
        (void)hipFree(c->d_zero);
        c->d_zero = nullptr;
        c->d_dGU = nullptr;
        return MOE_ENOMEM;
      }
    }
    const void* const* tabs[MOE_WTAB_ROWS] = {W1,
                                              W3,
                                              W2,
                                              reinterpret_cast<const void* const*>(dW1),
                                              reinterpret_cast<const void* const*>(dW3),
                                              reinterpret_cast<const void* const*>(dW2)};
    st = sync_tables(c, tabs, s);
    if (st != MOE_OK) return st;
    return launch_ffn_bwd_mfma(c, gated, dy_packed, x_packed, G_save, U_save, expert_counts,
                               expert_offsets, dx_packed, s);
  }
  if (c->d_dG == nullptr) {  // first backward call on this path: allocate the temporaries
    if (hipMalloc(&c->d_dG, sf_bytes) != hipSuccess || hipMalloc(&c->d_dU, sf_bytes) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipFree(c->d_dG);
      c->d_dG = nullptr;
      return MOE_ENOMEM;
    }
  }
  const void* const* tabs[MOE_WTAB_ROWS] = {W1,
                                            W3,
                                            W2,
                                            reinterpret_cast<const void* const*>(dW1),
                                            reinterpret_cast<const void* const*>(dW3),
                                            reinterpret_cast<const void* const*>(dW2)};
  st = sync_tables(c, tabs, s);
  if (st != MOE_OK) return st;
  st = launch_build_sched(c, expert_counts, expert_offsets, 0, s);
  if (st != MOE_OK) return st;
  return launch_ffn_bwd_generic(c, gated, dy_packed, x_packed, G_save, U_save, expert_counts,
                                expert_offsets, dx_packed, c->d_dG, c->d_dU, c->d_H, s);
}

int moe_dispatch_bwd(moe_ctx* c, const void* dx_packed, const int32_t* slot_to_row, int32_t T,
                     void* dx, void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T == 0) return MOE_OK;
  if (dx_packed == nullptr || slot_to_row == nullptr || dx == nullptr) return MOE_EINVAL;
  if (!aligned16(dx_packed) || !aligned16(dx)) return MOE_EINVAL;
  return launch_dispatch_bwd(c, dx_packed, slot_to_row, T, dx, (hipStream_t)stream);
}

int moe_route_bwd(moe_ctx* c, const void* x, const void* Wg, const float* logits,
                  const int32_t* topk_idx, const float* topk_w, const float* dtopk_w, int32_t T,
                  float* dlogits, float* dWg, float* dbias, void* dx, void* stream) {
  int st = check_ctx_T(c, T);
  if (st != MOE_OK) return st;
  if (T > 0 && (topk_idx == nullptr || topk_w == nullptr || dtopk_w == nullptr ||
                dlogits == nullptr))
    return MOE_EINVAL;
  if (T > 0 && c->cfg.renormalize == 0 && logits == nullptr) return MOE_EINVAL;
  if (T > 0 && dWg != nullptr && x == nullptr) return MOE_EINVAL;
  if (T > 0 && dx != nullptr && (Wg == nullptr || !aligned16(dx) || !aligned16(Wg))) return MOE_EINVAL;
  if (T > 0 && dWg != nullptr && c->d_rbwd_ws == nullptr) {
    if (hipMalloc(reinterpret_cast<void**>(&c->d_rbwd_ws),
                  std::max<size_t>(route_bwd_workspace_floats(c), 4) * sizeof(float)) != hipSuccess) {
      (void)hipGetLastError();
      c->d_rbwd_ws = nullptr;
      return MOE_ENOMEM;
    }
  }
  return launch_route_bwd(c, x, Wg, logits, topk_idx, topk_w, dtopk_w, T, dlogits, dWg, dbias, dx,
                          (hipStream_t)stream);
}

}  // extern "C"
