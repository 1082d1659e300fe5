// Chunked overlap schedule of the forward path (paper Sec. 3.2, stream model: the computation
// stream and the communication streams work on different chunks of the data at the same time;
// Fig. "overlap" shows the chunks of one layer in flight together).  On one GPU the transfers
// are absent, so what overlaps is the HBM-bound part of one chunk (gating, dispatch, combine)
// with the matrix-core part (expert GEMMs) of another: the T tokens are cut into contiguous
// chunks, chunk c runs moe_route -> moe_dispatch -> moe_expert_ffn -> moe_combine on internal
// stream c mod n_streams with that stream's own context (workspace), and the caller's stream
// is forked into / joined from the internal streams with events.  Host code only: every step
// is one of the library's own calls.
#include <algorithm>
#include <new>
#include <vector>

#include "moe_internal.h"

struct moe_pipeline {
  moe_config cfg;          // cfg.T_max: most tokens of one call (all chunks together)
  int n_chunks, n_streams;
  int chunk_max;           // tokens a chunk can hold
  int elem;
  std::vector<moe_ctx*> ctx;
  std::vector<hipStream_t> streams;
  std::vector<hipEvent_t> done;
  hipEvent_t fork;
};

namespace {

// Chunks are equal, a multiple of 4 tokens (every chunk's slices of the caller's buffers stay
// 16-byte aligned), the last one takes what is left (possibly nothing).
int chunk_tokens(int T, int n_chunks) {
  const int per = (T + n_chunks - 1) / n_chunks;
  return ((per + 3) / 4) * 4;
}

void destroy(moe_pipeline* p) {
  for (moe_ctx* c : p->ctx) (void)moe_destroy(c);
  for (hipStream_t s : p->streams) (void)hipStreamDestroy(s);
  for (hipEvent_t e : p->done) (void)hipEventDestroy(e);
  if (p->fork != nullptr) (void)hipEventDestroy(p->fork);
  delete p;
}

}  // namespace

extern "C" {

int moe_pipeline_create(moe_pipeline** out, const moe_config* cfg, int32_t n_chunks,
                        int32_t n_streams) {
  if (out == nullptr) return MOE_EINVAL;
  *out = nullptr;
  if (cfg == nullptr || n_chunks < 1 || n_chunks > 64 || n_streams < 1 || n_streams > 8 ||
      cfg->T_max < 0)
    return MOE_EINVAL;
  moe_pipeline* p = new (std::nothrow) moe_pipeline();
  if (p == nullptr) return MOE_ENOMEM;
  p->cfg = *cfg;
  p->n_chunks = n_chunks;
  p->n_streams = std::min(n_streams, n_chunks);
  p->chunk_max = chunk_tokens(cfg->T_max, n_chunks);
  p->elem = cfg->dtype == MOE_BF16 ? 2 : 4;
  p->fork = nullptr;
  moe_config cc = *cfg;
  cc.T_max = p->chunk_max;
  for (int i = 0; i < p->n_streams; ++i) {
    moe_ctx* c = nullptr;
    const int st = moe_create(&c, &cc);
    if (st != MOE_OK) {
      destroy(p);
      return st;
    }
    p->ctx.push_back(c);
    hipStream_t s = nullptr;
    hipEvent_t e = nullptr;
    // default priority on purpose; non-blocking: no implicit ordering with the null stream
    if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) {
      destroy(p);
      return MOE_EHIP;
    }
    p->streams.push_back(s);
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
      destroy(p);
      return MOE_EHIP;
    }
    p->done.push_back(e);
  }
  if (hipEventCreateWithFlags(&p->fork, hipEventDisableTiming) != hipSuccess) {
    p->fork = nullptr;
    destroy(p);
    return MOE_EHIP;
  }
  *out = p;
  return MOE_OK;
}

int moe_pipeline_destroy(moe_pipeline* p) {
  if (p == nullptr) return MOE_OK;
  (void)hipDeviceSynchronize();
  destroy(p);
  return MOE_OK;
}

int moe_pipeline_set_placement(moe_pipeline* p, const int32_t* expert_dest_rank) {
  if (p == nullptr) return MOE_EINVAL;
  for (moe_ctx* c : p->ctx) {
    const int st = moe_set_placement(c, expert_dest_rank);
    if (st != MOE_OK) return st;
  }
  return MOE_OK;
}

int moe_pipeline_chunk_range(const moe_pipeline* p, int32_t T, int32_t chunk, int32_t* t_begin,
                             int32_t* t_end) {
  if (p == nullptr || t_begin == nullptr || t_end == nullptr || T < 0 || T > p->cfg.T_max ||
      chunk < 0 || chunk >= p->n_chunks)
    return MOE_EINVAL;
  const int per = chunk_tokens(T, p->n_chunks);
  *t_begin = std::min(T, chunk * per);
  *t_end = std::min(T, (chunk + 1) * per);
  return MOE_OK;
}

int moe_pipeline_forward(moe_pipeline* p, const void* x, const void* Wg, const float* bias,
                         int32_t T, const void* const* W1, const void* const* W3,
                         const void* const* W2, int32_t* topk_idx, float* topk_w, void* x_packed,
                         int32_t* slot_to_row, int32_t* row_to_slot, int32_t* expert_counts,
                         int32_t* expert_offsets, int32_t* rank_counts, int32_t* rank_offsets,
                         void* y_packed, void* out, void* stream) {
  if (p == nullptr || T < 0 || T > p->cfg.T_max) return MOE_EINVAL;
  if (expert_counts == nullptr || expert_offsets == nullptr || rank_counts == nullptr ||
      rank_offsets == nullptr)
    return MOE_EINVAL;
  if (T > 0 && (x == nullptr || Wg == nullptr || topk_idx == nullptr || topk_w == nullptr ||
                x_packed == nullptr || slot_to_row == nullptr || row_to_slot == nullptr ||
                y_packed == nullptr || out == nullptr))
    return MOE_EINVAL;
  hipStream_t user = (hipStream_t)stream;
  const int E = p->cfg.E, R = p->cfg.R, k = p->cfg.k, d = p->cfg.d;
  const size_t row_bytes = (size_t)d * p->elem;
  if (hipEventRecord(p->fork, user) != hipSuccess) return MOE_EHIP;
  for (int i = 0; i < p->n_streams; ++i)
    if (hipStreamWaitEvent(p->streams[i], p->fork, 0) != hipSuccess) return MOE_EHIP;
  int status = MOE_OK;
  for (int c = 0; c < p->n_chunks && status == MOE_OK; ++c) {
    int32_t t0 = 0, t1 = 0;
    (void)moe_pipeline_chunk_range(p, T, c, &t0, &t1);
    const int Tc = t1 - t0;
    // an empty chunk (T below the chunk count's reach) starts at T, which need not be a multiple
    // of 4: its calls write only the per-chunk counts, so they get the buffers' own (aligned)
    // addresses
    if (Tc == 0) t0 = 0;
    moe_ctx* ctx = p->ctx[c % p->n_streams];
    hipStream_t s = p->streams[c % p->n_streams];
    const size_t s0 = (size_t)t0 * k;   // first slot (= first packed row) of the chunk
    const char* xc = (const char*)x + (size_t)t0 * row_bytes;
    int32_t* idx = topk_idx + s0;
    float* w = topk_w + s0;
    char* xp = (char*)x_packed + s0 * row_bytes;
    char* yp = (char*)y_packed + s0 * row_bytes;
    int32_t* cnt = expert_counts + (size_t)c * E;
    int32_t* off = expert_offsets + (size_t)c * E;
    status = moe_route(ctx, xc, Wg, bias, Tc, nullptr, idx, w, s);
    if (status == MOE_OK)
      status = moe_dispatch_routed(ctx, Tc > 0 ? xc : nullptr, idx, Tc, Tc > 0 ? xp : nullptr,
                            slot_to_row + s0, row_to_slot + s0, cnt, off,
                            rank_counts + (size_t)c * R, rank_offsets + (size_t)c * (R + 1), s);
    if (status == MOE_OK)
      status = moe_expert_ffn(ctx, xp, cnt, off, W1, W3, W2, Tc, yp, nullptr, nullptr, s);
    if (status == MOE_OK)
      status = moe_combine(ctx, yp, slot_to_row + s0, w, Tc, (char*)out + (size_t)t0 * row_bytes, s);
  }
  // join even after an error: the caller's stream must not run ahead of work already queued
  for (int i = 0; i < p->n_streams; ++i) {
    if (hipEventRecord(p->done[i], p->streams[i]) != hipSuccess ||
        hipStreamWaitEvent(user, p->done[i], 0) != hipSuccess)
      return status != MOE_OK ? status : MOE_EHIP;
  }
  return status;
}

}  // extern "C"
