// Stage 1 launcher: the dense indexer score (every score written).
// The kernel is in index_kernel.h.
#include "index_kernel.h"

using namespace ess_idx;

int ess_launch_index_score(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                           const int32_t* ctx_len, int B, int T, float* score, hipStream_t st,
                           const int32_t* block_table, int n_pages, hipEvent_t ev_start, hipEvent_t ev_stop, ess_xcd xcd) {
  IdxArgs a{};
  a.q = q; a.w = w; a.key = key; a.ctx_len = ctx_len; a.score = score;
  a.Lmax = c.max_ctx; a.Hi = c.idx_heads; a.chunk = pick_chunk(B, c.max_ctx);
  a.block_table = block_table; a.n_pages = n_pages;
  a.xcd = xcd; a.nx = (c.max_ctx + a.chunk - 1) / a.chunk; a.nb_seq = B;
  return launch_series<false>(c, T, dim3(a.nx, B), st, a, ev_start, ev_stop);
}
