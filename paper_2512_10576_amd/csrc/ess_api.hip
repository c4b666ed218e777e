// C ABI of libess: argument validation, context life cycle and the stream
// choreography of one layer-step (ESS paper Sec. 3.3: without overlap the
// miss fetch serialises between indexer and attention; with DA overlap Attn0
// over the resident entries runs while the fetch is in flight, Attn1 waits
// for it, and the two are merged).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "index_tile.h"

// Workgroups that Attn0 of the whole batch aims at when entries are offloaded: half a workgroup per CU.  Attn0 runs
// beside a fetch and has time to spare, while every split adds a partial result (128 KiB per row) that the merge,
// which runs after the last fetch, has to read: 128 against 256 took 15 % off Attn0 itself and 0.3-0.7 % off the step.
#ifndef ESS_ATTN0_WGS
#define ESS_ATTN0_WGS 128
#endif

namespace {

thread_local char g_err[512] = "";

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int entry_bytes(int fmt) { return fmt == ESS_FMT_BF16 ? 1152 : 648; }

int validate_config(const ess_config* c) {
  if (!c) return ess_fail(ESS_ERR_INVALID_ARG, "config is NULL");
  if (c->struct_size != sizeof(ess_config))
    return ess_fail(ESS_ERR_INVALID_ARG, "struct_size %u != %zu", c->struct_size, sizeof(ess_config));
  if (c->max_batch < 1 || c->max_batch > 4096) return ess_fail(ESS_ERR_INVALID_ARG, "max_batch %d outside [1, 4096]", c->max_batch);
  if (c->max_q_tokens < 1 || c->max_q_tokens > 4)
    return ess_fail(ESS_ERR_UNSUPPORTED, "max_q_tokens %d (supported: 1 to 4)", c->max_q_tokens);
  if (c->max_ctx < 1 || c->max_ctx > ESS_MAX_CTX)
    return ess_fail(ESS_ERR_INVALID_ARG, "max_ctx %d outside [1, %d]", c->max_ctx, ESS_MAX_CTX);
  if (c->idx_heads < 1 || c->idx_heads > 64)
    return ess_fail(ESS_ERR_UNSUPPORTED, "idx_heads %d outside [1, 64]", c->idx_heads);
  if (c->idx_dim != 32 && c->idx_dim != 64 && c->idx_dim != 128)
    return ess_fail(ESS_ERR_UNSUPPORTED, "idx_dim %d (supported: 32, 64, 128)", c->idx_dim);
  if (c->topk < 1 || c->topk > ESS_MAX_TOPK)
    return ess_fail(ESS_ERR_INVALID_ARG, "topk %d outside [1, %d]", c->topk, ESS_MAX_TOPK);
  if (c->max_q_tokens * c->topk > ESS_MAX_SEL)
    return ess_fail(ESS_ERR_CAPACITY, "T*k = %d exceeds %d", c->max_q_tokens * c->topk, ESS_MAX_SEL);
  if (c->attn_heads < 1 || c->attn_heads > 128)
    return ess_fail(ESS_ERR_UNSUPPORTED, "attn_heads %d outside [1, 128]", c->attn_heads);
  if (c->latent_fmt != ESS_FMT_BF16 && c->latent_fmt != ESS_FMT_FP8)
    return ess_fail(ESS_ERR_UNSUPPORTED, "latent_fmt %d", c->latent_fmt);
  if (c->row_stride < entry_bytes(c->latent_fmt) || (c->row_stride & 15) || c->row_stride > 2048)
    return ess_fail(ESS_ERR_INVALID_ARG, "row_stride %d must be a multiple of 16, >= %d and <= 2048", c->row_stride,
                    entry_bytes(c->latent_fmt));
  if (c->slots_per_seq < 1 || c->slots_per_seq > c->max_ctx)
    return ess_fail(ESS_ERR_INVALID_ARG, "slots_per_seq %d outside [1, max_ctx]", c->slots_per_seq);
  const long need = (long)c->max_q_tokens * c->topk;
  if (c->slots_per_seq < need && c->slots_per_seq < c->max_ctx)
    return ess_fail(ESS_ERR_CAPACITY, "slots_per_seq %d cannot hold one step's selection (T*k = %ld)",
                    c->slots_per_seq, need);
  if (!(c->sm_scale > 0.f)) return ess_fail(ESS_ERR_INVALID_ARG, "sm_scale must be positive");
  return ESS_OK;
}

struct WsLayout {
  size_t score, slot_idx, hit, miss, n_hit, n_miss, fill_tok, fill_slot, miss_cnt, o_part, lse_part, stats, seq_stats, zero_row, topk_cand, topk_cnt, topk_tau, sel_sample, sel_tau, sel_cand, sel_cnt, tickets, total;
};

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

WsLayout ws_layout(const ess_config& c) {
  const size_t B = c.max_batch, T = c.max_q_tokens, k = c.topk, H = c.attn_heads, L = c.max_ctx;
  WsLayout w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
  w.score = take(B * T * L * 4);
  w.slot_idx = take(B * T * k * 4);
  w.hit = take(B * T * k * 4);
  w.miss = take(B * T * k * 4);
  w.n_hit = take(B * T * 4);
  w.n_miss = take(B * T * 4);
  w.fill_tok = take(B * T * k * 4);
  w.fill_slot = take(B * T * k * 4);
  w.miss_cnt = take(B * 4);
  w.o_part = take(B * T * ESS_MAX_SPLITS * H * ESS_LATENT_DIM * 2);
  w.lse_part = take(B * T * ESS_MAX_SPLITS * H * 8);
  w.stats = take(4 * 8);
  w.seq_stats = take(B * 4 * 8);
  w.zero_row = take(ESS_ZERO_ROW_BYTES);
  w.topk_cand = take(ess_topk_cand_bytes());
  w.topk_cnt = take(ESS_TOPK_SHARED_ROWS * sizeof(uint32_t));
  w.topk_tau = take(ESS_TOPK_SHARED_ROWS * 2 * sizeof(uint32_t));
  w.sel_sample = take(B * T * (size_t)ess_sample_count(c.max_ctx) * 64 * 4);
  w.sel_tau = take(B * T * 8);
  w.sel_cand = take(B * T * (size_t)ess_sel_cand_cap() * 8);
  w.sel_cnt = take(B * T * 4);
  w.tickets = take(ESS_N_TICKETS * ESS_TICKET_WORDS * sizeof(uint32_t));
  w.total = off;
  return w;
}

int check_bt(const ess_ctx* ctx, int B, int T) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (B < 1 || B > ctx->cfg.max_batch) return ess_fail(ESS_ERR_INVALID_ARG, "B %d outside [1, %d]", B, ctx->cfg.max_batch);
  if (T < 1 || T > ctx->cfg.max_q_tokens)
    return ess_fail(ESS_ERR_INVALID_ARG, "T %d outside [1, %d]", T, ctx->cfg.max_q_tokens);
  return ESS_OK;
}

int check_cache(const ess_ctx* ctx, const ess_cache* c) {
  if (!c) return ess_fail(ESS_ERR_INVALID_ARG, "cache is NULL");
  if (!c->slot_pool || !c->slot_of || !c->token_of || !c->stamp)
    return ess_fail(ESS_ERR_INVALID_ARG, "cache has a NULL array");
  if (!aligned16(c->slot_pool) || !aligned16(c->host_pool_dev))
    return ess_fail(ESS_ERR_INVALID_ARG, "slot_pool / host_pool_dev must be 16-byte aligned");
  if (!c->host_pool_dev && ctx->cfg.slots_per_seq != ctx->cfg.max_ctx)
    return ess_fail(ESS_ERR_INVALID_ARG, "without a host pool slots_per_seq must equal max_ctx");
  return ESS_OK;
}

// number of attention splits for a list of up to k entries: a workgroup is sized to own a CU, so aim at
// a small multiple of the CU count; never fewer than the kernel's tiles-per-split limit allows
// `long_lists`: the lists are about topk entries long (Attn0, resident attention); then no workgroup
// gets more than 32 tiles: with several rounds of workgroups per CU, shorter ones overlap one's end
// (the write of its partial result) with another's work (measured: 9 % at batch 128 x 2 tokens)
int pick_splits(const ess_config& c, int B, int T, int cap, int target_wgs = 256, bool long_lists = true) {
  const int tiles = (c.topk + ESS_ATTN_TILE - 1) / ESS_ATTN_TILE;
  const int hgroups = (c.attn_heads + 127) / 128;      // a workgroup covers 128 heads
  int want = (target_wgs + B * T * hgroups - 1) / (B * T * hgroups);   // one workgroup per CU: fewer partial results to merge
  if (want > tiles) want = tiles;
  if (want > cap) want = cap;
  int lo = ess_attn_min_splits(c);
  if (long_lists && lo < (tiles + 31) / 32) lo = (tiles + 31) / 32;
  if (want < lo) want = lo;
  return want < 1 ? 1 : want;
}

// A view of the caller's cache arrays starting at sequence b0.
ess_cache shift_cache(const ess_config& c, const ess_cache& in, int b0) {
  ess_cache o = in;
  o.slot_pool = in.slot_pool + (size_t)b0 * c.slots_per_seq * c.row_stride;
  if (in.host_pool_dev) o.host_pool_dev = in.host_pool_dev + (size_t)b0 * c.max_ctx * c.row_stride;
  o.slot_of = in.slot_of + (size_t)b0 * c.max_ctx;
  o.token_of = in.token_of + (size_t)b0 * c.slots_per_seq;
  o.stamp = in.stamp + (size_t)b0 * c.slots_per_seq;
  return o;
}

// Bookkeeping + fetch of the sub-batch [b0, b0+B) (`cache`, `idx`, `slot_idx`, `miss_count` already
// point at sequence b0), the fetch on the side stream unless serial, tracked by event pair `half`.
// After return, work enqueued on `st` is ordered after the bookkeeping; *fill_pending tells whether
// ev_fill[half] must still be waited for before the fetched rows are read.
int run_cache_step(ess_ctx* ctx, const ess_cache& cache, const int32_t* idx, int B, int T, int kk, uint32_t step,
                   int32_t* slot_idx, int32_t* miss_count, hipStream_t st, bool* fill_pending, int b0 = 0,
                   int half = 0, hipEvent_t* fill_ev = nullptr, int fill_wgs = 64, bool confine = false) {
  *fill_pending = false;
  // confine: the fetch runs on the XCDs of ESS_FETCH_XCD_MASK and the kernels beside it stay off them, taking their work
  // through counters that this bookkeeping clears (counter 0: the fetch itself)
  int rc = ess_launch_bookkeeping(ctx, cache, idx, B, T, kk, step, slot_idx, miss_count, st, b0, half == 0,
                                  ess_xcd{nullptr, 0, nullptr, 0}, confine ? ctx->tickets : nullptr, ESS_TKT_FETCH2);
  if (rc != ESS_OK) return rc;
  if (!cache.host_pool_dev) return ESS_OK;      // nothing offloaded: no entry can be missing
  if (ctx->cfg.flags & ESS_FLAG_SERIAL) {
    if (fill_ev) ESS_HIP(hipEventRecord(fill_ev[0], st));
    rc = ess_launch_fill(ctx, cache, B, st, b0, fill_wgs);
    if (rc == ESS_OK && fill_ev) ESS_HIP(hipEventRecord(fill_ev[1], st));
    return rc;
  }
  ESS_HIP(hipEventRecord(ctx->ev_book[half], st));
  ESS_HIP(hipStreamWaitEvent(ctx->side, ctx->ev_book[half], 0));
  if (fill_ev) ESS_HIP(hipEventRecord(fill_ev[0], ctx->side));
  rc = ess_launch_fill(ctx, cache, B, ctx->side, b0, fill_wgs, confine ? ESS_FETCH_XCD_MASK : 0u, ctx->tickets);
  if (rc != ESS_OK) return rc;
  if (fill_ev) ESS_HIP(hipEventRecord(fill_ev[1], ctx->side));
  ESS_HIP(hipEventRecord(ctx->ev_fill[half], ctx->side));
  *fill_pending = true;
  return ESS_OK;
}

}  // namespace

int ess_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

extern "C" {

const char* ess_last_error(void) { return g_err; }

int ess_workspace_bytes(const ess_config* cfg, size_t* out) {
  int rc = validate_config(cfg);
  if (rc != ESS_OK) return rc;
  if (!out) return ess_fail(ESS_ERR_INVALID_ARG, "out is NULL");
  *out = ws_layout(*cfg).total;
  return ESS_OK;
}

int ess_create(const ess_config* cfg, ess_ctx** out) {
  int rc = validate_config(cfg);
  if (rc != ESS_OK) return rc;
  if (!out) return ess_fail(ESS_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  ess_ctx* ctx = new (std::nothrow) ess_ctx();
  if (!ctx) return ess_fail(ESS_ERR_NOMEM, "host allocation failed");
  memset(ctx, 0, sizeof(*ctx));
  ctx->cfg = *cfg;
  ctx->prof_mask = 0x3Fu;
  ctx->prof_every = 1;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) { delete ctx; return ess_fail(ESS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e)); }
  const WsLayout w = ws_layout(*cfg);
  uint8_t* base = nullptr;
  e = hipMalloc(reinterpret_cast<void**>(&base), w.total);
  if (e != hipSuccess) {
    delete ctx;
    (void)hipGetLastError();
    return ess_fail(ESS_ERR_NOMEM, "workspace of %zu bytes: %s", w.total, hipGetErrorString(e));
  }
  ctx->ws_bytes = w.total;
  ctx->score_ws = reinterpret_cast<float*>(base + w.score);
  ctx->slot_idx_ws = reinterpret_cast<int32_t*>(base + w.slot_idx);
  ctx->hit_list = reinterpret_cast<int32_t*>(base + w.hit);
  ctx->miss_list = reinterpret_cast<int32_t*>(base + w.miss);
  ctx->n_hit = reinterpret_cast<int32_t*>(base + w.n_hit);
  ctx->n_miss = reinterpret_cast<int32_t*>(base + w.n_miss);
  ctx->fill_tok = reinterpret_cast<int32_t*>(base + w.fill_tok);
  ctx->fill_slot = reinterpret_cast<int32_t*>(base + w.fill_slot);
  ctx->miss_cnt = reinterpret_cast<int32_t*>(base + w.miss_cnt);
  ctx->o_part = reinterpret_cast<uint16_t*>(base + w.o_part);
  ctx->lse_part = reinterpret_cast<float*>(base + w.lse_part);
  ctx->stats = reinterpret_cast<unsigned long long*>(base + w.stats);
  ctx->seq_stats = reinterpret_cast<unsigned long long*>(base + w.seq_stats);
  ctx->zero_row = base + w.zero_row;
  ctx->topk_cand = reinterpret_cast<unsigned long long*>(base + w.topk_cand);
  ctx->topk_cnt = reinterpret_cast<uint32_t*>(base + w.topk_cnt);
  ctx->topk_tau = reinterpret_cast<uint32_t*>(base + w.topk_tau);
  ctx->sel_sample = reinterpret_cast<float*>(base + w.sel_sample);
  ctx->sel_tau = reinterpret_cast<uint32_t*>(base + w.sel_tau);
  ctx->sel_cand = reinterpret_cast<unsigned long long*>(base + w.sel_cand);
  ctx->sel_cnt = reinterpret_cast<uint32_t*>(base + w.sel_cnt);
  ctx->tickets = reinterpret_cast<uint32_t*>(base + w.tickets);
  auto bail = [&](const char* what, hipError_t err) {
    for (int h = 0; h < 2; ++h) {
      if (ctx->ev_book[h]) (void)hipEventDestroy(ctx->ev_book[h]);
      if (ctx->ev_fill[h]) (void)hipEventDestroy(ctx->ev_fill[h]);
    }
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->host_miss) (void)hipHostFree(ctx->host_miss);
    (void)hipFree(base);
    delete ctx;
    return ess_fail(ESS_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
  };
  if ((e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking)) != hipSuccess) return bail("hipStreamCreate", e);
  for (int h = 0; h < 2; ++h) {
    if ((e = hipEventCreateWithFlags(&ctx->ev_book[h], hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
    if ((e = hipEventCreateWithFlags(&ctx->ev_fill[h], hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  }
  if ((e = hipMemset(ctx->stats, 0, 32)) != hipSuccess) return bail("hipMemset", e);
  if ((e = hipMemset(ctx->seq_stats, 0, (size_t)cfg->max_batch * 32)) != hipSuccess) return bail("hipMemset", e);
  if ((e = hipMemset(ctx->zero_row, 0, ESS_ZERO_ROW_BYTES)) != hipSuccess) return bail("hipMemset", e);
  if ((e = hipMemset(ctx->topk_cnt, 0, ESS_TOPK_SHARED_ROWS * sizeof(uint32_t))) != hipSuccess) return bail("hipMemset", e);
  if ((e = hipMemset(ctx->tickets, 0, ESS_N_TICKETS * ESS_TICKET_WORDS * sizeof(uint32_t))) != hipSuccess) return bail("hipMemset", e);
  {
    int irc = ess_init_cache_kernels(*cfg, &ctx->book_fits);
    if (irc == ESS_OK) irc = ess_init_attn_kernels();
    if (irc != ESS_OK) {                        // the text of the failure is already set
      char keep[sizeof(g_err)];
      memcpy(keep, g_err, sizeof(keep));
      (void)bail("", hipSuccess);
      memcpy(g_err, keep, sizeof(keep));
      return irc;
    }
  }
  ctx->xcds_even = false;
  if (ess_probe_xcds(ctx->tickets, &ctx->xcds_even) != ESS_OK) return bail("XCD probe", hipGetLastError());
  if ((e = hipHostMalloc(reinterpret_cast<void**>(&ctx->host_miss), ((size_t)cfg->max_batch + 1) * sizeof(int32_t),
                         hipHostMallocMapped)) != hipSuccess) return bail("hipHostMalloc", e);
  memset(ctx->host_miss, 0, ((size_t)cfg->max_batch + 1) * sizeof(int32_t));
  if ((e = hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->host_miss_dev), ctx->host_miss, 0)) != hipSuccess)
    return bail("hipHostGetDevicePointer", e);
  ctx->auto_threshold = 150;
  ctx->auto_calibrated = false;
  ctx->last_confined = 0;
  ctx->check_extra = 0;
  *out = ctx;
  return ESS_OK;
}

int ess_destroy(ess_ctx* ctx) {
  if (!ctx) return ESS_OK;
  (void)hipStreamSynchronize(ctx->side);
  (void)ess_profile_enable(ctx, 0);
  for (int h = 0; h < 2; ++h) {
    (void)hipEventDestroy(ctx->ev_book[h]);
    (void)hipEventDestroy(ctx->ev_fill[h]);
  }
  (void)hipStreamDestroy(ctx->side);
  (void)hipHostFree(ctx->host_miss);
  (void)hipFree(ctx->score_ws);                 // base of the workspace
  delete ctx;
  return ESS_OK;
}

int ess_cache_reset(ess_ctx* ctx, const ess_cache* cache, int32_t B, void* stream) {
  int rc = check_bt(ctx, B, 1);
  if (rc != ESS_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != ESS_OK) return rc;
  return ess_launch_cache_reset(ctx->cfg, *cache, B, static_cast<hipStream_t>(stream));
}

int ess_cache_admit(ess_ctx* ctx, const ess_cache* cache, const int32_t* tok, int32_t B, int32_t n, uint32_t step,
                    void* stream) {
  int rc = check_bt(ctx, B, 1);
  if (rc != ESS_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != ESS_OK) return rc;
  if (!tok) return ess_fail(ESS_ERR_INVALID_ARG, "tok is NULL");
  if (n < 1 || n > ctx->cfg.max_q_tokens * ctx->cfg.topk)
    return ess_fail(ESS_ERR_CAPACITY, "n %d outside [1, T*k = %d]", n, ctx->cfg.max_q_tokens * ctx->cfg.topk);
  if (n > ctx->cfg.slots_per_seq) return ess_fail(ESS_ERR_CAPACITY, "n %d exceeds the slot pool", n);
  if (step < 1) return ess_fail(ESS_ERR_INVALID_ARG, "step must be >= 1");
  hipStream_t st = static_cast<hipStream_t>(stream);
  bool pending = false;
  // one list of n entries per sequence, no per-query outputs
  rc = run_cache_step(ctx, *cache, tok, B, 1, n, step, nullptr, nullptr, st, &pending);
  if (rc != ESS_OK) return rc;
  if (pending) ESS_HIP(hipStreamWaitEvent(st, ctx->ev_fill[0], 0));
  return ESS_OK;
}

int ess_index_score(ess_ctx* ctx, const uint8_t* q, const float* w, const uint8_t* key, const int32_t* ctx_len,
                    int32_t B, int32_t T, float* score, void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if (!q || !w || !key || !ctx_len || !score) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(q) || !aligned16(key) || !aligned16(score))
    return ess_fail(ESS_ERR_INVALID_ARG, "q, key and score must be 16-byte aligned");
  return ess_launch_index_score(ctx->cfg, q, w, key, ctx_len, B, T, score, static_cast<hipStream_t>(stream));
}

namespace {
// The assertion of a step that fed launches by ticket (see ess_ticket_check): every launch handed out at least as
// many tickets as it had work items.  Workgroups draw tickets until none is left, wherever they run, so a
// failure means a defect in the hand-out itself; it is seen at the next call, and nothing is confined afterwards.
int check_tickets(ess_ctx* ctx) {
  volatile int32_t* flag = ctx->host_miss + ctx->cfg.max_batch;
  if (!*flag) return ESS_OK;
  *flag = 0;
  ctx->xcds_even = false;
  return ess_fail(ESS_ERR_INTERNAL, "assertion failed in an earlier decode step: a ticket-fed launch handed out fewer tickets "
                                    "than it had work items; XCD-confined schedules are now off");
}

int check_paged(const ess_ctx* ctx, const uint8_t* pool, const int32_t* block_table, int n_pages) {
  if (!block_table) return ess_fail(ESS_ERR_INVALID_ARG, "block_table is NULL");
  if (ctx->cfg.max_ctx % ESS_PAGE_TOKENS) return ess_fail(ESS_ERR_UNSUPPORTED, "paged Indexer-Cache needs max_ctx %% 64 == 0");
  if (n_pages < 1) return ess_fail(ESS_ERR_INVALID_ARG, "n_pages %d", n_pages);
  if (!aligned16(pool)) return ess_fail(ESS_ERR_INVALID_ARG, "the page pool must be 16-byte aligned");
  return ESS_OK;
}
}  // namespace

int ess_index_score_paged(ess_ctx* ctx, const uint8_t* q, const float* w, const uint8_t* key_pages,
                          const int32_t* block_table, int32_t n_pages, const int32_t* ctx_len, int32_t B, int32_t T,
                          float* score, void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if (!q || !w || !key_pages || !ctx_len || !score) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(q) || !aligned16(score)) return ess_fail(ESS_ERR_INVALID_ARG, "q and score must be 16-byte aligned");
  if ((rc = check_paged(ctx, key_pages, block_table, n_pages)) != ESS_OK) return rc;
  return ess_launch_index_score(ctx->cfg, q, w, key_pages, ctx_len, B, T, score, static_cast<hipStream_t>(stream),
                                block_table, n_pages);
}

int ess_index_topk(ess_ctx* ctx, const uint8_t* q, const float* w, const uint8_t* key, const int32_t* block_table,
                   int32_t n_pages, const int32_t* ctx_len, int32_t B, int32_t T, int32_t* idx, void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if (!q || !w || !key || !ctx_len || !idx) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(q) || !aligned16(key)) return ess_fail(ESS_ERR_INVALID_ARG, "q and key must be 16-byte aligned");
  if (block_table && (rc = check_paged(ctx, key, block_table, n_pages)) != ESS_OK) return rc;
  // index score and top-k as one stage without a score array (see ess_internal.h)
  hipStream_t st = static_cast<hipStream_t>(stream);
  const ess_config& c = ctx->cfg;
  const ess_xcd none{nullptr, 0, nullptr, 0};
  const int np = block_table ? n_pages : 0, cap = ess_sel_cand_cap();
  if ((rc = ess_launch_index_sample(c, q, w, key, ctx_len, B, T, ctx->sel_sample, st, block_table, np, none)) != ESS_OK) return rc;
  if ((rc = ess_launch_index_tau(ctx, ctx_len, B, T, 0, st, none)) != ESS_OK) return rc;
  rc = ess_launch_index_emit(c, q, w, key, ctx_len, B, T, ctx->sel_tau, ctx->sel_cand, ctx->sel_cnt, cap, st, block_table, np,
                             nullptr, nullptr, none);
  if (rc != ESS_OK) return rc;
  return ess_launch_topk_finish(ctx, q, w, key, block_table, np, ctx_len, B, T, 0, idx, st, none);
}

int ess_topk(ess_ctx* ctx, const float* score, const int32_t* ctx_len, int32_t B, int32_t T, int32_t* idx,
             void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if (!score || !ctx_len || !idx) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  return ess_launch_topk(ctx, score, ctx_len, B, T, idx, static_cast<hipStream_t>(stream));
}

int ess_gather_latent(ess_ctx* ctx, const ess_cache* cache, const int32_t* idx, const int32_t* ctx_len, int32_t B,
                      int32_t T, uint32_t step, int32_t* slot_idx, uint8_t* rows_out, int32_t* miss_count,
                      void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != ESS_OK) return rc;
  if (!idx || !slot_idx) return ess_fail(ESS_ERR_INVALID_ARG, "idx / slot_idx is NULL");
  if (!aligned16(rows_out)) return ess_fail(ESS_ERR_INVALID_ARG, "rows_out must be 16-byte aligned");
  if (step < 1) return ess_fail(ESS_ERR_INVALID_ARG, "step must be >= 1");
  (void)ctx_len;                                // visibility was already applied by the selection
  hipStream_t st = static_cast<hipStream_t>(stream);
  bool pending = false;
  rc = run_cache_step(ctx, *cache, idx, B, T, ctx->cfg.topk, step, slot_idx, miss_count, st, &pending);
  if (rc != ESS_OK) return rc;
  if (pending) ESS_HIP(hipStreamWaitEvent(st, ctx->ev_fill[0], 0));
  if (rows_out) return ess_launch_gather_rows(ctx->cfg, cache->slot_pool, slot_idx, B, T, rows_out, st);
  return ESS_OK;
}

int ess_sparse_mla_decode(ess_ctx* ctx, const void* q_bf16, const uint8_t* slot_pool, const int32_t* slot_idx,
                          int32_t B, int32_t T, void* out_bf16, float* lse, void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if (!q_bf16 || !slot_pool || !slot_idx || !out_bf16) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(q_bf16) || !aligned16(slot_pool) || !aligned16(out_bf16))
    return ess_fail(ESS_ERR_INVALID_ARG, "q, slot_pool and out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int ns = pick_splits(ctx->cfg, B, T, 16);
  rc = ess_launch_attn_partial(ctx, q_bf16, slot_pool, slot_idx, nullptr, B, T, 0, ns, st);
  if (rc != ESS_OK) return rc;
  return ess_launch_attn_merge(ctx, B, T, ns, out_bf16, lse, st);
}

int ess_decode_step(ess_ctx* ctx, const ess_cache* cache, const ess_step_args* a, void* stream) {
  if (!a) return ess_fail(ESS_ERR_INVALID_ARG, "args is NULL");
  int rc = check_bt(ctx, a->B, a->T);
  if (rc != ESS_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != ESS_OK) return rc;
  if (!a->q_idx_fp8 || !a->w || !a->key_fp8 || !a->ctx_len || !a->q_bf16 || !a->idx_out || !a->out_bf16)
    return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(a->q_idx_fp8) || !aligned16(a->key_fp8) || !aligned16(a->q_bf16) || !aligned16(a->out_bf16))
    return ess_fail(ESS_ERR_INVALID_ARG, "q_idx_fp8, key_fp8, q_bf16 and out_bf16 must be 16-byte aligned");
  if (a->step < 1) return ess_fail(ESS_ERR_INVALID_ARG, "step must be >= 1");
  if (a->block_table && (rc = check_paged(ctx, a->key_fp8, a->block_table, a->n_pages)) != ESS_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const ess_config& c = ctx->cfg;
  const int B = a->B, T = a->T;
  if ((rc = check_tickets(ctx)) != ESS_OK) return rc;

  // stage marks of this step, when profiling: a mark closes the interval since the previous mark and
  // books it under `tag` (0 index score, 1 top-k, 2 bookkeeping, 3 Attn0, 4 Attn1 + merge)
  hipEvent_t* pev = nullptr;
  int8_t* ptag = nullptr;
  int pslot = -1, nmark = 0;
  if (ctx->prof_ev && ctx->prof_n < ctx->prof_cap && (ctx->prof_calls++ % ctx->prof_every) == 0) {
    pslot = ctx->prof_n++;
    pev = ctx->prof_ev + (size_t)pslot * ESS_PROF_EVENTS;
    ptag = ctx->prof_tag + (size_t)pslot * ESS_PROF_MAIN;
    ctx->prof_nmark[pslot] = 0;
    ctx->prof_nfill[pslot] = 0;
    for (int f = 0; f < ESS_PROF_FILL; ++f) ctx->prof_pair_stage[(size_t)pslot * ESS_PROF_FILL + f] = 5;
  }
  // ESS_BEGIN(tag) / ESS_END(tag) bracket the launches of one stage; only selected stages are timed
  bool adjacent = false;                        // the last recorded mark sits right before this point
#define ESS_RECORD(tag)                                        \
  do {                                                         \
    if (nmark < ESS_PROF_MAIN) {                               \
      ESS_HIP(hipEventRecord(pev[nmark], st));                 \
      ptag[nmark] = (int8_t)(tag);                             \
      ctx->prof_nmark[pslot] = ++nmark;                        \
    }                                                          \
    adjacent = true;                                           \
  } while (0)
#define ESS_BEGIN(tag) do { if (pev && ((ctx->prof_mask >> (tag)) & 1u) && !adjacent) ESS_RECORD(-1); } while (0)
#define ESS_END(tag)                                           \
  do {                                                         \
    if (pev && ((ctx->prof_mask >> (tag)) & 1u)) ESS_RECORD(tag); \
    else adjacent = false;                                     \
  } while (0)

  const bool offloaded = cache->host_pool_dev != nullptr;
  // DualBatch-Attention overlap (Sec. 3.3): the batch is cut in two halves so that the second half's
  // indexer and top-k run while the first half's fetch is in flight
  bool want_dba = (c.flags & ESS_FLAG_DBA) != 0;
  long mean_miss = -1;                          // misses per sequence of the latest bookkeeping, if known
  if ((c.flags & ESS_FLAG_AUTO) && offloaded) {
    // miss counts of the latest bookkeeping as the host sees them now (no wait: possibly a step old)
    const volatile int32_t* hm = ctx->host_miss;
    long sum = 0;
    for (int b = 0; b < B; ++b) sum += hm[b];
    mean_miss = sum / B;
    // the split pays by hiding half the batch's index score behind a fetch: it must be long enough to be
    // worth two rounds of top-k and bookkeeping (at 32K context and batch 64 it is not, whatever the misses)
    const double idx_half_us = 0.5 * B * (double)c.max_ctx * (c.idx_dim + 4.0 * T) / 5.3e6;   // at 5.3 TB/s
    want_dba = sum > (long)ctx->auto_threshold * B && (ctx->auto_calibrated || idx_half_us >= 50.0);
  }
  const bool dba = offloaded && want_dba && !(c.flags & ESS_FLAG_SERIAL) && B >= 2;
  ctx->last_overlap = (c.flags & ESS_FLAG_SERIAL) ? 2 : (dba ? 1 : 0);
  const bool da_swap = offloaded && !dba && !(c.flags & ESS_FLAG_SERIAL);
  const int nh = dba ? 2 : 1;
  // A fetch confined to a few XCDs (ESS_FETCH_XCD_MASK), with the kernels beside it kept off them (see ess_xcd),
  // pays when the fetch is long: the kernels beside it then run as if alone, but on the other XCDs only.  With few misses the lost
  // CUs cost more (Attn0, in more rounds of workgroups, becomes the longer side).  Measured (with three XCDs) at batch 64,
  // 128K context, 1152-byte entries (step time, confined vs not): single-fetch schedule 0.436 vs 0.398 ms
  // at 31 misses per sequence, 0.447 vs 0.482 at 114, 0.557 vs 0.570 at 195; split-batch, first fetch:
  // 0.497 vs 0.476 at 114, 0.529 vs 0.529 at 195, 0.607 vs 0.631 at 289; second fetch as well: 0.546 vs
  // 0.529 at 195, 0.605 vs 0.607 at 289, 0.891 vs 0.933 at 494; at batch 128 with two query tokens and
  // quantised entries, where attention is as long as the fetches, the second confinement costs 5 %.
  // The rules below compare rough times (microseconds) of the fetch and of what runs beside it; the miss
  // count of the previous step is only known under ESS_FLAG_AUTO, without it nothing is confined.
  bool confine = false, confine2 = false, confine_da = false;
  ess_ticket_check chk{};                       // filled in by the launches that take their work by ticket
  chk.tickets = ctx->tickets;
  chk.flag = ctx->host_miss_dev + c.max_batch;
  if (mean_miss >= 0 && ctx->xcds_even) {
    const double link = 50e3;                                       // bytes per microsecond
    const double fetch_all = (double)B * mean_miss * c.row_stride / link, fetch_half = 0.5 * fetch_all;
    const double idx_half = 0.5 * B * (double)c.max_ctx * (c.idx_dim + 4.0 * T) / 5.3e6;
    // Attn0 on the XCDs the fetch leaves free (one workgroup per CU): rounds x (tiles x time per tile + start and end)
    const int work_cus = 32 * (8 - __builtin_popcount(ESS_FETCH_XCD_MASK & 0xffu));
    const int hg = (c.attn_heads + 127) / 128;
    const int ns0e = pick_splits(c, B, T, 16, ESS_ATTN0_WGS);
    const double hits = c.topk - (mean_miss / T < c.topk ? mean_miss / T : c.topk);
    const double tiles_item = (hits / ESS_ATTN_TILE) / ns0e + 1.0;
    const double rounds = (double)((long)B * T * hg * ns0e + work_cus - 1) / work_cus;
    // (a tile of 32 entries x 128 heads: 2.6 us, 4.2 us when the entries are dequantised on the way; 16 us of start and end)
    const double attn5 = (double)(long)rounds * (tiles_item * (c.latent_fmt == ESS_FMT_BF16 ? 2.6 : 4.2) + 16.0);
    // (one work counter serves one index-score launch: two query tokens at most)
    confine = dba && T <= 2 && fetch_half >= 1.5 * idx_half;
    confine2 = confine && attn5 + 40.0 <= 1.15 * fetch_half;        // + Attn1 and merge of the first half
    confine_da = da_swap && attn5 <= 1.6 * fetch_all;
  }
  ctx->last_confined = confine_da ? 1 : (confine2 ? 2 : (confine ? 1 : 0));
  const uint32_t check_extra = ctx->last_confined ? ctx->check_extra : 0u;   // test hook, one confined step
  if (ctx->last_confined) ctx->check_extra = 0;
  const uint32_t mask2 = ESS_FETCH_XCD_MASK;
  // launch `counter` of the step's ticket-fed launches: its counters, the XCDs it stays off, where its item count goes
  auto tk_xcd = [&](int counter) {
    return ess_xcd{ctx->tickets + counter * ESS_TICKET_WORDS, ESS_FETCH_XCD_MASK, chk.need + counter, ctx->ticket_grid};
  };
  const int wgs2 = ESS_FETCH_CONFINED_WGS;
  const int hb0[2] = {0, B / 2};
  const int hB[2] = {dba ? B / 2 : B, B - B / 2};
  const size_t k = (size_t)c.topk;
  bool pending[2] = {false, false};

  // attention splits: chosen from the whole batch and the same for both halves, so that every schedule
  // sums in the same order and gives the same bits
  const int ns0 = pick_splits(c, B, T, 16, offloaded ? ESS_ATTN0_WGS : 256);
  int ns1 = 0;
  if (offloaded) {
    // Attn1 works on the short miss lists: as many splits as give the whole batch one workgroup per CU
    ns1 = pick_splits(c, B, T, ESS_MAX_SPLITS - 16, 256, false);
  }

  // Stages 1 and 2 come in two forms: through the score array (index score, then top-k), or fused (the score array
  // never exists: a sample pass gives each row a lower bound, the index pass emits only candidates, the top-k is
  // finished among them: ess_index_topk).  Alone, on batch 64 at 128K, the fused form is the faster one (sample pass
  // 11 + 7 us, main pass 176 us against 189, finish 11 us against 17 + 15 for the two-kernel top-k: 211 against
  // 223 us), but inside a step it is not: its main pass, launched for half a batch, takes the time of the dense one
  // (99 against 98 us: the workgroup's wait for its place in the row's list weighs more the shorter the launch),
  // its sample pass is two more launches in a chain of dependent ones, and beside a running fetch its main pass
  // starts 10-15 us later than the dense one does.  Step time, batch 64 x 128K, split-batch with confined fetches:
  // 0.620 ms fused against 0.606 through the score array, and 0.614 with the second half fused and its sample
  // pass hidden on the side stream beside the first half's index score (which it slows by 8 us); batch 32 x 32K
  // resident 0.101 against 0.096; batch 64 x 32K 0.398 against 0.394.  So the step goes through the score array
  // unless ESS_FLAG_FUSED_SELECT asks for the fused form.
  const bool fused = (c.flags & ESS_FLAG_FUSED_SELECT) && !(c.flags & ESS_FLAG_DENSE_SCORES);
  const size_t sel_pitch = (size_t)ess_sample_count(c.max_ctx) * 64, sel_cap = (size_t)ess_sel_cand_cap();

  // stages 1-2 (+ 3, 5 when offloaded) per half; the fetch goes to the side stream
  for (int h = 0; h < nh; ++h) {
    const int b0 = hb0[h], Bh = hB[h];
    const size_t bt0 = (size_t)b0 * T;
    float* sc = ctx->score_ws + bt0 * c.max_ctx;
    int32_t* idx_h = a->idx_out + bt0 * k;
    // the index-score kernel is timed by its own start and end (events handed to the launch), not by
    // marks on the stream, which would add the dispatch gaps to the figure the roofline is taken from
    hipEvent_t ev_s = nullptr, ev_e = nullptr;
    auto take_index_events = [&]() {
      if (pev && (ctx->prof_mask & 1u) && nmark + 2 <= ESS_PROF_MAIN) {
        ev_s = pev[nmark];
        ev_e = pev[nmark + 1];
        ptag[nmark] = -1;
        ptag[nmark + 1] = 0;
        nmark += 2;
        ctx->prof_nmark[pslot] = nmark;
        adjacent = true;
      } else {
        adjacent = false;
      }
    };
    // second half of the split-batch schedule: these kernels run beside the first fetch, which is confined
    // to the XCDs of ESS_FETCH_XCD_MASK; they stay off those (counter blocks ESS_TKT_INDEX .. ESS_TKT_BOOK, cleared by the first half's bookkeeping)
    const bool beside = confine && h == 1;
    auto xcd_of = [&](int counter) { return beside ? tk_xcd(counter) : ess_xcd{nullptr, 0, nullptr, 0}; };
    const uint8_t* q_h = a->q_idx_fp8 + bt0 * c.idx_heads * c.idx_dim;
    const float* w_h = a->w + bt0 * c.idx_heads;
    // paged: one pool for the whole batch, the table rows of this sub-batch
    const uint8_t* key_h = a->block_table ? a->key_fp8 : a->key_fp8 + (size_t)b0 * c.max_ctx * c.idx_dim;
    const int32_t* table_h = a->block_table ? a->block_table + (size_t)b0 * (c.max_ctx / ESS_PAGE_TOKENS) : nullptr;
    const int np_h = a->block_table ? a->n_pages : 0;
    if (!fused) {
      take_index_events();
      rc = ess_launch_index_score(c, q_h, w_h, key_h, a->ctx_len + b0, Bh, T, sc, st, table_h, np_h, ev_s, ev_e, xcd_of(ESS_TKT_INDEX));
      if (rc != ESS_OK) return rc;
      ESS_BEGIN(1);
      rc = ess_launch_topk(ctx, sc, a->ctx_len + b0, Bh, T, idx_h, st, xcd_of(ESS_TKT_SAMPLE));
      if (rc != ESS_OK) return rc;
      ESS_END(1);
    } else {
      // the two small launches in front of the emitting pass are booked with the top-k, whose threshold search they are
      const size_t cap = sel_cap;
      ESS_BEGIN(1);
      rc = ess_launch_index_sample(c, q_h, w_h, key_h, a->ctx_len + b0, Bh, T, ctx->sel_sample + bt0 * sel_pitch, st, table_h, np_h,
                                   xcd_of(ESS_TKT_SAMPLE));
      if (rc != ESS_OK) return rc;
      if ((rc = ess_launch_index_tau(ctx, a->ctx_len + b0, Bh, T, b0, st, xcd_of(ESS_TKT_TAU))) != ESS_OK) return rc;
      ESS_END(1);
      take_index_events();
      rc = ess_launch_index_emit(c, q_h, w_h, key_h, a->ctx_len + b0, Bh, T, ctx->sel_tau + 2 * bt0, ctx->sel_cand + bt0 * cap,
                                 ctx->sel_cnt + bt0, (int)cap, st, table_h, np_h, ev_s, ev_e, xcd_of(ESS_TKT_INDEX));
      if (rc != ESS_OK) return rc;
      ESS_BEGIN(1);
      rc = ess_launch_topk_finish(ctx, q_h, w_h, key_h, table_h, np_h, a->ctx_len + b0, Bh, T, b0, idx_h, st, xcd_of(ESS_TKT_FINISH));
      if (rc != ESS_OK) return rc;
      ESS_END(1);
    }
    if (!offloaded) continue;
    const int32_t* used = a->topk_override ? a->topk_override + bt0 * k : idx_h;
    const ess_cache ch = shift_cache(c, *cache, b0);
    hipEvent_t* fev = (pev && h < ESS_PROF_FILL && ((ctx->prof_mask >> 5) & 1u)) ? pev + ESS_PROF_MAIN + 2 * h : nullptr;
    ESS_BEGIN(2);
    if (da_swap || (dba && h == 1)) {      // bookkeeping only; the fetch follows on this stream further down
      rc = ess_launch_bookkeeping(ctx, ch, used, Bh, T, c.topk, a->step, ctx->slot_idx_ws + bt0 * k,
                                  a->miss_count ? a->miss_count + b0 : nullptr, st, b0, h == 0, xcd_of(ESS_TKT_BOOK),
                                  (confine2 || (da_swap && confine_da)) ? ctx->tickets + (da_swap ? 0 : ESS_TKT_FETCH2) * ESS_TICKET_WORDS : nullptr,
                                  da_swap ? ESS_N_TICKETS : ESS_N_TICKETS - ESS_TKT_FETCH2);
      if (rc != ESS_OK) return rc;
    } else {
      rc = run_cache_step(ctx, ch, used, Bh, T, c.topk, a->step, ctx->slot_idx_ws + bt0 * k,
                          a->miss_count ? a->miss_count + b0 : nullptr, st, &pending[h], b0, h, fev, dba ? (confine ? ESS_FETCH_CONFINED_WGS : 28) : 64, confine);
      if (rc != ESS_OK) return rc;
      if (fev) { ctx->prof_nfill[pslot] = h + 1; ctx->prof_pair_stage[(size_t)pslot * ESS_PROF_FILL + h] = 5; }
    }
    ESS_END(2);
  }

  if (!offloaded) {
    // nothing offloaded: slot == position, attention straight over the selection
    const int32_t* used = a->topk_override ? a->topk_override : a->idx_out;
    ESS_BEGIN(3);
    rc = ess_launch_attn_partial(ctx, a->q_bf16, cache->slot_pool, used, nullptr, B, T, 0, ns0, st);
    if (rc != ESS_OK) return rc;
    ESS_END(3);
    ESS_BEGIN(4);
    rc = ess_launch_attn_merge(ctx, B, T, ns0, a->out_bf16, a->lse, st, a->miss_count, B);   // no misses: the counts are zero
    if (rc != ESS_OK) return rc;
    ESS_END(4);
    return ESS_OK;
  }

  const uint16_t* q16 = static_cast<const uint16_t*>(a->q_bf16);
  if (da_swap) {
    // DA schedule.  The fetch is the critical path, so it stays on the caller's stream, right behind the
    // bookkeeping and right before Attn1; Attn0, which has time to spare, goes to the side stream.  A
    // wait on another stream's event costs several microseconds when the event fires late and almost
    // nothing when it has fired long before: this way both waits of the step are of the second kind
    // (the side stream's wait for the bookkeeping delays only Attn0).
    ESS_HIP(hipEventRecord(ctx->ev_book[0], st));
    ESS_HIP(hipStreamWaitEvent(ctx->side, ctx->ev_book[0], 0));
    hipEvent_t* aev = (pev && ((ctx->prof_mask >> 3) & 1u)) ? pev + ESS_PROF_MAIN : nullptr;
    if (aev) ESS_HIP(hipEventRecord(aev[0], ctx->side));
    rc = ess_launch_attn_partial(ctx, q16, cache->slot_pool, ctx->hit_list, ctx->n_hit, B, T, 0, ns0, ctx->side, 0,
                                 confine_da ? tk_xcd(ESS_TKT_ATTN0) : ess_xcd{nullptr, 0, nullptr, 0});
    if (rc != ESS_OK) return rc;
    if (aev) {
      ESS_HIP(hipEventRecord(aev[1], ctx->side));
      ctx->prof_nfill[pslot] = 1;
      ctx->prof_pair_stage[(size_t)pslot * ESS_PROF_FILL] = 3;
    }
    ESS_HIP(hipEventRecord(ctx->ev_fill[0], ctx->side));          // here: Attn0 done
    ESS_BEGIN(5);
    rc = confine_da ? ess_launch_fill(ctx, *cache, B, st, 0, wgs2, mask2, ctx->tickets) : ess_launch_fill(ctx, *cache, B, st, 0, 64);
    if (rc != ESS_OK) return rc;
    ESS_END(5);
    ESS_BEGIN(4);
    ESS_HIP(hipStreamWaitEvent(st, ctx->ev_fill[0], 0));
    rc = ess_launch_attn_partial(ctx, q16, cache->slot_pool, ctx->miss_list, ctx->n_miss, B, T, ns0, ns1, st, 0);
    if (rc != ESS_OK) return rc;
    chk.need[ESS_TKT_ATTN0] += check_extra;
    rc = ess_launch_attn_merge(ctx, B, T, ns0 + ns1, a->out_bf16, a->lse, st, nullptr, 0, 0, confine_da ? &chk : nullptr);
    if (rc != ESS_OK) return rc;
    ESS_END(4);
    return ESS_OK;
  }

  if (dba) {
    // DBA schedule.  Two chains are critical: the two fetches, and the second half's index score, top-k
    // and bookkeeping, which the second fetch waits for.  A wait on another stream's event costs several
    // microseconds when the event fires late, so the second fetch follows its bookkeeping on the caller's
    // stream (it may start while the first fetch is still finishing: the link just stays busy), and what
    // has time to spare goes to the side stream behind the first fetch: Attn0 of the whole batch and Attn1
    // of the first half.  The caller's stream ends with Attn1 of the second half and the merge.
    const ess_cache c0 = shift_cache(c, *cache, hb0[0]), c1 = shift_cache(c, *cache, hb0[1]);
    const size_t bt1 = (size_t)hb0[1] * T;
    ESS_HIP(hipEventRecord(ctx->ev_book[1], st));                    // second half's bookkeeping done
    ESS_BEGIN(5);
    rc = confine2 ? ess_launch_fill(ctx, c1, hB[1], st, hb0[1], wgs2, mask2, ctx->tickets + ESS_TKT_FETCH2 * ESS_TICKET_WORDS)
                  : ess_launch_fill(ctx, c1, hB[1], st, hb0[1], 28);
    if (rc != ESS_OK) return rc;
    ESS_END(5);
    // side-stream attention is timed by event pairs 1 and 2 (pair 0 brackets the first fetch): all three or none
    hipEvent_t* aev = (pev && ctx->prof_nfill[pslot] == 1 && ((ctx->prof_mask >> 3) & 1u)) ? pev + ESS_PROF_MAIN + 2 : nullptr;
    ESS_HIP(hipStreamWaitEvent(ctx->side, ctx->ev_book[1], 0));
    if (aev) ESS_HIP(hipEventRecord(aev[0], ctx->side));
    // Attn0 of the whole batch in one launch (behind the first fetch it could not start much earlier
    // anyway): one workgroup per CU, the same splits as in the other schedules
    rc = ess_launch_attn_partial(ctx, q16, cache->slot_pool, ctx->hit_list, ctx->n_hit, B, T, 0, ns0, ctx->side, 0,
                                 confine2 ? tk_xcd(ESS_TKT_ATTN0) : ess_xcd{nullptr, 0, nullptr, 0});
    if (rc != ESS_OK) return rc;
    if (aev) {
      ESS_HIP(hipEventRecord(aev[1], ctx->side));
      ESS_HIP(hipEventRecord(aev[2], ctx->side));
    }
    rc = ess_launch_attn_partial(ctx, q16, c0.slot_pool, ctx->miss_list, ctx->n_miss, hB[0], T, ns0, ns1, ctx->side, hb0[0],
                                 confine2 ? tk_xcd(ESS_TKT_ATTN1) : ess_xcd{nullptr, 0, nullptr, 0});
    if (rc != ESS_OK) return rc;
    // each half is merged on the stream its Attn1 ran on: only half a merge is left behind the last fetch
    rc = ess_launch_attn_merge(ctx, hB[0], T, ns0 + ns1, a->out_bf16, a->lse, ctx->side, nullptr, 0, hb0[0]);
    if (rc != ESS_OK) return rc;
    if (aev) {
      ESS_HIP(hipEventRecord(aev[3], ctx->side));
      ctx->prof_nfill[pslot] = 3;
      ctx->prof_pair_stage[(size_t)pslot * ESS_PROF_FILL + 1] = 3;
      ctx->prof_pair_stage[(size_t)pslot * ESS_PROF_FILL + 2] = 4;
    }
    ESS_HIP(hipEventRecord(ctx->ev_fill[1], ctx->side));           // here: everything on the side stream done
    ESS_BEGIN(4);
    rc = ess_launch_attn_partial(ctx, q16 + bt1 * c.attn_heads * ESS_ROW_DIM, c1.slot_pool, ctx->miss_list + bt1 * k,
                                 ctx->n_miss + bt1, hB[1], T, ns0, ns1, st, hb0[1]);
    if (rc != ESS_OK) return rc;
    ESS_HIP(hipStreamWaitEvent(st, ctx->ev_fill[1], 0));          // Attn0 of the second half ran on the side stream
    chk.need[ESS_TKT_INDEX] += check_extra;
    rc = ess_launch_attn_merge(ctx, hB[1], T, ns0 + ns1, a->out_bf16, a->lse, st, nullptr, 0, hb0[1], confine ? &chk : nullptr);
    if (rc != ESS_OK) return rc;
    ESS_END(4);
    return ESS_OK;
  }

  // stage 4: Attn0 over resident entries while the fetches run, Attn1 over fetched ones, merge
  ESS_BEGIN(3);
  for (int h = 0; h < nh; ++h) {
    const int b0 = hb0[h], Bh = hB[h];
    const size_t bt0 = (size_t)b0 * T;
    const ess_cache ch = shift_cache(c, *cache, b0);
    rc = ess_launch_attn_partial(ctx, q16 + bt0 * c.attn_heads * ESS_ROW_DIM, ch.slot_pool, ctx->hit_list + bt0 * k,
                                 ctx->n_hit + bt0, Bh, T, 0, ns0, st, b0);
    if (rc != ESS_OK) return rc;
  }
  ESS_END(3);
  ESS_BEGIN(4);
  for (int h = 0; h < nh; ++h) {
    const int b0 = hb0[h], Bh = hB[h];
    const size_t bt0 = (size_t)b0 * T;
    const ess_cache ch = shift_cache(c, *cache, b0);
    if (pending[h]) ESS_HIP(hipStreamWaitEvent(st, ctx->ev_fill[h], 0));
    rc = ess_launch_attn_partial(ctx, q16 + bt0 * c.attn_heads * ESS_ROW_DIM, ch.slot_pool, ctx->miss_list + bt0 * k,
                                 ctx->n_miss + bt0, Bh, T, ns0, ns1, st, b0);
    if (rc != ESS_OK) return rc;
  }
  rc = ess_launch_attn_merge(ctx, B, T, ns0 + ns1, a->out_bf16, a->lse, st);
  if (rc != ESS_OK) return rc;
  ESS_END(4);
  return ESS_OK;
#undef ESS_RECORD
#undef ESS_BEGIN
#undef ESS_END
}

int ess_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) || !aligned16(dst) || !aligned16(src))
    return ess_fail(ESS_ERR_INVALID_ARG, "calib copy needs 16-byte aligned pointers and size");
  return ess_launch_calib_copy(dst, src, bytes, static_cast<hipStream_t>(stream));
}

int ess_calib_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink || (bytes & 15) || !aligned16(src))
    return ess_fail(ESS_ERR_INVALID_ARG, "calib read needs a 16-byte aligned pointer and size, and a sink");
  return ess_launch_calib_read(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int ess_append(ess_ctx* ctx, const ess_cache* cache, const uint8_t* new_key_fp8, const uint8_t* new_rows,
               uint8_t* key_fp8, int32_t* ctx_len, int32_t B, int32_t T, uint32_t step, int32_t* placed,
               const float* new_key_scale, const int32_t* block_table, int32_t n_pages, void* stream) {
  int rc = check_bt(ctx, B, T);
  if (rc != ESS_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != ESS_OK) return rc;
  if (!new_key_fp8 || !new_rows || !key_fp8 || !ctx_len) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (!aligned16(new_key_fp8) || !aligned16(new_rows) || !aligned16(key_fp8))
    return ess_fail(ESS_ERR_INVALID_ARG, "new_key_fp8, new_rows and key_fp8 must be 16-byte aligned");
  if (step < 1) return ess_fail(ESS_ERR_INVALID_ARG, "step must be >= 1");
  if (block_table) {
    if ((rc = check_paged(ctx, key_fp8, block_table, n_pages)) != ESS_OK) return rc;
    if (!new_key_scale) return ess_fail(ESS_ERR_INVALID_ARG, "new_key_scale is NULL");
  }
  return ess_launch_append(ctx->cfg, *cache, new_key_fp8, new_rows, key_fp8, ctx_len, B, T, step, placed,
                           new_key_scale, block_table, n_pages, static_cast<hipStream_t>(stream));
}

int ess_set_overlap_threshold(ess_ctx* ctx, int32_t misses_per_seq) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (misses_per_seq < 0) return ess_fail(ESS_ERR_INVALID_ARG, "threshold %d", misses_per_seq);
  ctx->auto_threshold = misses_per_seq;
  ctx->auto_calibrated = true;        // the caller's threshold is taken as measured for its workload: it applies alone
  return ESS_OK;
}

int ess_last_confined(const ess_ctx* ctx, int32_t* fetches) {
  if (!ctx || !fetches) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  *fetches = ctx->last_confined;
  return ESS_OK;
}

int ess_selfcheck_inject(ess_ctx* ctx, int32_t extra_items) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (extra_items < 0) return ess_fail(ESS_ERR_INVALID_ARG, "extra_items %d", extra_items);
  ctx->check_extra = (uint32_t)extra_items;
  return ESS_OK;
}

int ess_debug_ticket_grid(ess_ctx* ctx, int32_t workgroups) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (workgroups < 0 || workgroups > 65535) return ess_fail(ESS_ERR_INVALID_ARG, "workgroups %d outside [0, 65535]", workgroups);
  ctx->ticket_grid = workgroups;
  return ESS_OK;
}

int ess_last_overlap(const ess_ctx* ctx, int32_t* mode) {
  if (!ctx || !mode) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  *mode = ctx->last_overlap;
  return ESS_OK;
}

int ess_calib_memcpy_rows(void* dst, const void* host_pool, const int64_t* host_rows, int64_t n, int32_t row_bytes,
                          int32_t row_stride, void* stream) {
  if (!dst || !host_pool || !host_rows || n < 0 || row_bytes < 1 || row_stride < row_bytes)
    return ess_fail(ESS_ERR_INVALID_ARG, "memcpy rows: bad argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int64_t i = 0; i < n; ++i) {
    if (host_rows[i] < 0) return ess_fail(ESS_ERR_INVALID_ARG, "memcpy rows: negative row index");
    ESS_HIP(hipMemcpyAsync(static_cast<uint8_t*>(dst) + (size_t)i * row_stride,
                           static_cast<const uint8_t*>(host_pool) + (size_t)host_rows[i] * row_stride, (size_t)row_bytes,
                           hipMemcpyHostToDevice, st));
  }
  return ESS_OK;
}

int ess_profile_select(ess_ctx* ctx, uint32_t stage_mask, int32_t every) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (every < 1) return ess_fail(ESS_ERR_INVALID_ARG, "every must be >= 1");
  ctx->prof_mask = stage_mask & 0x3Fu;
  ctx->prof_every = every;
  ctx->prof_calls = 0;
  return ESS_OK;
}

int ess_profile_enable(ess_ctx* ctx, int32_t max_steps) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  if (max_steps < 0 || max_steps > 65536) return ess_fail(ESS_ERR_INVALID_ARG, "max_steps %d", max_steps);
  if (ctx->prof_ev) {
    for (int i = 0; i < ctx->prof_cap * ESS_PROF_EVENTS; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
    delete[] ctx->prof_ev;
    delete[] ctx->prof_tag;
    delete[] ctx->prof_nmark;
    delete[] ctx->prof_nfill;
    delete[] ctx->prof_pair_stage;
    ctx->prof_ev = nullptr;
  }
  ctx->prof_cap = ctx->prof_n = 0;
  if (max_steps == 0) return ESS_OK;
  const int n = max_steps * ESS_PROF_EVENTS;
  ctx->prof_ev = new (std::nothrow) hipEvent_t[n];
  ctx->prof_tag = new (std::nothrow) int8_t[(size_t)max_steps * ESS_PROF_MAIN];
  ctx->prof_nmark = new (std::nothrow) int[max_steps]();
  ctx->prof_nfill = new (std::nothrow) int[max_steps]();
  ctx->prof_pair_stage = new (std::nothrow) int[(size_t)max_steps * ESS_PROF_FILL]();
  if (!ctx->prof_ev || !ctx->prof_tag || !ctx->prof_nmark || !ctx->prof_nfill || !ctx->prof_pair_stage) {
    delete[] ctx->prof_ev; delete[] ctx->prof_tag; delete[] ctx->prof_nmark; delete[] ctx->prof_nfill;
    delete[] ctx->prof_pair_stage;
    ctx->prof_ev = nullptr;
    return ess_fail(ESS_ERR_NOMEM, "host allocation failed");
  }
  for (int i = 0; i < n; ++i) {
    hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
    if (e != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->prof_ev[j]);
      delete[] ctx->prof_ev; delete[] ctx->prof_tag; delete[] ctx->prof_nmark; delete[] ctx->prof_nfill;
      delete[] ctx->prof_pair_stage;
      ctx->prof_ev = nullptr;
      return ess_fail(ESS_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
    }
  }
  ctx->prof_cap = max_steps;
  return ESS_OK;
}

int ess_profile_intervals(ess_ctx* ctx, int32_t step, float* host_ms, int32_t* stage, int32_t cap, int32_t* n) {
  if (!ctx || !host_ms || !stage || !n) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (step < 0 || step >= ctx->prof_n) return ess_fail(ESS_ERR_INVALID_ARG, "step %d of %d recorded", step, ctx->prof_n);
  hipEvent_t* ev = ctx->prof_ev + (size_t)step * ESS_PROF_EVENTS;
  const int8_t* tag = ctx->prof_tag + (size_t)step * ESS_PROF_MAIN;
  const int nm = ctx->prof_nmark[step];
  if (nm > 0) ESS_HIP(hipEventSynchronize(ev[nm - 1]));
  int k = 0;
  for (int m = 1; m < nm && k < cap; ++m, ++k) {
    ESS_HIP(hipEventElapsedTime(&host_ms[k], ev[m - 1], ev[m]));
    stage[k] = tag[m];
  }
  *n = k;
  return ESS_OK;
}

int ess_profile_read(ess_ctx* ctx, float* host_ms, int32_t* n_steps) {
  if (!ctx || !host_ms || !n_steps) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  *n_steps = ctx->prof_n;
  for (int s = 0; s < ctx->prof_n; ++s) {
    hipEvent_t* ev = ctx->prof_ev + (size_t)s * ESS_PROF_EVENTS;
    const int8_t* tag = ctx->prof_tag + (size_t)s * ESS_PROF_MAIN;
    float* out = host_ms + (size_t)s * ESS_PROFILE_STAGES;
    for (int i = 0; i < ESS_PROFILE_STAGES; ++i) out[i] = 0.f;
    const int nm = ctx->prof_nmark[s];
    if (nm > 0) ESS_HIP(hipEventSynchronize(ev[nm - 1]));
    for (int m = 1; m < nm; ++m) {
      float ms = 0.f;
      ESS_HIP(hipEventElapsedTime(&ms, ev[m - 1], ev[m]));
      if (tag[m] >= 0 && tag[m] < ESS_PROFILE_STAGES) out[tag[m]] += ms;
    }
    for (int f = 0; f < ctx->prof_nfill[s]; ++f) {
      float ms = 0.f;
      ESS_HIP(hipEventSynchronize(ev[ESS_PROF_MAIN + 2 * f + 1]));
      ESS_HIP(hipEventElapsedTime(&ms, ev[ESS_PROF_MAIN + 2 * f], ev[ESS_PROF_MAIN + 2 * f + 1]));
      out[ctx->prof_pair_stage[(size_t)s * ESS_PROF_FILL + f]] += ms;
    }
  }
  ctx->prof_n = 0;
  return ESS_OK;
}

int ess_get_stats(ess_ctx* ctx, ess_stats* host_out, void* stream) {
  if (!ctx || !host_out) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  ESS_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  ESS_HIP(hipStreamSynchronize(ctx->side));
  const int rc = check_tickets(ctx);
  if (rc != ESS_OK) return rc;
  unsigned long long h[4];
  ESS_HIP(hipMemcpy(h, ctx->stats, sizeof(h), hipMemcpyDeviceToHost));
  host_out->steps = h[0];
  host_out->selected = h[1];
  host_out->misses = h[2];
  host_out->bytes_filled = h[3];
  return ESS_OK;
}

int ess_get_seq_stats(ess_ctx* ctx, int32_t B, ess_stats* host_out, void* stream) {
  if (!ctx || !host_out) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (B < 1 || B > ctx->cfg.max_batch) return ess_fail(ESS_ERR_INVALID_ARG, "B %d outside [1, %d]", B, ctx->cfg.max_batch);
  ESS_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  ESS_HIP(hipStreamSynchronize(ctx->side));
  static_assert(sizeof(ess_stats) == 32, "ess_stats is four 64-bit counters, the layout of the device arrays");
  ESS_HIP(hipMemcpy(host_out, ctx->seq_stats, (size_t)B * sizeof(ess_stats), hipMemcpyDeviceToHost));
  return ESS_OK;
}

int ess_reset_stats(ess_ctx* ctx, void* stream) {
  if (!ctx) return ess_fail(ESS_ERR_INVALID_ARG, "context is NULL");
  int rc = ess_launch_fill_u32(reinterpret_cast<uint32_t*>(ctx->stats), 8, 0u, static_cast<hipStream_t>(stream));
  if (rc != ESS_OK) return rc;
  return ess_launch_fill_u32(reinterpret_cast<uint32_t*>(ctx->seq_stats), 8 * ctx->cfg.max_batch, 0u, static_cast<hipStream_t>(stream));
}

}  // extern "C"
