/*
 * ess.h -- C ABI of libess: the decode-step hot path of ESS (Extended Sparse
 * Server, arXiv 2512.10576) for DeepSeek-V3.2-Exp-style sparse attention,
 * written for AMD MI355X (gfx950).
 *
 * Per layer and decode step the paper's design runs (Sec. 3, Sec. 3.3):
 *   indexer over the GPU-resident Indexer-Cache -> Top-2K selection ->
 *   look-up of the selected entries in the GPU-side Sparse Memory Pool under
 *   an LRU policy (Sec. 3.2) -> fetch of the missed entries from the CPU-side
 *   Total Memory Pool by direct GPU access to pinned host memory (Sec. 3.1,
 *   FlashTrans) -> SparseMLA over the selected entries, split in Attn0
 *   (resident entries, overlapping the fetch) and Attn1 (fetched entries),
 *   merged (Sec. 3.3, DA overlap).
 * Each of these stages is one call below; ess_decode_step chains them.
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary.  Every call returns an int:
 *     ESS_OK (0) or a negative ess_status.  ess_last_error() gives a text for
 *     the last failure on the calling thread.
 *   - Argument checks are synchronous.  GPU work is ENQUEUED on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns without waiting, except where stated.
 *   - Pointers are DEVICE pointers unless the name starts with host_.  The
 *     caller owns every data buffer, the cache state arrays and the pinned
 *     host pool; the library owns only the opaque ess_ctx (workspace, one
 *     side stream, events).  No call frees or reallocates caller memory.
 *   - Row bases must be 16-byte aligned; row_stride must be a multiple of 16.
 *   - Shapes use: B sequences, T query tokens per sequence (1 or 2), Lmax
 *     cached positions per sequence (row pitch of key/score/slot_of), Hi x Di
 *     indexer heads x dim, k = topk, H attention heads, S slots per sequence.
 *     Visible positions of query t: vis(b,t) = ctx_len[b] - (T-1-t), i.e. the
 *     cache already holds the T new tokens and query t sees itself and all
 *     earlier positions (multi-token decode, the paper's MTP setting, Table 1).
 *   - A context is not thread-safe; calls on one context must not overlap.
 */
#ifndef ESS_H
#define ESS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ESS_OK = 0,
  ESS_ERR_INVALID_ARG = -1, /* null / misaligned pointer, size out of the configured range */
  ESS_ERR_UNSUPPORTED = -2, /* a shape no kernel was compiled for */
  ESS_ERR_CAPACITY = -3,    /* slot pool smaller than one step's selection (S < T*k), or over a stated maximum */
  ESS_ERR_NOMEM = -4,       /* workspace allocation failed */
  ESS_ERR_HIP = -5,         /* a HIP runtime call failed; text in ess_last_error() */
  ESS_ERR_INTERNAL = -6     /* a device-side assertion of an EARLIER ess_decode_step failed (a defect in the library,
                               not a property of the inputs or of the machine); reported by the next ess_decode_step
                               or ess_get_stats */
} ess_status;

#define ESS_LATENT_DIM 512 /* value part of a Latent-Cache entry */
#define ESS_ROPE_DIM 64    /* rotary part */
#define ESS_FMT_BF16 0     /* entry = 576 bf16 (1152 bytes) */
#define ESS_FMT_FP8 1      /* entry = 512 e4m3 + 4 bf16 scales (one per 128) + 64 bf16 rope (648 bytes) */

#define ESS_FLAG_SERIAL 1u /* run the miss fill on the caller's stream (no side stream, no overlap) */
#define ESS_FLAG_DBA 2u    /* ess_decode_step: DualBatch-Attention overlap (Sec. 3.3): the batch is processed in two
                              halves so that the second half's indexer and top-k overlap the first half's fetch */

#define ESS_FLAG_AUTO 4u   /* ess_decode_step chooses per step between the DA and the DBA schedule from the miss
                              counts of the previous step (the paper's switch on the number of misses, Sec. 3.3);
                              threshold: ess_set_overlap_threshold.  Ignored with ESS_FLAG_SERIAL. */

/* ess_decode_step computes stages 1 and 2 as ess_index_score + ess_topk do, through a full score array, unless
 * ESS_FLAG_FUSED_SELECT asks for the form of ess_index_topk (no score array).  The results are the same bits; on
 * MI355X the first form gives the shorter step (the second is faster only as a stand-alone call on large batches). */
#define ESS_FLAG_DENSE_SCORES 8u  /* through the score array (the default; overrides ESS_FLAG_FUSED_SELECT) */
#define ESS_FLAG_FUSED_SELECT 16u /* as ess_index_topk */

typedef struct ess_ctx ess_ctx;

/* Fixed for the life of a context. */
typedef struct {
  uint32_t struct_size;   /* sizeof(ess_config), checked */
  int32_t max_batch;      /* largest B any call will pass; <= 4096 */
  int32_t max_q_tokens;   /* largest T (1 to 4, and T * topk <= 8192); the index score handles two query
                             tokens per pass over the keys, so T = 3, 4 read the Indexer-Cache twice */
  int32_t max_ctx;        /* Lmax: row pitch of key, score and slot_of; <= 524288 */
  int32_t idx_heads;      /* Hi, 1..64 */
  int32_t idx_dim;        /* Di, 32 | 64 | 128 */
  int32_t topk;           /* k, 1..4096, with T*k <= 8192 */
  int32_t attn_heads;     /* H, 1..128 */
  int32_t latent_fmt;     /* ESS_FMT_BF16 | ESS_FMT_FP8 */
  int32_t row_stride;     /* bytes between entries in slot pool and host pool (>= entry size, multiple of 16) */
  int32_t slots_per_seq;  /* S; = max_ctx when nothing is offloaded */
  float sm_scale;         /* softmax scale of the attention logits */
  uint32_t flags;         /* ESS_FLAG_* */
} ess_config;

/* Caller-owned Sparse Memory Pool state of ONE layer (Sec. 3.2).  Entry
 * granularity (Sec. 3.1: one Latent-Cache entry is the swap unit). */
typedef struct {
  uint8_t* slot_pool;           /* [B,S,row_stride] device: the GPU-side pool */
  const uint8_t* host_pool_dev; /* [B,Lmax,row_stride] pinned host memory, DEVICE-side address of it
                                   (hipHostMalloc'ed / torch pinned memory is directly addressable);
                                   NULL = nothing is offloaded: then S == Lmax and slot s holds token s */
  int32_t* slot_of;             /* [B,Lmax] slot of a token, -1 = not resident */
  int32_t* token_of;            /* [B,S]    token held by a slot, -1 = empty */
  uint32_t* stamp;              /* [B,S]    step of last use, 0 = never used */
} ess_cache;

/* Per-call inputs and outputs of ess_decode_step. */
typedef struct {
  const uint8_t* q_idx_fp8;     /* [B,T,Hi,Di] e4m3 indexer queries */
  const float* w;               /* [B,T,Hi] indexer head weights */
  const uint8_t* key_fp8;       /* [B,Lmax,Di] e4m3 Indexer-Cache, one key per token */
  const int32_t* ctx_len;       /* [B] cached positions per sequence (<= Lmax) */
  const void* q_bf16;           /* [B,T,H,576] absorbed attention queries */
  const int32_t* topk_override; /* [B,T,k] or NULL.  When given, stages 1-2 still run and fill
                                   idx_out, but the cache and the attention use these indices
                                   (trace replay); entries must be distinct per (b,t), < vis, or -1 */
  int32_t B, T;
  uint32_t step;                /* LRU clock: >= 1 and strictly increasing per cache */
  int32_t* idx_out;             /* [B,T,k] selected positions, ascending, -1 padded */
  void* out_bf16;               /* [B,T,H,512] attention output */
  float* lse;                   /* [B,T,H] log-sum-exp of the logits, or NULL */
  int32_t* miss_count;          /* [B] entries fetched from the host pool this step, or NULL */
  const int32_t* block_table;   /* NULL: key_fp8 is flat [B,max_ctx,idx_dim].  Else [B, max_ctx/64] page ids and
                                   key_fp8 is a page pool, see ess_index_score_paged */
  int32_t n_pages;              /* pages in the pool (with block_table) */
  int32_t reserved;             /* 0 */
} ess_step_args;

/* A context owns scratch memory that its calls share (scores, candidate lists and counters, partial
 * attention results, event objects): calls on one context must not overlap in time -- enqueue them
 * on one stream, or order the streams.  Different contexts are independent. */
/* Create a context: validates the configuration, allocates the workspace
 * (see ess_workspace_bytes), a side stream and events on the current device.
 * ESS_ERR_INVALID_ARG / ESS_ERR_UNSUPPORTED / ESS_ERR_CAPACITY (S < T*k) / ESS_ERR_NOMEM.
 * The calls that update the Sparse Memory Pool (ess_cache_admit, ess_gather_latent, ess_decode_step and ess_append
 * with an offloaded cache) keep a bitmap of max_ctx bits, the larger of a 32 KiB histogram and 8 bytes per
 * selected entry (max_q_tokens * topk, rounded up to a power of two), and 4 bytes per selected entry in the 160 KiB
 * of a CU's LDS: max_ctx / 8 + max(32768, 8 * pow2(T*k)) + 4 * T*k + 1 KiB <= 160 KiB.  Every max_ctx fits with
 * T*k <= 4096; with T*k = 8192 (64 + 32 KiB for the selection) max_ctx up to about 516000 does.  A configuration that
 * does not fit is accepted by ess_create, and those calls return ESS_ERR_UNSUPPORTED. */
int ess_create(const ess_config* cfg, ess_ctx** out);
/* Waits for the context's side stream, frees what ess_create allocated. */
int ess_destroy(ess_ctx* ctx);
/* Text of the last failure on this thread ("" if none).  Never NULL. */
const char* ess_last_error(void);
/* Device bytes ess_create will allocate for this configuration. */
int ess_workspace_bytes(const ess_config* cfg, size_t* out);

/* Sparse Memory Pool set-up.  With host_pool_dev == NULL: identity residency
 * (slot_of[b,s] = s, token_of[b,s] = s, stamp 0).  Otherwise all slots empty. */
int ess_cache_reset(ess_ctx* ctx, const ess_cache* cache, int32_t B, void* stream);
/* LRU-Warmup (Sec. 3.2): insert the given entries as one LRU step, fetching
 * missing ones from the host pool.  tok [B,n] (-1 = none), n <= T*k. */
int ess_cache_admit(ess_ctx* ctx, const ess_cache* cache, const int32_t* tok, int32_t B, int32_t n,
                    uint32_t step, void* stream);

/* Stage 1, indexer (Sec. 3: the Indexer-Cache scores every Latent-Cache entry):
 *   score[b,t,s] = sum_j w[b,t,j] * max(0, sum_d q[b,t,j,d] * key[b,s,d]),  s < vis(b,t);
 * fp8 x fp8 products accumulated in fp32.  score [B,T,Lmax] fp32; positions
 * s >= vis(b,t) hold unspecified values, and so does the score of a key when its
 * bytes, or those of the query, hold an e4m3 NaN (0x7f, 0xff). */
int ess_index_score(ess_ctx* ctx, const uint8_t* q_idx_fp8, const float* w, const uint8_t* key_fp8,
                    const int32_t* ctx_len, int32_t B, int32_t T, float* score, void* stream);

/* Stage 1 over a paged Indexer-Cache with one scale per key (Sec. 3: an Indexer-Cache entry is 132
 * bytes, 128 fp8 + one float; Sec. 3.3 names the kernel paged_mqa_logits).  key_pages is a pool of
 * n_pages pages of ESS_PAGE_TOKENS * (idx_dim + 4) bytes: 64 keys of idx_dim fp8 bytes, then 64
 * float32 scales.  Token s of sequence b is row s % 64 of page block_table[b, s / 64]
 * (block_table [B, max_ctx/64] int32, device; entries for pages at or past ctx_len are not read;
 * ids outside [0, n_pages) are clamped into the pool).  The stored key stands for scale * key with
 * scale > 0, and
 *   score[b,t,s] = scale_s * sum_j w[b,t,j] * max(0, q[b,t,j,:] . key_s),
 * the sum as in ess_index_score, then one float32 multiplication.  Needs max_ctx % 64 == 0 and
 * key_pages 16-byte aligned. */
#define ESS_PAGE_TOKENS 64
int ess_index_score_paged(ess_ctx* ctx, const uint8_t* q_idx_fp8, const float* w, const uint8_t* key_pages,
                          const int32_t* block_table, int32_t n_pages, const int32_t* ctx_len, int32_t B,
                          int32_t T, float* score, void* stream);

/* Stage 2, Top-K (Sec. 3: the top 2,048 entries): idx[b,t,:] = the min(k,vis)
 * positions largest under (score descending, position ascending), written in
 * ascending position order, then -1.  NaN ranks as -inf; +0 and -0 are equal. */
int ess_topk(ess_ctx* ctx, const float* score, const int32_t* ctx_len, int32_t B, int32_t T,
             int32_t* idx, void* stream);

/* Stages 1 and 2 as one: idx as ess_topk gives it for the scores ess_index_score (block_table NULL, key_fp8
 * [B,Lmax,Di]) or ess_index_score_paged (block_table given, key_fp8 = the page pool) would give -- the same bits --
 * without the score array (Sec. 3: only the top-k positions leave the indexer).  ess_decode_step runs this form
 * under ESS_FLAG_FUSED_SELECT.  Four launches: the scores of a sample of each sequence's keys (one block of 64 in every 2048) give, per
 * row (b,t), a lower bound that very probably leaves at least k and at most a few thousand scores at or above it;
 * the main pass over all keys computes every score and keeps only (position, score) of those that reach the bound;
 * the selection is finished among them, exactly.  A row whose candidates number fewer than k or more than 8192
 * (a misleading sample, massive ties at the bound) is recomputed from all its scores by one workgroup: correct, but
 * slow (about 0.2 ms for a row of 128K keys). */
int ess_index_topk(ess_ctx* ctx, const uint8_t* q_idx_fp8, const float* w, const uint8_t* key_fp8,
                   const int32_t* block_table, int32_t n_pages, const int32_t* ctx_len, int32_t B, int32_t T,
                   int32_t* idx, void* stream);

/* ess_topk for callers that cannot allocate device memory and therefore cannot create a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as ess_topk for
 * score [B,T,max_ctx] and k (idx [B,T,k]).  The call allocates nothing: its scratch memory (candidate
 * lists of rows that several workgroups share, and their counters) is an array inside the library's
 * image, 8 MiB + 1536 bytes, which every GPU the library runs on holds until the process ends.  Limits:
 * B*T <= ESS_TOPK_STATIC_MAX_ROWS, T <= 4, max_ctx <= 524288, k <= 4096; beyond them ESS_ERR_CAPACITY.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams or
 * threads) race; serialise them. */
#define ESS_TOPK_STATIC_MAX_ROWS 128
int ess_topk_static(const float* score, const int32_t* ctx_len, int32_t B, int32_t T, int32_t max_ctx, int32_t k,
                    int32_t* idx, void* stream);

/* Stages 3 + 5, Sparse Memory Pool look-up, LRU update and miss fetch
 * (Sec. 3.1, 3.2).  Per sequence: R = distinct valid entries of idx[b]; resident
 * ones are hits (stamp := step); the others, in ascending position, take the
 * slots smallest in (stamp, slot) among slots with stamp < step, whose former
 * tokens become non-resident; their rows are copied host pool -> slot.
 *   slot_idx [B,T,k]  slot of every selected entry after the step (-1 where idx is -1)
 *   rows_out [B,T,k,row_stride] or NULL: the selected rows, gathered (zero where idx is -1)
 *   miss_count [B] or NULL
 * The fetch runs on the context's side stream unless ESS_FLAG_SERIAL; either
 * way it is ordered before anything enqueued on `stream` after this call. */
int ess_gather_latent(ess_ctx* ctx, const ess_cache* cache, const int32_t* idx, const int32_t* ctx_len,
                      int32_t B, int32_t T, uint32_t step, int32_t* slot_idx, uint8_t* rows_out,
                      int32_t* miss_count, void* stream);

/* Stage 4, SparseMLA decode (Sec. 3.3) in absorbed form: an entry's 576 values
 * are the key, its first 512 the value.
 *   z_s = sm_scale * q . c_s ; lse = log sum_s exp z_s ; out = sum_s exp(z_s - lse) c_s[:512]
 * over the entries slot_idx[b,t,:] >= 0 of slot_pool [B,S,row_stride].  bf16
 * operands (fp8 entries are dequantised to bf16), fp32 accumulation and softmax.
 * The entry list is processed in several parts whose normalised results are
 * merged; they are held as fp16 in between (11 significant bits, against the 8
 * of the bf16 output), each head's part divided by the power of two that keeps
 * its largest value below 2^15, so entry values of any bf16 magnitude pass
 * (values more than 2^29 below the largest one of their head and part are
 * flushed to zero).  Empty selection: out = 0, lse = -inf. */
int ess_sparse_mla_decode(ess_ctx* ctx, const void* q_bf16, const uint8_t* slot_pool,
                          const int32_t* slot_idx, int32_t B, int32_t T, void* out_bf16, float* lse,
                          void* stream);

/* One layer-step: stages 1-5 in order, with the miss fetch overlapping Attn0, the attention over the
 * entries that were resident (Sec. 3.3, DA overlap), then Attn1 over the fetched ones, merged.  With
 * ESS_FLAG_DBA the fetch of the first half of the batch also overlaps the second half's indexer,
 * top-k and bookkeeping (DBA overlap).  Part of the work runs on the context's side stream; all of it
 * is ordered after what was enqueued on `stream` before the call and before what is enqueued on it
 * afterwards.  Results are identical, bit for bit, in all modes. */
int ess_decode_step(ess_ctx* ctx, const ess_cache* cache, const ess_step_args* args, void* stream);

/* ESS_FLAG_AUTO: the DBA schedule is used for a step when the previous bookkeeping of this context
 * saw more than `misses_per_seq` misses per sequence on average (Sec. 3.3: DBA pays when the fetch is
 * long), else the DA schedule.  The counts travel through pinned host memory and are read without
 * waiting for the GPU, so the decision may lag by a step; results do not depend on it.  Default 150
 * (measured crossover for 1152-byte entries, batch 64, 128K context on MI355X).  With the default
 * threshold the DBA schedule is only chosen when the index score of half the batch is long enough to
 * be worth hiding (estimated from batch x max_ctx: at least about 50 us, i.e. not at batch 64 and 32K
 * context, where the DA schedule was faster at every miss count); a threshold set with
 * ess_set_overlap_threshold is taken as measured for the caller's workload and applies alone.
 * ess_last_overlap: schedule the latest ess_decode_step used: 0 DA, 1 DBA, 2 serial. */
int ess_set_overlap_threshold(ess_ctx* ctx, int32_t misses_per_seq);
int ess_last_overlap(const ess_ctx* ctx, int32_t* mode);

/* Under ESS_FLAG_AUTO a step may confine its fetches from host memory to two of the eight XCDs and
 * keep the kernels that run beside them on the other six (FlashTrans reads, Sec. 3.1, slow every
 * memory access of the XCD they are issued from).  Those kernels take their work items by ticket:
 * every workgroup that runs on an XCD that takes work draws items from a counter until none is left,
 * and should no workgroup of a launch sit on such an XCD, the last one to arrive does all the work.
 * The results therefore do not depend on where the hardware places workgroups; ess_create only
 * probes whether workgroups go round the XCDs evenly, which is when confining pays.  Each such step
 * ends with a device-side assertion that every launch handed out at least as many tickets as it had
 * work items; a failure is reported, as ESS_ERR_INTERNAL, by the next ess_decode_step or
 * ess_get_stats on the context, and the context confines nothing from then on.
 * ess_last_confined: fetches of the latest ess_decode_step that were confined (0, 1 or 2).
 * ess_selfcheck_inject: test hook.  The assertion of the next confined step expects `extra_items`
 * more work items than there are, so that it fails (for extra_items > the workgroups of the launch)
 * although the step itself is complete; every kernel runs and ends as usual.
 * ess_debug_ticket_grid: test hook.  Ticket-fed launches (and confined fetches) of later steps use
 * exactly `workgroups` workgroups, whatever their number of work items (0 = the library's own
 * sizing); results are the same for every value >= 1. */
int ess_last_confined(const ess_ctx* ctx, int32_t* fetches);
int ess_selfcheck_inject(ess_ctx* ctx, int32_t extra_items);
int ess_debug_ticket_grid(ess_ctx* ctx, int32_t workgroups);

/* Append (Sec. 3.3, the write-back of newly generated entries): for each sequence b with
 * L0 = ctx_len[b], the t-th of its T new tokens takes position p = L0 + t:
 *   - key_fp8[b,p,:]  = new_key_fp8[b,t,:]            (Indexer-Cache, device, written)
 *   - host pool[b,p,:] = new_rows[b,t,:]              (through cache->host_pool_dev, which must then be a
 *                                                     writable mapping; skipped when it is NULL)
 *   - the entry is admitted to the slot pool as most recently used: it takes the slot smallest in
 *     (stamp, slot index) among slots with stamp < step (the victim rule of the bookkeeping; the
 *     former token of that slot becomes non-resident), gets stamp `step` and its bytes are written
 *     into the slot.  If every slot carries stamp `step` the entry is not admitted (it is in the host
 *     pool).  Without a host pool the slot is p itself.
 *   - ctx_len[b] = L0 + min(T, max_ctx - L0)  (device, in/out); tokens past max_ctx are dropped.
 * new_key_fp8 [B,T,idx_dim], new_rows [B,T,row_stride] (entries in the pool's storage format), both
 * device, 16-byte aligned.  placed [B,T] (device, may be NULL) receives the slot of each new token,
 * -1 if dropped or not admitted.  Call it on the stream of the decode steps, after the step that
 * produced the entries; `step` is that step's number or a later one.
 * Paged Indexer-Cache: with block_table != NULL, key_fp8 is the page pool of ess_index_score_paged,
 * the key goes to row p % 64 of page block_table[b, p / 64] and new_key_scale[b,t] (float32 [B,T],
 * device, required then) beside it.  The caller maps pages ahead of the context: a token whose page
 * id is outside [0, n_pages) is dropped like one past max_ctx, and so are the tokens after it. */
int ess_append(ess_ctx* ctx, const ess_cache* cache, const uint8_t* new_key_fp8, const uint8_t* new_rows,
               uint8_t* key_fp8, int32_t* ctx_len, int32_t B, int32_t T, uint32_t step, int32_t* placed,
               const float* new_key_scale, const int32_t* block_table, int32_t n_pages, void* stream);

/* Counters accumulated by ess_gather_latent / ess_cache_admit / ess_decode_step
 * since the last ess_reset_stats.  ess_get_stats WAITS for `stream` and the
 * side stream. */
typedef struct {
  uint64_t steps;        /* bookkeeping steps */
  uint64_t selected;     /* valid entries requested (an entry selected by both query tokens counts twice) */
  uint64_t misses;       /* entries fetched from the host pool */
  uint64_t bytes_filled; /* misses * row_stride */
} ess_stats;
int ess_get_stats(ess_ctx* ctx, ess_stats* host_out, void* stream);
/* The same counters per sequence (Sec. 3.2 evaluates miss counts; Sec. 3.3 switches on them): host_out[b] for the
 * first B sequences of the context, `steps` = bookkeeping steps of that sequence (admissions included).  Waits like
 * ess_get_stats; ess_reset_stats clears both. */
int ess_get_seq_stats(ess_ctx* ctx, int32_t B, ess_stats* host_out, void* stream);
int ess_reset_stats(ess_ctx* ctx, void* stream);

/* Measurement support.  After ess_profile_enable(ctx, n) every ess_decode_step records HIP
 * events on its stream between the stages (up to n steps; n = 0 disables and frees them).
 * ess_profile_read WAITS for the recorded events and returns, per recorded step, the
 * milliseconds of: [0] index score, [1] top-k, [2] cache bookkeeping, [3] Attn0,
 * [4] Attn1 (including any wait for the fetch) + merge, [5] the miss fetch kernel on its own
 * stream (0 when nothing is offloaded).  host_ms holds n*6 floats. */
#define ESS_PROFILE_STAGES 6
int ess_profile_enable(ess_ctx* ctx, int32_t max_steps);
int ess_profile_read(ess_ctx* ctx, float* host_ms, int32_t* n_steps);
/* Before ess_profile_read: the intervals between the events that recorded step `step` (0-based among the
 * recorded ones) left on the caller's stream, in stream order: host_ms[i] milliseconds, stage[i] the stage the
 * interval was booked under (as above) or -1 (not booked: the gap in front of a kernel that carries its own
 * events).  A stage that appears twice was launched twice (the two halves of a split-batch step).  At most cap
 * intervals; *n = how many.  WAITS for the events. */
int ess_profile_intervals(ess_ctx* ctx, int32_t step, float* host_ms, int32_t* stage, int32_t cap, int32_t* n);
/* Restrict the timing to some stages (bit i = stage i above; default all) and to every `every`-th
 * ess_decode_step (default 1): recorded events cost a few percent of a step, so a run whose
 * throughput matters samples one kernel on a few steps.  ess_profile_read then returns the sampled
 * steps only. */
int ess_profile_select(ess_ctx* ctx, uint32_t stage_mask, int32_t every);
/* A plain device-to-device copy kernel (reads `bytes`, writes `bytes`; bytes a multiple of 16,
 * pointers 16-byte aligned): known traffic against which hardware counters can be scaled. */
int ess_calib_copy(void* dst, const void* src, size_t bytes, void* stream);
/* A plain read kernel (reads `bytes` once, 16-byte loads, four per thread in flight; bytes a multiple of 16, src
 * 16-byte aligned): the rate a pure read stream reaches on the device, the measured counterpart of the nominal
 * HBM peak.  sink: ESS_CALIB_READ_WGS uint32 words (device) that receive a checksum, so that the loads are used. */
#define ESS_CALIB_READ_WGS 4096
int ess_calib_read(const void* src, size_t bytes, uint32_t* sink, void* stream);
/* The transfer the paper starts from (Sec. 3.1, the per-block copy that FlashTrans replaces): one
 * hipMemcpyAsync per entry, n entries of row_bytes each, entry i from
 * host_pool + host_rows[i] * row_stride (pinned host memory, HOST pointer) to
 * dst + i * row_stride (device).  host_rows is a HOST array.  Enqueues on `stream`, returns without
 * synchronizing.  For the granularity comparison only; no stage of the path uses it. */
int ess_calib_memcpy_rows(void* dst, const void* host_pool, const int64_t* host_rows, int64_t n,
                          int32_t row_bytes, int32_t row_stride, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ESS_H */
