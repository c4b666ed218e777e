// Internal declarations shared by the translation units of libess (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "ess.h"

#define ESS_MAX_CTX 524288      // selection bitmap of one sequence must fit in LDS (64 KiB)
#define ESS_MAX_TOPK 4096
#define ESS_MAX_SEL 8192        // T * k
#define ESS_ATTN_TILE 32        // entries per attention tile
#define ESS_MAX_SPLITS 20       // partial results per (b,t): Attn0 splits + Attn1 splits
#define ESS_ROW_DIM 576
#define ESS_ZERO_ROW_BYTES 2048  // >= the largest row_stride
#define ESS_TOPK_SHARED_ROWS 128 // rows (b,t) up to which a top-k row is shared by several workgroups
#define ESS_N_TICKETS 9         // ticket-fed launches of one step:
enum {                          // which launch uses which counter block
  ESS_TKT_FETCH1 = 0,           // the first (or only) fetch
  ESS_TKT_INDEX = 1,            // index score (dense or emitting)
  ESS_TKT_SAMPLE = 2,           // fused selection: sample pass; two-kernel top-k: candidate pass
  ESS_TKT_TAU = 3,              // fused selection: lower bounds; two-kernel top-k: its finish (the block after its candidate pass)
  ESS_TKT_FINISH = 4,           // top-k finish
  ESS_TKT_BOOK = 5,             // bookkeeping
  ESS_TKT_FETCH2 = 6,           // the second fetch of the split-batch schedule
  ESS_TKT_ATTN0 = 7,
  ESS_TKT_ATTN1 = 8
};
// Counters of one such launch.  They are device-scope atomics from all XCDs, which the memory side executes one
// after the other per address range, so each counter has 256 bytes to itself: [ESS_TK_WORK] work items handed out,
// [ESS_TK_ARRIVE] workgroups that arrived on XCDs that take no work, [ESS_TK_CLASS + 64 c] per-XCD counters of
// launches that hand out work XCD by XCD (attention).  ESS_TICKET_USED counters at a stride of 64 words.
#define ESS_TICKET_WORDS 1024
#define ESS_TK_STRIDE 64
#define ESS_TK_WORK 0
#define ESS_TK_ARRIVE 64
#define ESS_TK_CLASS 128
#define ESS_TICKET_USED 10
// A confined fetch runs on these XCDs, and the kernels beside it stay off them.  Measured at batch 64, 128K
// context (step time), with the kernels of the time: one XCD 0.668 ms (the fetch drops to 40 GB/s behind a single
// XCD's port when the other seven stream from HBM), two 0.614, three 0.605, four 0.631 (the index score is short
// of CUs), unconfined 0.631.  With the current kernels two and three XCDs give the same step there (0.590 ms), and
// two give the kernels beside the fetch more of the chip: the index score beside it runs at 4.3 instead of 3.9
// TB/s, and at batch 128 with two query tokens and quantised entries the step is 3 % shorter (1.078 against 1.113
// ms).  48 workgroups on the two XCDs (40: the same; 64: 10 % longer steps).
#ifndef ESS_FETCH_XCD_MASK
#define ESS_FETCH_XCD_MASK 3u
#endif
#ifndef ESS_FETCH_CONFINED_WGS
#define ESS_FETCH_CONFINED_WGS 48
#endif
#define ESS_PROF_MAIN 24        // stage marks on the caller's stream per step
#define ESS_PROF_FILL 3         // event pairs per step for work off the caller's stream (fetches, side-stream attention)
#define ESS_PROF_EVENTS (ESS_PROF_MAIN + 2 * ESS_PROF_FILL)

struct ess_ctx {
  ess_config cfg;
  int device;
  hipStream_t side;             // miss fetch stream (default priority)
  hipEvent_t ev_book[2], ev_fill[2];  // bookkeeping done / fetch done, per batch half
  // workspace (device)
  float* score_ws;              // [B,T,Lmax]
  int32_t* slot_idx_ws;         // [B,T,k]
  int32_t* hit_list;            // [B,T,k] slots of entries resident before the step, compacted
  int32_t* miss_list;           // [B,T,k] slots of entries fetched in this step, compacted
  int32_t* n_hit;               // [B,T]
  int32_t* n_miss;              // [B,T]
  int32_t* fill_tok;            // [B,T*k] token to fetch
  int32_t* fill_slot;           // [B,T*k] slot to fetch into
  int32_t* miss_cnt;            // [B]
  uint16_t* o_part;             // [B*T, ESS_MAX_SPLITS, H, 512] partial attention results, fp16 bits (times lse_part[..][1])
  float* lse_part;              // [B*T, ESS_MAX_SPLITS, H, 2]: log-sum-exp of a partial result and the power of two its fp16 values were divided by
  unsigned long long* stats;    // [4]
  unsigned long long* seq_stats; // [max_batch][4] the same four counters per sequence
  uint8_t* zero_row;            // ESS_ZERO_ROW_BYTES of zeros, never written: source of masked attention rows
  unsigned long long* topk_cand; // [ESS_TOPK_SHARED_ROWS][8192] candidate keys of rows shared by several workgroups
  uint32_t* topk_cnt;           // [ESS_TOPK_SHARED_ROWS] candidates listed per row: zero between steps
  uint32_t* topk_tau;           // [ESS_TOPK_SHARED_ROWS][2] the bounds the candidate pass worked with (see sample_bins)
  // fused selection inside ess_decode_step / ess_index_topk (no score array): per row (b,t)
  float* sel_sample;            // [B,T,64 * ess_sample_count(max_ctx)] scores of the sequence's sample blocks
  uint32_t* sel_tau;            // [B,T][2] bounds of the row's selection (ess_orderable images): candidates reach [0]; the k-th largest score very probably lies below [1]
  unsigned long long* sel_cand; // [B,T][ess_sel_cand_cap()] candidate keys
  uint32_t* sel_cnt;            // [B,T] candidates appended
  uint32_t* tickets;            // [ESS_N_TICKETS][ESS_TICKET_WORDS] work counters of kernels that run beside a fetch (see ess_xcd)
  bool xcds_even;               // workgroups go round the eight XCDs evenly (probed at creation): confining a fetch pays
  bool book_fits;               // the bookkeeping kernel's LDS arrays fit this configuration (else the cache calls are refused)
  int ticket_grid;              // > 0: ticket-fed launches use exactly this many workgroups (ess_debug_ticket_grid)
  int last_confined;            // fetches of the latest decode step that were confined to ESS_FETCH_XCD_MASK
  uint32_t check_extra;         // ess_selfcheck_inject: work items the next confined step's check expects on top
  size_t ws_bytes;
  // overlap switch (ESS_FLAG_AUTO): per-sequence miss counts of the latest bookkeeping, written by the
  // kernel into pinned host memory and read by the host, without a synchronisation, at the next step
  int32_t* host_miss;           // [max_batch] host address
  int32_t* host_miss_dev;       // device alias of the same memory
  int32_t auto_threshold;       // mean misses per sequence above which the split-batch schedule is used
  bool auto_calibrated;         // threshold set by the caller: no further condition on the index-score time
  int32_t last_overlap;         // schedule of the latest ess_decode_step: 0 DA, 1 DBA, 2 serial
  // optional stage timing (ess_profile_enable)
  hipEvent_t* prof_ev;          // [prof_cap][ESS_PROF_EVENTS]: marks on the caller's stream, then pairs around each fetch
  int8_t* prof_tag;             // [prof_cap][ESS_PROF_MAIN] stage a mark closes (-1 = start)
  int* prof_nmark;              // [prof_cap] marks recorded
  int* prof_nfill;              // [prof_cap] event pairs recorded off the caller's stream
  int* prof_pair_stage;         // [prof_cap][ESS_PROF_FILL] stage each pair times (5 fetch, 3 Attn0, 4 Attn1)
  int prof_cap, prof_n;
  uint32_t prof_mask;           // stages that are timed (bit i = stage i of ess_profile_read)
  int prof_every, prof_calls;   // every prof_every-th ess_decode_step is timed
};

// A fetch from host memory slows every memory access of the XCD its workgroups run on (the long
// reads fill that XCD's L2 request queues): a latency-bound kernel beside a 28-workgroup fetch spread
// over the chip takes 3.4x its time, beside the same fetch confined to one XCD -- which costs the fetch
// 3 % of its rate -- and kept off that XCD it is not slowed at all (measured).  A kernel launched with
// an ess_xcd therefore does not map workgroups to work by their index: workgroups on the XCDs in
// `avoid` exit, the others take work items from a counter until it runs out, however many they are.
// The launch is complete wherever the hardware puts its workgroups: should none of them sit on an XCD
// that takes work, the last workgroup to arrive does all of it.
struct ess_xcd {
  uint32_t* ticket;             // the launch's counters (ESS_TICKET_WORDS words), zero at launch; null: work by workgroup index
  uint32_t avoid;               // bit i: XCD i takes no work
  uint32_t* host_need;          // host memory, may be null: the launcher leaves the number of work items here
  int grid_override;            // > 0: launch exactly this many workgroups (test hook)
};
// The last kernel of a step that used such launches compares each launch's counters with its number of
// work items, as an assertion: a counter below it means a bug in the hand-out, reported through `flag`
// (pinned host memory) at the host's next call.
struct ess_ticket_check {
  const uint32_t* tickets;      // null: no check
  int32_t* flag;
  uint32_t need[ESS_N_TICKETS];
};
#ifdef __HIPCC__
// Non-temporal 16-byte store.  The large outputs of a step (scores, fetched rows, partial attention results, the
// attention output) are written this way: lines written with ordinary stores stay in the memory-side cache as
// modified lines until something displaces them, and that something is the next index-score launch, whose key
// stream then shares the HBM with their write-back (measured: a launch that streams 470 MB takes 9 us longer after
// 64 MiB of ordinary stores, 32 us longer after 256 MiB, and not a microsecond longer after the same bytes
// stored non-temporally).  The readers of these outputs lose nothing: they run on other XCDs than the writers,
// whose L2 they could not read from anyway.
typedef unsigned ess_uintx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void ess_store_nt(uint4* p, const uint4& v) {
  __builtin_nontemporal_store(ess_uintx4{v.x, v.y, v.z, v.w}, reinterpret_cast<ess_uintx4*>(p));
}
__device__ __forceinline__ int ess_xcc_id() { return __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15; }   // hwreg XCC_ID, bits 3:0
// Does this workgroup of a ticket-fed launch take work?  Same answer in all threads; `slot` is a __shared__ int.
// `on`: this workgroup sits on an XCD that takes work.  One that does not counts itself in and leaves -- unless it
// finds that every workgroup of the launch has done the same (it is the last, and none sits where work is
// taken): then it does the work.  Workgroups that take work touch no counter here.
__device__ __forceinline__ bool ess_ticket_join(uint32_t* ticket, bool on, int* slot) {
  if (on) return true;
  if (threadIdx.x == 0) {
    const uint32_t a = atomicAdd(ticket + ESS_TK_ARRIVE, 1u);
    *slot = (a + 1u == gridDim.x * gridDim.y * gridDim.z) ? 1 : 0;
  }
  __syncthreads();
  const int r = __builtin_amdgcn_readfirstlane(*slot);
  __syncthreads();
  return r != 0;
}
__device__ __forceinline__ bool ess_ticket_join(const ess_xcd& x, int* slot) {
  return ess_ticket_join(x.ticket, !((x.avoid >> ess_xcc_id()) & 1u), slot);
}
// Thread 0 draws the next work item of counter `c` and hands it to the whole workgroup (also a barrier between two
// work items): the item, or -1 past the end.  The ticket is asked for when it is needed, not ahead of time: memory
// operations of a wave complete in order, so a ticket requested before an item's first loads makes those loads
// wait for the atomic's round trip through the memory side (measured: 8 % on the index-score kernel).
__device__ __forceinline__ int ess_ticket_take(uint32_t* c, int items, int* slot) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t mine = atomicAdd(c, 1u);
    *slot = mine < (uint32_t)items ? (int)mine : -1;
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*slot);      // the same in every lane: let the compiler keep it in a scalar register
}
// ESS_WORK_LOOP(DYN, xcd, static_item, items, slot, item) { body } runs the body for the one work item of this
// workgroup's index (DYN false: a compile-time constant, the loop folds away and the kernel is straight-line code),
// or for every item this workgroup draws (DYN true: ticket-fed launch).  Kernels are compiled in both forms: in
// the looping form the compiler keeps more in registers across items, which the plain launches should not pay for.
#define ESS_WORK_LOOP(DYN, xcd, static_item, items, slot, item)                                              \
  if ((DYN) && !ess_ticket_join((xcd), (slot))) return;                                                      \
  for (int ess_round_ = 0, item = 0;                                                                         \
       (DYN) ? ((item = ess_ticket_take((xcd).ticket + ESS_TK_WORK, (items), (slot))) >= 0)                  \
             : (ess_round_ == 0 && (item = (static_item)) < (items));                                        \
       ++ess_round_)
#endif
// Workgroups to launch for a ticket-fed kernel: enough to put `per_cu` of them on every CU of the XCDs that
// take work (32 CUs each; any 8 consecutive workgroups are expected to cover the 8 XCDs, which only sizes the
// launch -- it is complete under any placement), never more working ones than there are items.
inline int ess_xcd_grid(int items, const ess_xcd& x, int per_cu = 1) {
  if (x.ticket && x.host_need) *x.host_need = (uint32_t)items;
  if (!x.ticket) return items;
  if (x.grid_override > 0) return x.grid_override;
  const int off = __builtin_popcount(x.avoid & 0xffu);
  int want = 32 * per_cu * (8 - off);
  if (want > items) want = items;
  if (want < 1) want = 1;
  return off ? (want + (8 - off) - 1) / (8 - off) * 8 : want;
}

int ess_fail(int code, const char* fmt, ...);

#define ESS_HIP(call)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return ess_fail(ESS_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),   \
                      __FILE__, __LINE__);                                                  \
  } while (0)

// Stage launchers.  All enqueue on `st` and return an ess_status.
int ess_launch_index_score(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                           const int32_t* ctx_len, int B, int T, float* score, hipStream_t st,
                           const int32_t* block_table = nullptr, int n_pages = 0,
                           // optional: events that take the kernel's own start and end times
                           hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, ess_xcd xcd = ess_xcd{nullptr, 0, nullptr, 0});
// The fused selection (index score + top-k without a score array) is four launches: scores of each sequence's
// sample blocks -> sel_sample; lower bounds -> sel_tau (and sel_cnt cleared); the emitting index-score pass ->
// sel_cand / sel_cnt; the top-k finish -> idx.  b0: first sequence of the (sub-)batch, for the context's arrays;
// caller-owned pointers are passed already shifted.
int ess_launch_index_sample(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                            const int32_t* ctx_len, int B, int T, float* sample, hipStream_t st,
                            const int32_t* block_table, int n_pages, ess_xcd xcd);
int ess_launch_index_tau(ess_ctx* ctx, const int32_t* ctx_len, int B, int T, int b0, hipStream_t st, ess_xcd xcd);
int ess_launch_index_emit(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                          const int32_t* ctx_len, int B, int T, const uint32_t* tau, unsigned long long* cand,
                          uint32_t* cnt, int cand_cap, hipStream_t st, const int32_t* block_table, int n_pages,
                          hipEvent_t ev_start, hipEvent_t ev_stop, ess_xcd xcd);
int ess_launch_topk_finish(ess_ctx* ctx, const uint8_t* q, const float* w, const uint8_t* key, const int32_t* block_table,
                           int n_pages, const int32_t* ctx_len, int B, int T, int b0, int32_t* idx, hipStream_t st,
                           ess_xcd xcd);
int ess_sel_cand_cap();
// xcd: its counter block and the next one are used (two kernels)
int ess_launch_topk(ess_ctx* ctx, const float* score, const int32_t* ctx_len, int B, int T, int32_t* idx,
                    hipStream_t st, ess_xcd xcd = ess_xcd{nullptr, 0, nullptr, 0});
size_t ess_topk_cand_bytes();
// fill kernel (used instead of hipMemsetAsync so that callers may capture the stream in a graph)
int ess_launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
int ess_launch_calib_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);
int ess_launch_append(const ess_config& c, const ess_cache& cache, const uint8_t* new_key, const uint8_t* new_rows,
                      uint8_t* key, int32_t* ctx_len, int B, int T, uint32_t step, int32_t* placed,
                      const float* new_scale, const int32_t* block_table, int n_pages, hipStream_t st);
int ess_launch_fill_u32(uint32_t* p, int n, uint32_t value, hipStream_t st);
int ess_probe_xcds(uint32_t* hist8, bool* even);   // blocking; at context creation
int ess_init_cache_kernels(const ess_config& c, bool* fits);                     // function attributes (dynamic LDS sizes); at context creation
int ess_init_attn_kernels();
int ess_launch_cache_reset(const ess_config& c, const ess_cache& cache, int B, hipStream_t st);
// look-up + LRU update + lists; n_sel = entries per sequence in idx ([B,n_sel], T lists of n_sel/T)
// b0 = first sequence of the (sub-)batch: caller-owned pointers are passed already shifted, the
// library's workspace arrays are shifted inside
int ess_launch_bookkeeping(ess_ctx* ctx, const ess_cache& cache, const int32_t* idx, int B, int T, int kk,
                           uint32_t step, int32_t* slot_idx, int32_t* miss_count_out, hipStream_t st, int b0 = 0,
                           bool count_step = true, ess_xcd xcd = ess_xcd{nullptr, 0, nullptr, 0}, uint32_t* zero_tickets = nullptr,
                           int n_zero_tickets = 0);
// only_xcds != 0: the fetch runs on these XCDs alone (`wgs` workgroups there, rows handed out through `ticket`)
int ess_launch_fill(ess_ctx* ctx, const ess_cache& cache, int B, hipStream_t st, int b0 = 0, int wgs = 64,
                    uint32_t only_xcds = 0, uint32_t* ticket = nullptr);
int ess_launch_gather_rows(const ess_config& c, const uint8_t* slot_pool, const int32_t* slot_idx, int B, int T,
                           uint8_t* rows_out, hipStream_t st);
// attention over list[b,t,0..n) (n = n_list[b,t], or k when n_list is NULL), written as `nsplit`
// partial results starting at partial index `split0`
int ess_launch_attn_partial(ess_ctx* ctx, const void* q, const uint8_t* slot_pool, const int32_t* list,
                            const int32_t* n_list, int B, int T, int split0, int nsplit, hipStream_t st, int b0 = 0,
                            ess_xcd xcd = ess_xcd{nullptr, 0, nullptr, 0});
int ess_attn_min_splits(const ess_config& c);   // fewest splits a list of k entries may be cut into
// zero_cnt (may be NULL): n_zero int32 counters that the merge kernel also clears; b0 = first sequence of the
// sub-batch of B sequences (out_bf16 and lse are the whole batch's arrays)
int ess_launch_attn_merge(ess_ctx* ctx, int B, int T, int nsplit_total, void* out_bf16, float* lse,
                          hipStream_t st, int32_t* zero_cnt = nullptr, int n_zero = 0, int b0 = 0,
                          const ess_ticket_check* check = nullptr);
