// Stages 3 + 5: Sparse Memory Pool look-up, LRU update, miss fetch and row
// gather (ESS paper Sec. 3.1 FlashTrans, Sec. 3.2 LRU-based eviction and
// admission).  The swap unit is one Latent-Cache entry (Sec. 3.1).
//
// Reading of "LRU-based" implemented here (step-granular, order-free):
//   R = distinct valid selected positions of a sequence; resident members are
//   hits and get stamp := step; the others, in ascending position, take the
//   slots smallest in (stamp, slot) among slots with stamp < step; the former
//   token of a taken slot becomes non-resident.
//
// One workgroup per sequence does the whole update without any serial list:
//   - the selection is turned into a bitmap in LDS (dedups the T query
//     tokens and yields misses in ascending position by a prefix sum);
//   - victims come from a 4-pass radix select on the 32-bit stamps
//     (conflict-free histogram: 32 interleaved copies, copy = lane & 31),
//     ties on the threshold stamp broken by slot order with one block scan,
//     then a bitonic sort of the (stamp, slot) pairs in LDS;
//   - the i-th miss is paired with the i-th victim and a fetch list is
//     written for the fill kernel;
//   - per (b,t), slots of hits and of fetched entries are compacted into two
//     lists, which drive Attn0 and Attn1 (Sec. 3.3).
// The fetch itself is a separate kernel so that it can run on a side stream:
// GPU threads read the pinned host pool by address (the paper's UVA idea),
// one wave per 1152- or 656-byte entry, many entries in flight.
#include "ess_internal.h"
#include "select_common.h"

namespace {

constexpr int BT = 1024;

struct BookShared {
  uint32_t wave_tot[BT / 64];
  uint32_t sel_digit, sel_below;
};
// The large arrays of the bookkeeping kernel live in dynamic LDS, sized by the configuration:
//   bm [W]  bitmap of the missed positions (W = max_ctx / 32 words, rounded up to an even number)
//   un      histogram of the radix passes (256 x 32 counters, 32 KiB), later the victims' (stamp, slot) keys
//           (vict_cap = sel_cap rounded up to a power of two, 8 bytes each)
//   mt [sel_cap]  missed positions in ascending order (sel_cap = max_q_tokens * topk)
constexpr int BOOK_HIST_BYTES = 256 * 32 * 4;
inline int book_pow2(int n) { int p = 1; while (p < n) p <<= 1; return p; }
inline size_t book_words(int max_ctx) { return (size_t)(((max_ctx + 31) / 32 + 1) & ~1); }
inline size_t book_union_bytes(int sel_cap) {
  const size_t v = (size_t)book_pow2(sel_cap) * 8;
  return v > (size_t)BOOK_HIST_BYTES ? v : (size_t)BOOK_HIST_BYTES;
}
inline size_t book_lds_bytes(int max_ctx, int sel_cap) {
  return book_words(max_ctx) * 4 + book_union_bytes(sel_cap) + (size_t)sel_cap * 4;
}

using ess_sel::wave_incl_scan;
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  return ess_sel::block_incl_scan<BT>(v, wave_tot, total);
}

__device__ void bitonic_sort_u64(unsigned long long* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int t = threadIdx.x; t < (n >> 1); t += BT) {
        const int lo = 2 * t - (t & (stride - 1));
        const int hi = lo + stride;
        const bool up = (lo & size) == 0;
        const unsigned long long x = a[lo], y = a[hi];
        if ((x > y) == up) { a[lo] = y; a[hi] = x; }
      }
    }
  }
  __syncthreads();
}

// idx: [B, T, kk] selected positions (-1 = none).  Dynamic LDS: bitmap of Lmax bits.
// REG: the slots a thread owns (S / 1024, rounded up, at most 16) are held in registers, so the
// stamps are read from memory once, all loads of a thread in flight together.
template <bool REG, bool DYN>
__global__ __launch_bounds__(BT) void k_bookkeeping(
    const int32_t* __restrict__ idx, int T, int kk, int Lmax, int S, int32_t* __restrict__ slot_of,
    int32_t* __restrict__ token_of, uint32_t* __restrict__ stamp, uint32_t step, int32_t* __restrict__ slot_idx_out,
    int32_t* __restrict__ hit_list, int32_t* __restrict__ miss_list, int32_t* __restrict__ n_hit,
    int32_t* __restrict__ n_miss, int32_t* __restrict__ fill_tok, int32_t* __restrict__ fill_slot, int fill_cap,
    int32_t* __restrict__ miss_cnt, int32_t* __restrict__ miss_count_out, unsigned long long* __restrict__ stats,
    unsigned long long* __restrict__ seq_stats,
    int row_stride, int count_step, int32_t* __restrict__ host_miss, ess_xcd xcd, int n_seq,
    uint32_t* __restrict__ zero_tickets, int n_zero_tickets, int bm_words, int union_bytes) {
  extern __shared__ __align__(16) uint32_t bm[];              // see the layout above
  uint32_t* const s_hist = bm + bm_words;
  unsigned long long* const s_vict = reinterpret_cast<unsigned long long*>(bm + bm_words);
  int32_t* const s_miss_tok = reinterpret_cast<int32_t*>(bm + bm_words + union_bytes / 4);
  const int vict_cap = union_bytes / 8;                       // >= the misses of one step, rounded up to a power of two
  __shared__ BookShared sm;
  __shared__ int s_item;
  constexpr int RS = 16;                       // register-held stamps per thread
  // work counters of the kernels that follow this one beside the fetch it feeds: cleared here, by the first
  // workgroup, so that no launch has to do it (this kernel itself never uses the counters it clears)
  if (zero_tickets && blockIdx.x == 0)            // n_zero_tickets launches' counters: the words in use
    for (int i = threadIdx.x; i < n_zero_tickets * ESS_TICKET_USED; i += BT)
      zero_tickets[(i / ESS_TICKET_USED) * ESS_TICKET_WORDS + (i % ESS_TICKET_USED) * ESS_TK_STRIDE] = 0;
  // work item = sequence: by workgroup index, or drawn from the launch's counter off the XCDs to be avoided
  ESS_WORK_LOOP(DYN, xcd, blockIdx.x, n_seq, &s_item, b) {
  // (looping form: the thread index passes through an empty asm statement, so that what is derived from it is
  // computed per work item instead of being carried in registers across the loop, where it led to spills)
  int tid_ = threadIdx.x;
  if constexpr (DYN) asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63;
  const int W = (Lmax + 31) >> 5;
  const int nsel = T * kk;
  const int32_t* sel = idx + (size_t)b * nsel;
  int32_t* so = slot_of + (size_t)b * Lmax;
  int32_t* to = token_of + (size_t)b * S;
  uint32_t* stp = stamp + (size_t)b * S;

  for (int j = tid; j < W; j += BT) bm[j] = 0;
  __syncthreads();
  // look-up straight from the selection list (all gathers of a thread in flight together): hits get
  // their stamp, misses set their bit; duplicates across the T query tokens do the same thing twice
  // (kept: when one round covers the selection and a query token's list is whole rounds of the workgroup, the
  // lists at the end are built from these registers instead of a second look-up)
  const bool keep = nsel <= 4 * BT && kk % BT == 0;
  uint32_t my_valid = 0;
  int sv[4] = {-1, -1, -1, -1}, slv[4] = {-1, -1, -1, -1};
  for (int e0 = 0; e0 < nsel; e0 += 4 * BT) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * BT + tid;
      sv[u] = e < nsel ? sel[e] : -1;
      if (sv[u] >= Lmax) sv[u] = -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) slv[u] = sv[u] >= 0 ? so[sv[u]] : -1;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (sv[u] < 0) continue;
      ++my_valid;
      if (slv[u] >= 0) stp[slv[u]] = step;
      else atomicOr(&bm[sv[u] >> 5], 1u << (sv[u] & 31));
    }
  }
  __syncthreads();

  // misses in ascending position: prefix sum over the bitmap words
  const int wpt = (W + BT - 1) / BT;
  const int w0 = min(tid * wpt, W), w1 = min(w0 + wpt, W);
  uint32_t my_miss = 0;
  for (int wd = w0; wd < w1; ++wd) my_miss += __popc(bm[wd]);
  // one scan for both counts (each at most T * k <= 8192: 16 bits apiece)
  uint32_t both;
  const uint32_t miss_inc = block_incl_scan(my_miss | (my_valid << 16), sm.wave_tot, &both) & 0xffffu;
  const uint32_t m = both & 0xffffu, nvalid = both >> 16;
  {
    uint32_t pos = miss_inc - my_miss;
    for (int wd = w0; wd < w1; ++wd) {
      uint32_t bits = bm[wd];
      while (bits) {
        const int bit = __ffs(bits) - 1;
        bits &= bits - 1;
        if (pos < (uint32_t)fill_cap) s_miss_tok[pos] = wd * 32 + bit;
        ++pos;
      }
    }
  }
  __syncthreads();                               // also: the stamps of the hits are visible

  if (m > 0) {
    // this thread's slots: [v0, v1), contiguous so that slot order is thread order
    const int spt = (S + BT - 1) / BT;
    const int v0 = min(tid * spt, S), v1 = min(v0 + spt, S);
    uint32_t sr[RS];
    if (REG) {
#pragma unroll
      for (int j = 0; j < RS; ++j) sr[j] = (v0 + j < v1) ? stp[v0 + j] : 0xffffffffu;   // never evictable
    }
    auto stamp_at = [&](int j) -> uint32_t { return REG ? sr[j] : stp[v0 + j]; };
    const int nj = REG ? RS : spt;
    // ---- m-th smallest stamp among evictable slots (stamp < step): 4 x 8-bit MSD radix passes
    // evictable stamps are < step, so digits above step's top byte are zero for all of them: skip those passes
    uint32_t prefix = 0, need = m;
    const int first_pass = step < (1u << 8) ? 3 : (step < (1u << 16) ? 2 : (step < (1u << 24) ? 1 : 0));
    for (int pass = first_pass; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      for (int j = tid; j < 256 * 32; j += BT) s_hist[j] = 0;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < nj; ++j) {
        if (v0 + j >= v1) continue;
        const uint32_t st = stamp_at(j);
        if (st < step && (pass == first_pass || (st >> (shift + 8)) == prefix))
          atomicAdd(&s_hist[((st >> shift) & 255u) * 32 + (lane & 31)], 1u);
      }
      __syncthreads();
      uint32_t c = 0;
      if (tid < 256) {
        // a thread's 32 copies are consecutive words, so consecutive threads start 32 words apart: the 16-byte
        // pieces are taken in an order rotated by the thread index, which spreads a read over the banks
        const uint4* h4 = reinterpret_cast<const uint4*>(s_hist + tid * 32);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
          const uint4 x = h4[(g + tid) & 7];
          c += x.x + x.y + x.z + x.w;
        }
      }
      uint32_t total;
      const uint32_t inc = block_incl_scan(c, sm.wave_tot, &total);
      const uint32_t below = inc - c;
      if (tid < 256 && below < need && below + c >= need) { sm.sel_digit = tid; sm.sel_below = below; }
      __syncthreads();
      need -= sm.sel_below;
      prefix = (prefix << 8) | sm.sel_digit;
      __syncthreads();
    }
    const uint32_t tau = prefix;               // threshold stamp; `need` slots with stamp == tau are taken, lowest slots first
    // ---- collect victims: stamp < tau, plus the first `need` slots (in slot order) with stamp == tau
    uint32_t my_eq = 0, my_lt = 0;
#pragma unroll
    for (int j = 0; j < nj; ++j)
      if (v0 + j < v1) {
        const uint32_t st = stamp_at(j);
        my_eq += (st == tau) ? 1u : 0u;
        my_lt += (st < tau) ? 1u : 0u;
      }
    // slots at the threshold stamp (their order decides which of them are taken) and slots below it (all taken)
    uint32_t tot_eq, tot_lt;
    uint32_t rank = block_incl_scan(my_eq, sm.wave_tot, &tot_eq) - my_eq;      // slots at the threshold stamp in front of this thread's
    // where this thread's victims go: those of the threads before it come first (the list is in slot order)
    uint32_t at = (block_incl_scan(my_lt, sm.wave_tot, &tot_lt) - my_lt) + min(rank, need);
#pragma unroll
    for (int j = 0; j < nj; ++j) {
      if (v0 + j >= v1) continue;
      const uint32_t st = stamp_at(j);
      bool take = st < tau;
      if (st == tau) { take = rank < need; ++rank; }
      if (take) {
        if (at < (uint32_t)vict_cap) s_vict[at] = ((unsigned long long)st << 32) | (uint32_t)(v0 + j);
        ++at;
      }
    }
    __syncthreads();
    // order the victims by (stamp, slot).  Up to 1024 of them: every thread ranks one victim by counting
    // the smaller keys (keys are distinct; no barriers, LDS broadcast reads); more: bitonic sort.
    const bool by_rank = m <= (uint32_t)BT;
    if (by_rank) {
      // every victim's rank = the number of smaller keys, counted by BT / m threads per victim, each over its share
      // of the list (LDS broadcast reads), and added up in LDS
      uint32_t* s_rank = reinterpret_cast<uint32_t*>(s_vict + vict_cap / 2);        // the list takes the lower half at most
      const int mr = ((int)m + 63) & ~63;            // threads of one share: whole waves
      const int shares = BT / mr;
      for (int j = tid; j < (int)m; j += BT) s_rank[j] = 0;
      __syncthreads();
      const int i = tid % mr, p = tid / mr;
      unsigned long long my_key = 0;
      if (i < (int)m && p < shares) {
        my_key = s_vict[i];
        const int j0 = (int)((long)m * p / shares), j1 = (int)((long)m * (p + 1) / shares);
        int rk = 0;
        int j = j0;
        for (; j + 8 <= j1; j += 8) {            // eight independent LDS reads in flight (the plain loop waits for each)
          unsigned long long x[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) x[u] = s_vict[j + u];
#pragma unroll
          for (int u = 0; u < 8; ++u) rk += x[u] < my_key ? 1 : 0;
        }
        for (; j < j1; ++j) rk += s_vict[j] < my_key ? 1 : 0;
        atomicAdd(&s_rank[i], (uint32_t)rk);
      }
      __syncthreads();
      const int my_rank = (tid < (int)m) ? (int)s_rank[tid] : -1;
      if (tid < (int)m) my_key = s_vict[tid];
      __syncthreads();
      if (my_rank >= 0) s_vict[my_rank] = my_key;
      __syncthreads();
    } else {
      int np = 1;
      while (np < (int)m) np <<= 1;
      for (int j = (int)m + tid; j < np; j += BT) s_vict[j] = ~0ull;
      bitonic_sort_u64(s_vict, np);
    }
    // ---- pair the i-th miss with the i-th victim
    for (uint32_t i = tid; i < m; i += BT) {
      const int s = s_miss_tok[i];
      const int v = (int)(uint32_t)s_vict[i];
      const int old = to[v];
      if (old >= 0) so[old] = -1;
      to[v] = s;
      so[s] = v;
      stp[v] = step;
      fill_tok[(size_t)b * fill_cap + i] = s;
      fill_slot[(size_t)b * fill_cap + i] = v;
    }
  }
  if (tid == 0) {
    miss_cnt[b] = (int32_t)m;
    if (miss_count_out) miss_count_out[b] = (int32_t)m;
    if (host_miss) host_miss[b] = (int32_t)m;       // pinned host memory: the host's view for the overlap switch
    if (b == 0 && count_step) atomicAdd(&stats[0], 1ull);
    atomicAdd(&stats[1], (unsigned long long)nvalid);
    atomicAdd(&stats[2], (unsigned long long)m);
    atomicAdd(&stats[3], (unsigned long long)m * (unsigned long long)row_stride);
    // the same per sequence (this workgroup is the only writer of its sequence's four counters)
    seq_stats[4 * b + 0] += 1ull;
    seq_stats[4 * b + 1] += (unsigned long long)nvalid;
    seq_stats[4 * b + 2] += (unsigned long long)m;
    seq_stats[4 * b + 3] += (unsigned long long)m * (unsigned long long)row_stride;
  }
  __syncthreads();                               // table updates visible to the whole workgroup

  // ---- per (b,t): slot of every selected entry, and the compacted hit / fetched lists
  if (slot_idx_out == nullptr && hit_list == nullptr) continue;
  for (int t = 0; t < T; ++t) {
    const size_t rowoff = ((size_t)b * T + t) * kk;
    uint32_t base_hit = 0, base_miss = 0;
    for (int j0 = 0; j0 < kk; j0 += BT) {
      const int j = j0 + tid;
      int slot = -1;
      bool fresh = false;
      if (keep) {
        // entry t * kk + j0 + tid was looked up by this thread in round u: a hit keeps the slot it had, a miss
        // got its slot in the pairing above
        const int u = (t * kk + j0) / BT;
        const int s = u == 0 ? sv[0] : (u == 1 ? sv[1] : (u == 2 ? sv[2] : sv[3]));
        const int s0 = u == 0 ? slv[0] : (u == 1 ? slv[1] : (u == 2 ? slv[2] : slv[3]));
        if (s >= 0) {
          fresh = s0 < 0;
          slot = fresh ? so[s] : s0;
        }
        if (slot_idx_out) slot_idx_out[rowoff + j] = slot;
      } else if (j < kk) {
        const int s = idx[rowoff + j];
        if (s >= 0 && s < Lmax) {
          slot = so[s];
          fresh = (bm[s >> 5] >> (s & 31)) & 1u;
        }
        if (slot_idx_out) slot_idx_out[rowoff + j] = slot;
      }
      if (hit_list) {
        const uint32_t is_hit = (slot >= 0 && !fresh) ? 1u : 0u;
        const uint32_t is_miss = (slot >= 0 && fresh) ? 1u : 0u;
        uint32_t tot;
        const uint32_t inc = block_incl_scan(is_hit | (is_miss << 16), sm.wave_tot, &tot);
        const uint32_t ex = inc - (is_hit | (is_miss << 16));
        if (is_hit) hit_list[rowoff + base_hit + (ex & 0xffffu)] = slot;
        if (is_miss) miss_list[rowoff + base_miss + (ex >> 16)] = slot;
        base_hit += tot & 0xffffu;
        base_miss += tot >> 16;
      }
    }
    if (hit_list && tid == 0) {
      n_hit[b * T + t] = (int32_t)base_hit;
      n_miss[b * T + t] = (int32_t)base_miss;
    }
  }
  }
}

// Fetch: one wave per missed entry, rows copied host pool -> slot pool in 16-byte pieces, two
// entries per wave in flight at once.  The kernel is a handful of 512-thread workgroups that loop
// over all sequences: its waves spend their life waiting on the host link.  The number of workgroups
// sets how many bytes are in flight on the link: 64 (1.2 MB in flight) reach 53 GB/s, 32 reach
// 50 GB/s, 16 reach 48 GB/s, 8 only 27 GB/s.  The long host reads also fill the L2 request queues of
// the XCDs the workgroups sit on, and every other memory access of those XCDs waits behind them: a
// kernel beside a 64-workgroup fetch spread over the chip takes about 2.2x its time alone (a
// latency-bound one more), beside 28-32 workgroups about 1.3x.  The launcher can therefore confine
// the fetch to some XCDs (`only_xcds`: the other workgroups exit, entries are handed out by ticket),
// and the kernels beside it stay off those (ess_xcd).
constexpr int FILL_WPB = 8;                                 // waves per workgroup
constexpr int FILL_MAX_B = 4096;

__global__ __launch_bounds__(FILL_WPB * 64) void k_fill(const uint8_t* __restrict__ host_pool, uint8_t* __restrict__ slot_pool,
                                               const int32_t* __restrict__ fill_tok,
                                               const int32_t* __restrict__ fill_slot, int fill_cap,
                                               const int32_t* __restrict__ miss_cnt, int B, int Lmax, int S,
                                               int row_stride, uint32_t only_xcds, uint32_t* __restrict__ ticket) {
  // confined fetch: only workgroups on the XCDs in `only_xcds` work (or, should none sit there, the last one to
  // arrive), entries are handed out through `ticket`
  __shared__ int s_join;
  if (only_xcds && !ess_ticket_join(ticket, (only_xcds >> ess_xcc_id()) & 1u, &s_join)) return;
  extern __shared__ int32_t pref[];                          // [B + 1] pref[b] = entries of sequences < b (kept small:
                                                             // the kernel must fit beside workgroups that fill the LDS)
  const int tid = threadIdx.x, lane = tid & 63;
  // exclusive prefix sum of the per-sequence miss counts, by the first wave
  if (tid < 64) {
    int run = 0;
    for (int b0 = 0; b0 <= B; b0 += 64) {
      const int b = b0 + lane;
      const int cnt = b < B ? min(miss_cnt[b], fill_cap) : 0;
      const int inc = (int)wave_incl_scan((uint32_t)cnt, lane);
      if (b <= B) pref[b] = run + inc - cnt;
      run += __shfl(inc, 63, 64);
    }
  }
  __syncthreads();
  const int M = pref[B];
  const int gw = blockIdx.x * FILL_WPB + (tid >> 6);         // wave index in the grid
  const int FILL_WAVES = gridDim.x * FILL_WPB;
  const int chunks = row_stride >> 4;                        // <= 128 for the supported entry sizes
  const int c0 = lane, c1 = lane + 64;
  auto locate = [&](int r, const uint4*& src, uint4*& dst) { // r-th entry of the flattened list
    int lo = 0, hi = B;                                      // largest b with pref[b] <= r
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pref[mid] <= r) lo = mid; else hi = mid;
    }
    const int i = r - pref[lo];
    const int tok = fill_tok[(size_t)lo * fill_cap + i], slot = fill_slot[(size_t)lo * fill_cap + i];
    src = reinterpret_cast<const uint4*>(host_pool + ((size_t)lo * Lmax + tok) * row_stride);
    dst = reinterpret_cast<uint4*>(slot_pool + ((size_t)lo * S + slot) * row_stride);
  };
  for (int r = gw;; r += 2 * FILL_WAVES) {                   // two entries of this wave in flight
    int rB;
    if (only_xcds) {                                         // entries r, r + 1 by ticket
      uint32_t tk = 0;
      if (lane == 0) tk = atomicAdd(ticket, 2u);
      r = (int)__shfl(tk, 0, 64);
      rB = r + 1;
    } else {
      rB = r + FILL_WAVES;
    }
    if (r >= M) break;
    const bool two = rB < M;
    const uint4 *srcA, *srcB;
    uint4 *dstA, *dstB;
    locate(r, srcA, dstA);
    locate(two ? rB : r, srcB, dstB);
    uint4 a0 = make_uint4(0, 0, 0, 0), a1 = a0, b0 = a0, b1 = a0;
    if (c0 < chunks) a0 = srcA[c0];
    if (c1 < chunks) a1 = srcA[c1];
    if (two && c0 < chunks) b0 = srcB[c0];
    if (two && c1 < chunks) b1 = srcB[c1];
    if (c0 < chunks) ess_store_nt(dstA + c0, a0);
    if (c1 < chunks) ess_store_nt(dstA + c1, a1);
    if (two && c0 < chunks) ess_store_nt(dstB + c0, b0);
    if (two && c1 < chunks) ess_store_nt(dstB + c1, b1);
  }
}

// rows_out[b,t,j,:] = slot_pool[b, slot_idx[b,t,j], :] (zeros where the slot is -1); one wave per row
__global__ __launch_bounds__(256) void k_gather_rows(const uint8_t* __restrict__ slot_pool,
                                                     const int32_t* __restrict__ slot_idx, int per_seq, int S,
                                                     int row_stride, uint8_t* __restrict__ rows_out) {
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int nw = gridDim.x * 4;
  const int chunks = row_stride >> 4;
  for (int i = blockIdx.x * 4 + (threadIdx.x >> 6); i < per_seq; i += nw) {
    const int v = slot_idx[(size_t)b * per_seq + i];
    uint4* dst = reinterpret_cast<uint4*>(rows_out + ((size_t)b * per_seq + i) * row_stride);
    if (v >= 0 && v < S) {
      const uint4* src = reinterpret_cast<const uint4*>(slot_pool + ((size_t)b * S + v) * row_stride);
      for (int c = lane; c < chunks; c += 64) dst[c] = src[c];
    } else {
      for (int c = lane; c < chunks; c += 64) dst[c] = make_uint4(0, 0, 0, 0);
    }
  }
}

// Append (Sec. 3.3): the entries a step produced enter the caches.  One workgroup per sequence; for each
// of its T new tokens, in order: index key -> Indexer-Cache row p, entry -> host pool row p (stores
// through the device mapping of the pinned pool: the write-back to the Total Memory Pool), and admission
// to the slot pool as most recently used: the slot smallest in (stamp, slot) among slots with a stamp
// below `step` is taken -- the victim rule of the bookkeeping -- or, with every slot on stamp `step`,
// none (the entry then lives in the host pool only).  Without a host pool slot = position.
constexpr int APPEND_NT = 1024;
__global__ __launch_bounds__(APPEND_NT) void k_append(
    const uint8_t* __restrict__ new_key, const uint8_t* __restrict__ new_rows, uint8_t* __restrict__ key,
    uint8_t* __restrict__ host_pool, uint8_t* __restrict__ slot_pool, int32_t* __restrict__ slot_of,
    int32_t* __restrict__ token_of, uint32_t* __restrict__ stamp, int32_t* __restrict__ ctx_len,
    int32_t* __restrict__ placed, int T, int Di, int Lmax, int S, int row_stride, uint32_t step,
    const float* __restrict__ new_scale, const int32_t* __restrict__ block_table, int n_pages) {
  __shared__ unsigned long long red[APPEND_NT / 64];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int L0 = max(0, min(ctx_len[b], Lmax));
  int n = min(T, Lmax - L0);
  // paged Indexer-Cache: a token needs a mapped page; the first one without stops the append
  const int32_t* bt = block_table ? block_table + (size_t)b * (Lmax / ESS_PAGE_TOKENS) : nullptr;
  if (bt)
    for (int t = 0; t < n; ++t) {
      const int pid = bt[(L0 + t) / ESS_PAGE_TOKENS];
      if (pid < 0 || pid >= n_pages) { n = t; break; }
    }
  const int kchunks = Di >> 4, rchunks = row_stride >> 4;
  int32_t* so = slot_of + (size_t)b * Lmax;
  int32_t* to = token_of + (size_t)b * S;
  uint32_t* stp = stamp + (size_t)b * S;
  for (int t = 0; t < T; ++t) {
    if (t >= n) {                                  // no room left in the buffers: dropped
      if (tid == 0 && placed) placed[(size_t)b * T + t] = -1;
      continue;
    }
    const int p = L0 + t;
    const uint4* krow = reinterpret_cast<const uint4*>(new_key + ((size_t)b * T + t) * Di);
    const uint4* erow = reinterpret_cast<const uint4*>(new_rows + ((size_t)b * T + t) * row_stride);
    if (bt) {
      uint8_t* page = key + (size_t)bt[p / ESS_PAGE_TOKENS] * ((size_t)ESS_PAGE_TOKENS * (Di + 4));
      const int r = p % ESS_PAGE_TOKENS;
      if (tid < kchunks) reinterpret_cast<uint4*>(page + (size_t)r * Di)[tid] = krow[tid];
      if (tid == 32) reinterpret_cast<float*>(page + (size_t)ESS_PAGE_TOKENS * Di)[r] = new_scale[(size_t)b * T + t];
    } else if (tid < kchunks) {
      reinterpret_cast<uint4*>(key + ((size_t)b * Lmax + p) * Di)[tid] = krow[tid];
    }
    if (host_pool && tid >= 64 && tid - 64 < rchunks)
      reinterpret_cast<uint4*>(host_pool + ((size_t)b * Lmax + p) * row_stride)[tid - 64] = erow[tid - 64];
    int v = p;
    if (host_pool) {
      unsigned long long best = ~0ull;
      for (int s = tid; s < S; s += APPEND_NT) {
        const uint32_t x = stp[s];
        if (x < step) {
          const unsigned long long cand = ((unsigned long long)x << 32) | (uint32_t)s;
          best = cand < best ? cand : best;
        }
      }
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = __shfl_xor(best, d, 64);
        best = o < best ? o : best;
      }
      if (lane == 0) red[tid >> 6] = best;
      __syncthreads();
      best = red[0];
#pragma unroll
      for (int i = 1; i < APPEND_NT / 64; ++i) best = red[i] < best ? red[i] : best;
      v = best == ~0ull ? -1 : (int)(uint32_t)best;
    }
    if (v >= 0) {
      if (tid >= 256 && tid - 256 < rchunks)
        reinterpret_cast<uint4*>(slot_pool + ((size_t)b * S + v) * row_stride)[tid - 256] = erow[tid - 256];
      if (tid == 0) {
        const int old = to[v];
        if (old >= 0) so[old] = -1;
        to[v] = p;
        so[p] = v;
        stp[v] = step;
      }
    }
    if (tid == 0 && placed) placed[(size_t)b * T + t] = v;
    __syncthreads();                               // the next token's search sees this stamp; red is free again
  }
  if (tid == 0) ctx_len[b] = L0 + n;               // every thread read ctx_len before the first barrier or exit
}

__global__ __launch_bounds__(256) void k_calib_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Reads `n` 16-byte pieces and leaves one word per workgroup, so that the loads are not dead.  A workgroup streams
// one contiguous range (`per_wg` pieces); its four waves interleave 8 KiB pieces, each wave instruction covering
// 1 KiB, eight of them in flight per wave -- the pattern with which a pure read stream is fastest on this chip.
__global__ __launch_bounds__(256) void k_calib_read(const uint4* __restrict__ src, size_t n, size_t per_wg,
                                                    uint32_t* __restrict__ sink) {
  constexpr int U = 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t lo = (size_t)blockIdx.x * per_wg;
  const size_t hi = lo + per_wg < n ? lo + per_wg : n;
  uint32_t acc = 0;
  for (size_t base = lo + (size_t)wave * U * 64; base < hi; base += (size_t)4 * U * 64) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = base + (size_t)u * 64 + lane;
      x[u] = i < hi ? src[i] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) acc ^= __shfl_xor(acc, d, 64);
  if (lane == 0) atomicXor(&sink[blockIdx.x], acc);
}

__global__ void k_fill_u32(uint32_t* p, int n, uint32_t value) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

__global__ void k_cache_reset(int32_t* slot_of, int32_t* token_of, uint32_t* stamp, int Lmax, int S, int identity) {
  const int b = blockIdx.y;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < Lmax) slot_of[(size_t)b * Lmax + i] = identity ? i : -1;
  if (i < S) {
    token_of[(size_t)b * S + i] = identity ? i : -1;
    stamp[(size_t)b * S + i] = 0;
  }
}

}  // namespace

int ess_launch_append(const ess_config& c, const ess_cache& cache, const uint8_t* new_key, const uint8_t* new_rows,
                      uint8_t* key, int32_t* ctx_len, int B, int T, uint32_t step, int32_t* placed,
                      const float* new_scale, const int32_t* block_table, int n_pages, hipStream_t st) {
  hipLaunchKernelGGL(k_append, dim3(B), dim3(APPEND_NT), 0, st, new_key, new_rows, key,
                     const_cast<uint8_t*>(cache.host_pool_dev), cache.slot_pool, cache.slot_of, cache.token_of,
                     cache.stamp, ctx_len, placed, T, c.idx_dim, c.max_ctx, c.slots_per_seq, c.row_stride, step,
                     new_scale, block_table, n_pages);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(k_calib_copy, dim3(8192), dim3(256), 0, st, static_cast<uint4*>(dst), static_cast<const uint4*>(src),
                     bytes / 16);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_calib_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  const size_t n = bytes / 16;
  size_t per_wg = 16384;                                     // 256 KiB per workgroup, more when that needs too many workgroups
  while ((n + per_wg - 1) / per_wg > ESS_CALIB_READ_WGS) per_wg *= 2;
  const unsigned grid = (unsigned)((n + per_wg - 1) / per_wg);
  hipLaunchKernelGGL(k_calib_read, dim3(grid ? grid : 1), dim3(256), 0, st, static_cast<const uint4*>(src), n, per_wg, sink);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

// hist[x] += 1 for the XCD x this workgroup runs on
__global__ void k_xcd_probe(uint32_t* hist) {
  if (threadIdx.x == 0) atomicAdd(&hist[ess_xcc_id() & 7], 1u);
}

// Are 64 workgroups spread evenly over eight XCDs (8 each)?  Only then may a launch count on finding
// eight minus n of any eight consecutive workgroups off a set of n XCDs.  `hist8`: eight zeroed counters, zero again on return.
int ess_probe_xcds(uint32_t* hist8, bool* even) {
  hipLaunchKernelGGL(k_xcd_probe, dim3(64), dim3(64), 0, 0, hist8);
  ESS_HIP(hipGetLastError());
  uint32_t h[8];
  ESS_HIP(hipMemcpy(h, hist8, sizeof(h), hipMemcpyDeviceToHost));
  ESS_HIP(hipMemset(hist8, 0, sizeof(h)));
  *even = true;
  for (int i = 0; i < 8; ++i) *even = *even && h[i] == 8u;
  return ESS_OK;
}

int ess_launch_fill_u32(uint32_t* p, int n, uint32_t value, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_u32, dim3((n + 255) / 256), dim3(256), 0, st, p, n, value);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_cache_reset(const ess_config& c, const ess_cache& cache, int B, hipStream_t st) {
  const int n = c.max_ctx > c.slots_per_seq ? c.max_ctx : c.slots_per_seq;
  hipLaunchKernelGGL(k_cache_reset, dim3((n + 255) / 256, B), dim3(256), 0, st, cache.slot_of, cache.token_of,
                     cache.stamp, c.max_ctx, c.slots_per_seq, cache.host_pool_dev == nullptr ? 1 : 0);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_bookkeeping(ess_ctx* ctx, const ess_cache& cache, const int32_t* idx, int B, int T, int kk,
                           uint32_t step, int32_t* slot_idx, int32_t* miss_count_out, hipStream_t st, int b0,
                           bool count_step, ess_xcd xcd, uint32_t* zero_tickets, int n_zero_tickets) {
  const ess_config& c = ctx->cfg;
  if (!ctx->book_fits)
    return ess_fail(ESS_ERR_UNSUPPORTED, "the cache bookkeeping of max_ctx %d with T*k = %d does not fit the LDS (max_ctx / 8 + "
                    "12 * T*k bytes must stay below 160 KiB)", c.max_ctx, c.max_q_tokens * c.topk);
  const int cap = c.max_q_tokens * c.topk;
  const size_t lds = book_lds_bytes(c.max_ctx, cap);
  const bool lists = (kk == c.topk);           // compacted lists have the pitch of the top-k
  const size_t lo = (size_t)b0 * T * c.topk;   // offset of this sub-batch in the per-(b,t) lists
  const bool reg = c.slots_per_seq <= BT * 16;
  auto kern = xcd.ticket ? (reg ? &k_bookkeeping<true, true> : &k_bookkeeping<false, true>)
                         : (reg ? &k_bookkeeping<true, false> : &k_bookkeeping<false, false>);
  hipLaunchKernelGGL(kern, dim3(ess_xcd_grid(B, xcd)), dim3(BT), lds, st, idx, T, kk, c.max_ctx, c.slots_per_seq,
                     cache.slot_of, cache.token_of, cache.stamp, step, slot_idx,
                     lists ? ctx->hit_list + lo : nullptr, lists ? ctx->miss_list + lo : nullptr,
                     ctx->n_hit + (size_t)b0 * T, ctx->n_miss + (size_t)b0 * T, ctx->fill_tok + (size_t)b0 * cap,
                     ctx->fill_slot + (size_t)b0 * cap, cap, ctx->miss_cnt + b0, miss_count_out, ctx->stats, ctx->seq_stats + 4 * (size_t)b0,
                     c.row_stride, count_step ? 1 : 0, (c.flags & ESS_FLAG_AUTO) ? ctx->host_miss_dev + b0 : nullptr, xcd, B,
                     zero_tickets, n_zero_tickets, (int)book_words(c.max_ctx), (int)book_union_bytes(cap));
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

// At context creation (on the context's device): the bookkeeping kernels keep their arrays in dynamic LDS (see
// BookShared).  The limit is a property of the function, shared by all contexts: it only grows.  A configuration
// whose arrays do not fit the CU's 160 KiB (a selection of 8192 entries per sequence together with a context
// above 500K) cannot use the cache calls: *fits tells.
int ess_init_cache_kernels(const ess_config& c, bool* fits) {
  static size_t have = 0;
  const size_t lds = book_lds_bytes(c.max_ctx, c.max_q_tokens * c.topk);
  *fits = lds + 256 <= 160 * 1024;             // + the kernel's small static arrays
  if (!*fits || lds <= have) return ESS_OK;
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bookkeeping<true, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bookkeeping<false, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bookkeeping<true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_bookkeeping<false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  have = lds;
  return ESS_OK;
}

int ess_launch_fill(ess_ctx* ctx, const ess_cache& cache, int B, hipStream_t st, int b0, int wgs, uint32_t only_xcds,
                    uint32_t* ticket) {
  wgs = wgs < 1 ? 1 : (wgs > 256 ? 256 : wgs);
  if (only_xcds) {                             // `wgs` workgroups on the chosen XCDs, if any 8 consecutive ones cover all XCDs
    if (!ticket) return ess_fail(ESS_ERR_INVALID_ARG, "internal: confined fetch without a ticket");
    const int on = __builtin_popcount(only_xcds & 0xffu);
    wgs = (wgs + on - 1) / on * 8;
    if (ctx->ticket_grid > 0) wgs = ctx->ticket_grid;
  }
  const ess_config& c = ctx->cfg;
  const int cap = c.max_q_tokens * c.topk;
  hipLaunchKernelGGL(k_fill, dim3(wgs), dim3(FILL_WPB * 64), (size_t)(B + 1) * sizeof(int32_t), st, cache.host_pool_dev, cache.slot_pool,
                     ctx->fill_tok + (size_t)b0 * cap, ctx->fill_slot + (size_t)b0 * cap, cap, ctx->miss_cnt + b0, B,
                     c.max_ctx, c.slots_per_seq, c.row_stride, only_xcds, ticket);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_gather_rows(const ess_config& c, const uint8_t* slot_pool, const int32_t* slot_idx, int B, int T,
                           uint8_t* rows_out, hipStream_t st) {
  hipLaunchKernelGGL(k_gather_rows, dim3(64, B), dim3(256), 0, st, slot_pool, slot_idx, T * c.topk,
                     c.slots_per_seq, c.row_stride, rows_out);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
