// Stage 2: per-query top-k over the indexer scores (ESS paper Sec. 3: the top
// 2,048 entries are selected).
//
// Selection order is (score descending, position ascending).  Every position
// gets a unique composite key  c = orderable_u32(score) << IB | (2^IB-1 - pos)
// (IB = bits needed for a position), so "the k largest composite keys" is a
// total order with no ties and any selection algorithm gives the same set.
//
// One workgroup per (b,t) row finds the threshold key T* = the k-th largest
// composite key, then emits every position whose key is >= T*:
//   A. long rows: a 14-bit histogram of a sample of the scores gives a key that is
//      below the k-th largest score with high probability yet keeps only a few
//      thousand positions at or above it; one pass over the row collects those
//      candidates (their composite keys) in LDS.  If their number is not in
//      [k, buffer size] (an unlucky sample, massive ties) path B runs instead.
//   B. general: MSD radix narrowing on the composite key straight from memory,
//      11 bits a pass (histogram in 8 interleaved copies, copy = lane & 7, so
//      that lanes hitting one hot bin do not serialise), until the positions
//      matching the decided prefix fit the buffer; one pass collects them.
//   C. both: radix select inside LDS over the candidates yields T* exactly.
//   D. the selected positions are marked in an LDS bitmap of the row and read
//      back in ascending order (a counting sort), so the output is ordered
//      and deterministic.
// Row passes keep four 16-byte loads per thread in flight; a workgroup that
// issued one load per thread and round would crawl at memory latency.
#include "index_tile.h"
#include "select_common.h"
#include <mutex>

namespace {

constexpr int NT = 1024;
constexpr int HBITS = 11;
constexpr int NBINS = 1 << HBITS;
constexpr int COPIES = 8;
using ess_sel::CAND_CAP;
using ess_sel::SBITS;
using ess_sel::SBINS;
constexpr int SAMPLE_TARGET = 4096;         // at most this many samples per row (four per thread), about every 16th score or fewer
static_assert(SAMPLE_TARGET <= 4 * NT, "the sample is loaded in one round of four per thread");
constexpr int FAST_MIN_VIS = 16384;

struct __align__(16) TopkShared {
  union {
    uint32_t hist[NBINS * COPIES];        // 64 KiB
    uint32_t shist[ess_sel::sample_words<NT>()];   // 68 KiB, bins placed by sample_slot
    unsigned long long cand[CAND_CAP];    // 64 KiB
  };
  int32_t out_list[ESS_MAX_TOPK];         // 16 KiB
  uint32_t lhist[NBINS];                  // 8 KiB: digit histogram of the candidates held in LDS
  uint32_t wave_tot[NT / 64];
  unsigned long long red_and[NT / 64], red_or[NT / 64];
  uint32_t out_n, cand_n;
  uint32_t sel_digit, sel_above, sel_count;
  uint32_t sbin[2];                       // sample_bins' result words
};

__device__ __forceinline__ uint32_t orderable(float v) { return ess_orderable(v); }

using ess_sel::wave_incl_scan;
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  return ess_sel::block_incl_scan<NT>(v, wave_tot, total);
}

// append `val` for lanes with pred, one LDS atomic per wave; entries past `cap` are counted, not stored
template <typename V>
__device__ __forceinline__ void wave_append(bool pred, V val, V* list, uint32_t* counter, uint32_t cap = 0xffffffffu) {
  const unsigned long long mask = __ballot(pred);
  if (mask == 0) return;
  const int lane = threadIdx.x & 63;
  uint32_t base = 0;
  const int leader = __ffsll((long long)mask) - 1;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(mask));
  base = __shfl(base, leader, 64);
  const uint32_t pos = base + __popcll(mask & ((1ull << lane) - 1ull));
  if (pred && pos < cap) list[pos] = val;
}

// Calls f(position, score, valid) for every position of the row, by all threads the same number of
// times (f may hold wave-wide operations).  Each thread has four 16-byte loads in flight per round,
// which is what makes one workgroup able to pull a 512 KiB row at cache bandwidth, not at latency.
template <typename F>
__device__ __forceinline__ void scan_row(const float* __restrict__ srow, int vis, bool vec_ok, F&& f) {
  constexpr int U = 4;
  const int tid = threadIdx.x;
  int done = 0;
  if (vec_ok) {
    const int nvec = vis >> 2;
    const float4* v4 = reinterpret_cast<const float4*>(srow);
    for (int base = 0; base < nvec; base += NT * U) {
      float4 x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * NT + tid;
        x[u] = j < nvec ? v4[j] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * NT + tid;
        const bool ok = j < nvec;
        f(4 * j + 0, x[u].x, ok);
        f(4 * j + 1, x[u].y, ok);
        f(4 * j + 2, x[u].z, ok);
        f(4 * j + 3, x[u].w, ok);
      }
    }
    done = nvec << 2;
  }
  for (int i0 = done; i0 < vis; i0 += NT) {
    const int i = i0 + tid;
    const bool ok = i < vis;
    f(i, ok ? srow[i] : 0.f, ok);
  }
}

// Same walk, handing f one round (16 positions of this thread) at a time.  The loads of the next
// round are issued before the current round is processed (two register sets); indices past the end
// are clamped, not predicated, so that every load is unconditional.
template <typename F>
__device__ __forceinline__ void scan_row_rounds(const float* __restrict__ srow, int vis, bool vec_ok, F&& f) {
  constexpr int U = 4;
  const int tid = threadIdx.x;
  int done = 0;
  int pos[16];
  float val[16];
  bool ok[16];
  if (vec_ok && vis >= 4) {
    const int nvec = vis >> 2;
    const float4* v4 = reinterpret_cast<const float4*>(srow);
    auto load = [&](int base, float4 (&x)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) x[u] = v4[min(base + u * NT + tid, nvec - 1)];
    };
    auto process = [&](int base, const float4 (&x)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * NT + tid;
        const bool in = j < nvec;
        pos[4 * u + 0] = 4 * j + 0; val[4 * u + 0] = x[u].x; ok[4 * u + 0] = in;
        pos[4 * u + 1] = 4 * j + 1; val[4 * u + 1] = x[u].y; ok[4 * u + 1] = in;
        pos[4 * u + 2] = 4 * j + 2; val[4 * u + 2] = x[u].z; ok[4 * u + 2] = in;
        pos[4 * u + 3] = 4 * j + 3; val[4 * u + 3] = x[u].w; ok[4 * u + 3] = in;
      }
      f(pos, val, ok);
    };
    constexpr int R = NT * U;                    // float4s per round
    float4 xa[U], xb[U];
    load(0, xa);
    for (int base = 0; base < nvec; base += 2 * R) {
      load(base + R, xb);
      process(base, xa);
      if (base + R >= nvec) break;
      load(base + 2 * R, xa);
      process(base + R, xb);
    }
    done = nvec << 2;
  }
  for (int i0 = done; i0 < vis; i0 += 16 * NT) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int i = i0 + e * NT + tid;
      pos[e] = i; ok[e] = i < vis; val[e] = ok[e] ? srow[i] : 0.f;
    }
    f(pos, val, ok);
  }
}

// D, second half: the positions marked in the bitmap bmp[0..W), in ascending order, to orow[0..k)
__device__ __forceinline__ void emit_bitmap(TopkShared& sm, const uint32_t* bmp, int W, int k, int32_t* __restrict__ orow) {
  const int tid = threadIdx.x;
  const int wpt = (W + NT - 1) / NT;
  const int w0 = min(tid * wpt, W), w1 = min(w0 + wpt, W);
  uint32_t mine = 0;
  for (int wd = w0; wd < w1; ++wd) mine += __popc(bmp[wd]);
  uint32_t total;
  uint32_t outp = block_incl_scan(mine, sm.wave_tot, &total) - mine;
  for (int wd = w0; wd < w1; ++wd) {
    uint32_t bits = bmp[wd];
    while (bits) {
      const int bit = __ffs(bits) - 1;
      bits &= bits - 1;
      if (outp < (uint32_t)k) orow[outp] = wd * 32 + bit;
      ++outp;
    }
  }
}

// Which of the 2048 digits the radix select's histogram sm.lhist holds contains the need-th largest key, counted
// from the top: sm.sel_digit, with sm.sel_above keys above it and sm.sel_count in it.  Ends with a barrier.
__device__ __forceinline__ void crossing_digit(TopkShared& sm, uint32_t need) {
  const int tid = threadIdx.x;
  const int d_hi = NBINS - 1 - 2 * tid, d_lo = d_hi - 1;      // thread tid owns two digits, descending
  const uint32_t c_hi = sm.lhist[d_hi], c_lo = sm.lhist[d_lo];
  uint32_t total;
  const uint32_t inc = block_incl_scan(c_hi + c_lo, sm.wave_tot, &total);
  const uint32_t above_hi = inc - c_hi - c_lo;
  const uint32_t above_lo = above_hi + c_hi;
  if (above_hi < need && above_hi + c_hi >= need) {
    sm.sel_digit = d_hi; sm.sel_above = above_hi; sm.sel_count = c_hi;
  } else if (above_lo < need && above_lo + c_lo >= need) {
    sm.sel_digit = d_lo; sm.sel_above = above_lo; sm.sel_count = c_lo;
  }
  __syncthreads();
}

// A row finished from its candidate list (`listed` keys at grow, k <= listed <= CAND_CAP; SRC_LDS: the list is
// sm.cand itself) when the k-th largest score very probably lies in [lo, hi) (ess_orderable images; see
// sample_bins).  The keys stay in registers.  One
// histogram pass spreads [lo, hi) over 2047 digits (whatever lies at or above hi goes into the top one), the digit
// that holds the k-th largest key is found, and inside it -- a handful of keys -- the key is found by counting.
// Returns false, with the keys copied to sm.cand, when that digit holds more keys than the counting step takes
// (massive ties, or a k-th largest score outside the range): the caller goes on with the general selection.
template <bool SRC_LDS>
__device__ __forceinline__ bool finish_fast(TopkShared& sm, const unsigned long long* grow, uint32_t listed,
                                            uint32_t lo, uint32_t hi, int vis, int k, int IB, int32_t* __restrict__ orow) {
  constexpr int PER = CAND_CAP / NT;
  constexpr uint32_t SMALL = 1024;           // keys the counting step takes: one per thread
  const int tid = threadIdx.x;
  const unsigned long long imask = (1ull << IB) - 1ull;
  unsigned long long c[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u)
    c[u] = (uint32_t)(u * NT + tid) < listed ? (SRC_LDS ? sm.cand[u * NT + tid] : grow[u * NT + tid]) : 0ull;
  if (SRC_LDS) __syncthreads();              // the bitmap shares its memory with the list: every thread holds its keys first
  // while the keys are on their way: clear the histogram and the row's bitmap
  uint32_t* bmp = sm.hist;
  const int W = (vis + 31) >> 5;
  for (int j = tid; j < W; j += NT) bmp[j] = 0;
  for (int j = tid; j < NBINS; j += NT) sm.lhist[j] = 0;
  if (tid == 0) sm.cand_n = 0;
  int sh = 0;
  while (((hi - lo) >> sh) > (uint32_t)(NBINS - 2)) ++sh;
  auto digit = [&](unsigned long long key) -> uint32_t {
    const uint32_t sc = (uint32_t)(key >> IB);
    return sc >= hi ? (uint32_t)(NBINS - 1) : (sc <= lo ? 0u : min((sc - lo) >> sh, (uint32_t)(NBINS - 2)));
  };
  __syncthreads();
#pragma unroll
  for (int u = 0; u < PER; ++u)
    if ((uint32_t)(u * NT + tid) < listed) atomicAdd(&sm.lhist[digit(c[u])], 1u);
  __syncthreads();
  crossing_digit(sm, (uint32_t)k);
  const uint32_t dsel = sm.sel_digit, take = (uint32_t)k - sm.sel_above, cnt = sm.sel_count;
  unsigned long long t_in = 0ull;            // inside the digit, keys at or above this one are taken
  if (cnt != take) {
    if (cnt > SMALL) {
#pragma unroll
      for (int u = 0; u < PER; ++u)
        if ((uint32_t)(u * NT + tid) < listed) sm.cand[u * NT + tid] = c[u];
      if (tid == 0) sm.cand_n = listed;
      __syncthreads();
      return false;
    }
    unsigned long long* few = reinterpret_cast<unsigned long long*>(sm.out_list);     // room for 2048 keys
#pragma unroll
    for (int u = 0; u < PER; ++u)
      wave_append<unsigned long long>((uint32_t)(u * NT + tid) < listed && digit(c[u]) == dsel, c[u], few, &sm.cand_n);
    __syncthreads();
    if ((uint32_t)tid < cnt) {
      const unsigned long long my = few[tid];
      uint32_t above = 0;
      for (uint32_t i = 0; i < cnt; ++i) above += few[i] > my ? 1u : 0u;
      if (above == take - 1u) sm.red_and[0] = my;            // keys are distinct: exactly one thread
    }
    __syncthreads();
    t_in = sm.red_and[0];
  }
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    if ((uint32_t)(u * NT + tid) < listed) {
      const uint32_t d = digit(c[u]);
      if (d > dsel || (d == dsel && c[u] >= t_in)) {
        const uint32_t pos = (uint32_t)(imask - (c[u] & imask));
        atomicOr(&bmp[pos >> 5], 1u << (pos & 31));
      }
    }
  }
  __syncthreads();
  emit_bitmap(sm, bmp, W, k, orow);
  return true;
}

// MODE 0: one workgroup does the whole row (grid: rows).
// MODE 1 + MODE 2, for small batches of long rows: the candidate pass of path A, the only part that
// scales with the row, is spread over `parts` workgroups per row in a kernel of its own (MODE 1, grid
// parts x rows: every workgroup finds the same threshold from the same samples, scans its slice and
// appends its candidates to the row's list in global memory, g_cnt[row] counting them), and the
// finishing kernel (MODE 2, grid rows) takes the list when its size is in [k, buffer] -- else it does
// the row by itself like MODE 0.  The hand-over is the kernel boundary: workgroups of one kernel
// never exchange data (an agent-scope fence inside a kernel costs tens of microseconds on this
// multi-die part, where it writes the L2 back).  g_cnt is zero between steps: MODE 2 clears it.
// MODE 3: the finishing kernel of the fused selection (grid rows).  The row's list was written by the emitting
// index-score pass (index_kernel.h), for rows of any length; `score` is scratch memory, not scores: a row whose list
// cannot be used (fewer than k or more than the buffer holds: a misleading sample, massive ties) has its scores
// computed here, by this workgroup, into its row of `score`, and is then done like MODE 0.
// one work item = (part, row) of k_topk<MODE>; every field of `sm` is set before it is read, so items may follow each other
struct TopkRecompute {                     // MODE 3: what it takes to compute a row's scores
  const uint8_t* q; const float* w; const uint8_t* key; const int32_t* block_table;
  int n_pages, Hi, Di;
};
template <int MODE>
__device__ __forceinline__ void topk_item(TopkShared& sm, int item, int parts, float* __restrict__ score,
                                          const int32_t* __restrict__ ctx_len, int T, int Lmax, int k, int IB,
                                          int32_t* __restrict__ idx_out, unsigned long long* __restrict__ g_cand,
                                          uint32_t* __restrict__ g_cnt, uint32_t* __restrict__ g_tau, const TopkRecompute& rc) {
  const int row = item / parts;
  const int part = item % parts;
  const int b = row / T, t = row % T;
  const int tid = threadIdx.x, lane = tid & 63;
  int vis = ctx_len[b] - (T - 1 - t);
  vis = max(0, min(vis, Lmax));
  float* srow = score + (size_t)row * Lmax;
  int32_t* orow = idx_out + (size_t)row * k;

  if (MODE == 1 && (vis <= k || vis < FAST_MIN_VIS)) return;      // nothing to prepare
  uint32_t listed = 0;
  if (MODE >= 2) {                         // candidates prepared by the kernel in front (0 if none)
    listed = g_cnt[row];
    __syncthreads();
    if (tid == 0) g_cnt[row] = 0;
  }
  if (vis <= k) {                          // everything visible is selected
    for (int j = tid; j < k; j += NT) orow[j] = j < vis ? j : -1;
    return;
  }

  const unsigned long long imask = (1ull << IB) - 1ull;
  const bool vec_ok = ((Lmax & 3) == 0) && ((reinterpret_cast<uintptr_t>(score) & 15) == 0);
  auto comp_of = [&](int i, float v) -> unsigned long long {
    return ((unsigned long long)orderable(v) << IB) | (imask - (unsigned long long)i);
  };

  // decided high bits of T* (`prefix`), number of undecided low bits (`rem`), and how many of the
  // keys matching the prefix are still to be taken (`need`); candidates matching it sit in sm.cand
  int rem = 32 + IB;
  unsigned long long prefix = 0;
  uint32_t need = (uint32_t)k;
  bool have_cand = false;                   // sm.cand[0..nc) holds every key matching the prefix
  bool all_in_cand = false;                 // ... and every key above it as well (path A)
  int nc = 0;

  // ---- A: sampled one-pass collection for long rows
  const bool use_list = MODE >= 2 && listed >= (uint32_t)k && listed <= (uint32_t)CAND_CAP;
  if (MODE == 3 && !use_list) {
    const uint8_t* q_row = rc.q + (size_t)row * rc.Hi * rc.Di;
    const float* w_row = rc.w + (size_t)row * rc.Hi;
    const int32_t* table_row = rc.block_table ? rc.block_table + (size_t)b * (Lmax / ESS_PAGE_TOKENS) : nullptr;
    const uint8_t* keys = rc.block_table ? rc.key : rc.key + (size_t)b * Lmax * rc.Di;
    if (rc.Di == 128) ess_idx::row_scores_slow<128>(q_row, w_row, rc.Hi, keys, Lmax, table_row, rc.n_pages, vis, srow);
    else if (rc.Di == 64) ess_idx::row_scores_slow<64>(q_row, w_row, rc.Hi, keys, Lmax, table_row, rc.n_pages, vis, srow);
    else ess_idx::row_scores_slow<32>(q_row, w_row, rc.Hi, keys, Lmax, table_row, rc.n_pages, vis, srow);
    __syncthreads();                       // the scores are read back by other threads of this workgroup
  }
  if (use_list) {
    const unsigned long long* grow = g_cand + (size_t)row * CAND_CAP;
    bool copied = false;
    {
      const uint32_t lo = g_tau[2 * row], hi = g_tau[2 * row + 1];       // left by the kernel that made the list
      if (lo != 0u && hi > lo) {
        if (finish_fast<false>(sm, grow, listed, lo, hi, vis, k, IB, orow)) return;
        copied = true;
      }
    }
    if (!copied) {
      for (int j = tid; j < (int)listed; j += NT) sm.cand[j] = grow[j];
      if (tid == 0) sm.cand_n = listed;
      __syncthreads();
    }
  }
  if (vis >= FAST_MIN_VIS || use_list) {
   uint32_t lo_bin = 0, hi_bin = 0xffffffffu;
   if (!use_list) {
    // samples: blocks of 16 consecutive scores (one 64-byte piece of a cache line), every bstride-th block,
    // about SAMPLE_TARGET scores in all.  (One score out of every 16th..32nd touches every cache line of the
    // row: in cache-line traffic the sample then costs as much as the pass that follows.)
    const int nblk_all = vis >> 4;
    int bstride = 1;
    while (nblk_all / bstride > SAMPLE_TARGET / 16) bstride <<= 1;
    const int ns = (nblk_all / bstride) << 4;
    // (at most SAMPLE_TARGET samples: four per thread, requested before the histogram is cleared)
    float sv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = u * NT + tid;
      sv[u] = j < ns ? srow[(size_t)(j >> 4) * bstride * 16 + (j & 15)] : 0.f;
    }
    for (int j = tid; j < ess_sel::sample_words<NT>(); j += NT) sm.shist[j] = 0;
    if (tid == 0) { sm.cand_n = 0; sm.sbin[0] = sm.sbin[1] = 0xffffffffu; }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (u * NT + tid < ns) atomicAdd(&sm.shist[ess_sel::sample_slot<NT>(orderable(sv[u]) >> (32 - SBITS))], 1u);
    __syncthreads();
    ess_sel::sample_bins<NT>(sm.shist, sm.wave_tot, sm.sbin, k, ns, vis, &lo_bin, &hi_bin);      // (ends with a barrier: shist is dead from here, cand may overwrite it)
   }
    if (MODE == 1 && lo_bin == 0xffffffffu) return;   // no usable threshold: the finishing kernel takes path B
    if (use_list || lo_bin != 0xffffffffu) {
     // the k-th largest score very probably lies in [tau, tau_hi) (see sample_bins)
     const uint32_t tau = lo_bin << (32 - SBITS);
     const uint32_t tau_hi = (hi_bin == 0xffffffffu || hi_bin == SBINS - 1) ? 0xffffffffu : (hi_bin + 1) << (32 - SBITS);
     if (!use_list) {
      // The pass only compares floats and stores (position, score) of the few positions at or above
      // the key: v >= tau_f is the same predicate as orderable(v) >= tau (NaN fails both, -0 == +0),
      // and the composite keys are computed afterwards, densely, for the candidates alone.
      const float tau_f = __uint_as_float((tau & 0x80000000u) ? (tau & 0x7fffffffu) : ~tau);
      uint2* raw = reinterpret_cast<uint2*>(sm.cand);
      // this workgroup's slice of the row (boundaries on 16-byte pieces)
      const int s_lo = parts > 1 ? (int)(((long)vis * part / parts) & ~3L) : 0;
      const int s_hi = (parts > 1 && part + 1 < parts) ? (int)(((long)vis * (part + 1) / parts) & ~3L) : vis;
      scan_row_rounds(srow + s_lo, s_hi - s_lo, vec_ok, [&](const int (&pos)[16], const float (&val)[16], const bool (&ok)[16]) {
        uint32_t cnt = 0, flags = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (ok[e] && val[e] >= tau_f) { flags |= 1u << e; ++cnt; }
        // one LDS atomic per wave and round
        const uint32_t winc = wave_incl_scan(cnt, lane);
        uint32_t base = 0;
        if (lane == 63 && winc) base = atomicAdd(&sm.cand_n, winc);
        base = __shfl(base, 63, 64) + winc - cnt;
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (flags & (1u << e)) {
            if (base < (uint32_t)CAND_CAP) raw[base] = make_uint2((uint32_t)(pos[e] + s_lo), __float_as_uint(val[e]));
            ++base;
          }
      });
      __syncthreads();
      if ((int)sm.cand_n <= CAND_CAP)
        for (int j = tid; j < (int)sm.cand_n; j += NT) {
          const uint2 pv = raw[j];
          sm.cand[j] = comp_of((int)pv.x, __uint_as_float(pv.y));
        }
      __syncthreads();
     }
      nc = (int)sm.cand_n;
      if (MODE == 1) {
        // append this slice's candidates to the row's list; the true count is added even when it overflows,
        // so that the finishing kernel sees the overflow
        unsigned long long* grow = g_cand + (size_t)row * CAND_CAP;
        if (tid == 0) {
          sm.sel_above = atomicAdd(&g_cnt[row], (uint32_t)nc);
          if (part == 0) { g_tau[2 * row] = tau; g_tau[2 * row + 1] = tau_hi; }    // (every part finds the same two)
        }
        __syncthreads();
        const uint32_t gbase = sm.sel_above;
        if (nc <= CAND_CAP)
          for (int j = tid; j < nc; j += NT)
            if (gbase + (uint32_t)j < (uint32_t)CAND_CAP) grow[gbase + j] = sm.cand[j];
        return;
      }
      if (!use_list && nc >= k && nc <= CAND_CAP && tau != 0u && tau_hi > tau &&
          finish_fast<true>(sm, sm.cand, (uint32_t)nc, tau, tau_hi, vis, k, IB, orow))
        return;
      if (nc >= k && nc <= CAND_CAP) {
        // bits on which the candidates differ: everything above is common and decided
        unsigned long long a = ~0ull, o = 0ull;
        for (int j = tid; j < nc; j += NT) { a &= sm.cand[j]; o |= sm.cand[j]; }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { a &= __shfl_xor(a, d, 64); o |= __shfl_xor(o, d, 64); }
        if (lane == 0) { sm.red_and[tid >> 6] = a; sm.red_or[tid >> 6] = o; }
        __syncthreads();
        a = ~0ull; o = 0ull;
#pragma unroll
        for (int i = 0; i < NT / 64; ++i) { a &= sm.red_and[i]; o |= sm.red_or[i]; }
        const unsigned long long diff = a ^ o;
        rem = diff ? 64 - __clzll((long long)diff) : 0;
        prefix = rem < 64 ? (o >> rem) : 0;
        have_cand = true;
        all_in_cand = true;
      }
      __syncthreads();
    }
  }

  // ---- B: general narrowing from memory
  if (!have_cand) {
    uint32_t cnt_match = (uint32_t)vis;
    while (cnt_match > (uint32_t)CAND_CAP && rem > 0) {
      const int bits = min(HBITS, rem);
      const int shift = rem - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int j = tid; j < NBINS * COPIES; j += NT) sm.hist[j] = 0;
      __syncthreads();
      scan_row(srow, vis, vec_ok, [&](int i, float v, bool ok) {
        const unsigned long long c = comp_of(i, v);
        if (ok && (c >> rem) == prefix)
          atomicAdd(&sm.hist[(((uint32_t)(c >> shift)) & dmask) * COPIES + (lane & 7)], 1u);
      });
      __syncthreads();
      // thread tid owns digits NBINS-1-2*tid and NBINS-2-2*tid (descending), scan = suffix counts
      const int d_hi = NBINS - 1 - 2 * tid, d_lo = d_hi - 1;
      uint32_t c_hi = 0, c_lo = 0;
#pragma unroll
      for (int r = 0; r < COPIES; ++r) {
        c_hi += sm.hist[d_hi * COPIES + r];
        c_lo += sm.hist[d_lo * COPIES + r];
      }
      uint32_t total;
      const uint32_t inc = block_incl_scan(c_hi + c_lo, sm.wave_tot, &total);
      const uint32_t above_hi = inc - c_hi - c_lo;      // keys with a digit > d_hi
      const uint32_t above_lo = above_hi + c_hi;        // keys with a digit > d_lo
      if (above_hi < need && above_hi + c_hi >= need) {
        sm.sel_digit = d_hi; sm.sel_above = above_hi; sm.sel_count = c_hi;
      } else if (above_lo < need && above_lo + c_lo >= need) {
        sm.sel_digit = d_lo; sm.sel_above = above_lo; sm.sel_count = c_lo;
      }
      __syncthreads();
      need -= sm.sel_above;
      prefix = (prefix << bits) | sm.sel_digit;
      cnt_match = sm.sel_count;
      rem = shift;
      __syncthreads();
    }
    if (tid == 0) sm.cand_n = 0;
    __syncthreads();
    scan_row(srow, vis, vec_ok, [&](int i, float v, bool ok) {
      const unsigned long long c = comp_of(i, v);
      wave_append<unsigned long long>(ok && (c >> rem) == prefix, c, sm.cand, &sm.cand_n, CAND_CAP);
    });
    __syncthreads();
    nc = (int)sm.cand_n;
  }

  // ---- C: radix select inside LDS: the need-th largest candidate among those matching the prefix
  while (rem > 0) {
    const int bits = min(HBITS, rem);
    const int shift = rem - bits;
    const uint32_t dmask = (1u << bits) - 1u;
    for (int j = tid; j < NBINS; j += NT) sm.lhist[j] = 0;
    __syncthreads();
    for (int j = tid; j < nc; j += NT) {
      const unsigned long long c = sm.cand[j];
      if ((c >> rem) == prefix) atomicAdd(&sm.lhist[((uint32_t)(c >> shift)) & dmask], 1u);
    }
    __syncthreads();
    crossing_digit(sm, need);
    need -= sm.sel_above;
    prefix = (prefix << bits) | sm.sel_digit;
    const uint32_t cnt = sm.sel_count;
    rem = shift;
    __syncthreads();
    if (cnt == need) break;                  // every key with this prefix is taken
  }
  const unsigned long long t_star = rem < 64 ? (prefix << rem) : 0ull;

  // ---- D: mark the selected positions in a bitmap of the row, read them back in ascending order
  uint32_t* bmp = sm.hist;                   // aliases cand: the keys are moved out first
  const int W = (vis + 31) >> 5;             // <= 16384 words
  if (all_in_cand) {
    if (tid == 0) sm.out_n = 0;
    __syncthreads();
    for (int j0 = 0; j0 < nc; j0 += NT) {
      const int j = j0 + tid;
      const unsigned long long c = j < nc ? sm.cand[j] : 0ull;
      wave_append<int32_t>(j < nc && c >= t_star, (int32_t)(imask - (c & imask)), sm.out_list, &sm.out_n, ESS_MAX_TOPK);
    }
    __syncthreads();
    for (int j = tid; j < W; j += NT) bmp[j] = 0;
    __syncthreads();
    for (int j = tid; j < k; j += NT) {
      const int pos = sm.out_list[j];
      atomicOr(&bmp[pos >> 5], 1u << (pos & 31));
    }
  } else {
    __syncthreads();
    for (int j = tid; j < W; j += NT) bmp[j] = 0;
    __syncthreads();
    scan_row(srow, vis, vec_ok, [&](int i, float v, bool ok) {
      if (ok && comp_of(i, v) >= t_star) atomicOr(&bmp[i >> 5], 1u << (i & 31));
    });
  }
  __syncthreads();
  emit_bitmap(sm, bmp, W, k, orow);
}

template <int MODE, bool DYN>
__global__ __launch_bounds__(NT) void k_topk(float* __restrict__ score, const int32_t* __restrict__ ctx_len,
                                             int T, int Lmax, int k, int IB, int32_t* __restrict__ idx_out,
                                             unsigned long long* __restrict__ g_cand, uint32_t* __restrict__ g_cnt,
                                             uint32_t* __restrict__ g_tau, ess_xcd xcd, int rows, int parts_arg,
                                             const TopkRecompute rc) {
  __shared__ TopkShared sm;
  __shared__ int s_item;
  const int parts = MODE == 1 ? parts_arg : 1;
  // work item = (part, row): by workgroup index, or drawn from the launch's counter off the XCDs to be avoided
  ESS_WORK_LOOP(DYN, xcd, MODE == 1 ? blockIdx.y * parts + blockIdx.x : blockIdx.x, rows * parts, &s_item, item) {
    topk_item<MODE>(sm, item, parts, score, ctx_len, T, Lmax, k, IB, idx_out, g_cand, g_cnt, g_tau, rc);
  }
}

// The bounds of every row's selection, from the scores of the sequence's sample blocks (one workgroup per row), as
// ess_orderable images of scores:
// tau[row][0] = a score that very probably has at least k and at most a few thousand of the row's scores at or above
// it; 0 (everything is a candidate) for rows that fit the candidate buffer whole or whose sample gives no bound;
// 0xffffffff (nothing) for rows with at most k visible positions, which need no list;
// tau[row][1] = a score that very probably has fewer than k of the row's scores at or above it (0xffffffff if the
// sample gives none; 0 with no lower bound): the k-th largest score very probably lies between the two, which lets
// the finishing kernel resolve that range in one pass.
// Also clears the row's candidate counter for the pass that follows.
template <bool DYN>
__global__ __launch_bounds__(NT) void k_index_tau(const float* __restrict__ sample, const int32_t* __restrict__ ctx_len,
                                                  int T, int Lmax, int k, int period, int nsamp,
                                                  uint32_t* __restrict__ tau, uint32_t* __restrict__ g_cnt, ess_xcd xcd,
                                                  int rows) {
  __shared__ uint32_t shist[ess_sel::sample_words<NT>()];
  __shared__ uint32_t wave_tot[NT / 64], sel[2];
  __shared__ int s_item;
  ESS_WORK_LOOP(DYN, xcd, blockIdx.x, rows, &s_item, row) {
    const int tid = threadIdx.x;
    const int b = row / T, t = row % T;
    const int len = min(ctx_len[b], Lmax);
    const int vis = max(0, len - (T - 1 - t));
    if (tid == 0) g_cnt[row] = 0;
    if (vis <= k || vis <= CAND_CAP) {
      if (tid == 0) {
        tau[2 * row] = vis <= k ? 0xffffffffu : 0u;
        tau[2 * row + 1] = 0u;
      }
      continue;
    }
    // the blocks that count are the first nv: starts grow with the block number
    const int lim = len - (T - 1);
    int nv = lim / period;
    if (nv < nsamp && ess_sample_start(nv, period) + 64 <= lim) ++nv;
    nv = min(nv, nsamp);
    const int ns = nv * 64;
    // the samples are requested before the histogram is cleared: one round trip to memory, not two
    const float* srow = sample + (size_t)row * nsamp * 64;
    constexpr int PER = ESS_SAMPLE_BLOCKS * 64 / NT;
    float sv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) sv[u] = u * NT + tid < ns ? srow[u * NT + tid] : 0.f;
    for (int j = tid; j < ess_sel::sample_words<NT>(); j += NT) shist[j] = 0;
    if (tid == 0) sel[0] = sel[1] = 0xffffffffu;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if (u * NT + tid < ns) atomicAdd(&shist[ess_sel::sample_slot<NT>(orderable(sv[u]) >> (32 - SBITS))], 1u);
    __syncthreads();
    uint32_t lo = 0xffffffffu, hi = 0xffffffffu;
    if (ns > 0) ess_sel::sample_bins<NT>(shist, wave_tot, sel, k, ns, vis, &lo, &hi);
    if (tid == 0) {
      tau[2 * row] = lo == 0xffffffffu ? 0u : lo << (32 - SBITS);
      // scores in the bins above `hi` are very probably fewer than k; no such bin: no upper bound
      tau[2 * row + 1] = lo == 0xffffffffu ? 0u : ((hi == 0xffffffffu || hi == SBINS - 1) ? 0xffffffffu : (hi + 1) << (32 - SBITS));
    }
  }
}

}  // namespace

namespace {
// Launches of one top-k call.  cand / cnt: candidate lists [ESS_TOPK_SHARED_ROWS][CAND_CAP] and their counters
// (zero at launch, zero again afterwards), only used when rows are shared by several workgroups.
int launch_topk(int max_ctx, int k, const float* score_in, const int32_t* ctx_len, int B, int T, int32_t* idx,
                unsigned long long* cand, uint32_t* cnt, uint32_t* tau, hipStream_t st, ess_xcd xcd) {
  float* score = const_cast<float*>(score_in);          // read only in these modes
  const TopkRecompute rc{};
  int IB = 1;
  while ((1 << IB) < max_ctx) ++IB;
  // small batches of long rows: the candidate pass goes to a kernel of its own that puts several
  // workgroups on every row (as many as fill the chip, at most 8)
  const int rows = B * T;
  int parts = 1;
  if (max_ctx >= 4 * FAST_MIN_VIS && rows <= ESS_TOPK_SHARED_ROWS) {
    parts = 256 / rows;
    if (parts > 8) parts = 8;
  }
  const ess_xcd x0 = xcd, x1 = ess_xcd{xcd.ticket ? xcd.ticket + ESS_TICKET_WORDS : nullptr, xcd.avoid,
                                       xcd.host_need ? xcd.host_need + 1 : nullptr, xcd.grid_override};
  const bool dyn = xcd.ticket != nullptr;
#define ESS_TOPK_LAUNCH(MODE, grid, x, np)                                                                           \
  do {                                                                                                               \
    if (dyn) hipLaunchKernelGGL((k_topk<MODE, true>), grid, dim3(NT), 0, st, score, ctx_len, T, max_ctx, k, IB, idx, \
                                cand, cnt, tau, x, rows, np, rc);                                                    \
    else hipLaunchKernelGGL((k_topk<MODE, false>), grid, dim3(NT), 0, st, score, ctx_len, T, max_ctx, k, IB, idx,    \
                            cand, cnt, tau, x, rows, np, rc);                                                        \
  } while (0)
  if (parts > 1) {
    const dim3 g1 = dyn ? dim3(ess_xcd_grid(parts * rows, x0)) : dim3(parts, rows);
    ESS_TOPK_LAUNCH(1, g1, x0, parts);
    ESS_TOPK_LAUNCH(2, dim3(ess_xcd_grid(rows, x1)), x1, 1);
  } else {
    ESS_TOPK_LAUNCH(0, dim3(ess_xcd_grid(rows, x1)), x1, 1);
  }
#undef ESS_TOPK_LAUNCH
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
}  // namespace

int ess_launch_topk(ess_ctx* ctx, const float* score, const int32_t* ctx_len, int B, int T, int32_t* idx,
                    hipStream_t st, ess_xcd xcd) {
  return launch_topk(ctx->cfg.max_ctx, ctx->cfg.topk, score, ctx_len, B, T, idx, ctx->topk_cand, ctx->topk_cnt, ctx->topk_tau, st, xcd);
}

// The two small kernels of the fused selection that live here (see ess_internal.h).
int ess_launch_index_tau(ess_ctx* ctx, const int32_t* ctx_len, int B, int T, int b0, hipStream_t st, ess_xcd xcd) {
  const ess_config& c = ctx->cfg;
  const int rows = B * T, nsamp = ess_sample_count(c.max_ctx);
  const size_t r0 = (size_t)b0 * T;
  const dim3 grid(ess_xcd_grid(rows, xcd));
  if (xcd.ticket)
    hipLaunchKernelGGL((k_index_tau<true>), grid, dim3(NT), 0, st, ctx->sel_sample + r0 * nsamp * 64, ctx_len, T, c.max_ctx,
                       c.topk, ess_sample_period(c.max_ctx), nsamp, ctx->sel_tau + 2 * r0, ctx->sel_cnt + r0, xcd, rows);
  else
    hipLaunchKernelGGL((k_index_tau<false>), grid, dim3(NT), 0, st, ctx->sel_sample + r0 * nsamp * 64, ctx_len, T, c.max_ctx,
                       c.topk, ess_sample_period(c.max_ctx), nsamp, ctx->sel_tau + 2 * r0, ctx->sel_cnt + r0, xcd, rows);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_topk_finish(ess_ctx* ctx, const uint8_t* q, const float* w, const uint8_t* key, const int32_t* block_table,
                           int n_pages, const int32_t* ctx_len, int B, int T, int b0, int32_t* idx, hipStream_t st,
                           ess_xcd xcd) {
  const ess_config& c = ctx->cfg;
  int IB = 1;
  while ((1 << IB) < c.max_ctx) ++IB;
  const int rows = B * T;
  const size_t r0 = (size_t)b0 * T;
  const TopkRecompute rc{q, w, key, block_table, n_pages, c.idx_heads, c.idx_dim};
  const dim3 grid(ess_xcd_grid(rows, xcd));
  if (xcd.ticket)
    hipLaunchKernelGGL((k_topk<3, true>), grid, dim3(NT), 0, st, ctx->score_ws + r0 * c.max_ctx, ctx_len, T, c.max_ctx, c.topk,
                       IB, idx, ctx->sel_cand + r0 * CAND_CAP, ctx->sel_cnt + r0, ctx->sel_tau + 2 * r0, xcd, rows, 1, rc);
  else
    hipLaunchKernelGGL((k_topk<3, false>), grid, dim3(NT), 0, st, ctx->score_ws + r0 * c.max_ctx, ctx_len, T, c.max_ctx, c.topk,
                       IB, idx, ctx->sel_cand + r0 * CAND_CAP, ctx->sel_cnt + r0, ctx->sel_tau + 2 * r0, xcd, rows, 1, rc);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_sel_cand_cap() { return CAND_CAP; }

size_t ess_topk_cand_bytes() { return (size_t)ESS_TOPK_SHARED_ROWS * CAND_CAP * sizeof(unsigned long long); }

// ---------------------------------------------------------------------------------------------
// ess_topk_static: the top-k for callers that cannot allocate.  Its scratch memory -- the candidate lists of rows
// shared by several workgroups, and their counters -- is this array, part of the library's image on every
// GPU it is loaded on (8 MiB + 1536 bytes).  In host code the array's name is not a device address: the address
// on the current device is asked for once per device and kept.
namespace {
constexpr size_t kStaticCand = (size_t)ESS_TOPK_SHARED_ROWS * CAND_CAP;          // candidate keys
constexpr size_t kStaticWords = kStaticCand + ESS_TOPK_SHARED_ROWS / 2 + ESS_TOPK_SHARED_ROWS;   // + the rows' counters (uint32 each) + their bounds (2 x uint32)
constexpr int kMaxDevices = 64;
static_assert(ESS_TOPK_STATIC_MAX_ROWS == ESS_TOPK_SHARED_ROWS, "the static scratch holds one candidate list per shared row");
}  // namespace
static __device__ __align__(256) unsigned long long ess_topk_scratch[kStaticWords];
namespace {
unsigned long long* g_static_ptr[kMaxDevices];                                   // per device: address of its copy of the array
std::mutex g_static_mu;
}  // namespace

extern "C" int ess_topk_static(const float* score, const int32_t* ctx_len, int32_t B, int32_t T, int32_t max_ctx,
                               int32_t k, int32_t* idx, void* stream) {
  if (!score || !ctx_len || !idx) return ess_fail(ESS_ERR_INVALID_ARG, "NULL argument");
  if (B < 1 || T < 1 || T > 4) return ess_fail(ESS_ERR_INVALID_ARG, "B %d, T %d (T: 1 to 4)", B, T);
  if ((long)B * T > ESS_TOPK_STATIC_MAX_ROWS)
    return ess_fail(ESS_ERR_CAPACITY, "ess_topk_static: B*T = %ld rows exceed the %d its static scratch memory holds",
                    (long)B * T, ESS_TOPK_STATIC_MAX_ROWS);
  if (max_ctx < 1 || max_ctx > ESS_MAX_CTX)
    return ess_fail(ESS_ERR_CAPACITY, "ess_topk_static: max_ctx %d outside [1, %d]", max_ctx, ESS_MAX_CTX);
  if (k < 1 || k > ESS_MAX_TOPK) return ess_fail(ESS_ERR_CAPACITY, "ess_topk_static: k %d outside [1, %d]", k, ESS_MAX_TOPK);
  int dev = 0;
  ESS_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return ess_fail(ESS_ERR_UNSUPPORTED, "ess_topk_static: device %d", dev);
  unsigned long long* base;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {                 // first call on this device: where does its copy of the array live?
      void* p = nullptr;
      ESS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(ess_topk_scratch)));
      if (!p) return ess_fail(ESS_ERR_HIP, "ess_topk_static: the scratch array has no address on device %d", dev);
      g_static_ptr[dev] = static_cast<unsigned long long*>(p);
    }
    base = g_static_ptr[dev];
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint32_t* cnt = reinterpret_cast<uint32_t*>(base + kStaticCand);
  // the array keeps what the last call left: the counters must start at zero (a fill kernel, not a memset node,
  // so that the call may be captured in a graph)
  int rc = ess_launch_fill_u32(cnt, ESS_TOPK_SHARED_ROWS, 0u, st);
  if (rc != ESS_OK) return rc;
  return launch_topk(max_ctx, k, score, ctx_len, B, T, idx, base, cnt, cnt + ESS_TOPK_SHARED_ROWS, st, ess_xcd{nullptr, 0, nullptr, 0});
}
