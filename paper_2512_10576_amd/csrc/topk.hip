// Stage 2: per-query top-k over the indexer scores (ESS paper Sec. 3: the top
// 2,048 entries are selected).
//
// Selection order is (score descending, position ascending).  Every position
// gets a unique composite key  c = orderable_u32(score) << IB | (2^IB-1 - pos)
// (IB = bits needed for a position), so "the k largest composite keys" is a
// total order with no ties and any selection algorithm gives the same set.
//
// One workgroup per (b,t) row:
//   1. MSD radix narrowing, 11 bits a pass, on the composite key: histogram
//      the next digit of the positions that still match the decided prefix,
//      find the digit that holds the k-th largest key, descend -- until the
//      positions matching the prefix fit a candidate buffer in LDS.
//   2. one collection pass: keys above the prefix are selected outright, keys
//      matching it go to the candidate buffer;
//   3. the candidates are sorted in LDS (bitonic) and the best `need` taken;
//   4. the k positions are sorted ascending and written.
// The histogram is kept in 8 interleaved copies (copy = lane & 7, one bank
// apart) so that lanes hitting the same hot bin do not serialise.
#include "ess_internal.h"

namespace {

constexpr int NT = 1024;
constexpr int HBITS = 11;
constexpr int NBINS = 1 << HBITS;
constexpr int COPIES = 8;
constexpr int CAND_CAP = 8192;

struct __align__(16) TopkShared {
  union {
    uint32_t hist[NBINS * COPIES];        // 64 KiB
    unsigned long long cand[CAND_CAP];    // 64 KiB
  };
  int32_t out_list[ESS_MAX_TOPK];         // 16 KiB
  uint32_t wave_tot[NT / 64];
  uint32_t out_n, cand_n;
  uint32_t sel_digit, sel_above, sel_count;
};

__device__ __forceinline__ uint32_t orderable(float v) {
  if (v != v) v = -__builtin_inff();      // NaN ranks as -inf
  v += 0.0f;                              // -0 -> +0
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

// inclusive scan over the NT threads in thread order; *total gets the sum
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_scan(v, lane);
  __syncthreads();                         // wave_tot may still be read from a previous call
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) {
    const uint32_t x = wave_tot[i];
    if (i < wave) off += x;
    tot += x;
  }
  *total = tot;
  return inc + off;
}

// append `val` for lanes with pred, one LDS atomic per wave
template <typename V>
__device__ __forceinline__ void wave_append(bool pred, V val, V* list, uint32_t* counter) {
  const unsigned long long mask = __ballot(pred);
  if (mask == 0) return;
  const int lane = threadIdx.x & 63;
  uint32_t base = 0;
  const int leader = __ffsll((long long)mask) - 1;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(mask));
  base = __shfl(base, leader, 64);
  if (pred) list[base + __popcll(mask & ((1ull << lane) - 1ull))] = val;
}

// ascending bitonic sort of a[0..n), n a power of two, by all NT threads
template <typename V>
__device__ void bitonic_sort(V* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int t = threadIdx.x; t < (n >> 1); t += NT) {
        const int lo = 2 * t - (t & (stride - 1));
        const int hi = lo + stride;
        const bool up = (lo & size) == 0;
        const V x = a[lo], y = a[hi];
        if ((x > y) == up) { a[lo] = y; a[hi] = x; }
      }
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(NT) void k_topk(const float* __restrict__ score, const int32_t* __restrict__ ctx_len,
                                             int T, int Lmax, int k, int IB, int32_t* __restrict__ idx_out) {
  __shared__ TopkShared sm;
  const int row = blockIdx.x;
  const int b = row / T, t = row % T;
  const int tid = threadIdx.x, lane = tid & 63;
  int vis = ctx_len[b] - (T - 1 - t);
  vis = max(0, min(vis, Lmax));
  const float* srow = score + (size_t)row * Lmax;
  int32_t* orow = idx_out + (size_t)row * k;

  if (vis <= k) {                          // everything visible is selected
    for (int j = tid; j < k; j += NT) orow[j] = j < vis ? j : -1;
    return;
  }

  const unsigned long long imask = (1ull << IB) - 1ull;
  auto comp = [&](int i) -> unsigned long long {
    return ((unsigned long long)orderable(srow[i]) << IB) | (imask - (unsigned long long)i);
  };

  int rem = 32 + IB;                       // undecided low bits of the composite key
  unsigned long long prefix = 0;           // decided high bits
  uint32_t need = (uint32_t)k;             // how many keys matching the prefix are still to be taken
  uint32_t cnt_match = (uint32_t)vis;

  while (cnt_match > (uint32_t)CAND_CAP && rem > 0) {
    const int bits = min(HBITS, rem);
    const int shift = rem - bits;
    const uint32_t dmask = (1u << bits) - 1u;
    for (int j = tid; j < NBINS * COPIES; j += NT) sm.hist[j] = 0;
    __syncthreads();
    for (int i = tid; i < vis; i += NT) {
      const unsigned long long c = comp(i);
      if ((c >> rem) == prefix) atomicAdd(&sm.hist[(((uint32_t)(c >> shift)) & dmask) * COPIES + (lane & 7)], 1u);
    }
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

  // collection
  if (tid == 0) { sm.out_n = 0; sm.cand_n = 0; }
  __syncthreads();
  for (int i0 = 0; i0 < vis; i0 += NT) {
    const int i = i0 + tid;
    bool sel = false, cnd = false;
    unsigned long long c = 0;
    if (i < vis) {
      c = comp(i);
      const unsigned long long top = c >> rem;
      sel = top > prefix;
      cnd = top == prefix;
    }
    wave_append<int32_t>(sel, i, sm.out_list, &sm.out_n);
    wave_append<unsigned long long>(cnd, c, sm.cand, &sm.cand_n);
  }
  __syncthreads();
  const int nc = (int)sm.cand_n;
  int np = 1;
  while (np < nc) np <<= 1;
  for (int j = nc + tid; j < np; j += NT) sm.cand[j] = 0ull;   // below every real key
  bitonic_sort<unsigned long long>(sm.cand, np);               // ascending: best keys at the end
  const uint32_t got = sm.out_n;                               // = k - need
  for (uint32_t j = tid; j < need; j += NT)
    sm.out_list[got + j] = (int32_t)(imask - (sm.cand[np - 1 - j] & imask));
  int kp = 1;
  while (kp < k) kp <<= 1;
  for (int j = k + tid; j < kp; j += NT) sm.out_list[j] = 0x7fffffff;
  bitonic_sort<int32_t>(sm.out_list, kp);
  for (int j = tid; j < k; j += NT) orow[j] = sm.out_list[j];
}

}  // namespace

int ess_launch_topk(const ess_config& c, const float* score, const int32_t* ctx_len, int B, int T, int32_t* idx,
                    hipStream_t st) {
  int IB = 1;
  while ((1 << IB) < c.max_ctx) ++IB;
  hipLaunchKernelGGL(k_topk, dim3(B * T), dim3(NT), 0, st, score, ctx_len, T, c.max_ctx, c.topk, IB, idx);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
