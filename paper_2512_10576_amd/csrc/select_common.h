// Pieces shared by the kernels of the selection (top-k, and the sampled lower bound of the fused selection).
#pragma once
#include "ess_internal.h"

namespace ess_sel {

constexpr int SBITS = 14;                  // sample histogram: top 14 bits of the orderable key
constexpr int SBINS = 1 << SBITS;
constexpr int CAND_CAP = 8192;             // candidate keys a row's list (and the LDS of the finishing kernel) holds

// Where bin i of a sample histogram lives in LDS when NTH threads scan it: each thread sums SBINS / NTH consecutive
// bins, so consecutive threads would read addresses a power of two apart -- the same bank in every lane.  One unused
// word after each thread's bins makes the stride odd.  The histogram takes SBINS + NTH words.
template <int NTH>
__device__ __forceinline__ int sample_slot(uint32_t bin) { return (int)(bin + bin / (SBINS / NTH)); }
template <int NTH>
constexpr int sample_words() { return SBINS + NTH; }

// Inclusive prefix sum over the 64 lanes of a wave, by data-parallel-primitive moves inside the vector ALU (seven
// adds; the same through ds_bpermute is six dependent trips through the LDS crossbar): sums of 4 neighbours inside
// each row of 16 lanes (row_shr 1, 2, 3), of 8 and 16 (row_shr 4 and 8 on the banks that have such neighbours), then
// lane 15 of a row added to the next row (row_bcast 15, rows 1 and 3) and lane 31 to the upper half (row_bcast 31).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int /*lane*/) {
  const int x = (int)v;
  int r = x + __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);
  r += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);
  r += __builtin_amdgcn_update_dpp(0, x, 0x113, 0xf, 0xf, true);
  r += __builtin_amdgcn_update_dpp(0, r, 0x114, 0xf, 0xe, true);
  r += __builtin_amdgcn_update_dpp(0, r, 0x118, 0xf, 0xc, true);
  r += __builtin_amdgcn_update_dpp(0, r, 0x142, 0xa, 0xf, false);
  r += __builtin_amdgcn_update_dpp(0, r, 0x143, 0xc, 0xf, false);
  return (uint32_t)r;
}

// inclusive scan over the NTH threads of the workgroup in thread order; *total gets the sum
template <int NTH>
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_scan(v, lane);
  __syncthreads();                         // wave_tot may still be read from a previous call
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t off = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NTH / 64; ++i) {
    const uint32_t x = wave_tot[i];
    if (i < wave) off += x;
    tot += x;
  }
  *total = tot;
  return inc + off;
}

// Two bins of a sample histogram shist (laid out by sample_slot<NTH>; ns samples of a row of vis scores), from the
// count of samples from the top down:
//   lo: down to which a pass must collect so that it very probably gets the k largest scores and not many more --
//       where the count reaches the expected number of samples above the k-th largest score plus a margin of about
//       4 sigma;
//   hi: where it reaches that number minus the margin -- the scores above this bin are very probably fewer than k.
// 0xffffffff: no such bin.  sel[0..1] (LDS) must hold 0xffffffff on entry, set before the barrier that completes the
// histogram; wave_tot: NTH / 64 words of LDS.  Ends with a barrier.
template <int NTH>
__device__ __forceinline__ void sample_bins(const uint32_t* shist, uint32_t* wave_tot, uint32_t* sel, int k, int ns,
                                            int vis, uint32_t* lo_bin, uint32_t* hi_bin) {
  const int tid = threadIdx.x;
  const float expct = (float)k * (float)ns / (float)vis;
  const float margin = 4.0f * sqrtf(expct) + 8.0f;
  const uint32_t target[2] = {(uint32_t)(expct + margin), expct - margin >= 1.0f ? (uint32_t)(expct - margin) : 0u};
  constexpr int BPT = SBINS / NTH;         // bins per thread, descending
  const int top_bin = SBINS - 1 - tid * BPT;
  const int top_slot = sample_slot<NTH>(top_bin);               // the thread's bins are consecutive words
  uint32_t mine = 0, bin[BPT];              // (kept in registers: the search below is a chain of dependent steps)
#pragma unroll
  for (int r = 0; r < BPT; ++r) { bin[r] = shist[top_slot - r]; mine += bin[r]; }
  uint32_t total;
  const uint32_t inc = block_incl_scan<NTH>(mine, wave_tot, &total);
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    uint32_t above = inc - mine;
    if (target[w] > 0 && above < target[w] && inc >= target[w]) {    // the crossing bin is one of mine
      int at = -1;
#pragma unroll
      for (int r = 0; r < BPT; ++r) {                                // the first r at which the count reaches the target
        above += bin[r];
        if (at < 0 && above >= target[w]) at = r;
      }
      sel[w] = (uint32_t)(top_bin - at);
    }
  }
  __syncthreads();
  *lo_bin = sel[0];
  *hi_bin = sel[1];
  __syncthreads();
}

}  // namespace ess_sel
