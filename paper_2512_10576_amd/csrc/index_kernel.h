// Stage 1: indexer score over the whole Indexer-Cache (ESS paper Sec. 3).
//
//   score[b,t,s] = sum_j w[b,t,j] * max(0, sum_d q[b,t,j,d] * key[b,s,d])
//
// The kernel is a key stream: every 128-byte key is read from HBM exactly
// once (for all T query tokens), the q.k contraction runs on the fp8 matrix
// cores (v_mfma_f32_16x16x128_f8f6f4 for 128-dimensional keys, else
// v_mfma_f32_16x16x32_fp8_fp8; heads = M, tokens = N, dim = K) and the
// ReLU / head-weighted reduction stays in registers (see index_tile.h).
//
// Two forms of the one kernel body:
//   * dense (EMIT false): every score is written to score[b,t,s];
//   * emit (EMIT true): no score is written; positions whose score reaches the row's lower bound tau[b,t]
//     (derived from a sample of the sequence's keys by the pass in front, index_sample.hip) are collected in LDS
//     as composite selection keys and appended, once per workgroup, to the row's candidate list, from which the
//     top-k is finished.  The score stream (4 bytes per key and query token, and the pass of the top-k that would
//     read it back) does not exist in this form.
//
// This header is compiled into two translation units (EMIT false / true), which halves the build time.
#pragma once
#include "index_tile.h"
#include <hip/hip_ext.h>

namespace ess_idx {

constexpr int kWaves = 4;                 // waves per workgroup
constexpr int kMaxChunk = 2048;           // keys per work item at most

struct IdxArgs {
  const uint8_t* q; const float* w; const uint8_t* key; const int32_t* ctx_len;
  float* score;                             // dense: [B,Ttot,Lmax]; emit: unused
  int Lmax, Hi, chunk;
  const int32_t* block_table; int n_pages;
  int Ttot, t0;                             // tokens per sequence in q / w / score, first token of this launch
  ess_xcd xcd; int nx, nb_seq;              // work distribution; work items per sequence, sequences
  // emit form
  const uint32_t* tau;                      // [B,Ttot][2] bounds (ess_orderable images of scores); [0], the lower one, is used
  unsigned long long* cand;                 // [B,Ttot][cand_cap] candidate keys
  uint32_t* cnt;                            // [B,Ttot] candidates appended (may exceed cand_cap: the list is then unusable)
  int cand_cap, IB;                         // IB = bits of a position in a composite key
};

// HB = 16-head blocks (Hi padded up), DI = indexer dim, T = query tokens per sequence handled by this
// launch (1 or 2): tokens t0 .. t0+T-1 of the Ttot the sequence has.  More than two tokens per
// sequence take further launches, which read the keys again.
// PAGED: `key` is a pool of pages (64 keys of DI bytes, then 64 float scales); token s of sequence b is
// row s % 64 of page block_table[b, s / 64] and its score is multiplied by its scale (positive, so the
// scale commutes with the ReLU and the head sum: one multiplication of the exact sum).  A wave's batch
// of 64 tokens is exactly one page.
// Two waves per SIMD are asked for (all forms fit 256 registers), which also makes the compiler give the MFMAs
// vector-register results: with one wave allowed it puts them in accumulation registers and copies every one back
// before the ReLU (64 v_accvgpr_read per batch of 64 keys).  The looping single-token form is left as it was: beside
// a fetch, on six XCDs, it measured 2 % slower in the other form.
template <int HB, int DI, int T, bool PAGED, bool DYN, bool EMIT>
__global__ __launch_bounds__(kWaves * 64, (T == 2 || !DYN) ? 2 : 1) void k_index_score(const IdxArgs a) {
  constexpr int KS = DI / 32;
  constexpr size_t kPageBytes = (size_t)kBatchTokens * (DI + 4);
  __shared__ int s_item;
  __shared__ unsigned long long s_cand[EMIT ? T : 1][EMIT ? kMaxChunk : 1];
  __shared__ uint32_t s_n[2], s_base[2];
  const uint8_t* __restrict__ key = a.key;
  float* __restrict__ score = a.score;
  const int Lmax = a.Lmax, Ttot = a.Ttot, t0 = a.t0;
  // work item = (chunk, sequence): by workgroup index, or drawn from the launch's counter off the XCDs to be avoided
  ESS_WORK_LOOP(DYN, a.xcd, blockIdx.y * a.nx + blockIdx.x, a.nx * a.nb_seq, &s_item, item) {
  const int b = item / a.nx;
  const int len = min(a.ctx_len[b], Lmax);

  // the thread index passes through an empty asm statement so that what is derived from it is computed per work
  // item instead of being carried in registers across the loop
  int tidx = threadIdx.x;
  if constexpr (DYN) asm volatile("" : "+v"(tidx));
  const int lane = tidx & 63;
  const int wave = tidx >> 6;
  const int g = lane >> 4;
  const int n = lane & 15;

  // this wave's keys: batches of 64 at base0, base0 + kStride, ... below blk_end
  constexpr int kStride = kWaves * kBatchTokens;
  const int blk_base = (item % a.nx) * a.chunk;
  if (blk_base >= len) continue;
  const int blk_end = min(blk_base + a.chunk, len);
  const int base0 = blk_base + wave * kBatchTokens;
  const int nb = base0 < blk_end ? (blk_end - base0 + kStride - 1) / kStride : 0;

  uint32_t tau[T];
  unsigned long long imask = 0;
  if constexpr (EMIT) {
#pragma unroll
    for (int t = 0; t < T; ++t) tau[t] = a.tau[2 * ((size_t)b * Ttot + t0 + t)];
    imask = (1ull << a.IB) - 1ull;
    if (tidx < 2) s_n[tidx] = 0;
    __syncthreads();
  }

  if (nb > 0) {
  QueryRegs<HB, DI, T> qr;                // 8 KiB per sequence and token, read from the L2 by every workgroup of the sequence
  load_query<HB, DI, T>(qr, a.q + (size_t)(b * Ttot + t0) * a.Hi * DI, a.w + (size_t)(b * Ttot + t0) * a.Hi, a.Hi, g, n);

  const uint8_t* kbase = key + (size_t)b * Lmax * DI;
  const int last_row = Lmax - 1;

  // paged: lane j holds the page of this wave's j-th batch (a workgroup covers at most 2048 tokens:
  // 8 batches per wave), read once, handed out with readlane
  int pidv = 0;
  if constexpr (PAGED) {
    if (lane < nb) {
      const int pid = a.block_table[(size_t)b * (Lmax / kBatchTokens) + base0 / kBatchTokens + lane * kWaves];
      pidv = min(max(pid, 0), a.n_pages - 1);                 // a bad table entry must not leave the pool
    }
  }

  struct Batch {
    KeyRegs<KS> k[kTilesPerBatch];
    float sc;                                                 // PAGED: scale of token base + lane
  };

  auto load_batch = [&](int j, Batch& dst) {
    const int base = base0 + j * kStride;
    if constexpr (PAGED) {
      const uint8_t* page = key + (size_t)__builtin_amdgcn_readlane(pidv, j) * kPageBytes;
#pragma unroll
      for (int u = 0; u < kTilesPerBatch; ++u) load_row_share<DI>(page + (size_t)(u * 16 + n) * DI, g, dst.k[u].v);
      dst.sc = *reinterpret_cast<const float*>(page + (size_t)kBatchTokens * DI + lane * 4);
    } else {
#pragma unroll
      for (int u = 0; u < kTilesPerBatch; ++u) {
        const int row = min(base + u * 16 + n, last_row);     // clamp keeps ragged tails in bounds
        load_row_share<DI>(kbase + (size_t)row * DI, g, dst.k[u].v);
      }
    }
  };

  auto compute_batch = [&](int j, const Batch& kr) {
    const int base = base0 + j * kStride;
    float res[T];
#pragma unroll
    for (int t = 0; t < T; ++t) res[t] = 0.f;
#pragma unroll
    for (int u = 0; u < kTilesPerBatch; ++u) {
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const float s = tile_score<HB, DI, T>(qr, t, kr.k[u]);
        res[t] = (g == u) ? s : res[t];                       // lane (g,n) keeps tile g's token n
      }
    }
    const int tok = base + lane;                              // = base + 16*g + n
    if constexpr (EMIT) {
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const uint32_t ok = ess_orderable(PAGED ? res[t] * kr.sc : res[t]);
        const bool take = tok < blk_end && tok < len - (Ttot - 1 - (t0 + t)) && ok >= tau[t];
        // one LDS atomic per wave, batch and token row; a work item holds at most kMaxChunk keys: the list cannot overflow
        const unsigned long long mask = __ballot(take);
        if (mask) {
          const int leader = __ffsll((long long)mask) - 1;
          uint32_t at = 0;
          if (lane == leader) at = atomicAdd(&s_n[t], (uint32_t)__popcll(mask));
          at = __shfl(at, leader, 64) + __popcll(mask & ((1ull << lane) - 1ull));
          if (take) s_cand[t][at] = ((unsigned long long)ok << a.IB) | (imask - (unsigned long long)tok);
        }
      }
    } else {
      if (tok < blk_end) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
          __builtin_nontemporal_store(PAGED ? res[t] * kr.sc : res[t], &score[(size_t)(b * Ttot + t0 + t) * Lmax + tok]);
        }
      }
    }
  };

  // Three register buffers: the loads of batches i+1 and i+2 are in flight while batch i is
  // computed (16 KiB per wave for Di = 128).  Inside the loop every prefetch is unconditional, so the
  // number of loads in flight is the same on every path (a prefetch under a branch makes the compiler
  // wait for the newest loads before it uses the oldest); the last batches are peeled off.
  Batch bufA, bufB, bufC;
#define ESS_LOAD(buf, j) load_batch((j), buf)
#define ESS_COMP(buf, j) compute_batch((j), buf)
  ESS_LOAD(bufA, 0);
  ESS_LOAD(bufB, min(1, nb - 1));            // invariant: A holds batch i, B batch i+1 (clamped)
  int i = 0;
  for (; i + 4 < nb; i += 3) {
    ESS_LOAD(bufC, i + 2); ESS_COMP(bufA, i);
    ESS_LOAD(bufA, i + 3); ESS_COMP(bufB, i + 1);
    ESS_LOAD(bufB, i + 4); ESS_COMP(bufC, i + 2);
  }
  const int r = nb - i;                      // 1..4 batches left
  if (r == 1) {
    ESS_COMP(bufA, i);
  } else if (r == 2) {
    ESS_COMP(bufA, i); ESS_COMP(bufB, i + 1);
  } else if (r == 3) {
    ESS_LOAD(bufC, i + 2); ESS_COMP(bufA, i); ESS_COMP(bufB, i + 1); ESS_COMP(bufC, i + 2);
  } else {
    ESS_LOAD(bufC, i + 2); ESS_COMP(bufA, i);
    ESS_LOAD(bufA, i + 3); ESS_COMP(bufB, i + 1);
    ESS_COMP(bufC, i + 2); ESS_COMP(bufA, i + 3);
  }
#undef ESS_LOAD
#undef ESS_COMP
  }

  if constexpr (EMIT) {
    // the item's candidates leave as one piece per token row: one device-wide atomic per workgroup and row
    __syncthreads();
    if (tidx < T && s_n[tidx]) s_base[tidx] = atomicAdd(&a.cnt[(size_t)b * Ttot + t0 + tidx], s_n[tidx]);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const uint32_t cn = s_n[t], at = s_base[t];
      unsigned long long* list = a.cand + ((size_t)b * Ttot + t0 + t) * a.cand_cap;
      for (uint32_t j = tidx; j < cn; j += kWaves * 64)
        if (at + j < (uint32_t)a.cand_cap) list[at + j] = s_cand[t][j];
    }
  }
  }
}

template <int HB, int DI, int T, bool PAGED, bool DYN, bool EMIT>
void launch_d(dim3 grid, hipStream_t st, const IdxArgs& a0, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const dim3 block(kWaves * 64);
  IdxArgs a = a0;
  if constexpr (DYN) {
    // ticket-fed: as many workgroups as the working XCDs hold at once; each draws items until none is left
    static int per_cu = 0;
    if (per_cu == 0) {
      int n = 0;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_index_score<HB, DI, T, PAGED, true, EMIT>, kWaves * 64, 0) != hipSuccess || n < 1) n = 1;
      per_cu = n;
    }
    grid = dim3(ess_xcd_grid(a.nx * a.nb_seq, a.xcd, per_cu));
  }
  if (ev_start || ev_stop)          // timed launch: the events take the kernel's own start and end
    hipExtLaunchKernelGGL((k_index_score<HB, DI, T, PAGED, DYN, EMIT>), grid, block, 0, st, ev_start, ev_stop, 0, a);
  else
    hipLaunchKernelGGL((k_index_score<HB, DI, T, PAGED, DYN, EMIT>), grid, block, 0, st, a);
}

template <int HB, int DI, int T, bool PAGED, bool EMIT>
void launch_k(dim3 grid, hipStream_t st, const IdxArgs& a, hipEvent_t e0, hipEvent_t e1) {
  if (a.xcd.ticket) launch_d<HB, DI, T, PAGED, true, EMIT>(grid, st, a, e0, e1);
  else launch_d<HB, DI, T, PAGED, false, EMIT>(grid, st, a, e0, e1);
}

template <int HB, int DI, int T, bool EMIT>
void launch_p(dim3 grid, hipStream_t st, const IdxArgs& a, hipEvent_t e0, hipEvent_t e1) {
  if (a.block_table) launch_k<HB, DI, T, true, EMIT>(grid, st, a, e0, e1);
  else launch_k<HB, DI, T, false, EMIT>(grid, st, a, e0, e1);
}

template <int HB, int DI, bool EMIT>
void launch_t(int T, dim3 grid, hipStream_t st, const IdxArgs& a, hipEvent_t e0, hipEvent_t e1) {
  if (T == 1) launch_p<HB, DI, 1, EMIT>(grid, st, a, e0, e1);
  else launch_p<HB, DI, 2, EMIT>(grid, st, a, e0, e1);
}

template <int DI, bool EMIT>
void launch_hb(int HB, int T, dim3 grid, hipStream_t st, const IdxArgs& a, hipEvent_t e0, hipEvent_t e1) {
  switch (HB) {
    case 1: launch_t<1, DI, EMIT>(T, grid, st, a, e0, e1); break;
    case 2: launch_t<2, DI, EMIT>(T, grid, st, a, e0, e1); break;
    case 3: launch_t<3, DI, EMIT>(T, grid, st, a, e0, e1); break;
    default: launch_t<4, DI, EMIT>(T, grid, st, a, e0, e1); break;
  }
}

// One launch per pair of query tokens; the events of a timed call bracket the whole series.  `a` describes the
// work of one launch except Ttot / t0, which are set here.
template <bool EMIT>
int launch_series(const ess_config& c, int T, dim3 grid, hipStream_t st, IdxArgs a, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const int HB = (c.idx_heads + 15) / 16;
  if (a.xcd.ticket && T > 2) return ess_fail(ESS_ERR_UNSUPPORTED, "internal: one ticket serves one index-score launch");
  a.Ttot = T;
  for (int t0 = 0; t0 < T; t0 += 2) {
    const int Tl = T - t0 < 2 ? T - t0 : 2;
    a.t0 = t0;
    hipEvent_t e0 = t0 == 0 ? ev_start : nullptr, e1 = t0 + 2 >= T ? ev_stop : nullptr;
    switch (c.idx_dim) {
      case 32: launch_hb<32, EMIT>(HB, Tl, grid, st, a, e0, e1); break;
      case 64: launch_hb<64, EMIT>(HB, Tl, grid, st, a, e0, e1); break;
      case 128: launch_hb<128, EMIT>(HB, Tl, grid, st, a, e0, e1); break;
      default: return ess_fail(ESS_ERR_UNSUPPORTED, "idx_dim %d (supported: 32, 64, 128)", c.idx_dim);
    }
  }
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

// tokens per workgroup: a multiple of the 256 tokens the four waves cover per round; 2048 when
// that still leaves several workgroups per CU, else 1024
inline int pick_chunk(int B, int Lmax) { return ((long)B * Lmax >= 2048L * 1024) ? 2048 : 1024; }

}  // namespace ess_idx
