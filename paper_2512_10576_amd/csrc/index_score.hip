// Stage 1: indexer score over the whole Indexer-Cache (ESS paper Sec. 3).
//
//   score[b,t,s] = sum_j w[b,t,j] * max(0, sum_d q[b,t,j,d] * key[b,s,d])
//
// The kernel is a key stream: every 128-byte key is read from HBM exactly
// once (for all T query tokens), the q.k contraction runs on the fp8 matrix
// cores (v_mfma_f32_16x16x128_f8f6f4 for 128-dimensional keys, else
// v_mfma_f32_16x16x32_fp8_fp8; heads = M, tokens = N, dim = K) and the
// ReLU / head-weighted reduction stays in registers.
//
// Register layout.  A wave handles 16 tokens per MFMA tile.  Lane l = 16*g + n
// (g = 0..3, n = 0..15) owns token n of the tile and the g-th quarter of the
// contraction dimension.  Because a dot product does not depend on the order
// of its terms, the hardware's k index is mapped onto the key dimension so
// that each lane's share is contiguous in memory: for Di = 128 lane (g,n)
// loads bytes [16g,16g+16) and [64+16g,64+16g+16) of its key row with two
// 16-byte loads, which makes every load instruction of the wave touch 64
// contiguous bytes per row; q is loaded with the same mapping.  The
// accumulator of lane (g,n) holds heads 16*mb + 4g + i (i = 0..3) of token n,
// so the head reduction is 4*HB fused multiply-adds in the lane plus two
// cross-lane steps (xor 16, xor 32).
#include "ess_internal.h"
#include <hip/hip_ext.h>

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int kWaves = 4;                 // waves per workgroup
constexpr int kTilesPerBatch = 4;         // 4 tiles x 16 tokens = 64 scores = one coalesced 256-byte store per wave
constexpr int kBatchTokens = 16 * kTilesPerBatch;

template <int KS>
struct KeyRegs {                          // one tile's key bytes held by a lane: KS x 8 bytes
  long v[KS];
};

template <int DI>
__device__ __forceinline__ void load_row_share(const uint8_t* row, int g, long (&dst)[DI / 32]) {
  constexpr int KS = DI / 32;
  if constexpr (KS == 1) {
    dst[0] = *reinterpret_cast<const long*>(row + g * 8);
  } else {
#pragma unroll
    for (int c = 0; c < KS / 2; ++c) {
      const uint4 x = *reinterpret_cast<const uint4*>(row + c * 64 + g * 16);
      dst[2 * c] = (long)(((unsigned long)x.y << 32) | x.x);
      dst[2 * c + 1] = (long)(((unsigned long)x.w << 32) | x.z);
    }
  }
}

// HB = 16-head blocks (Hi padded up), DI = indexer dim, T = query tokens per sequence handled by this
// launch (1 or 2): tokens t0 .. t0+T-1 of the Ttot the sequence has.  More than two tokens per
// sequence take further launches, which read the keys again.
// PAGED: `key` is a pool of pages (64 keys of DI bytes, then 64 float scales); token s of sequence b is
// row s % 64 of page block_table[b, s / 64] and its score is multiplied by its scale (positive, so the
// scale commutes with the ReLU and the head sum: one multiplication of the exact sum).  A wave's batch
// of 64 tokens is exactly one page.
template <int HB, int DI, int T, bool PAGED, bool DYN>
__global__ __launch_bounds__(kWaves * 64, T == 2 ? 2 : 1) void k_index_score(const uint8_t* __restrict__ q,
                                                              const float* __restrict__ w,
                                                              const uint8_t* __restrict__ key,
                                                              const int32_t* __restrict__ ctx_len,
                                                              float* __restrict__ score, int Lmax, int Hi,
                                                              int chunk_tokens,
                                                              const int32_t* __restrict__ block_table, int n_pages,
                                                              int Ttot, int t0, ess_xcd xcd, int nx, int nb_seq) {
  constexpr int KS = DI / 32;
  constexpr size_t kPageBytes = (size_t)kBatchTokens * (DI + 4);
  __shared__ int s_item;
  // work item = (chunk, sequence): by workgroup index, or drawn from the launch's counter off the XCDs to be avoided
  ESS_WORK_LOOP(DYN, xcd, blockIdx.y * nx + blockIdx.x, nx * nb_seq, &s_item, item) {
  const int b = item / nx;
  const int len = min(ctx_len[b], Lmax);
  const int blk_base = (item % nx) * chunk_tokens;
  if (blk_base >= len) continue;
  const int blk_end = min(blk_base + chunk_tokens, len);

  // the thread index passes through an empty asm statement so that what is derived from it is computed per work
  // item instead of being carried in registers across the loop
  int tidx = threadIdx.x;
  if constexpr (DYN) asm volatile("" : "+v"(tidx));
  const int lane = tidx & 63;
  const int wave = tidx >> 6;
  const int g = lane >> 4;
  const int n = lane & 15;

  // stationary operands of the item: q as the A matrix (row = head), w per accumulator row (8 KiB per sequence
  // and token, read from the L2 by every workgroup that works on the sequence)
  long qa[T][HB][KS];
  float wr[T][HB][4];
#pragma unroll
  for (int t = 0; t < T; ++t) {
#pragma unroll
    for (int mb = 0; mb < HB; ++mb) {
      const int head = mb * 16 + n;
      if (head < Hi) {
        load_row_share<DI>(q + ((size_t)(b * Ttot + t0 + t) * Hi + head) * DI, g, qa[t][mb]);
      } else {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) qa[t][mb][kk] = 0;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int hrow = mb * 16 + g * 4 + i;
        wr[t][mb][i] = hrow < Hi ? w[(size_t)(b * Ttot + t0 + t) * Hi + hrow] : 0.f;
      }
    }
  }

  const uint8_t* kbase = key + (size_t)b * Lmax * DI;
  const int last_row = Lmax - 1;
  constexpr int kStride = kWaves * kBatchTokens;
  const int base0 = blk_base + wave * kBatchTokens;
  if (base0 >= blk_end) continue;
  const int nb = (blk_end - base0 + kStride - 1) / kStride;

  // paged: lane j holds the page of this wave's j-th batch (a workgroup covers at most 2048 tokens:
  // 8 batches per wave), read once, handed out with readlane
  int pidv = 0;
  if constexpr (PAGED) {
    if (lane < nb) {
      const int pid = block_table[(size_t)b * (Lmax / kBatchTokens) + base0 / kBatchTokens + lane * kWaves];
      pidv = min(max(pid, 0), n_pages - 1);                   // a bad table entry must not leave the pool
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
        // the HB head blocks are independent accumulation chains: stepping through them inside the
        // contraction loop keeps dependent MFMAs HB instructions apart (head block outermost, the
        // compiler issued each chain back to back and every MFMA waited for the one before)
        float s = 0.f;
        floatx4 acc[HB];
#pragma unroll
        for (int mb = 0; mb < HB; ++mb) acc[mb] = floatx4{0.f, 0.f, 0.f, 0.f};
        if constexpr (KS == 4) {
          // 128-dimensional keys: one v_mfma_f32_16x16x128_f8f6f4 per head block (both formats e4m3, no
          // block scales) in place of four 16x16x32 fp8 MFMAs -- a quarter of the instructions and, on
          // gfx950, twice the rate.  A lane's 32 key bytes pair with its 32 query bytes as before.
          const intx8 kv = __builtin_bit_cast(intx8, kr.k[u]);
#pragma unroll
          for (int mb = 0; mb < HB; ++mb) {
            KeyRegs<4> ql;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) ql.v[kk] = qa[t][mb][kk];
            acc[mb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(__builtin_bit_cast(intx8, ql), kv, acc[mb], 0, 0, 0, 0, 0, 0);
          }
        } else {
#pragma unroll
          for (int kk = 0; kk < KS; ++kk)
#pragma unroll
            for (int mb = 0; mb < HB; ++mb)
              acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(qa[t][mb][kk], kr.k[u].v[kk], acc[mb], 0, 0, 0);
        }
#pragma unroll
        for (int mb = 0; mb < HB; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i) s = fmaf(wr[t][mb][i], fmaxf(acc[mb][i], 0.f), s);
        s += __shfl_xor(s, 16, 64);
        s += __shfl_xor(s, 32, 64);
        res[t] = (g == u) ? s : res[t];                       // lane (g,n) keeps tile g's token n
      }
    }
    const int tok = base + lane;                              // = base + 16*g + n
    if (tok < blk_end) {
#pragma unroll
      for (int t = 0; t < T; ++t) score[(size_t)(b * Ttot + t0 + t) * Lmax + tok] = PAGED ? res[t] * kr.sc : res[t];
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
}

struct IdxArgs {
  const uint8_t* q; const float* w; const uint8_t* key; const int32_t* ctx_len; float* score;
  int Lmax, Hi, chunk;
  const int32_t* block_table; int n_pages;
  hipEvent_t ev_start, ev_stop;             // optional: take the kernel's own start and end times
  int Ttot, t0;                             // tokens per sequence in q / w / score, first token of this launch
  ess_xcd xcd; int nx, nb_seq;              // work distribution; chunks per sequence, sequences
};

template <int HB, int DI, int T, bool PAGED, bool DYN>
void launch_d(dim3 grid, hipStream_t st, const IdxArgs& a) {
  const dim3 block(kWaves * 64);
  if constexpr (DYN) {
    // ticket-fed: as many workgroups as the working XCDs hold at once; each draws items until none is left
    static int per_cu = 0;
    if (per_cu == 0) {
      int n = 0;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_index_score<HB, DI, T, PAGED, true>, kWaves * 64, 0) != hipSuccess || n < 1) n = 1;
      per_cu = n;
    }
    grid = dim3(ess_xcd_grid(a.nx * a.nb_seq, a.xcd, per_cu));
  }
  if (a.ev_start || a.ev_stop)      // timed launch: the events take the kernel's own start and end
    hipExtLaunchKernelGGL((k_index_score<HB, DI, T, PAGED, DYN>), grid, block, 0, st, a.ev_start, a.ev_stop, 0, a.q, a.w, a.key,
                          a.ctx_len, a.score, a.Lmax, a.Hi, a.chunk, a.block_table, a.n_pages, a.Ttot, a.t0, a.xcd, a.nx, a.nb_seq);
  else
    hipLaunchKernelGGL((k_index_score<HB, DI, T, PAGED, DYN>), grid, block, 0, st, a.q, a.w, a.key, a.ctx_len, a.score, a.Lmax,
                       a.Hi, a.chunk, a.block_table, a.n_pages, a.Ttot, a.t0, a.xcd, a.nx, a.nb_seq);
}

template <int HB, int DI, int T, bool PAGED>
void launch_k(dim3 grid, hipStream_t st, const IdxArgs& a) {
  if (a.xcd.ticket) launch_d<HB, DI, T, PAGED, true>(grid, st, a);
  else launch_d<HB, DI, T, PAGED, false>(grid, st, a);
}

template <int HB, int DI, int T>
void launch_p(dim3 grid, hipStream_t st, const IdxArgs& a) {
  if (a.block_table) launch_k<HB, DI, T, true>(grid, st, a);
  else launch_k<HB, DI, T, false>(grid, st, a);
}

template <int HB, int DI>
void launch_t(int T, dim3 grid, hipStream_t st, const IdxArgs& a) {
  if (T == 1) launch_p<HB, DI, 1>(grid, st, a);
  else launch_p<HB, DI, 2>(grid, st, a);
}

template <int DI>
void launch_hb(int HB, int T, dim3 grid, hipStream_t st, const IdxArgs& a) {
  switch (HB) {
    case 1: launch_t<1, DI>(T, grid, st, a); break;
    case 2: launch_t<2, DI>(T, grid, st, a); break;
    case 3: launch_t<3, DI>(T, grid, st, a); break;
    default: launch_t<4, DI>(T, grid, st, a); break;
  }
}

}  // namespace

int ess_launch_index_score(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                           const int32_t* ctx_len, int B, int T, float* score, hipStream_t st,
                           const int32_t* block_table, int n_pages, hipEvent_t ev_start, hipEvent_t ev_stop, ess_xcd xcd) {
  const int Hi = c.idx_heads, Di = c.idx_dim, Lmax = c.max_ctx;
  const int HB = (Hi + 15) / 16;
  // tokens per workgroup: a multiple of the 256 tokens the four waves cover per round; 2048 when
  // that still leaves several workgroups per CU, else 1024
  const int chunk = ((long)B * Lmax >= 2048L * 1024) ? 2048 : 1024;
  const int nx = (Lmax + chunk - 1) / chunk;
  if (xcd.ticket && T > 2) return ess_fail(ESS_ERR_UNSUPPORTED, "internal: one ticket serves one index-score launch");
  const dim3 grid(nx, B);
  // two query tokens per launch; the events of a timed call bracket the whole series
  for (int t0 = 0; t0 < T; t0 += 2) {
    const int Tl = T - t0 < 2 ? T - t0 : 2;
    const IdxArgs a{q, w, key, ctx_len, score, Lmax, Hi, chunk, block_table, n_pages,
                    t0 == 0 ? ev_start : nullptr, t0 + 2 >= T ? ev_stop : nullptr, T, t0, xcd, nx, B};
    switch (Di) {
      case 32: launch_hb<32>(HB, Tl, grid, st, a); break;
      case 64: launch_hb<64>(HB, Tl, grid, st, a); break;
      case 128: launch_hb<128>(HB, Tl, grid, st, a); break;
      default: return ess_fail(ESS_ERR_UNSUPPORTED, "idx_dim %d (supported: 32, 64, 128)", Di);
    }
  }
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
