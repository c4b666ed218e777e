// Device code shared by the kernels that compute indexer scores (ESS paper Sec. 3):
//
//   score[b,t,s] = sum_j w[b,t,j] * max(0, sum_d q[b,t,j,d] * key[b,s,d])
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
#pragma once
#include "ess_internal.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx8 __attribute__((ext_vector_type(8)));

namespace ess_idx {

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

// The stationary operands of T query tokens of one sequence: q as the A matrix (row = head), w per accumulator row.
template <int HB, int DI, int T>
struct QueryRegs {
  long qa[T][HB][DI / 32];
  float wr[T][HB][4];
};

// q, w: first of the T tokens' rows ([Hi][DI] bytes and [Hi] floats each, the tokens back to back)
template <int HB, int DI, int T>
__device__ __forceinline__ void load_query(QueryRegs<HB, DI, T>& r, const uint8_t* __restrict__ q, const float* __restrict__ w,
                                           int Hi, int g, int n) {
  constexpr int KS = DI / 32;
#pragma unroll
  for (int t = 0; t < T; ++t) {
#pragma unroll
    for (int mb = 0; mb < HB; ++mb) {
      const int head = mb * 16 + n;
      if (head < Hi) {
        load_row_share<DI>(q + ((size_t)t * Hi + head) * DI, g, r.qa[t][mb]);
      } else {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) r.qa[t][mb][kk] = 0;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int hrow = mb * 16 + g * 4 + i;
        r.wr[t][mb][i] = hrow < Hi ? w[(size_t)t * Hi + hrow] : 0.f;
      }
    }
  }
}

// max(x, 0) in one instruction: as signed integers, the bit patterns of the floats below zero (and of -0) are
// negative and those of the others are themselves, so an integer max with 0 is the ReLU.  Written as fmaxf it costs
// two (the compiler first quiets a possible signalling NaN with a v_max of the value with itself).  A NaN, which
// only q or key bytes that encode one can produce, passes with its sign bit clear and becomes 0 with it set.
__device__ __forceinline__ float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

// Scores of one tile of 16 keys for token t: every lane (g,n) returns the score of key n.
template <int HB, int DI, int T>
__device__ __forceinline__ float tile_score(const QueryRegs<HB, DI, T>& r, int t, const KeyRegs<DI / 32>& key) {
  constexpr int KS = DI / 32;
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
    const intx8 kv = __builtin_bit_cast(intx8, key);
#pragma unroll
    for (int mb = 0; mb < HB; ++mb) {
      KeyRegs<4> ql;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) ql.v[kk] = r.qa[t][mb][kk];
      acc[mb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(__builtin_bit_cast(intx8, ql), kv, acc[mb], 0, 0, 0, 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
#pragma unroll
      for (int mb = 0; mb < HB; ++mb)
        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(r.qa[t][mb][kk], key.v[kk], acc[mb], 0, 0, 0);
  }
#pragma unroll
  for (int mb = 0; mb < HB; ++mb)
#pragma unroll
    for (int i = 0; i < 4; ++i) s = fmaf(r.wr[t][mb][i], relu(acc[mb][i]), s);
  s += __shfl_xor(s, 16, 64);
  s += __shfl_xor(s, 32, 64);
  return s;
}

// All scores of one row (b,t), positions [0, vis), by the calling workgroup (any number of whole waves), one block
// of 64 keys per wave at a time: slow, for the rare row whose candidate list could not be used.  The head blocks
// beyond Hi are zero, which leaves the sums as the kernels specialised on the number of head blocks form them.
// table_row: the sequence's row of the block table (paged Indexer-Cache) or null (key = the sequence's keys).
template <int DI>
__device__ __forceinline__ void row_scores_slow(const uint8_t* __restrict__ q_row, const float* __restrict__ w_row, int Hi,
                                                const uint8_t* __restrict__ key, int Lmax,
                                                const int32_t* __restrict__ table_row, int n_pages, int vis,
                                                float* __restrict__ out) {
  constexpr int KS = DI / 32;
  constexpr size_t kPageBytes = (size_t)kBatchTokens * (DI + 4);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int g = lane >> 4, n = lane & 15;
  QueryRegs<4, DI, 1> qr;
  load_query<4, DI, 1>(qr, q_row, w_row, Hi, g, n);
  for (int base = wave * kBatchTokens; base < vis; base += nw * kBatchTokens) {
    KeyRegs<KS> kr[kTilesPerBatch];
    float sc = 1.f;
    if (table_row) {
      const int pid = min(max(table_row[base / kBatchTokens], 0), n_pages - 1);
      const uint8_t* page = key + (size_t)pid * kPageBytes;
#pragma unroll
      for (int u = 0; u < kTilesPerBatch; ++u) load_row_share<DI>(page + (size_t)(u * 16 + n) * DI, g, kr[u].v);
      sc = *reinterpret_cast<const float*>(page + (size_t)kBatchTokens * DI + lane * 4);
    } else {
#pragma unroll
      for (int u = 0; u < kTilesPerBatch; ++u)
        load_row_share<DI>(key + (size_t)min(base + u * 16 + n, Lmax - 1) * DI, g, kr[u].v);
    }
    float res = 0.f;
#pragma unroll
    for (int u = 0; u < kTilesPerBatch; ++u) {
      const float s = tile_score<4, DI, 1>(qr, 0, kr[u]);
      res = (g == u) ? s : res;
    }
    const int tok = base + lane;
    if (tok < vis) out[tok] = table_row ? res * sc : res;
  }
}

}  // namespace ess_idx

// Where the sample of a sequence's keys lies, from which the selection's lower bound is taken before the main
// pass: one block of 64 consecutive keys out of every `period` (2048 keys, more for contexts beyond 256K so that
// a sequence has at most ESS_SAMPLE_BLOCKS of them), at an offset inside its period that changes from period to
// period.  A block counts when it lies wholly inside what every query token of the sequence sees.
#define ESS_SAMPLE_BLOCKS 128
__host__ __device__ inline int ess_sample_period(int max_ctx) {
  const int chunks = (max_ctx + 2047) / 2048;
  return 2048 * ((chunks + ESS_SAMPLE_BLOCKS - 1) / ESS_SAMPLE_BLOCKS);
}
__host__ __device__ inline int ess_sample_count(int max_ctx) {           // blocks a sequence of max_ctx keys has
  const int p = ess_sample_period(max_ctx);
  return (max_ctx + p - 1) / p;
}
__host__ __device__ inline int ess_sample_start(int s, int period) {
  return s * period + 64 * (int)(((unsigned)s * 11u + 5u) % (unsigned)(period / 64));
}

#ifdef __HIPCC__
// float -> unsigned key with the same order; NaN ranks as -inf, -0 as +0
__device__ __forceinline__ uint32_t ess_orderable(float v) {
  if (v != v) v = -__builtin_inff();
  v += 0.0f;
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
#endif
