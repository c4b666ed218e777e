// The pass in front of the emitting index-score pass (fused selection, see index_kernel.h): the scores of every
// sequence's sample blocks (ess_sample_start: 64 consecutive keys out of every 2048),
//   sample[b,t,64 s + i] = score of key ess_sample_start(s) + i   for the blocks s that count,
// from which k_index_tau (topk.hip) takes the rows' lower bounds.  A thirty-second of the main pass's arithmetic and
// a latency-bound kernel: it is spread over the chip, eight blocks per workgroup (two per wave, both requested at
// once), and does not run beside anything.
#include "index_tile.h"
#include "select_common.h"

using namespace ess_idx;

namespace {

constexpr int kSWaves = 4;
constexpr int kThreads = kSWaves * 64;
constexpr int G = 2;                        // blocks per wave
constexpr int kPartBlocks = kSWaves * G;

struct SampleArgs {
  const uint8_t* q; const float* w; const uint8_t* key; const int32_t* ctx_len;
  int Lmax, Hi;
  const int32_t* block_table; int n_pages;
  int Ttot, t0;                             // tokens per sequence in q / w / sample, first token of this launch
  ess_xcd xcd; int nparts, nb_seq;          // work items per sequence (groups of kPartBlocks sample blocks), sequences
  int period, nsamp;                        // ess_sample_period / ess_sample_count of the context
  float* sample;                            // [B,Ttot,64 * nsamp]
};

template <int HB, int DI, int T, bool PAGED, bool DYN>
__global__ __launch_bounds__(kThreads, 1) void k_index_sample(const SampleArgs a) {
  constexpr int KS = DI / 32;
  constexpr size_t kPageBytes = (size_t)kBatchTokens * (DI + 4);
  __shared__ int s_item;
  const int Lmax = a.Lmax, Ttot = a.Ttot, t0 = a.t0;
  ESS_WORK_LOOP(DYN, a.xcd, blockIdx.y * a.nparts + blockIdx.x, a.nparts * a.nb_seq, &s_item, item) {
    int tidx = threadIdx.x;
    if constexpr (DYN) asm volatile("" : "+v"(tidx));
    const int lane = tidx & 63, wave = tidx >> 6, g = lane >> 4, n = lane & 15;
    const int b = item / a.nparts;
    const int len = min(a.ctx_len[b], Lmax);
    const int lim = len - (Ttot - 1);                           // what every query token of the sequence sees
    // this wave's blocks: s0, s0 + kSWaves; those that count come first (starts grow with the block number)
    const int s0 = (item % a.nparts) * kPartBlocks + wave;
    int nbw = 0;
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int s = s0 + u * kSWaves;
      nbw += (s < a.nsamp && ess_sample_start(s, a.period) + kBatchTokens <= lim) ? 1 : 0;
    }
    if (nbw == 0) continue;
    QueryRegs<HB, DI, T> qr;
    load_query<HB, DI, T>(qr, a.q + (size_t)(b * Ttot + t0) * a.Hi * DI, a.w + (size_t)(b * Ttot + t0) * a.Hi, a.Hi, g, n);
    const uint8_t* kbase = a.key + (size_t)b * Lmax * DI;
    struct Batch {
      KeyRegs<KS> k[kTilesPerBatch];
      float sc;
    };
    Batch buf[G];
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int base = ess_sample_start(s0 + min(u, nbw - 1) * kSWaves, a.period);   // past the end: the last block again, not used
      if constexpr (PAGED) {
        const int pid = a.block_table[(size_t)b * (Lmax / kBatchTokens) + base / kBatchTokens];
        const uint8_t* page = a.key + (size_t)min(max(pid, 0), a.n_pages - 1) * kPageBytes;
#pragma unroll
        for (int x = 0; x < kTilesPerBatch; ++x) load_row_share<DI>(page + (size_t)(x * 16 + n) * DI, g, buf[u].k[x].v);
        buf[u].sc = *reinterpret_cast<const float*>(page + (size_t)kBatchTokens * DI + lane * 4);
      } else {
#pragma unroll
        for (int x = 0; x < kTilesPerBatch; ++x)
          load_row_share<DI>(kbase + (size_t)(base + x * 16 + n) * DI, g, buf[u].k[x].v);   // a block that counts lies inside the sequence
      }
    }
#pragma unroll
    for (int u = 0; u < G; ++u) {
      float res[T];
#pragma unroll
      for (int t = 0; t < T; ++t) res[t] = 0.f;
#pragma unroll
      for (int x = 0; x < kTilesPerBatch; ++x) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const float s = tile_score<HB, DI, T>(qr, t, buf[u].k[x]);
          res[t] = (g == x) ? s : res[t];
        }
      }
      if (u < nbw) {
#pragma unroll
        for (int t = 0; t < T; ++t)
          a.sample[((size_t)(b * Ttot + t0 + t) * a.nsamp + (s0 + u * kSWaves)) * kBatchTokens + lane] = PAGED ? res[t] * buf[u].sc : res[t];
      }
    }
  }
}

template <int HB, int DI, int T, bool PAGED, bool DYN>
int launch_d(hipStream_t st, const SampleArgs& a) {
  const ess_xcd x = a.xcd;
  const dim3 grid = DYN ? dim3(ess_xcd_grid(a.nparts * a.nb_seq, x)) : dim3(a.nparts, a.nb_seq);
  hipLaunchKernelGGL((k_index_sample<HB, DI, T, PAGED, DYN>), grid, dim3(kThreads), 0, st, a);
  return ESS_OK;
}

template <int HB, int DI, int T>
int launch_p(hipStream_t st, const SampleArgs& a) {
  if (a.block_table) return a.xcd.ticket ? launch_d<HB, DI, T, true, true>(st, a) : launch_d<HB, DI, T, true, false>(st, a);
  return a.xcd.ticket ? launch_d<HB, DI, T, false, true>(st, a) : launch_d<HB, DI, T, false, false>(st, a);
}

template <int DI>
int launch_hb(int HB, int T, hipStream_t st, const SampleArgs& a) {
  switch (HB) {
    case 1: return T == 1 ? launch_p<1, DI, 1>(st, a) : launch_p<1, DI, 2>(st, a);
    case 2: return T == 1 ? launch_p<2, DI, 1>(st, a) : launch_p<2, DI, 2>(st, a);
    case 3: return T == 1 ? launch_p<3, DI, 1>(st, a) : launch_p<3, DI, 2>(st, a);
    default: return T == 1 ? launch_p<4, DI, 1>(st, a) : launch_p<4, DI, 2>(st, a);
  }
}

}  // namespace

int ess_launch_index_sample(const ess_config& c, const uint8_t* q, const float* w, const uint8_t* key,
                            const int32_t* ctx_len, int B, int T, float* sample, hipStream_t st,
                            const int32_t* block_table, int n_pages, ess_xcd xcd) {
  SampleArgs a{};
  a.q = q; a.w = w; a.key = key; a.ctx_len = ctx_len;
  a.Lmax = c.max_ctx; a.Hi = c.idx_heads;
  a.block_table = block_table; a.n_pages = n_pages;
  a.Ttot = T; a.xcd = xcd; a.nb_seq = B;
  a.period = ess_sample_period(c.max_ctx); a.nsamp = ess_sample_count(c.max_ctx);
  a.nparts = (a.nsamp + kPartBlocks - 1) / kPartBlocks;
  a.sample = sample;
  if (xcd.ticket && T > 2) return ess_fail(ESS_ERR_UNSUPPORTED, "internal: one ticket serves one sample launch");
  const int HB = (c.idx_heads + 15) / 16;
  for (int t0 = 0; t0 < T; t0 += 2) {
    a.t0 = t0;
    const int Tl = T - t0 < 2 ? T - t0 : 2;
    int rc;
    switch (c.idx_dim) {
      case 32: rc = launch_hb<32>(HB, Tl, st, a); break;
      case 64: rc = launch_hb<64>(HB, Tl, st, a); break;
      case 128: rc = launch_hb<128>(HB, Tl, st, a); break;
      default: return ess_fail(ESS_ERR_UNSUPPORTED, "idx_dim %d (supported: 32, 64, 128)", c.idx_dim);
    }
    if (rc != ESS_OK) return rc;
  }
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
