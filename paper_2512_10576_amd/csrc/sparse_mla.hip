// Stage 4: SparseMLA decode over the selected Latent-Cache entries (ESS paper
// Sec. 3.3), absorbed form: the 576 values of an entry are the key, the first
// 512 the value.  Flash-decoding layout: every (b,t) is cut into `nsplit`
// ranges of its entry list; each workgroup produces a softmax-normalised
// partial output and its log-sum-exp for all heads, and a merge kernel
// combines the partial results -- the same merge that joins Attn0 (resident
// entries) and Attn1 (fetched entries) of the DA overlap.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, wave64).  A workgroup is four
// waves, one per SIMD, each owning 32 heads with the whole 512-wide output row
// in 256 accumulator registers and its queries stationary (144 VGPRs): 128 heads
// per workgroup, so the entries of a range are brought from memory once for all
// heads.  The kernel is built for one wave per SIMD and the register budget that
// comes with it.  Both products are computed transposed so that nothing is
// re-laid out between them; see the comment at the kernel.
#include "ess_internal.h"
#include <utility>
#include <hip/hip_bf16.h>

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
// Partial results travel from the partial-attention kernels to the merge kernel as fp16: they are
// softmax-normalised (|value| <= the largest entry value), fp16 keeps 11 bits of them while the merged
// output is rounded to bf16's 8, and the traffic between the two kernels, which is most of what both
// cost beyond their tile loops, is halved.  The split weights (log-sum-exp) stay fp32.
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int TILE = ESS_ATTN_TILE;            // 32 entries
constexpr int NTH = 256;                       // four waves
constexpr int KSTEPS = ESS_ROW_DIM / 32;       // 18
constexpr int VBLOCKS = ESS_LATENT_DIM / 16;   // 32
constexpr int MAX_TPS = 64;                    // tiles per split (the launcher picks nsplit accordingly): a list of 2048 entries fits one split
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const __hip_bfloat16 x = __float2bfloat16(a), y = __float2bfloat16(b);
  return (uint32_t)(*reinterpret_cast<const uint16_t*>(&x)) | ((uint32_t)(*reinterpret_cast<const uint16_t*>(&y)) << 16);
}

// rope piece (dims 512 + 8*rc ..): bf16 in both formats
template <int FMT>
__device__ __forceinline__ uint4 load_rope(const uint8_t* row, int rc) {
  return *reinterpret_cast<const uint4*>(row + (FMT == ESS_FMT_BF16 ? 1024 : 520) + rc * 16);
}

// ---------------------------------------------------------------------------------------------
// bf16 entries are brought into LDS by the memory system itself
// (global_load_lds_dwordx4: a wave instruction moves 64 x 16 bytes from per-lane global addresses to
// consecutive LDS addresses, no registers involved).  One wave instruction per 1024-byte latent
// part of a row, one per eight 128-byte rope parts.  The loads are issued through inline assembly
// because the compiler, seeing an LDS-writing load, would wait for every outstanding one before the
// next LDS read; completion is tracked by hand with s_waitcnt vmcnt (memory loads complete in issue
// order, 9 of them per wave and tile).
constexpr int RP_BYTES = TILE * 128;           // 4096: rope parts, 16-byte pieces XOR-swizzled by row
constexpr int DMA_PER_TILE = 9;                // wave instructions per tile: 8 latent rows + 1 rope group

__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// 64 lanes x 16 bytes from `gptr` (per lane) to LDS address `lds_dst` + 16 * lane (lds_dst wave-uniform)
// The statement writes m0 and says so (m0 is reserved: the compiler never keeps a value of its own there across
// statements, but the clobber makes the write visible to it; clang warns about reserved registers in clobber lists).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_dst) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void wait_vmcnt() {     // vmcnt <= N, other counters untouched
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// ---------------------------------------------------------------- the partial-attention kernel
// Four waves, one per SIMD, 32 heads each: a workgroup covers all (up to 128) heads of one range of the entry
// list, so an entry is brought from memory once per range.  Tiles of 32 entries sit in LDS as bf16 rows: bf16
// entries gathered by global_load_lds, quantised entries (512 fp8 + 4 scales + rope) loaded into registers a tile
// ahead, dequantised and written in the same layout.  Matrix-core mapping (v_mfma_f32_32x32x16_bf16), both
// products transposed so that nothing is re-laid out between them:
//   S^T[r,h] = sum_d K[r,d] Q[h,d]      A = entry rows from LDS (lane: row l%32, 8 dims), B = Q^T (registers)
//   O^T[v,h] = sum_r V^T[v,r] P^T[r,h]  A = V^T, read transposed from the same rows, B = P^T (registers)
// The accumulator of S^T gives lane (hh = l/32, h = l%32) the sixteen logits of head h for tile rows
// 8q + 4hh + i (q, i = 0..3), and registers 8s..8s+7 are, in that order, the eight k-values the lane supplies for
// the B operand of k-step s of the second product: P^T never leaves registers.  Softmax state is per lane = per
// (head, half); the two halves of a head meet in one v_permlane32_swap.
// 32 heads per wave halve the LDS bytes per flop against 16 (a K or V^T fragment of 1 KiB feeds twice the
// multiply-adds).  That is what counts, because the tile loop is bound by the LDS: per tile a SIMD issues 68 MFMAs
// of 32 cycles (2176 cycles), but the four waves read 278 KiB of fragments, and the LDS delivers them at about
// 64 bytes per clock for ds_read_b128 and 41 for the transposing reads, CU-wide (phase timers: 2000 cycles for
// the first product's 144 reads, 3200 for the second product's 256), whatever the prefetch depth and whatever
// else is interleaved.
//  * V^T is never built.  ds_read_b64_tr_b16 delivers, in each group of 16 lanes, column n of four consecutive
//    rows to lane n (source lane 4i+j points at columns 4j..4j+3 of row i); two such reads (rows 16s+4hh+i and
//    16s+8+4hh+i) make one A fragment whose k order is the order in which S^T leaves the first product.
//  * Rows have no padding (pitch 1024 bytes); the 16-byte granules of a row are XOR-swizzled with
//    f(row) = (row&3)<<2 | (row>>2)&3, applied on the way in by letting lane l of the gather fetch granule
//    l ^ f(row).  The LDS has 64 banks (256 bytes per clock): K fragments (16 rows of one granule per clock) are
//    conflict-free because f is a bijection of the row's low four bits, transposing reads (4 rows x 64 bytes per
//    clock) because f puts the row's low two bits above the granule pair.
//  * The running maximum is only moved when a tile exceeds it by more than 2^8, so the 256 accumulator registers
//    are rescaled a few times per split instead of once per tile.
//  * Four raw buffers: the gathers of three tiles are in flight; those of tile it+3 are issued between the MFMAs of
//    tile it.
// Masked entries (slot < 0) are gathered from a row of zeros, so that no product meets stale LDS.
constexpr int TRP = 1024;                        // latent row pitch in LDS
constexpr int TR_KL_BYTES = TILE * TRP;          // 32768
constexpr int TR_RAW_BYTES = TR_KL_BYTES + RP_BYTES;
constexpr int tr_nbuf(int fmt) { return fmt == ESS_FMT_BF16 ? 4 : 2; }
constexpr int Q_PITCH = ESS_ROW_DIM * 2 + 16;    // 1168: pitch of the query rows while they are staged in LDS
constexpr int O_PITCH = ESS_LATENT_DIM * 2 + 8;  // 1032: pitch of the fp16 result rows while they are staged in LDS
constexpr int tr_lds_bytes(int fmt) {            // tile buffers + slot list, and room for the staged queries: 155648 | 149504
  const int tiles = tr_nbuf(fmt) * TR_RAW_BYTES + MAX_TPS * TILE * 4, stage = 128 * Q_PITCH;
  return tiles > stage ? tiles : stage;
}
constexpr float kLazyMax = 8.0f;
constexpr int HPW = 32;                          // heads per wave
constexpr int HPG = 4 * HPW;                     // heads per workgroup
constexpr int KS16 = ESS_ROW_DIM / 16;           // 36 k-steps of the first product
constexpr int VB32 = ESS_LATENT_DIM / 32;        // 16 blocks of 32 value columns

typedef float floatx16 __attribute__((ext_vector_type(16)));

// The 256 output accumulators of a wave (16 blocks of 32 value columns x 32 heads, 16 registers each) live in
// AGPRs a0..a255 under fixed names, outside the compiler's register allocation: every access is an asm statement
// that names them by number.  (Left to the allocator -- as MFMA builtins, or as asm operands with the "a"
// constraint -- they are copied around or spilled, because the rare rescale multiplies them with vector ALU
// instructions and the loop leaves no spare 16-register tuple.)  This file is compiled with
// -amdgpu-mfma-vgpr-form, which keeps the results of the compiler's own MFMAs (the first product) in VGPRs, and
// the AGPR file is claimed as a whole (see AgprHold below), so that the compiler has no use for AGPRs of its own:
// tests/test_abi.py checks in the generated code that nothing but these statements names one and that nothing is
// spilled.
// The compiler's hazard logic does not look into asm statements, and an MFMA that directly follows the vector ALU
// instruction producing one of its VGPR operands was seen to read the register's previous contents: an MFMA
// marked WAIT carries wait states inside its own statement, where no scheduling can separate them from it.
// The compiler must keep its hands off the AGPRs that these statements use behind its back.  It is told that they
// are taken: eight 32-register values with the "a" constraint are defined at the start of the kernel (by an empty
// statement) and passed through empty statements (agpr_fence) at the top of every tile iteration and at the end, so
// they are live throughout and fill the AGPR file -- the allocator has no AGPR left for a temporary or a spill of
// its own, and the launch reserves all 256.  What the values "hold" is of no interest to the compiler's code.
typedef float floatx32 __attribute__((ext_vector_type(32)));
struct AgprHold { floatx32 d0, d1, d2, d3, d4, d5, d6, d7; };
// (the comments inside the statements mark the claimed stretch in the generated code, for the test that reads it)
__device__ __forceinline__ void agpr_claim(AgprHold& h) {
  asm volatile("; ess_agpr_claim" : "=a"(h.d0), "=a"(h.d1), "=a"(h.d2), "=a"(h.d3), "=a"(h.d4), "=a"(h.d5), "=a"(h.d6), "=a"(h.d7));
}
__device__ __forceinline__ void agpr_fence(AgprHold& h) {
  asm volatile("; ess_agpr_fence" : "+a"(h.d0), "+a"(h.d1), "+a"(h.d2), "+a"(h.d3), "+a"(h.d4), "+a"(h.d5), "+a"(h.d6), "+a"(h.d7));
}
__device__ __forceinline__ void agpr_release(AgprHold& h) {
  asm volatile("; ess_agpr_release" : "+a"(h.d0), "+a"(h.d1), "+a"(h.d2), "+a"(h.d3), "+a"(h.d4), "+a"(h.d5), "+a"(h.d6), "+a"(h.d7));
}
template <int VB, bool WAIT>
__device__ __forceinline__ void pv_mfma(const bf16x8& a, const bf16x8& b) {
  if constexpr (WAIT)
    asm volatile("s_nop 7\n\tv_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]" : : "v"(a), "v"(b), "n"(16 * VB), "n"(16 * VB + 15));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]" : : "v"(a), "v"(b), "n"(16 * VB), "n"(16 * VB + 15));
}
template <int R> __device__ __forceinline__ void acc_zero1() { asm volatile("v_accvgpr_write_b32 a[%0], 0" : : "n"(R)); }
template <int R> __device__ __forceinline__ void acc_scale1(float alpha) {
  float t;
  asm volatile("v_accvgpr_read_b32 %0, a[%2]\n\ts_nop 0\n\tv_mul_f32 %0, %0, %1\n\ts_nop 0\n\tv_accvgpr_write_b32 a[%2], %0" : "=&v"(t) : "v"(alpha), "n"(R));
}
template <int R> __device__ __forceinline__ float acc_read1() {
  float t;
  asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(t) : "n"(R));
  return t;
}
template <int... R> __device__ __forceinline__ void acc_zero_seq(std::integer_sequence<int, R...>) { (acc_zero1<R>(), ...); }
template <int... R> __device__ __forceinline__ void acc_scale_seq(float alpha, std::integer_sequence<int, R...>) { (acc_scale1<R>(alpha), ...); }
__device__ __forceinline__ void acc_zero() { acc_zero_seq(std::make_integer_sequence<int, 256>{}); }
// every register of a lane belongs to the lane's head: all scale by the lane's alpha
__device__ __forceinline__ void acc_scale(float alpha) { acc_scale_seq(alpha, std::make_integer_sequence<int, 256>{}); }
// the 16 registers of block VB: rows (value columns) 32 VB + 8q + 4hh + i at index 4q + i
template <int VB, int... I>
__device__ __forceinline__ void acc_read_block(float (&o)[16], std::integer_sequence<int, I...>) { ((o[I] = acc_read1<16 * VB + I>()), ...); }

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v lds_short4v;
typedef unsigned uint2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int tr_swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ bf16x8 tr_frag(uint32_t addr_lo, uint32_t addr_hi) {
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(addr_lo));
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4v*>(addr_hi));
  typedef short short8v __attribute__((ext_vector_type(8)));
  const short8v x = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, x);
}

// max / sum over the two lanes that hold one head (l and l ^ 32), result in both
__device__ __forceinline__ float pair_max(float x) {
  uint2v a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
}
__device__ __forceinline__ float pair_sum(float x) {
  uint2v a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(a.x) + __uint_as_float(a.y);
}

template <int FMT, bool DYN>
__global__ __launch_bounds__(NTH, 1) void k_attn_partial_tr(
    const uint16_t* __restrict__ q, const uint8_t* __restrict__ pool, const int32_t* __restrict__ list,
    const int32_t* __restrict__ n_list, int T, int H, int kk, int S, int row_stride, float scale_log2e, int split0,
    int nsplit, _Float16* __restrict__ o_part, float* __restrict__ lse_part, const uint8_t* __restrict__ zero_row,
    ess_xcd xcd, int n_bt, int n_hg) {
  extern __shared__ __align__(16) uint8_t lds[];
  __shared__ int s_item;
  constexpr bool kDma = FMT == ESS_FMT_BF16;       // rows go to LDS as they are; else through registers, dequantised
  constexpr int NBUF = tr_nbuf(FMT);
  int32_t* slot_cache = reinterpret_cast<int32_t*>(lds + NBUF * TR_RAW_BYTES);   // [MAX_TPS][32]
  const uint32_t lds0 = lds_addr_of(lds);
  // Work item = (bt, split, head group).  The work items of one (b,t) share its queries (144 KiB for 128 heads),
  // so they should meet in one L2.  By workgroup index: bt is the fastest grid dimension, and consecutive
  // workgroups go round the eight XCDs, so the splits of a row land on one XCD whenever the number of rows is a
  // multiple of eight.  Drawn from counters (off the XCDs to be avoided): every XCD that takes work has a counter
  // of its own (class c of nw) that hands out the items of rows c, c + nw, c + 2 nw .. one after the other; a
  // workgroup whose class has run out goes on with the next class, so any one workgroup could finish the launch.
  const int per_row = nsplit * n_hg, n_items = n_bt * per_row;
  constexpr bool dyn = DYN;
  int cls = 0, nw = 1, tried = 1;
  if (dyn) {
    if (!ess_ticket_join(xcd, &s_item)) return;
    const uint32_t work = ~xcd.avoid & 0xffu;
    const int x = ess_xcc_id() & 7;
    nw = max(__popc(work), 1);
    cls = ((work >> x) & 1u) ? __popc(work & ((1u << x) - 1u)) : 0;
  }
  for (int round = 0;; ++round) {
  int split, bt, hg;
  if (dyn) {
    int item;
    for (;;) {
      // ticket v of class cls: row (v / per_row) * nw + cls, item v % per_row of that row
      __syncthreads();
      if (threadIdx.x == 0) {
        const uint32_t tk = atomicAdd(xcd.ticket + ESS_TK_CLASS + ESS_TK_STRIDE * cls, 1u);
        const uint32_t row = (tk / (uint32_t)per_row) * (uint32_t)nw + (uint32_t)cls;
        s_item = row < (uint32_t)n_bt ? (int)(row * (uint32_t)per_row + tk % (uint32_t)per_row) : -1;
      }
      __syncthreads();
      item = __builtin_amdgcn_readfirstlane(s_item);
      if (item >= 0 || tried == nw) break;
      ++tried;
      cls = cls + 1 == nw ? 0 : cls + 1;
    }
    if (item < 0) break;
    bt = item / per_row;
    split = (item % per_row) / n_hg;
    hg = item % n_hg;
  } else {
    if (round) break;
    bt = blockIdx.x; split = blockIdx.y; hg = blockIdx.z;
  }
  const int b = bt / T;
  // the thread index passes through an empty asm statement so that what is derived from it (lane constants, LDS
  // offsets) is computed per work item, where it is needed, instead of being kept in registers across the loop
  int tid = threadIdx.x;
  if constexpr (DYN) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hh = lane >> 5, h32 = lane & 31;       // half of the wave, head within the wave
  const int head0 = hg * HPG + wave * HPW;
  const bool wave_active = head0 < H;

  const int n = n_list ? min(n_list[bt], kk) : kk;
  const int tiles_total = (n + TILE - 1) / TILE;
  const int tps = min((tiles_total + nsplit - 1) / nsplit, MAX_TPS);
  const int tile_begin = split * tps;
  const int tile_end = min(tile_begin + tps, tiles_total);
  const int my_tiles = max(tile_end - tile_begin, 0);

  // this thread's share of the split's entry list: asked for first, so that it arrives while the queries are staged
  const int32_t* lrow = list + (size_t)bt * kk;
  const uint8_t* pbase = pool + (size_t)b * S * row_stride;
  constexpr int SLOTS_PT = MAX_TPS * TILE / NTH;   // 8 list entries per thread at most
  int my_slot[SLOTS_PT];
#pragma unroll
  for (int u = 0; u < SLOTS_PT; ++u) {
    const int j = tid + NTH * u, e = tile_begin * TILE + j;
    int sl = (j < my_tiles * TILE && e < n) ? lrow[e] : -1;
    if (sl >= S) sl = -1;
    my_slot[u] = sl;
  }

  // Q^T as the B operand, stationary: lane (hh, h) holds dims 16 ks + 8 hh .. + 7 of head h for every k-step.
  // The queries of the workgroup's heads are one contiguous block in memory: the threads read it piece by piece
  // (whole cache lines per wave instruction) into the still empty tile buffers, rows at a pitch of 1168 bytes so
  // that sixteen rows' pieces fall on different banks, and every lane takes its fragments from there.  (Read
  // straight from memory, a wave instruction touches 32 bytes of each of 32 rows and every cache line is asked for
  // four times: most of what a workgroup cost beyond its tiles.)
  bf16x8 qb[KS16];
  {
    constexpr int QPIECES = ESS_ROW_DIM * 2 / 16;    // 72 pieces of 16 bytes per head
    const int nh = min(HPG, H - hg * HPG);
    const uint4* qsrc = reinterpret_cast<const uint4*>(q + ((size_t)bt * H + (size_t)hg * HPG) * ESS_ROW_DIM);
    const int npieces = nh * QPIECES;
    uint4 x[HPG * QPIECES / NTH];                    // 36 loads of a thread in flight
#pragma unroll
    for (int i = 0; i < HPG * QPIECES / NTH; ++i) {
      const int pc = tid + NTH * i;
      x[i] = pc < npieces ? qsrc[pc] : make_uint4(0, 0, 0, 0);       // heads past H: zeros
    }
#pragma unroll
    for (int i = 0; i < HPG * QPIECES / NTH; ++i) {
      const int pc = tid + NTH * i, row = pc / QPIECES, col = pc - row * QPIECES;
      *reinterpret_cast<uint4*>(lds + row * Q_PITCH + col * 16) = x[i];
    }
    __syncthreads();
    const uint8_t* qrow = lds + (wave * HPW + h32) * Q_PITCH + hh * 16;
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) qb[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 32);
    __syncthreads();                                 // the staging area becomes tile buffers and slot list
  }
  AgprHold hold;
  agpr_claim(hold);
  acc_zero();
  float m_ref = -__builtin_inff(), l_run = 0.f;

#pragma unroll
  for (int u = 0; u < SLOTS_PT; ++u)
    if (tid + NTH * u < my_tiles * TILE) slot_cache[tid + NTH * u] = my_slot[u];
  wait_vmcnt<0>();                             // q and list loads are done: from here only the gathers count
  __syncthreads();

  // Gathers of one tile into raw buffer it % 4: this wave brings rows 8w..8w+7 (steps 0..7, one
  // instruction per row) and the rope parts of the same rows (step 8).
  const int rr = wave * 8 + (lane >> 3);
  const int rope_off = 1024 + (((lane & 7) ^ (rr & 7)) * 16);
  // slots of one tile's rows: read from LDS in one go, so that no gather waits on the LDS queue later; the
  // address of a row is computed when its gather is issued (scalar arithmetic for the eight whole-row
  // gathers: it then runs while the matrix pipe is busy)
  auto gather_sources = [&](int it, int (&sl)[DMA_PER_TILE]) {
    const int32_t* ts = slot_cache + it * TILE;
#pragma unroll
    for (int r8 = 0; r8 < 8; ++r8) sl[r8] = __builtin_amdgcn_readfirstlane(ts[wave * 8 + r8]);   // the same in all lanes: scalar registers
    sl[8] = ts[rr];
  };
  auto gather_step = [&](int it, int step, const int (&sl)[DMA_PER_TILE]) {
    const uint32_t raw = lds0 + (uint32_t)((it % NBUF) * TR_RAW_BYTES);
    if (step < 8) {
      const int row = wave * 8 + step;
      const int u = sl[step];
      const uint8_t* src = u >= 0 ? pbase + (size_t)u * row_stride : zero_row;
      dma16(src + ((lane ^ tr_swz(row)) << 4), raw + (uint32_t)(row * TRP));
    } else {
      const uint8_t* src = sl[8] >= 0 ? pbase + (size_t)sl[8] * row_stride : zero_row;
      dma16(src + rope_off, raw + (uint32_t)(TR_KL_BYTES + wave * 1024));
    }
  };
  // Quantised entries: a tile's share of a thread -- row tid/8: four 16-byte pieces of fp8 values (piece
  // c + 8j, c = tid%8, belongs to scale group j), the row's four bf16 scales, one 16-byte rope piece --
  // is loaded into registers two tiles ahead and written to LDS one tile ahead, as bf16 in the layout
  // that the gathers of bf16 entries produce (two buffers).
  struct StagedF8 { uint4 lat[4]; uint2 sc; uint4 rope; };
  auto f8_load = [&](int it, StagedF8& st) {
    const int row = tid >> 3, c = tid & 7;
    const int sl = slot_cache[it * TILE + row];
    const uint8_t* src = sl >= 0 ? pbase + (size_t)sl * row_stride : zero_row;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) st.lat[jj] = *reinterpret_cast<const uint4*>(src + (c + 8 * jj) * 16);
    st.sc = *reinterpret_cast<const uint2*>(src + 512);
    st.rope = load_rope<ESS_FMT_FP8>(src, c);
  };
  auto f8_store = [&](int it, const StagedF8& st) {
    uint8_t* KL = lds + (it % NBUF) * TR_RAW_BYTES;
    const int row = tid >> 3, c = tid & 7;
    const int f = tr_swz(row);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const uint32_t sbits = (jj < 2 ? st.sc.x : st.sc.y) >> (16 * (jj & 1));
      const float sc = __uint_as_float(sbits << 16);
      const uint32_t w[4] = {st.lat[jj].x, st.lat[jj].y, st.lat[jj].z, st.lat[jj].w};
      uint32_t o[8];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[d], false);
        const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[d], true);
        o[2 * d] = pack_bf16(lo[0] * sc, lo[1] * sc);
        o[2 * d + 1] = pack_bf16(hi[0] * sc, hi[1] * sc);
      }
      const int G = 2 * (c + 8 * jj);
      *reinterpret_cast<uint4*>(KL + row * TRP + ((G ^ f) << 4)) = make_uint4(o[0], o[1], o[2], o[3]);
      *reinterpret_cast<uint4*>(KL + row * TRP + (((G + 1) ^ f) << 4)) = make_uint4(o[4], o[5], o[6], o[7]);
    }
    *reinterpret_cast<uint4*>(KL + TR_KL_BYTES + row * 128 + ((c ^ (row & 7)) * 16)) = st.rope;
  };
  StagedF8 stg;
  if constexpr (kDma) {
    for (int it = 0; it < min(my_tiles, 2); ++it) {
      int src[DMA_PER_TILE];
      gather_sources(it, src);
#pragma unroll
      for (int step = 0; step < DMA_PER_TILE; ++step) gather_step(it, step, src);
    }
  } else {
    if (my_tiles > 0) { f8_load(0, stg); f8_store(0, stg); }
    if (my_tiles > 1) f8_load(1, stg);
  }

  // lane constants of the two LDS access patterns.  K fragment of k-step ks: row h32, granule 2 ks + hh, i.e.
  // kbase ^ ((ks & 7) << 5) plus 256 (ks >> 3) (the swizzle touches the low four granule bits only); rope
  // k-steps read the rope region.  V^T fragment of block vb, k-step s: rows 16 s + 4 hh + ti (+ 8), columns
  // 32 vb + 16 gi + 4 tj ..: vbase{0,1} ^ ((vb & 3) << 6) plus 256 (vb >> 2) plus 16 s rows.
  const int fk = tr_swz(h32);
  const uint32_t kbase = (uint32_t)(h32 * TRP + ((hh ^ fk) << 4));
  const int gi = (lane >> 4) & 1, ti = (lane & 15) >> 2, tj = lane & 3;
  const int vrow0 = 4 * hh + ti, vrow1 = 8 + 4 * hh + ti;
  const uint32_t vbase0 = (uint32_t)(vrow0 * TRP + (((2 * gi + (tj >> 1)) ^ tr_swz(vrow0)) << 4) + (tj & 1) * 8);
  const uint32_t vbase1 = (uint32_t)(vrow1 * TRP + (((2 * gi + (tj >> 1)) ^ tr_swz(vrow1)) << 4) + (tj & 1) * 8);

  // pieces of a tile's work, shared by the two loops below
  auto load_k = [&](const uint8_t* KL, int ks) -> bf16x8 {
    if (ks < 32) return *reinterpret_cast<const bf16x8*>(KL + (kbase ^ (uint32_t)((ks & 7) << 5)) + 256 * (ks >> 3));
    const int p = (ks - 32) * 2 + hh;
    return *reinterpret_cast<const bf16x8*>(KL + TR_KL_BYTES + h32 * 128 + ((p ^ (h32 & 7)) * 16));
  };
  auto load_v = [&](uint32_t KLa, int j) -> bf16x8 {       // j = 16 s + vb: all blocks of k-step 0, then all of k-step 1
    const int vb = j & 15, s = j >> 4;
    const uint32_t x = (uint32_t)((vb & 3) << 6), off = 256u * (uint32_t)(vb >> 2) + (uint32_t)(16 * s * TRP);
    return tr_frag(KLa + (vbase0 ^ x) + off, KLa + (vbase1 ^ x) + off);
  };
  // logits of the lane's sixteen rows (8 q + 4 hh + i at index 4 q + i), masked rows at -inf
  auto logits = [&](const floatx16& sacc, const int32_t* tile_slot, float (&z)[16]) {
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      const int4 v = *reinterpret_cast<const int4*>(tile_slot + 8 * qd + 4 * hh);
      z[4 * qd] = v.x >= 0 ? sacc[4 * qd] * scale_log2e : -__builtin_inff();
      z[4 * qd + 1] = v.y >= 0 ? sacc[4 * qd + 1] * scale_log2e : -__builtin_inff();
      z[4 * qd + 2] = v.z >= 0 ? sacc[4 * qd + 2] * scale_log2e : -__builtin_inff();
      z[4 * qd + 3] = v.w >= 0 ? sacc[4 * qd + 3] * scale_log2e : -__builtin_inff();
    }
  };
  auto max16 = [](const float (&z)[16]) {
    return fmaxf(fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7]))),
                 fmaxf(fmaxf(fmaxf(z[8], z[9]), fmaxf(z[10], z[11])), fmaxf(fmaxf(z[12], z[13]), fmaxf(z[14], z[15]))));
  };

  if constexpr (kDma) {
    // ---- bf16 entries.  One wave per SIMD issues its instructions one at a time, and what a tile costs is the
    // sum of their issue times (a vector ALU instruction 4 cycles, an LDS read 13-16), not the 2176 cycles its 68
    // MFMAs keep the matrix pipe busy.  The loop is therefore a software pipeline in which the vector ALU work of
    // the softmax rides in the shadow of MFMAs: iteration `it`
    //   1. computes S^T of tile it (a chain of 36 dependent MFMAs) and, between them, turns the logits of tile
    //      it-1 into P^T (exponentials, row sums, bf16 pairs);
    //   2. issues the second product of tile it-1 and, between its MFMAs, turns S^T of tile it into logits and
    //      takes their maximum (which may move the softmax reference: the accumulators are then rescaled after
    //      these MFMAs, before those of tile it).
    // A tile's buffer is in use for two iterations, and the gathers of tile it+2 (into the buffer tile it-2 used)
    // are issued during iteration it: two tiles in flight.
    float z[16];                                 // logits of the previous tile (rows 8 q + 4 hh + i at index 4 q + i)
    float m_use = 0.f;                           // the reference they are taken against
    float alpha_pending = 1.f;                   // rescale of the accumulators due before the next second product
    bool scale_pending = false;
    // one iteration; QK: there is a tile `it` to start, PV: there is a tile it-1 to finish
    auto iteration = [&](int it, auto qkc, auto pvc) {
      constexpr bool QK = decltype(qkc)::value, PV = decltype(pvc)::value;
      const uint8_t* KL = lds + (it % NBUF) * TR_RAW_BYTES;
      const uint32_t KLp = lds0 + (uint32_t)(((it + NBUF - 1) % NBUF) * TR_RAW_BYTES);     // tile it-1
      const bool more = it + 2 < my_tiles;
      int src[DMA_PER_TILE];
      agpr_fence(hold);
      if constexpr (QK) {
        // this wave's gathers of tile `it` have landed when at most those of tile it+1 are outstanding
        if (it + 1 < my_tiles) wait_vmcnt<DMA_PER_TILE>(); else wait_vmcnt<0>();
      }
      __syncthreads();                           // ... everyone's did; and everyone is done with tile it-2
      if (more) gather_sources(it + 2, src);
      if (!wave_active) {
        if (more) {
#pragma unroll
          for (int step = 0; step < DMA_PER_TILE; ++step) gather_step(it + 2, step, src);
        }
        return;
      }
      floatx16 sacc;
      uint32_t pq[8];                            // P^T of tile it-1 as bf16 pairs: k-step 0 in [0..3], k-step 1 in [4..7]
      float psum = 0.f;
      // one row of tile it-1: exponential against the reference, row sum, and (every second row) a bf16 pair
      auto exp_row = [&](auto ic) {
        constexpr int i = decltype(ic)::value;
        z[i] = __builtin_amdgcn_exp2f(z[i] - m_use);     // the argument is <= 2^kLazyMax: no range reduction needed
        psum += z[i];
        if constexpr (i & 1) pq[i >> 1] = pack_bf16(z[i - 1], z[i]);
      };
      if constexpr (QK) {
        // S^T = K Q^T: 36 k-steps, A fragments read CK k-steps ahead; a gather instruction after every fourth
        // k-step; rows of tile it-1 after every second one
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
        constexpr int CK = 3;
        bf16x8 fa[CK];
#pragma unroll
        for (int j = 0; j < CK; ++j) fa[j] = load_k(KL, j);
        auto qk_step = [&](auto ksc) {
          constexpr int ks = decltype(ksc)::value;
          const bf16x8 a = fa[ks % CK];
          if (ks + CK < KS16) fa[ks % CK] = load_k(KL, ks + CK);
          if (more && (ks & 3) == 3) gather_step(it + 2, ks >> 2, src);
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[ks], sacc, 0, 0, 0);
          if constexpr (PV && (ks & 1) == 1 && (ks >> 1) < 16) exp_row(std::integral_constant<int, (ks >> 1)>{});
        };
        [&]<int... K>(std::integer_sequence<int, K...>) { (qk_step(std::integral_constant<int, K>{}), ...); }
        (std::make_integer_sequence<int, KS16>{});
      } else {
        [&]<int... I>(std::integer_sequence<int, I...>) { (exp_row(std::integral_constant<int, I>{}), ...); }
        (std::make_integer_sequence<int, 16>{});
      }
      if constexpr (PV) l_run += psum;
      agpr_fence(hold);
      if (scale_pending) {                       // wave-uniform; rare
        acc_scale(alpha_pending);
        scale_pending = false;
      }
      // second product of tile it-1 (32 MFMAs) with the logits of tile it taken between them
      constexpr int CV = 5;
      bf16x8 fv[CV];
      if constexpr (PV) {
#pragma unroll
        for (int j = 0; j < CV; ++j) fv[j] = load_v(KLp, j);
      }
      const int32_t* tile_slot = slot_cache + it * TILE;
      auto step = [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        if constexpr (PV) {
          const bf16x8 a = fv[j % CV];
          if (j + CV < 2 * VB32) fv[j % CV] = load_v(KLp, j + CV);
          uint4 pw = j < 16 ? make_uint4(pq[0], pq[1], pq[2], pq[3]) : make_uint4(pq[4], pq[5], pq[6], pq[7]);
          pv_mfma<(j & 15), (j == 0 || j == 16)>(a, *reinterpret_cast<bf16x8*>(&pw));
        }
        if constexpr (QK) {
          if constexpr (j >= 2 && j < 18 && (j & 3) == 2) {      // logits of rows 8 qd + 4 hh + i, masked rows at -inf
            constexpr int qd = (j - 2) >> 2;
            const int4 v = *reinterpret_cast<const int4*>(tile_slot + 8 * qd + 4 * hh);
            z[4 * qd] = v.x >= 0 ? sacc[4 * qd] * scale_log2e : -__builtin_inff();
            z[4 * qd + 1] = v.y >= 0 ? sacc[4 * qd + 1] * scale_log2e : -__builtin_inff();
            z[4 * qd + 2] = v.z >= 0 ? sacc[4 * qd + 2] * scale_log2e : -__builtin_inff();
            z[4 * qd + 3] = v.w >= 0 ? sacc[4 * qd + 3] * scale_log2e : -__builtin_inff();
          }
          if constexpr (j == 20) {
            const float tmax = pair_max(max16(z));
            // move the reference only when this tile exceeds it by more than 2^kLazyMax (always from -inf)
            const bool move = tmax > m_ref + kLazyMax;
            if (__any(move)) {
              const float m_new = move ? tmax : m_ref;
              alpha_pending = m_new == -__builtin_inff() ? 1.f : exp2f(m_ref - m_new);   // m_ref = -inf: 0, acc is 0 anyway
              l_run *= alpha_pending;
              m_ref = m_new;
              scale_pending = true;              // the accumulators are rescaled once the MFMAs of tile it-1 are through
            }
            m_use = (m_ref == -__builtin_inff()) ? 0.f : m_ref;
          }
        }
      };
      [&]<int... J>(std::integer_sequence<int, J...>) { (step(std::integral_constant<int, J>{}), ...); }
      (std::make_integer_sequence<int, 2 * VB32>{});
    };
    if (my_tiles > 0) {
      iteration(0, std::true_type{}, std::false_type{});
      for (int it = 1; it < my_tiles; ++it) iteration(it, std::true_type{}, std::true_type{});
      iteration(my_tiles, std::false_type{}, std::true_type{});
    }
  } else {
  for (int it = 0; it < my_tiles; ++it) {
    // ---- quantised entries: the tile's three phases one after the other
    const uint32_t KLa = lds0 + (uint32_t)((it % NBUF) * TR_RAW_BYTES);
    const uint8_t* KL = lds + (it % NBUF) * TR_RAW_BYTES;
    agpr_fence(hold);
    __syncthreads();                           // tile `it` is in LDS (written a tile ago); everyone is done with tile it-1
    if (it + 1 < my_tiles) f8_store(it + 1, stg);   // into the buffer tile it-1 used
    if (it + 2 < my_tiles) f8_load(it + 2, stg);
    if (!wave_active) continue;

    floatx16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
    constexpr int CK = 2;                      // the staged tile needs the registers
    bf16x8 fa[CK];
#pragma unroll
    for (int j = 0; j < CK; ++j) fa[j] = load_k(KL, j);
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      const bf16x8 a = fa[ks % CK];
      if (ks + CK < KS16) fa[ks % CK] = load_k(KL, ks + CK);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[ks], sacc, 0, 0, 0);
    }
    agpr_fence(hold);
    float z[16];
    logits(sacc, slot_cache + it * TILE, z);
    const float tmax = pair_max(max16(z));
    const bool move = tmax > m_ref + kLazyMax;
    if (__any(move)) {
      const float m_new = move ? tmax : m_ref;
      const float alpha = m_new == -__builtin_inff() ? 1.f : exp2f(m_ref - m_new);
      l_run *= alpha;
      m_ref = m_new;
      acc_scale(alpha);
    }
    const float m_safe = (m_ref == -__builtin_inff()) ? 0.f : m_ref;
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      z[j] = __builtin_amdgcn_exp2f(z[j] - m_safe);     // the argument is <= 2^kLazyMax: no range reduction needed
      psum += z[j];
    }
    l_run += psum;
    uint4 pw0 = make_uint4(pack_bf16(z[0], z[1]), pack_bf16(z[2], z[3]), pack_bf16(z[4], z[5]), pack_bf16(z[6], z[7]));
    uint4 pw1 = make_uint4(pack_bf16(z[8], z[9]), pack_bf16(z[10], z[11]), pack_bf16(z[12], z[13]), pack_bf16(z[14], z[15]));
    const bf16x8 pb0 = *reinterpret_cast<bf16x8*>(&pw0), pb1 = *reinterpret_cast<bf16x8*>(&pw1);
    agpr_fence(hold);
    constexpr int CV = 4;
    bf16x8 fv[CV];
#pragma unroll
    for (int j = 0; j < CV; ++j) fv[j] = load_v(KLa, j);
    auto pv_step = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const bf16x8 a = fv[j % CV];
      if (j + CV < 2 * VB32) fv[j % CV] = load_v(KLa, j + CV);
      pv_mfma<(j & 15), (j == 0 || j == 16)>(a, j < 16 ? pb0 : pb1);
    };
    [&]<int... J>(std::integer_sequence<int, J...>) { (pv_step(std::integral_constant<int, J>{}), ...); }
    (std::make_integer_sequence<int, 2 * VB32>{});
  }
  }
  // the hazard logic does not see the MFMAs inside the asm statements: let the last ones retire
  // before their results are read
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  agpr_fence(hold);

  {
    // lane constants afresh (see above): nothing of the epilogue is carried through the tile loop
    int tid2 = threadIdx.x;
    asm volatile("" : "+v"(tid2));
    const int lane2 = tid2 & 63, hh2 = (tid2 >> 5) & 1, h2 = tid2 & 31, head = head0 + h2;
    const float l_tot = pair_sum(l_run);
    float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    const size_t prow = ((size_t)bt * ESS_MAX_SPLITS + split0 + split) * H + min(head, H - 1);
    // The partial result goes through LDS (the tile buffers are free now) so that it leaves as whole rows: a lane
    // holds four consecutive columns at a time, of a row 1 KiB away from its neighbour's.  fp16 rows at a pitch of
    // 1032 bytes: the 32 heads of a half-wave write 8 bytes each to 64 different banks.
    // fp16 holds magnitudes below 65504.  The rows are staged as they are, the largest magnitude noted on the way;
    // should a head's reach 2^15 (entry values of that size: rare) the wave stages once more, such heads divided by
    // the power of two that brings their largest value below 2^15 -- exact, and undone by the merge.
    __syncthreads();                                 // every wave is done with the last tile
    uint8_t* orow = lds + (wave * HPW + h2) * O_PITCH + 8 * hh2;
    float amax = 0.f, down = 1.f;
    auto stage_rows = [&]() {
      auto stage_block = [&](auto vbc) {
        constexpr int vb = decltype(vbc)::value;
        float o[16];
        acc_read_block<vb>(o, std::make_integer_sequence<int, 16>{});
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          floatx4 ov = floatx4{o[4 * qd] * inv, o[4 * qd + 1] * inv, o[4 * qd + 2] * inv, o[4 * qd + 3] * inv};
          amax = fmaxf(fmaxf(amax, fmaxf(fabsf(ov[0]), fabsf(ov[1]))), fmaxf(fabsf(ov[2]), fabsf(ov[3])));
#pragma unroll
          for (int i = 0; i < 4; ++i) ov[i] = __builtin_amdgcn_fmed3f(ov[i], -65504.f, 65504.f);   // never inf in the fp16 image
          *reinterpret_cast<halfx4*>(orow + (vb * 32 + 8 * qd) * 2) = __builtin_convertvector(ov, halfx4);   // round to nearest even
        }
      };
      [&]<int... V>(std::integer_sequence<int, V...>) { (stage_block(std::integral_constant<int, V>{}), ...); }
      (std::make_integer_sequence<int, VB32>{});
    };
    stage_rows();
    amax = pair_max(amax);
    if (__any(amax >= 32768.f)) {
      int ex = 0;
      (void)frexpf(amax, &ex);                       // amax < 2^ex
      down = (amax >= 32768.f && amax <= 3.0e38f) ? ldexpf(1.f, ex - 15) : 1.f;
      inv = inv / down;
      stage_rows();
    }
    agpr_release(hold);                              // the accumulators are read out: the AGPRs are the compiler's again
    __syncthreads();
    // a wave writes its own 32 rows, 1 KiB per instruction
    const int rows_here = min(HPW, H - head0);
    _Float16* obase = o_part + (((size_t)bt * ESS_MAX_SPLITS + split0 + split) * H + head0) * ESS_LATENT_DIM;
    for (int r = 0; r < rows_here; ++r) {
      const uint2* src = reinterpret_cast<const uint2*>(lds + (wave * HPW + r) * O_PITCH + lane2 * 16);
      const uint2 lo = src[0], hi = src[1];
      ess_store_nt(reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(obase + (size_t)r * ESS_LATENT_DIM) + lane2 * 16), make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
    if (head < H && hh2 == 0)
      *reinterpret_cast<float2*>(lse_part + 2 * prow) = make_float2(l_tot > 0.f ? (m_ref + log2f(l_tot)) * kLn2 : -__builtin_inff(), down);
  }
  }
}

// out[bt,h,:] = sum_s exp(lse_s - lse) * o_s ;  lse = log sum_s exp(lse_s).  One wave per (bt,h).
// The partial results of four splits are requested before any is used (the kernel is a chain of
// dependent loads otherwise); those of empty splits are not read at all.  `zero_cnt` (may be NULL): n_zero counters the first workgroup clears,
// for steps that have no other kernel to do it in.
__global__ __launch_bounds__(256) void k_attn_merge(const _Float16* __restrict__ o_part, const float* __restrict__ lse_part,
                                                    int H, int nsplit, int total_rows, uint16_t* __restrict__ out,
                                                    float* __restrict__ lse_out, int32_t* __restrict__ zero_cnt,
                                                    int n_zero, ess_ticket_check chk) {
  if (zero_cnt && blockIdx.x == 0)
    for (int i = threadIdx.x; i < n_zero; i += 256) zero_cnt[i] = 0;
  if (chk.tickets && blockIdx.x == 0 && threadIdx.x == 0) {
    bool short_of = false;
#pragma unroll
    for (int i = 0; i < ESS_N_TICKETS; ++i) {
      uint32_t handed = chk.tickets[i * ESS_TICKET_WORDS + ESS_TK_WORK];   // the launch's counter, or its per-XCD counters
      for (int c = 0; c < 8; ++c) handed += chk.tickets[i * ESS_TICKET_WORDS + ESS_TK_CLASS + ESS_TK_STRIDE * c];
      short_of |= chk.need[i] != 0 && handed < chk.need[i];
    }
    if (short_of) *chk.flag = 1;
  }
  const int rowi = blockIdx.x * 4 + (threadIdx.x >> 6);      // bt*H + h
  if (rowi >= total_rows) return;
  const int lane = threadIdx.x & 63;
  const int bt = rowi / H, h = rowi % H;
  const size_t base = ((size_t)bt * ESS_MAX_SPLITS) * H + h;
  // the split weights first (one small load each, kept in registers), then only the partial results
  // of splits that hold something: a miss list usually fills one of its splits and leaves the rest empty
  float lsv[ESS_MAX_SPLITS], up[ESS_MAX_SPLITS];     // up: the power of two a split's fp16 values were divided by
  float mx = -__builtin_inff();
#pragma unroll
  for (int s = 0; s < ESS_MAX_SPLITS; ++s) {
    const float2 lu = s < nsplit ? *reinterpret_cast<const float2*>(lse_part + 2 * (base + (size_t)s * H)) : make_float2(-__builtin_inff(), 1.f);
    lsv[s] = lu.x;
    up[s] = lu.y;
    mx = fmaxf(mx, lsv[s]);
  }
  float den = 0.f;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (mx > -__builtin_inff()) {
#pragma unroll
    for (int s0 = 0; s0 < ESS_MAX_SPLITS; s0 += 4) {
      if (s0 >= nsplit) break;
      halfx8 xy[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        xy[u] = halfx8{0, 0, 0, 0, 0, 0, 0, 0};
        if (lsv[s0 + u] != -__builtin_inff())                   // same for the whole wave: one row per wave
          xy[u] = *reinterpret_cast<const halfx8*>(o_part + (base + (size_t)(s0 + u) * H) * ESS_LATENT_DIM + lane * 8);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (lsv[s0 + u] == -__builtin_inff()) continue;
        const float wgt = __expf(lsv[s0 + u] - mx);
        den += wgt;
        const float wu = wgt * up[s0 + u];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] += wu * (float)xy[u][i];
      }
    }
  }
  const float inv = den > 0.f ? 1.0f / den : 0.f;
  uint4 o = make_uint4(pack_bf16(a[0] * inv, a[1] * inv), pack_bf16(a[2] * inv, a[3] * inv),
                       pack_bf16(a[4] * inv, a[5] * inv), pack_bf16(a[6] * inv, a[7] * inv));
  ess_store_nt(reinterpret_cast<uint4*>(out + (size_t)rowi * ESS_LATENT_DIM + lane * 8), o);
  if (lse_out && lane == 0) lse_out[rowi] = den > 0.f ? mx + __logf(den) : -__builtin_inff();
}

}  // namespace

int ess_attn_min_splits(const ess_config& c) {
  const int tiles = (c.topk + TILE - 1) / TILE;
  return (tiles + MAX_TPS - 1) / MAX_TPS;
}

// At context creation (on the context's device): the partial-attention kernels use more dynamic LDS than the default limit.
int ess_init_attn_kernels() {
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_partial_tr<ESS_FMT_BF16, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, tr_lds_bytes(ESS_FMT_BF16)));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_partial_tr<ESS_FMT_BF16, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, tr_lds_bytes(ESS_FMT_BF16)));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_partial_tr<ESS_FMT_FP8, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, tr_lds_bytes(ESS_FMT_FP8)));
  ESS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_partial_tr<ESS_FMT_FP8, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, tr_lds_bytes(ESS_FMT_FP8)));
  return ESS_OK;
}

int ess_launch_attn_partial(ess_ctx* ctx, const void* q, const uint8_t* slot_pool, const int32_t* list,
                            const int32_t* n_list, int B, int T, int split0, int nsplit, hipStream_t st, int b0, ess_xcd xcd) {
  const ess_config& c = ctx->cfg;
  if (nsplit < ess_attn_min_splits(c)) return ess_fail(ESS_ERR_INVALID_ARG, "internal: too few attention splits");
  const int n_hg = (c.attn_heads + HPG - 1) / HPG;      // 128 heads per workgroup
  dim3 grid(B * T, nsplit, n_hg);
  if (xcd.ticket) grid = dim3(ess_xcd_grid(nsplit * B * T * n_hg, xcd));     // one workgroup per CU
  const float sc = c.sm_scale * kLog2e;
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  // partial results of sequence b0 onward
  _Float16* op = reinterpret_cast<_Float16*>(ctx->o_part) + (size_t)b0 * T * ESS_MAX_SPLITS * c.attn_heads * ESS_LATENT_DIM;
  float* lp = ctx->lse_part + (size_t)b0 * T * ESS_MAX_SPLITS * c.attn_heads * 2;
#define ESS_ATTN_LAUNCH(FMT, DYN)                                                                                      \
  hipLaunchKernelGGL((k_attn_partial_tr<FMT, DYN>), grid, dim3(NTH), tr_lds_bytes(FMT), st, qq, slot_pool, list, n_list, T, \
                     c.attn_heads, c.topk, c.slots_per_seq, c.row_stride, sc, split0, nsplit, op, lp, ctx->zero_row, xcd,  \
                     B * T, n_hg)
  if (c.latent_fmt == ESS_FMT_BF16) {
    if (xcd.ticket) ESS_ATTN_LAUNCH(ESS_FMT_BF16, true); else ESS_ATTN_LAUNCH(ESS_FMT_BF16, false);
  } else {
    if (xcd.ticket) ESS_ATTN_LAUNCH(ESS_FMT_FP8, true); else ESS_ATTN_LAUNCH(ESS_FMT_FP8, false);
  }
#undef ESS_ATTN_LAUNCH
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}

int ess_launch_attn_merge(ess_ctx* ctx, int B, int T, int nsplit_total, void* out_bf16, float* lse, hipStream_t st,
                          int32_t* zero_cnt, int n_zero, int b0, const ess_ticket_check* check) {
  const int H = ctx->cfg.attn_heads;
  ess_ticket_check chk{};
  if (check) chk = *check;
  const int rows = B * T * H;
  const size_t r0 = (size_t)b0 * T * H;                       // first (bt, h) row of the sub-batch
  hipLaunchKernelGGL(k_attn_merge, dim3((rows + 3) / 4), dim3(256), 0, st,
                     reinterpret_cast<const _Float16*>(ctx->o_part) + r0 * ESS_MAX_SPLITS * ESS_LATENT_DIM,
                     ctx->lse_part + r0 * ESS_MAX_SPLITS * 2, H, nsplit_total, rows,
                     static_cast<uint16_t*>(out_bf16) + r0 * ESS_LATENT_DIM, lse ? lse + r0 : nullptr, zero_cnt, n_zero, chk);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
