// Stage 4: SparseMLA decode over the selected Latent-Cache entries (ESS paper
// Sec. 3.3), absorbed form: the 576 values of an entry are the key, the first
// 512 the value.  Flash-decoding layout: every (b,t) is cut into `nsplit`
// ranges of its entry list; each workgroup produces a softmax-normalised
// partial output and its log-sum-exp for all heads, and a merge kernel
// combines the partial results -- the same merge that joins Attn0 (resident
// entries) and Attn1 (fetched entries) of the DA overlap.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, wave64).  A workgroup is four
// waves, one per SIMD, each owning 16 heads with the whole 512-wide output row
// in 128 accumulator registers and its queries stationary (72 VGPRs); 64 heads
// per workgroup, head groups in grid.z.  The kernel is built for one wave per
// SIMD and the large register budget that comes with it.  Both products are
// computed transposed so that nothing is re-laid out between them:
//   S^T[r,h] = sum_d K[r,d] Q[h,d]      A = entry rows from LDS (row-major), B = Q^T (registers)
//   O^T[v,h] = sum_r V^T[v,r] P^T[r,h]  A = V^T, read transposed from the same rows, B = P^T (registers)
// The accumulator of S^T gives lane (g,h) the eight logits of head h for tile rows
// {4g..4g+3} and {16+4g..16+4g+3}; in exactly that order they are the eight
// k-values the lane supplies for the B operand of the second product, so P^T
// never leaves registers.  Softmax state is per lane = per head.
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
// Four waves x 16 heads, tiles of 32 entries in LDS as bf16 rows: bf16 entries gathered by
// global_load_lds, quantised entries (512 fp8 + 4 scales + rope) loaded into registers a tile ahead,
// dequantised and written in the same layout.  What the kernel is
// built around (a first version that built V^T in LDS, rescaled every tile and left the accumulators
// to the register allocator spent 1100 instructions per tile and wave, 68 of them MFMAs):
//  * V^T is never built.  The A operand of O^T += V^T P^T wants, per lane, 8 entries of one value
//    column; ds_read_b64_tr_b16 delivers exactly that from rows stored entry-major: in each group
//    of 16 lanes, source lane 4i+j points at 4 consecutive columns (4j..4j+3) of row i and lane n
//    receives column n of rows 0..3.  Two such reads (rows 4g+i and 16+4g+i) make one A fragment
//    whose k order is the order in which S^T leaves the first product.
//  * Rows have no padding (pitch 1024 bytes); the 16-byte granules of a row are XOR-swizzled with
//    f(row) = (row&3)<<2 | (row>>2)&3, applied on the way in by letting lane l of the gather fetch
//    granule l ^ f(row).  The LDS has 64 banks (256 bytes per clock), so a group of 16 lanes is
//    conflict-free when its 16-byte granules differ mod 16: K fragments (16 rows, one granule each)
//    because f is a bijection of the row's low four bits, transposing reads (rows 4g..4g+3, 32
//    bytes each) because f puts the row's low two bits above the granule pair.  (A three-bit f,
//    enough for 32 banks, made both products 1.7x slower.)
//  * The running maximum is only moved when a tile exceeds it by more than 2^8 (exponentials stay
//    below 2^8 relative to the reference, far inside fp32 and bf16 range), so the 128 accumulator
//    registers are rescaled a few times per split instead of once per tile.
//  * Four raw buffers: the gathers of three tiles are in flight; those of tile it+3 are issued one at
//    a time between the MFMAs of tile it, so that a gather instruction that waits for the texture
//    path does so while the matrix and LDS pipes are busy.
//  * Cross-lane maxima and sums over the four 16-lane groups use v_permlane32_swap / 16_swap, not LDS.
// Masked entries (slot < 0) are gathered from a row of zeros, so that no product meets stale LDS.
constexpr int TRP = 1024;                        // latent row pitch in LDS
constexpr int TR_KL_BYTES = TILE * TRP;          // 32768
constexpr int TR_RAW_BYTES = TR_KL_BYTES + RP_BYTES;
constexpr int tr_nbuf(int fmt) { return fmt == ESS_FMT_BF16 ? 4 : 2; }
constexpr int tr_lds_bytes(int fmt) { return tr_nbuf(fmt) * TR_RAW_BYTES + MAX_TPS * TILE * 4; }   // 155648 | 81920
constexpr float kLazyMax = 8.0f;

// The 128 output accumulators of a wave live in AGPRs a0..a127 under fixed names, outside the
// compiler's register allocation: every access is an asm statement that names them.  (Left to the
// allocator they are copied to VGPRs and back once per tile, 256 moves, because the rare rescale
// multiplies them with vector ALU instructions.)  The statements clobber what they write, so the
// kernel's register count covers them.  This file is compiled with -amdgpu-mfma-vgpr-form, which
// keeps the results of the compiler's own MFMAs (the first product) in VGPRs, and the kernel needs
// fewer than 256 VGPRs, so the compiler itself uses no AGPR here; tests/test_abi.py checks in the
// generated code that nothing but these statements names one.  368 registers per lane in all, which
// leaves room on every SIMD for the waves of the fetch kernel that runs beside Attn0.
#define ESS_ACC_TUPLES(X) X(0, 0, 1, 2, 3) X(1, 4, 5, 6, 7) X(2, 8, 9, 10, 11) X(3, 12, 13, 14, 15) X(4, 16, 17, 18, 19) X(5, 20, 21, 22, 23) X(6, 24, 25, 26, 27) X(7, 28, 29, 30, 31) X(8, 32, 33, 34, 35) X(9, 36, 37, 38, 39) X(10, 40, 41, 42, 43) X(11, 44, 45, 46, 47) X(12, 48, 49, 50, 51) X(13, 52, 53, 54, 55) X(14, 56, 57, 58, 59) X(15, 60, 61, 62, 63) X(16, 64, 65, 66, 67) X(17, 68, 69, 70, 71) X(18, 72, 73, 74, 75) X(19, 76, 77, 78, 79) X(20, 80, 81, 82, 83) X(21, 84, 85, 86, 87) X(22, 88, 89, 90, 91) X(23, 92, 93, 94, 95) X(24, 96, 97, 98, 99) X(25, 100, 101, 102, 103) X(26, 104, 105, 106, 107) X(27, 108, 109, 110, 111) X(28, 112, 113, 114, 115) X(29, 116, 117, 118, 119) X(30, 120, 121, 122, 123) X(31, 124, 125, 126, 127)
#define ESS_ACC_REGS(X) X(0, 0) X(1, 1) X(2, 2) X(3, 3) X(4, 4) X(5, 5) X(6, 6) X(7, 7) X(8, 8) X(9, 9) X(10, 10) X(11, 11) X(12, 12) X(13, 13) X(14, 14) X(15, 15) X(16, 16) X(17, 17) X(18, 18) X(19, 19) X(20, 20) X(21, 21) X(22, 22) X(23, 23) X(24, 24) X(25, 25) X(26, 26) X(27, 27) X(28, 28) X(29, 29) X(30, 30) X(31, 31) X(32, 32) X(33, 33) X(34, 34) X(35, 35) X(36, 36) X(37, 37) X(38, 38) X(39, 39) X(40, 40) X(41, 41) X(42, 42) X(43, 43) X(44, 44) X(45, 45) X(46, 46) X(47, 47) X(48, 48) X(49, 49) X(50, 50) X(51, 51) X(52, 52) X(53, 53) X(54, 54) X(55, 55) X(56, 56) X(57, 57) X(58, 58) X(59, 59) X(60, 60) X(61, 61) X(62, 62) X(63, 63) X(64, 64) X(65, 65) X(66, 66) X(67, 67) X(68, 68) X(69, 69) X(70, 70) X(71, 71) X(72, 72) X(73, 73) X(74, 74) X(75, 75) X(76, 76) X(77, 77) X(78, 78) X(79, 79) X(80, 80) X(81, 81) X(82, 82) X(83, 83) X(84, 84) X(85, 85) X(86, 86) X(87, 87) X(88, 88) X(89, 89) X(90, 90) X(91, 91) X(92, 92) X(93, 93) X(94, 94) X(95, 95) X(96, 96) X(97, 97) X(98, 98) X(99, 99) X(100, 100) X(101, 101) X(102, 102) X(103, 103) X(104, 104) X(105, 105) X(106, 106) X(107, 107) X(108, 108) X(109, 109) X(110, 110) X(111, 111) X(112, 112) X(113, 113) X(114, 114) X(115, 115) X(116, 116) X(117, 117) X(118, 118) X(119, 119) X(120, 120) X(121, 121) X(122, 122) X(123, 123) X(124, 124) X(125, 125) X(126, 126) X(127, 127)

// The compiler's hazard logic does not look into asm statements, and an MFMA that directly follows the vector
// ALU instruction producing one of its VGPR operands was seen to read the register's previous contents.  The
// first MFMA of every chunk (WAIT) therefore carries its wait states inside its own statement, where no
// scheduling can separate them from it; the later ones of a chunk follow an MFMA.
template <int VB, bool WAIT> __device__ __forceinline__ void pv_mfma(const bf16x8& a, const bf16x8& b);
#define X(vb, r0, r1, r2, r3)                                                                            \
  template <> __device__ __forceinline__ void pv_mfma<vb, false>(const bf16x8& a, const bf16x8& b) {     \
    asm volatile("v_mfma_f32_16x16x32_bf16 a[" #r0 ":" #r3 "], %0, %1, a[" #r0 ":" #r3 "]"               \
                 : : "v"(a), "v"(b) : "a" #r0, "a" #r1, "a" #r2, "a" #r3);                               \
  }                                                                                                      \
  template <> __device__ __forceinline__ void pv_mfma<vb, true>(const bf16x8& a, const bf16x8& b) {      \
    asm volatile("s_nop 7\n\tv_mfma_f32_16x16x32_bf16 a[" #r0 ":" #r3 "], %0, %1, a[" #r0 ":" #r3 "]"    \
                 : : "v"(a), "v"(b) : "a" #r0, "a" #r1, "a" #r2, "a" #r3);                               \
  }
ESS_ACC_TUPLES(X)
#undef X
template <int BASE, int... I>
__device__ __forceinline__ void pv_chunk(const bf16x8 (&fv)[sizeof...(I)], const bf16x8& pb, std::integer_sequence<int, I...>) {
  (pv_mfma<BASE + I, I == 0>(fv[I], pb), ...);
}
__device__ __forceinline__ void acc_zero() {
#define X(n, r) asm volatile("v_accvgpr_write_b32 a" #r ", 0" : : : "a" #r);
  ESS_ACC_REGS(X)
#undef X
}
// a[4 vb + i] holds row 4g+i of value block vb for head n16: every register of a lane scales by the lane's alpha
__device__ __forceinline__ void acc_scale(float alpha) {
  float t;
#define X(n, r) asm volatile("v_accvgpr_read_b32 %0, a" #r "\n\tv_mul_f32 %0, %0, %1\n\tv_accvgpr_write_b32 a" #r ", %0" \
                             : "=&v"(t) : "v"(alpha) : "a" #r);
  ESS_ACC_REGS(X)
#undef X
}
__device__ __forceinline__ void acc_read(float (&o)[128]) {
#define X(n, r) asm volatile("v_accvgpr_read_b32 %0, a" #r : "=v"(o[n]));
  ESS_ACC_REGS(X)
#undef X
}

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

// max / sum over the four lanes that share lane % 16 (one per 16-lane group), result in all four
__device__ __forceinline__ float group_max(float x) {
  uint2v a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
  uint2v b = __builtin_amdgcn_permlane16_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}
__device__ __forceinline__ float group_sum(float x) {
  uint2v a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = __uint_as_float(a.x) + __uint_as_float(a.y);
  uint2v b = __builtin_amdgcn_permlane16_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return __uint_as_float(b.x) + __uint_as_float(b.y);
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
  // Work item = (split, bt, head group): by workgroup index, or drawn from counters off the XCDs to be avoided.
  // The head groups of one (split, bt) read the same entries, so they should meet in one L2: every XCD that takes
  // work has a counter of its own (class c of nw) that hands out pairs c, c + nw, c + 2 nw .. head group by head
  // group; a workgroup whose class has run out goes on with the next class, so any one workgroup could finish
  // the whole launch.
  const int n_pairs = nsplit * n_bt, n_items = n_pairs * n_hg;
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
      // ticket v of class cls stands for pair (v / n_hg) * nw + cls, head group v % n_hg
      __syncthreads();
      if (threadIdx.x == 0) {
        const uint32_t tk = atomicAdd(xcd.ticket + ESS_TK_CLASS + ESS_TK_STRIDE * cls, 1u);
        const uint32_t pair = (tk / (uint32_t)n_hg) * (uint32_t)nw + (uint32_t)cls;
        s_item = pair < (uint32_t)n_pairs ? (int)(pair * (uint32_t)n_hg + tk % (uint32_t)n_hg) : -1;
      }
      __syncthreads();
      item = __builtin_amdgcn_readfirstlane(s_item);
      if (item >= 0 || tried == nw) break;
      ++tried;
      cls = cls + 1 == nw ? 0 : cls + 1;
    }
    if (item < 0) break;
    hg = item % n_hg;
    split = (item / n_hg) % nsplit;
    bt = item / (n_hg * nsplit);
  } else {
    if (round) break;
    split = blockIdx.x; bt = blockIdx.y; hg = blockIdx.z;
  }
  const int b = bt / T;
  // the thread index passes through an empty asm statement so that what is derived from it (lane constants, LDS
  // offsets) is computed per work item, where it is needed, instead of being kept in registers across the loop
  int tid = threadIdx.x;
  if constexpr (DYN) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n16 = lane & 15;
  const int head0 = (hg * 4 + wave) * 16;
  const bool wave_active = head0 < H;

  const int n = n_list ? min(n_list[bt], kk) : kk;
  const int tiles_total = (n + TILE - 1) / TILE;
  const int tps = min((tiles_total + nsplit - 1) / nsplit, MAX_TPS);
  const int tile_begin = split * tps;
  const int tile_end = min(tile_begin + tps, tiles_total);
  const int my_tiles = max(tile_end - tile_begin, 0);

  bf16x8 qb[KSTEPS];
  {
    const int head = head0 + n16;
    const uint16_t* qrow = q + ((size_t)bt * H + min(head, H - 1)) * ESS_ROW_DIM;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      uint4 x = *reinterpret_cast<const uint4*>(qrow + ks * 32 + g * 8);
      if (head >= H) x = make_uint4(0, 0, 0, 0);
      qb[ks] = *reinterpret_cast<bf16x8*>(&x);
    }
  }
  acc_zero();
  float m_ref = -__builtin_inff(), l_run = 0.f;

  const int32_t* lrow = list + (size_t)bt * kk;
  const uint8_t* pbase = pool + (size_t)b * S * row_stride;
  for (int j = tid; j < my_tiles * TILE; j += NTH) {
    const int e = tile_begin * TILE + j;
    int sl = e < n ? lrow[e] : -1;
    if (sl >= S) sl = -1;
    slot_cache[j] = sl;
  }
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
    for (int r8 = 0; r8 < 8; ++r8) sl[r8] = ts[wave * 8 + r8];
    sl[8] = ts[rr];
  };
  auto gather_step = [&](int it, int step, const int (&sl)[DMA_PER_TILE]) {
    const uint32_t raw = lds0 + (uint32_t)((it % NBUF) * TR_RAW_BYTES);
    if (step < 8) {
      const int row = wave * 8 + step;
      const int u = __builtin_amdgcn_readfirstlane(sl[step]);
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
    for (int it = 0; it < min(my_tiles, NBUF - 1); ++it) {
      int src[DMA_PER_TILE];
      gather_sources(it, src);
#pragma unroll
      for (int step = 0; step < DMA_PER_TILE; ++step) gather_step(it, step, src);
    }
  } else {
    if (my_tiles > 0) { f8_load(0, stg); f8_store(0, stg); }
    if (my_tiles > 1) f8_load(1, stg);
  }

  // lane constants of the two LDS access patterns
  const int fk = tr_swz(n16);                                   // K fragments: row n16 (and 16 + n16)
  uint32_t koff[4];                                             // by ks & 3; + 256 * (ks >> 2) is an immediate
#pragma unroll
  for (int c = 0; c < 4; ++c) koff[c] = (uint32_t)(n16 * TRP + (((4 * c + g) ^ fk) << 4));
  const int ti = n16 >> 2, tj = n16 & 3;                        // transposing reads: source row 4g + ti, columns 4 tj ..
  const int trow = 4 * g + ti;
  const uint32_t c4 = (uint32_t)((((tj >> 1) ^ tr_swz(trow)) & 15) << 4);
  uint32_t voff[8];                                             // by vb & 7; + 256 * (vb >> 3) is an immediate
#pragma unroll
  for (int c = 0; c < 8; ++c) voff[c] = (uint32_t)(trow * TRP + (tj & 1) * 8) + (((uint32_t)(32 * c)) ^ c4);

  for (int it = 0; it < my_tiles; ++it) {
    const uint32_t KLa = lds0 + (uint32_t)((it % NBUF) * TR_RAW_BYTES);
    const uint8_t* KL = lds + (it % NBUF) * TR_RAW_BYTES;
    const uint8_t* RP = KL + TR_KL_BYTES;
    const int32_t* tile_slot = slot_cache + it * TILE;
    const bool more = kDma && it + NBUF - 1 < my_tiles;   // tile it+3 goes into the buffer tile it-1 used
    int src[DMA_PER_TILE];
    if constexpr (kDma) {
      // this wave's gathers of tile `it` have landed when at most those of the later tiles are outstanding
      const int later = min(my_tiles - 1 - it, NBUF - 2);
      if (later >= 2) wait_vmcnt<2 * DMA_PER_TILE>(); else if (later == 1) wait_vmcnt<DMA_PER_TILE>(); else wait_vmcnt<0>();
      __syncthreads();                         // ... everyone's did; and everyone is done with tile it-1
      if (more) gather_sources(it + NBUF - 1, src);
    } else {
      __syncthreads();                         // tile `it` is in LDS (written a tile ago); everyone is done with tile it-1
      if (it + 1 < my_tiles) f8_store(it + 1, stg);   // into the buffer tile it-1 used
      if (it + 2 < my_tiles) f8_load(it + 2, stg);
    }
    if (!wave_active) {
      if (more) {
#pragma unroll
        for (int step = 0; step < DMA_PER_TILE; ++step) gather_step(it + NBUF - 1, step, src);
      }
      continue;
    }

    // ---- S^T = K Q^T; A fragments read six k-steps ahead of the MFMAs that use them; three gather
    // instructions of tile it+3 after each chunk of fragment reads
    floatx4 s0 = floatx4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
    constexpr int CH = kDma ? 6 : 3;           // quantised entries: the staged tile needs the registers
    bf16x8 fa[2][CH], fb[2][CH];
    auto load_chunk = [&](int c, bf16x8 (&da)[CH], bf16x8 (&db)[CH]) {
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        const int ks = c * CH + j;
        if (ks < 16) {
          da[j] = *reinterpret_cast<const bf16x8*>(KL + koff[ks & 3] + 256 * (ks >> 2));
          db[j] = *reinterpret_cast<const bf16x8*>(KL + koff[ks & 3] + 256 * (ks >> 2) + 16 * TRP);
        } else {
          const int p = (ks - 16) * 4 + g;
          da[j] = *reinterpret_cast<const bf16x8*>(RP + n16 * 128 + ((p ^ (n16 & 7)) * 16));
          db[j] = *reinterpret_cast<const bf16x8*>(RP + (16 + n16) * 128 + ((p ^ (n16 & 7)) * 16));
        }
      }
    };
    load_chunk(0, fa[0], fb[0]);
#pragma unroll
    for (int c = 0; c < KSTEPS / CH; ++c) {
      if (c + 1 < KSTEPS / CH) load_chunk(c + 1, fa[(c + 1) & 1], fb[(c + 1) & 1]);
      if (more) {
#pragma unroll
        for (int step = 9 * c / (KSTEPS / CH); step < 9 * (c + 1) / (KSTEPS / CH); ++step) gather_step(it + NBUF - 1, step, src);
      }
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[c & 1][j], qb[c * CH + j], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[c & 1][j], qb[c * CH + j], s1, 0, 0, 0);
      }
    }
    const int4 v0 = *reinterpret_cast<const int4*>(tile_slot + g * 4);
    const int4 v1 = *reinterpret_cast<const int4*>(tile_slot + 16 + g * 4);
    // the first V fragments do not depend on the softmax: request them now, they arrive while it runs
    constexpr int CV = 8;
    bf16x8 fv[2][CV];
    auto load_v = [&](int c, bf16x8 (&d)[CV]) {
#pragma unroll
      for (int j = 0; j < CV; ++j) {
        const int vb = c * CV + j;
        const uint32_t a = KLa + voff[vb & 7] + 256u * (uint32_t)(vb >> 3);
        d[j] = tr_frag(a, a + 16 * TRP);
      }
    };
    load_v(0, fv[0]);
    load_v(1, fv[1]);
    const bool ok[8] = {v0.x >= 0, v0.y >= 0, v0.z >= 0, v0.w >= 0, v1.x >= 0, v1.y >= 0, v1.z >= 0, v1.w >= 0};
    float z[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      z[i] = ok[i] ? s0[i] * scale_log2e : -__builtin_inff();
      z[4 + i] = ok[4 + i] ? s1[i] * scale_log2e : -__builtin_inff();
    }
    const float tmax = group_max(fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7]))));
    // move the reference only when this tile exceeds it by more than 2^kLazyMax (always from -inf)
    const bool move = tmax > m_ref + kLazyMax;
    if (__any(move)) {
      const float m_new = move ? tmax : m_ref;
      const float alpha = m_new == -__builtin_inff() ? 1.f : exp2f(m_ref - m_new);   // m_ref = -inf: 0, acc is 0 anyway
      l_run *= alpha;
      m_ref = m_new;
      acc_scale(alpha);
    }
    const float m_safe = (m_ref == -__builtin_inff()) ? 0.f : m_ref;
    float p[8], psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p[j] = exp2f(z[j] - m_safe);
      psum += p[j];
    }
    l_run += psum;
    uint4 pw = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
    const bf16x8 pb = *reinterpret_cast<bf16x8*>(&pw);

    // ---- O^T += V^T P^T, A fragments by transposing reads, eight blocks ahead
    static_assert(VBLOCKS / CV == 4, "four chunks of value blocks");
    constexpr auto seq = std::make_integer_sequence<int, CV>{};
    pv_chunk<0 * CV>(fv[0], pb, seq);
    load_v(2, fv[0]);
    pv_chunk<1 * CV>(fv[1], pb, seq);
    load_v(3, fv[1]);
    pv_chunk<2 * CV>(fv[0], pb, seq);
    pv_chunk<3 * CV>(fv[1], pb, seq);
  }
  // the hazard logic does not see the MFMAs inside the asm statements: let the last ones retire
  // before their results are read
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

  {
    const int head = head0 + n16;
    const float l_tot = group_sum(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    float o[128];
    acc_read(o);
    if (head < H) {
      const size_t prow = ((size_t)bt * ESS_MAX_SPLITS + split0 + split) * H + head;
      _Float16* op = o_part + prow * ESS_LATENT_DIM;
#pragma unroll
      for (int vb = 0; vb < VBLOCKS; ++vb) {
        floatx4 ov = floatx4{o[4 * vb] * inv, o[4 * vb + 1] * inv, o[4 * vb + 2] * inv, o[4 * vb + 3] * inv};
#pragma unroll
        for (int i = 0; i < 4; ++i) ov[i] = __builtin_amdgcn_fmed3f(ov[i], -65504.f, 65504.f);   // an average of entry values: saturate, never inf
        *reinterpret_cast<halfx4*>(op + vb * 16 + g * 4) = __builtin_convertvector(ov, halfx4);   // round to nearest even
      }
      if (g == 0) lse_part[prow] = l_tot > 0.f ? (m_ref + log2f(l_tot)) * kLn2 : -__builtin_inff();
    }
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
  float lsv[ESS_MAX_SPLITS];
  float mx = -__builtin_inff();
#pragma unroll
  for (int s = 0; s < ESS_MAX_SPLITS; ++s) {
    lsv[s] = s < nsplit ? lse_part[base + (size_t)s * H] : -__builtin_inff();
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
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] += wgt * (float)xy[u][i];
      }
    }
  }
  const float inv = den > 0.f ? 1.0f / den : 0.f;
  uint4 o = make_uint4(pack_bf16(a[0] * inv, a[1] * inv), pack_bf16(a[2] * inv, a[3] * inv),
                       pack_bf16(a[4] * inv, a[5] * inv), pack_bf16(a[6] * inv, a[7] * inv));
  *reinterpret_cast<uint4*>(out + (size_t)rowi * ESS_LATENT_DIM + lane * 8) = o;
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
  const int n_hg = (c.attn_heads + 63) / 64;            // 64 heads per workgroup
  dim3 grid(nsplit, B * T, n_hg);
  if (xcd.ticket) grid = dim3(ess_xcd_grid(nsplit * B * T * n_hg, xcd));     // one workgroup per CU
  const float sc = c.sm_scale * kLog2e;
  const uint16_t* qq = static_cast<const uint16_t*>(q);
  // partial results of sequence b0 onward
  _Float16* op = reinterpret_cast<_Float16*>(ctx->o_part) + (size_t)b0 * T * ESS_MAX_SPLITS * c.attn_heads * ESS_LATENT_DIM;
  float* lp = ctx->lse_part + (size_t)b0 * T * ESS_MAX_SPLITS * c.attn_heads;
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
                     ctx->lse_part + r0 * ESS_MAX_SPLITS, H, nsplit_total, rows,
                     static_cast<uint16_t*>(out_bf16) + r0 * ESS_LATENT_DIM, lse ? lse + r0 : nullptr, zero_cnt, n_zero, chk);
  ESS_HIP(hipGetLastError());
  return ESS_OK;
}
