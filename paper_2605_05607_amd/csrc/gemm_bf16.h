// Grouped GEMMs on the matrix cores: tile, work item, the per-item kernels and the resident kernel, for bf16
// operands and (template flag FP8) for E4M3 operands.
#pragma once
#include <type_traits>

#include "combine_kernels.h"
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Grouped bf16 GEMM on the matrix cores.  C[rows of one expert tile, kBN/2 or kBN columns] = A * W_e.
//   A rows   : row_map == nullptr -> A[m0 + r, :]; else A[row_map[m0 + r], :] (token gather of Dispatch).
//   B tiles  : packed in operand order (pack_kernels.h), streamed linearly into the LDS and read linearly from it.
//   GATED    : epilogue h = silu(g) * u, written as bf16   (GEMM-1)
//   !GATED   : epilogue o = acc * row_w[row], written fp32 (GEMM-2, gate weight of Sec. III-C)
// Tile 256 x 256 x 64, one workgroup of 512 threads per CU.  Every operand byte enters the CU once (global ->
// registers -> LDS) because the L2 -> CU path, not the matrix core, is what saturates first on this chip;
// sharing goes through the LDS, which has bandwidth to spare.  8 waves = 2 (rows) x 4 (columns), each wave
// owns 128 x 64 as 4 x 2 MFMA 32x32x16 accumulators; two waves per SIMD cover each other's LDS latency.
// LDS is double buffered (2 x 64 KiB) with one barrier per k-step; the next slab is in flight in registers
// while the current one is multiplied.  NB = number of 32-row blocks of this wave that hold valid rows (the
// others are skipped: small experts are weight-streaming bound and need no padding math).
// ------------------------------------------------------------------------------------------------

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// FP8 operands (E4M3): a 16-byte fragment holds 16 reduction indices per lane; two fragments (32 bytes per lane)
// feed one 32x32x64 instruction.  Which reduction indices share an instruction, and where in the operand they sit,
// does not matter as long as A and B agree: both put the same two 16-byte chunks of the reduction range side by side.
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f32x16 mfma_fp8_pair(bf16x8 a_lo, bf16x8 a_hi, bf16x8 b_lo, bf16x8 b_hi, f32x16 c) {
  const i32x8 a = __builtin_shufflevector(__builtin_bit_cast(i32x4, a_lo), __builtin_bit_cast(i32x4, a_hi), 0, 1, 2, 3,
                                          4, 5, 6, 7);
  const i32x8 b = __builtin_shufflevector(__builtin_bit_cast(i32x4, b_lo), __builtin_bit_cast(i32x4, b_hi), 0, 1, 2, 3,
                                          4, 5, 6, 7);
  // both operands E4M3 (format selectors 0), no block scales (all scale operands 0)
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

constexpr int kGemmThreads = 512;

// s_waitcnt immediate of the gfx9 encoding (gfx950 included) for "vmcnt(0)": the vector-memory counter at zero (bits
// 3:0 and 15:14), the export and LDS/scalar counters left at their maxima (bits 6:4 = 7, bits 11:8 = 15).  Used where
// a wait has to be spelled out around the device-scope hand-over of the resident kernel (see gemm_bf16_drain); any
// other instruction set encodes the counters differently, so the build is pinned to the target the waits were
// written for.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "the explicit s_waitcnt encodings of the hand-over are written for gfx950"
#endif
constexpr int kWaitVmcnt0 = 0x0F70;
constexpr int kAStageBytes = kBM * kBK * 2;               // 32 KiB
constexpr int kStageBytes = kAStageBytes + kTileBytes;    // 64 KiB: A slab then B slab
constexpr int kPatchBytes = 32 * 288;                     // per-wave epilogue patch (fits 8 x in the stages)

// FP8: A and the packed B hold E4M3 codes; a k-step then covers 128 reduction indices in the same 128 bytes per row,
// so the staging, the LDS image and the fragment reads are byte for byte those of the bf16 tile.  The scales
// (g.a_scale per token, g.b_scale per expert and output column, g.h_scale per expert) are applied in the epilogues
// and GEMM-1 writes h as codes.
// TRAIN selects the epilogues of the training path (bf16 only):
//   GATED  : as GEMM-1, and g and u are kept as well (g.aux = gu [rows, 2 N] bf16: g, then u) for the backward pass;
//   !GATED : the first GEMM of the backward pass, dh_raw = dy Wd^T (N = f).  With the kept g, u and the gate weight w:
//            dh = w dh_raw, dg = dh u silu'(g), du = dh silu(g)  ->  g.out = dgu [rows, 2 N] bf16 (dg, then du), and
//            g.aux2 = w silu(g) u [rows, N] bf16 (the h operand of the down-projection weight gradient, weight folded in).
template <bool GATED, bool RESIDENT, int NB, int NA, int DEPTH, bool FP8 = false, bool TRAIN = false, bool LONE = false>
__device__ __forceinline__ void gemm_bf16_tile(const GemmArgs &g, unsigned char *smem, int nt, int le, int m0,
                                               int rows, int nblk_total, int poison = 0,
                                               int32_t *pre_ctr = nullptr, int *pre_slot = nullptr) {
  // RESIDENT (the kernel that loops over items): the thread index goes through an empty asm so that nothing
  // derived from it counts as loop invariant; hoisting those values across items costs more registers than the
  // tile has to spare.
  int tid = threadIdx.x;
  if (RESIDENT) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int w8 = tid >> 6;
  const int wm = w8 >> 2, wn = w8 & 3;

  // ---- global -> register staging (scalars, not arrays, so nothing lands in scratch) ----
  // A: thread t stages chunk t & 7 (8 reduction indices) of rows (t >> 3) + 64 i; B: chunks t + 512 i
  const int a_chunk = tid & 7;
  const int a_row0 = tid >> 3;  // 0..63
  typedef typename std::conditional<FP8, uint8_t, bf16_t>::type elt_t;
  constexpr int EPC = FP8 ? 16 : 8;    // elements per 16-byte chunk
  constexpr int KS = FP8 ? 128 : kBK;  // reduction indices per k-step
  const elt_t *a_base = static_cast<const elt_t *>(g.A) + a_chunk * EPC;
#define MOE355_A_ROW(i)                                                                          \
  const int a_rc##i = a_row0 + 64 * i < rows ? a_row0 + 64 * i : rows - 1; /* padding: a valid row */ \
  const uint32_t a_off##i =                                                                      \
      (uint32_t)(g.row_map ? g.row_map[m0 + a_rc##i] : m0 + a_rc##i) * (uint32_t)g.lda;
  MOE355_A_ROW(0) MOE355_A_ROW(1) MOE355_A_ROW(2) MOE355_A_ROW(3)
#undef MOE355_A_ROW
  // LDS destination of row a_row0; row + 64 i lies 8192 bytes further (64 i keeps the swizzle bits)
  const int a_dst = (a_row0 * 8 + (a_chunk ^ ((a_row0 >> 1) & 7))) * 16;
  const unsigned char *b_src =
      static_cast<const unsigned char *>(g.Bp) + ((size_t)(le * g.n_ntiles + nt) * g.n_ktiles) * kTileBytes + tid * 16;

  // Register slab sets.  Set x always exists; set y is used when DEPTH == 2 (two slabs in flight: tiles with at
  // most 64 rows are pure weight streaming, their accumulators are small, and what limits them is the number of
  // bytes a CU keeps in flight towards HBM).
  u32x4 ra0x, ra1x, ra2x, ra3x, rb0x, rb1x, rb2x, rb3x;
  u32x4 ra0y, ra1y, ra2y, ra3y, rb0y, rb1y, rb2y, rb3y;
  // A slab is moved in three portions: {ra0, ra1, rb0}, {ra2, ra3, rb1}, {rb2, rb3}
  // k tail: a chunk past K is replaced by chunk 0 of the same row (valid memory, finite data); the packed B
  // tile is zero there, so it contributes nothing and no select has to wait on the load
#define MOE355_A_OFF(KT) ((KT) * KS + a_chunk * EPC < g.K ? (KT) * KS : -a_chunk * EPC)
  // NA = row loads per thread that reach valid rows (1: rows < 64, 2: rows < 128, 4: all); the others are skipped
  // Weight tiles of a streaming item (at most 64 rows), and of any item that is its expert's only M tile (LONE), are
  // read once by one workgroup: loaded with the non-temporal hint so that they do not push the operands that other
  // tiles share out of the L2.
#define MOE355_B_LOAD(PTR)                                                                          \
  ((NA == 1 || LONE) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(PTR))                        \
           : *reinterpret_cast<const u32x4 *>(PTR))
#define MOE355_LOAD_P0(S, KT)                                                                       \
  do {                                                                                              \
    ra0##S = *reinterpret_cast<const u32x4 *>(a_base + a_off0 + MOE355_A_OFF(KT));                  \
    if (NA > 1) ra1##S = *reinterpret_cast<const u32x4 *>(a_base + a_off1 + MOE355_A_OFF(KT));      \
    rb0##S = MOE355_B_LOAD(b_src + (size_t)(KT) * kTileBytes);                                      \
  } while (0)
#define MOE355_LOAD_P1(S, KT)                                                                       \
  do {                                                                                              \
    if (NA > 2) ra2##S = *reinterpret_cast<const u32x4 *>(a_base + a_off2 + MOE355_A_OFF(KT));      \
    if (NA > 2) ra3##S = *reinterpret_cast<const u32x4 *>(a_base + a_off3 + MOE355_A_OFF(KT));      \
    rb1##S = MOE355_B_LOAD(b_src + (size_t)(KT) * kTileBytes + 8192);                               \
  } while (0)
#define MOE355_LOAD_P2(S, KT)                                                                       \
  do {                                                                                              \
    rb2##S = MOE355_B_LOAD(b_src + (size_t)(KT) * kTileBytes + 16384);                              \
    rb3##S = MOE355_B_LOAD(b_src + (size_t)(KT) * kTileBytes + 24576);                              \
  } while (0)
#define MOE355_STORE_P0(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    *reinterpret_cast<u32x4 *>(s_ + a_dst) = ra0##S;                                                \
    if (NA > 1) *reinterpret_cast<u32x4 *>(s_ + a_dst + 8192) = ra1##S;                             \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16) = rb0##S;                              \
  } while (0)
#define MOE355_STORE_P1(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    if (NA > 2) *reinterpret_cast<u32x4 *>(s_ + a_dst + 16384) = ra2##S;                            \
    if (NA > 2) *reinterpret_cast<u32x4 *>(s_ + a_dst + 24576) = ra3##S;                            \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 8192) = rb1##S;                       \
  } while (0)
#define MOE355_STORE_P2(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 16384) = rb2##S;                      \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 24576) = rb3##S;                      \
  } while (0)

  f32x16 acc[NB > 0 ? NB : 1][2];
#pragma unroll
  for (int mi = 0; mi < NB; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;

  // ---- LDS -> MFMA operand addressing: lane l reads row l & 31 of a 32-row block, k half l >> 5 ----
  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  const int a_rd = (wm * 128 + l31) * 128;                  // + mi * 4096
  const int b_rd = kAStageBytes + wn * 8192 + lane * 16;    // + j * 4096 + kk * 1024: operands are stored per lane

  constexpr int NF = NB > 0 ? NB : 1;
  bf16x8 fa0[NF], fb0[2], fa1[NF], fb1[2];  // operand fragments of two consecutive k-substeps
#define MOE355_READ_FRAGS(FA, FB, STAGE, KK)                                                           \
  do {                                                                                                 \
    const int slot_ = (((KK) * 2 + khalf) ^ sw) * 16;                                                  \
    _Pragma("unroll") for (int mi = 0; mi < NB; ++mi) FA[mi] =                                         \
        *reinterpret_cast<const bf16x8 *>((STAGE) + a_rd + mi * 4096 + slot_);                         \
    if (NB > 0) {                                                                                      \
      FB[0] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + (KK) * 1024);                         \
      FB[1] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + 4096 + (KK) * 1024);                  \
    }                                                                                                  \
  } while (0)
#define MOE355_MFMAS(FA, FB)                                                                           \
  do {                                                                                                 \
    _Pragma("unroll") for (int mi = 0; mi < NB; ++mi) {                                                \
      acc[mi][0] = mfma_bf16(FA[mi], FB[0], acc[mi][0]);                                               \
      acc[mi][1] = mfma_bf16(FA[mi], FB[1], acc[mi][1]);                                               \
    }                                                                                                  \
  } while (0)

  // Pipeline.  At the top of k-step kt: LDS stage kt & 1 holds slab kt, a register set holds slab kt + 1 (its
  // loads were issued DEPTH k-steps ago, in three portions), and fa0 / fb0 hold the operands of substep 0.
  // Substeps 0..2 each multiply, fetch the next substep's operands, move one portion of the register set into the
  // other stage and reissue that portion's loads for slab kt + 1 + DEPTH, so the global loads, the LDS stores and
  // the LDS reads are all spread under the MFMAs instead of forming a burst around the barrier.  The single
  // barrier sits before substep 3, whose operands are already in registers; substep 3 also fetches substep 0 of
  // the next slab.  Reloads past the last k-step repeat the last slab: in bounds, never used.
  // Requested instruction order (sched_group_barrier masks: 0x008 MFMA, 0x020 VMEM read, 0x100 DS read,
  // 0x200 DS write).
#define MOE355_ORDER(NW)                                                                                \
  do {                                                                                                 \
    if (NB >= 3) {                                                                                     \
      /* the LDS reads two behind each of the first MFMAs, then one staging store and one global load  \
         behind each of the next ones, the rest of the MFMAs last: the LDS queue never sees more than  \
         two requests in a row (measured 3-4 % faster than all reads, all MFMAs, all stores, all       \
         loads; the stores as early as the reads: 7 % slower, they wait for the global loads) */       \
      _Pragma("unroll") for (int i_ = 0; i_ < (NB + 2) / 2; ++i_) {                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                             \
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                             \
      }                                                                                                \
      if ((NB + 2) & 1) {                                                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                             \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                             \
      }                                                                                                \
      _Pragma("unroll") for (int i_ = 0; i_ < (NW); ++i_) {                                            \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                             \
        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                             \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                             \
      }                                                                                                \
      if (2 * NB - (NB + 3) / 2 - (NW) > 0)                                                            \
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NB - (NB + 3) / 2 - (NW), 0);                  \
    } else {                                                                                           \
      if (NB > 0) {                                                                                    \
        __builtin_amdgcn_sched_group_barrier(0x100, NB + 2, 0);                                        \
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NB, 0);                                        \
      }                                                                                                \
      if ((NW) > 0) {                                                                                  \
        __builtin_amdgcn_sched_group_barrier(0x200, (NW), 0);                                          \
        __builtin_amdgcn_sched_group_barrier(0x020, (NW), 0);                                          \
      }                                                                                                \
    }                                                                                                  \
  } while (0)
#define MOE355_KSTEP(S, KT_, KPRE)                                                                      \
  do {                                                                                                 \
    const unsigned char *sCur = smem + ((KT_) & 1) * kStageBytes;                                      \
    const int nxt = ((KT_) & 1) ^ 1;                                                                   \
    const int kp_ = min((KPRE), kt_last);                                                              \
    MOE355_READ_FRAGS(fa1, fb1, sCur, 1);                                                              \
    MOE355_MFMAS(fa0, fb0);                                                                            \
    MOE355_STORE_P0(S, nxt);                                                                           \
    MOE355_LOAD_P0(S, kp_);                                                                            \
    MOE355_READ_FRAGS(fa0, fb0, sCur, 2);                                                              \
    MOE355_MFMAS(fa1, fb1);                                                                            \
    MOE355_STORE_P1(S, nxt);                                                                           \
    MOE355_LOAD_P1(S, kp_);                                                                            \
    MOE355_READ_FRAGS(fa1, fb1, sCur, 3);                                                              \
    MOE355_MFMAS(fa0, fb0);                                                                            \
    MOE355_STORE_P2(S, nxt);                                                                           \
    MOE355_LOAD_P2(S, kp_);                                                                            \
    MOE355_ORDER(NA > 1 ? 3 : 2);                                                                      \
    MOE355_ORDER(NA > 2 ? 3 : 1);                                                                      \
    MOE355_ORDER(2);                                                                                   \
    __syncthreads();                                                                                   \
    MOE355_READ_FRAGS(fa0, fb0, smem + nxt * kStageBytes, 0);                                          \
    MOE355_MFMAS(fa1, fb1);                                                                            \
    MOE355_ORDER(0);                                                                                   \
  } while (0)

  // FP8 k-step: the operands of substeps 0 and 1 (then 2 and 3) sit in fa0 / fa1 and go into one instruction per
  // accumulator; the fragments of the next pair are read once those instructions have been issued, the staging
  // traffic is spread between the two groups as above, and the barrier again sits in front of the last group.
#define MOE355_MFMAS8()                                                                                \
  do {                                                                                                 \
    _Pragma("unroll") for (int mi = 0; mi < NB; ++mi) {                                                \
      acc[mi][0] = mfma_fp8_pair(fa0[mi], fa1[mi], fb0[0], fb1[0], acc[mi][0]);                        \
      acc[mi][1] = mfma_fp8_pair(fa0[mi], fa1[mi], fb0[1], fb1[1], acc[mi][1]);                        \
    }                                                                                                  \
  } while (0)
#define MOE355_KSTEP8(S, KT_, KPRE)                                                                     \
  do {                                                                                                 \
    const unsigned char *sCur = smem + ((KT_) & 1) * kStageBytes;                                      \
    const int nxt = ((KT_) & 1) ^ 1;                                                                   \
    const int kp_ = min((KPRE), kt_last);                                                              \
    MOE355_MFMAS8();                                                                                   \
    MOE355_STORE_P0(S, nxt);                                                                           \
    MOE355_LOAD_P0(S, kp_);                                                                            \
    MOE355_READ_FRAGS(fa0, fb0, sCur, 2);                                                              \
    MOE355_READ_FRAGS(fa1, fb1, sCur, 3);                                                              \
    MOE355_STORE_P1(S, nxt);                                                                           \
    MOE355_LOAD_P1(S, kp_);                                                                            \
    MOE355_STORE_P2(S, nxt);                                                                           \
    MOE355_LOAD_P2(S, kp_);                                                                            \
    __syncthreads();                                                                                   \
    MOE355_MFMAS8();                                                                                   \
    MOE355_READ_FRAGS(fa0, fb0, smem + nxt * kStageBytes, 0);                                          \
    MOE355_READ_FRAGS(fa1, fb1, smem + nxt * kStageBytes, 1);                                          \
  } while (0)

  const int KT = g.n_ktiles;
  const int kt_last = KT - 1;
  MOE355_LOAD_P0(x, 0); MOE355_LOAD_P1(x, 0); MOE355_LOAD_P2(x, 0);
  MOE355_STORE_P0(x, 0); MOE355_STORE_P1(x, 0); MOE355_STORE_P2(x, 0);
  {
    const int k1 = min(1, kt_last);
    MOE355_LOAD_P0(x, k1); MOE355_LOAD_P1(x, k1); MOE355_LOAD_P2(x, k1);
    if (DEPTH == 2) {
      const int k2 = min(2, kt_last);
      MOE355_LOAD_P0(y, k2); MOE355_LOAD_P1(y, k2); MOE355_LOAD_P2(y, k2);
    }
  }
  __syncthreads();
  MOE355_READ_FRAGS(fa0, fb0, smem, 0);
  if (FP8) MOE355_READ_FRAGS(fa1, fb1, smem, 1);

  if (FP8 && DEPTH == 1) {
    for (int kt = 0; kt < KT; ++kt) MOE355_KSTEP8(x, kt, kt + 2);
  } else if (FP8) {
    for (int kt = 0; kt < KT; kt += 2) {
      MOE355_KSTEP8(x, kt, kt + 3);
      if (kt + 1 < KT) MOE355_KSTEP8(y, kt + 1, kt + 4);
    }
  } else if (DEPTH == 1) {
    for (int kt = 0; kt < KT; ++kt) MOE355_KSTEP(x, kt, kt + 2);
  } else {
    // set x carries the odd slabs, set y the even ones
    for (int kt = 0; kt < KT; kt += 2) {
      MOE355_KSTEP(x, kt, kt + 3);
      if (kt + 1 < KT) MOE355_KSTEP(y, kt + 1, kt + 4);
    }
  }
#undef MOE355_KSTEP
#undef MOE355_KSTEP8
#undef MOE355_MFMAS8
#undef MOE355_ORDER
#undef MOE355_READ_FRAGS
#undef MOE355_MFMAS
#undef MOE355_LOAD_P0
#undef MOE355_B_LOAD
#undef MOE355_LOAD_P1
#undef MOE355_LOAD_P2
#undef MOE355_STORE_P0
#undef MOE355_STORE_P1
#undef MOE355_STORE_P2
#undef MOE355_A_OFF

  // ---- epilogue ----
  // Accumulator register r of lane l holds C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 block, i.e. a lane
  // owns one column.  Each wave turns its blocks around through a private LDS patch (the stages are dead now)
  // so that the global stores are 16 bytes per lane along a row instead of one element per lane.
  __syncthreads();  // every wave has finished reading the stages
  // RESIDENT: the ticket of this workgroup's next item is drawn now, by thread 0, so that the atomic's round trip
  // runs under the epilogue instead of in front of the next item; the value is parked in the LDS at the very end.
  int pre_v = -1;
  if (RESIDENT && pre_ctr && threadIdx.x == 0) pre_v = atomicAdd(pre_ctr, 1);
  unsigned char *patch = smem + w8 * kPatchBytes;
  // GEMM-2: the gate weights and the sole-slot marks of this wave's 128 rows come in once, coalesced, and wait in the
  // LDS behind the patches (1 KiB per wave), instead of 24 scattered loads in front of every 32-row block
  float *meta_w = reinterpret_cast<float *>(smem + 8 * kPatchBytes + w8 * 1024);
  int *meta_s = reinterpret_cast<int *>(meta_w + 128);
  if (!GATED && !TRAIN && NB > 0) {
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int row_l = wm * 128 + hh * 64 + lane;
      meta_w[hh * 64 + lane] = row_l < rows ? (g.row_w ? g.row_w[m0 + row_l] : 1.f) : 0.f;
      meta_s[hh * 64 + lane] = (g.row_sole && row_l < rows) ? g.row_sole[m0 + row_l] : -1;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (!GATED && TRAIN && NB > 0) {
    // first backward GEMM: the gate weights of this wave's rows, parked behind the wave's three blocks (which take
    // 13824 of its 16 KiB)
    meta_w = reinterpret_cast<float *>(smem + w8 * 16384 + 13824);
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int row_l = wm * 128 + hh * 64 + lane;
      meta_w[hh * 64 + lane] = row_l < rows ? g.row_w[m0 + row_l] : 0.f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (GATED && FP8 && NB > 0) {
    // FP8 GEMM-1: the same for the scales of the tokens behind this wave's rows (rows past the end repeat the last)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int row_l = min(wm * 128 + hh * 64 + lane, rows - 1);
      meta_w[hh * 64 + lane] = g.a_scale[g.row_map ? g.row_map[m0 + row_l] : m0 + row_l];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  // FP8: the scales of this lane's columns, read once (inside the loop over the blocks the compiler would have to
  // read them again behind every global store).  GEMM-1: scale of the gate and of the up column of h column col_h
  // and the expert's scale of h; GEMM-2: the expert's scale of h times the scales of the lane's two output columns.
  float f8_s0 = 1.f, f8_s1 = 1.f, f8_sh = 1.f;
  if (FP8 && GATED && NB > 0) {
    const int col_h = nt * (kBN / 2) + wn * 32 + l31;
    const float *bs = g.b_scale + (size_t)le * 2 * g.N;
    f8_s0 = col_h < g.N ? bs[col_h] : 0.f;
    f8_s1 = col_h < g.N ? bs[g.N + col_h] : 0.f;
    f8_sh = g.h_scale[le];
  }
  if (FP8 && !GATED && NB > 0) {
    const int c0 = nt * kBN + wn * 64 + l31;
    const float sh = g.h_scale[le];
    f8_s0 = c0 < g.N ? sh * g.b_scale[(size_t)le * g.N + c0] : 0.f;
    f8_s1 = c0 + 32 < g.N ? sh * g.b_scale[(size_t)le * g.N + c0 + 32] : 0.f;
  }
#pragma unroll
  for (int mi = 0; mi < NB; ++mi) {
    const int blk_row0 = wm * 128 + mi * 32;  // first tile row of this 32-row block
    if (!GATED && TRAIN) {
      // This wave's 32 x 64 block of g and of u comes in through the LDS in 16-byte pieces (row pitch 144 bytes, g
      // at 0, u at 4608 of a private 16 KiB region: the stages are dead), every lane replaces the elements it holds
      // accumulators for by dg and du in place and puts w silu(g) u into a third block at 9216, and the three
      // blocks leave in 16-byte pieces.
      unsigned char *blk = smem + w8 * 16384;
      const bf16_t *gu = static_cast<const bf16_t *>(g.aux);
      bf16_t *dgu = static_cast<bf16_t *>(g.out), *hw = static_cast<bf16_t *>(g.aux2);
      const int col0 = nt * kBN + wn * 64;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int c = it * 64 + lane;  // 16-byte chunk: 8 chunks per row
        const int rl = c >> 3, cc = c & 7;
        const int row_l = blk_row0 + rl, col = col0 + cc * 8;
        if (row_l < rows && col < g.N) {
          const bf16_t *src = gu + (size_t)(m0 + row_l) * 2 * g.N + col;
          *reinterpret_cast<u32x4 *>(blk + rl * 144 + cc * 16) = *reinterpret_cast<const u32x4 *>(src);
          *reinterpret_cast<u32x4 *>(blk + 4608 + rl * 144 + cc * 16) = *reinterpret_cast<const u32x4 *>(src + g.N);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // gate weights of the 16 rows this lane holds accumulators for (rows past the end: 0, the math stays finite
      // and nothing of them is stored)
      float wv[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 w4 = *reinterpret_cast<const f32x4 *>(meta_w + mi * 32 + q * 8 + khalf * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) wv[q * 4 + e] = w4[e];
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        // all reads of this half first, then the arithmetic, then all writes: the LDS operations of one kind go
        // out back to back instead of waiting on one another
        const int cb = (j * 32 + l31) * 2;
        float gv[16], uv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
          gv[r] = (float)*reinterpret_cast<const bf16_t *>(blk + rl * 144 + cb);
          uv[r] = (float)*reinterpret_cast<const bf16_t *>(blk + 4608 + rl * 144 + cb);
        }
        bf16_t o_dg[16], o_du[16], o_hw[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-gv[r])), silu = gv[r] * sg;
          const float dh = wv[r] * acc[mi][j][r];
          o_dg[r] = (bf16_t)(dh * uv[r] * (sg * (1.0f + gv[r] * (1.0f - sg))));
          o_du[r] = (bf16_t)(dh * silu);
          o_hw[r] = (bf16_t)(wv[r] * silu * uv[r]);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
          *reinterpret_cast<bf16_t *>(blk + rl * 144 + cb) = o_dg[r];
          *reinterpret_cast<bf16_t *>(blk + 4608 + rl * 144 + cb) = o_du[r];
          *reinterpret_cast<bf16_t *>(blk + 9216 + rl * 144 + cb) = o_hw[r];
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int c = it * 64 + lane;
        const int rl = c >> 3, cc = c & 7;
        const int row_l = blk_row0 + rl, col = col0 + cc * 8;
        if (row_l < rows && col < g.N) {
          bf16_t *dst = dgu + (size_t)(m0 + row_l) * 2 * g.N + col;
          *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(blk + rl * 144 + cc * 16);
          *reinterpret_cast<u32x4 *>(dst + g.N) = *reinterpret_cast<const u32x4 *>(blk + 4608 + rl * 144 + cc * 16);
          *reinterpret_cast<u32x4 *>(hw + (size_t)(m0 + row_l) * g.N + col) =
              *reinterpret_cast<const u32x4 *>(blk + 9216 + rl * 144 + cc * 16);
        }
      }
    } else if (GATED && FP8) {
      // h block: 32 rows x 32 columns of E4M3 codes, row pitch 48 bytes.  g and u get the scales of their token
      // and of their columns; h = silu(g) * u is divided by the expert's scale for h and converted.
      const float sg = f8_s0, su = f8_s1, rsh = __builtin_amdgcn_rcpf(f8_sh);
      f32x4 sx4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) sx4[q] = *reinterpret_cast<const f32x4 *>(meta_w + mi * 32 + q * 8 + khalf * 4);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
        const float sx = sx4[r >> 2][r & 3];
        const float gv = acc[mi][0][r] * (sx * sg), uv = acc[mi][1][r] * (sx * su);
        patch[rl * 48 + l31] = to_e4m3((gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv))) * uv * rsh);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      {
        const int rl = lane >> 1, cc = lane & 1;  // 16-byte chunk: 2 chunks per row
        const int row_l = blk_row0 + rl;
        const int col = nt * (kBN / 2) + wn * 32 + cc * 16;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(patch + rl * 48 + cc * 16);
        if (row_l < rows && col < g.N)
          *reinterpret_cast<u32x4 *>(static_cast<uint8_t *>(g.out) + (size_t)(m0 + row_l) * g.ldo + col) = v;
      }
    } else if (GATED) {
      // h block: 32 rows x 32 columns bf16, row pitch 80 bytes (keeps the two half-waves on different banks);
      // TRAIN: two more such blocks for g and u, 2560 bytes apart
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
        const float gv = acc[mi][0][r], uv = acc[mi][1][r];
        // (the hardware reciprocal, 1 ulp, instead of the correctly rounded division: h is rounded to bf16 next)
        *reinterpret_cast<bf16_t *>(patch + rl * 80 + l31 * 2) =
            (bf16_t)((gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv))) * uv);
        if (TRAIN) {
          *reinterpret_cast<bf16_t *>(patch + 2560 + rl * 80 + l31 * 2) = (bf16_t)gv;
          *reinterpret_cast<bf16_t *>(patch + 5120 + rl * 80 + l31 * 2) = (bf16_t)uv;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int c = it * 64 + lane;        // 16-byte chunk: 4 chunks per row
        const int rl = c >> 2, cc = c & 3;
        const int row_l = blk_row0 + rl;
        const int col = nt * (kBN / 2) + wn * 32 + cc * 8;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(patch + rl * 80 + cc * 16);
        if (row_l < rows && col < g.N) {
          *reinterpret_cast<u32x4 *>(static_cast<bf16_t *>(g.out) + (size_t)(m0 + row_l) * g.ldo + col) = v;
          if (TRAIN) {
            bf16_t *gu = static_cast<bf16_t *>(g.aux) + (size_t)(m0 + row_l) * 2 * g.N + col;
            *reinterpret_cast<u32x4 *>(gu) = *reinterpret_cast<const u32x4 *>(patch + 2560 + rl * 80 + cc * 16);
            *reinterpret_cast<u32x4 *>(gu + g.N) = *reinterpret_cast<const u32x4 *>(patch + 5120 + rl * 80 + cc * 16);
          }
        }
      }
    } else {
      // o block: 32 rows x 64 columns fp32, row pitch 288 bytes.  A row whose token has no other local slot
      // is final already (the Combine sum would have one term): it goes to y in the output type, skipping o.
      // FP8: the scale of the expert's h times the scale of the lane's two output columns
      const float cs0 = f8_s0, cs1 = f8_s1;
      int sole[8];
#pragma unroll
      for (int it = 0; it < 8; ++it) sole[it] = meta_s[mi * 32 + it * 4 + (lane >> 4)];
      f32x4 w4[4];  // gate weights of the 16 rows this lane holds accumulators for (0 past the end)
#pragma unroll
      for (int q = 0; q < 4; ++q) w4[q] = *reinterpret_cast<const f32x4 *>(meta_w + mi * 32 + q * 8 + khalf * 4);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
        float wgt = w4[r >> 2][r & 3];
        if (poison) wgt = __builtin_nanf("");  // the wait for this item's h gave up: mark what it writes
        *reinterpret_cast<float *>(patch + rl * 288 + l31 * 4) = FP8 ? acc[mi][0][r] * cs0 * wgt : acc[mi][0][r] * wgt;
        *reinterpret_cast<float *>(patch + rl * 288 + 128 + l31 * 4) =
            FP8 ? acc[mi][1][r] * cs1 * wgt : acc[mi][1][r] * wgt;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int rl = it * 4 + (lane >> 4), cc = lane & 15;  // 16 chunks of 16 bytes per row
        const int row_l = blk_row0 + rl;
        const int col = nt * kBN + wn * 64 + cc * 4;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 16);
        if (row_l < rows && col < g.N) {
          if (sole[it] >= 0) {
            bf16x4 b;
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = (bf16_t)(v[q] + 0.0f);  // + 0 as in the sum that starts from zero
            // (y is not read again by this launch: streamed past the L2, which the operands need)
            __builtin_nontemporal_store(
                b, reinterpret_cast<bf16x4 *>(static_cast<bf16_t *>(g.y) + (size_t)sole[it] * g.ldo + col));
          } else {
            *reinterpret_cast<f32x4 *>(static_cast<float *>(g.out) + (size_t)(m0 + row_l) * g.ldo + col) = v;
          }
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the patch is reused by the next block
  }
  if (RESIDENT && pre_ctr && threadIdx.x == 0) *pre_slot = pre_v;
}

// One work item on the matrix cores.  Wave-uniform dispatch on the number of valid 32-row blocks: every variant
// executes the same sequence of barriers.  poison != 0 (GEMM-2 inside the resident kernel, after a wait that gave up):
// the rows are written as NaN.
template <bool GATED, bool RESIDENT, bool FP8 = false, bool TRAIN = false>
__device__ __forceinline__ void gemm_bf16_item(const GemmArgs &g, unsigned char *smem, const int4 item,
                                               int poison = 0, int32_t *pre_ctr = nullptr,
                                               int *pre_slot = nullptr) {
  const int le = item.x, m0 = item.y, rows = item.z & kItemRowsMask, nt = item.w & ((1 << kTileShift) - 1);
  // the expert's only M tile (uniform).  Only the resident kernels, which run the layers made of such tiles, have
  // the variants with streaming weight loads: in the per-item kernels they cost six more registers, and those
  // kernels leave 16 registers per SIMD to the kernels that run beside them in the backward pass.
  const bool lone = (item.z & kItemLone) != 0;
  const int nblk_total = (rows + 31) >> 5;                        // 1..8
  const int wm = threadIdx.x >> 8;                                // wave row (wave-uniform)
  const int nb = max(0, min(4, nblk_total - 4 * wm));             // valid 32-row blocks of this wave
#define MOE355_TILE_(NB_, NA_, LONE_)                                                                              \
  gemm_bf16_tile<GATED, RESIDENT, NB_, NA_, (NA_ == 1 ? 2 : 1), FP8, TRAIN, LONE_>(g, smem, nt, le, m0, rows, nblk_total, \
                                                                                 poison, pre_ctr, pre_slot)
#define MOE355_TILE(NB_, NA_)                                                                  \
  do {                                                                                         \
    if (RESIDENT && NA_ > 1 && lone) MOE355_TILE_(NB_, NA_, (RESIDENT && NA_ > 1)); else MOE355_TILE_(NB_, NA_, false); \
  } while (0)
  if (nblk_total <= 2) {
    if (nb == 2) MOE355_TILE(2, 1); else if (nb == 1) MOE355_TILE(1, 1); else MOE355_TILE(0, 1);
  } else if (nblk_total <= 4) {
    if (nb == 4) MOE355_TILE(4, 2); else if (nb == 3) MOE355_TILE(3, 2); else MOE355_TILE(0, 2);
  } else {
    if (nb == 4) MOE355_TILE(4, 4); else if (nb == 3) MOE355_TILE(3, 4); else if (nb == 2) MOE355_TILE(2, 4);
    else MOE355_TILE(1, 4);
  }
#undef MOE355_TILE
#undef MOE355_TILE_
}

// One workgroup per work item; workgroup -> item by chunked_item.
template <bool GATED, bool FP8 = false, bool TRAIN = false>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  const int q = chunked_item(blockIdx.x, *g.n_items);
  if (q < 0) return;
  gemm_bf16_item<GATED, false, FP8, TRAIN>(g, smem, g.work[q]);
}

// ------------------------------------------------------------------------------------------------
// GEMM-1 and GEMM-2 of a layer in ONE launch of resident workgroups (one per CU), the one-GPU form of the
// tile-granular GEMM-1 => GEMM-2 hand-over of the fused kernel (Sec. IV-A, IV-B): a GEMM-2 tile starts as soon
// as the h rows of its M tile are complete, so the CUs that run out of GEMM-1 work (a launch of a few hundred
// tiles of ~100 us ends with many CUs idle) continue with GEMM-2 instead of waiting for a kernel boundary.
// moe_fused_forward uses it for bf16 layers whose experts get less than one full M tile of rows on average: the
// launches are then dominated by partial tiles and, under skewed routing, by the tail of the few large experts
// (measured 5 % faster than two launches on the DeepSeek-shaped skewed load, 1 % slower on the same shape with
// uniform routing).  With fuller experts a whole step is 1-3 % slower than with two launches (7-9 % on layers of
// 0.1-0.2 ms), and the kernel boundary of moe_fused_forward_two_launch is used instead.
//
// Work distribution: both lists are cut into 8 queues exactly as a plain launch would spread them over the XCDs
// (queue x = virtual blocks x, x + 8, ...; see chunked_item); a workgroup draws tickets from its home queue
// (blockIdx % 8, the XCD it runs on) and, when that is empty, from the others.  It moves on to GEMM-2 only after
// it has seen every GEMM-1 queue empty, i.e. when every GEMM-1 item is already in the hands of a running
// workgroup; GEMM-1 items never wait, so the counter a GEMM-2 item polls is always completed by workgroups that
// make progress: no deadlock for any number of resident workgroups and any placement.
// Hand-over: the producers of an M tile store h, fence at device scope, and count themselves in tile_ready;
// the consumer polls the counter, then fences before it loads h (the L2s of the XCDs are not coherent with
// each other, the device-scope fences write back / invalidate them).
// ------------------------------------------------------------------------------------------------
struct PipelineArgs {
  GemmArgs g1, g2;
  int32_t *tickets;     // [16]: queues of GEMM-1, then of GEMM-2
  int32_t *tile_ready;  // [M tiles] GEMM-1 items finished per M tile
  int32_t *error;       // set if a wait gave up (cannot happen unless the lists are corrupt)
  int nt1;              // GEMM-1 items per M tile a GEMM-2 item waits for
  int max_polls;        // bound on the polls of one wait (x ~1 us), so that no wave can wait forever
  // Combine stage (gemm_bf16_combine_kernel only)
  int32_t *tile_done;         // [M tiles] GEMM-2 items finished per M tile
  const int32_t *row_tile;    // [P] M tile of each local row
  const int32_t *topk_idx, *inv_perm, *offsets, *header;
  int T, k, e_lo, E_loc, P_cap, nt2, n_mtiles_cap;
};

constexpr int kMaxPolls = 1 << 22;  // default bound: several seconds

// All items of one GEMM that this workgroup can get hold of: home queue first, then the other queues.
// tile_done (GEMM-2 only, may be null): counter per M tile that every finished item of the tile is counted in, for
// the Combine stage that follows in the same launch; s_done: kDoneCap ints of LDS (tiles of the finished items).
constexpr int kDoneCap = 256;
template <bool GATED, bool FP8 = false, bool TRAIN = false>
__device__ __forceinline__ void gemm_bf16_drain(const GemmArgs &g, unsigned char *smem, int *s_item,
                                                int32_t *__restrict__ tickets, int32_t *__restrict__ tile_ready,
                                                int32_t *__restrict__ error, int nt1, int max_polls,
                                                int32_t *__restrict__ tile_done = nullptr, int *s_done = nullptr) {
  const int home = blockIdx.x & 7;
  const int n_items = *g.n_items;
  const int n_virtual = (n_items + 8 * kChunk - 1) / (8 * kChunk) * (8 * kChunk);
  int qsel = 0;  // queues tried so far, in the order home, home + 1, ... (only thread 0's copy is used)
  // Next list position for this workgroup, or -1 when every queue is empty (thread 0 only).
  // pre >= 0: a ticket of the queue this workgroup is on, drawn ahead under the previous item's epilogue
  auto draw = [&](int pre) {
    int q = -1;
    while (qsel < 8) {
      const int queue = (home + qsel) & 7;
      const int v = queue + 8 * (pre >= 0 ? pre : atomicAdd(&tickets[queue], 1));
      pre = -1;
      if (v < n_virtual) {
        if ((q = chunked_item(v, n_items)) >= 0) break;
        continue;  // a virtual block without an item
      }
      // this queue is empty: read all counters at once and go on with the next queue that still has positions
      // (an empty queue stays empty, so every queue is seen empty before the loop ends)
      unsigned open_queues = 0;  // bit i: queue i still has positions
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = __hip_atomic_load(&tickets[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        open_queues |= (unsigned)(i + 8 * t < n_virtual) << i;
      }
      int next = 8;
#pragma unroll
      for (int i = 7; i >= 1; --i) {
        const int s2 = qsel + i;  // candidate position in the visiting order
        if (s2 < 8 && ((open_queues >> ((home + s2) & 7)) & 1u)) next = s2;
      }
      qsel = next;
    }
    return q;
  };
  // GEMM-2 items that feed Combine in the same launch: the o rows (and the y rows of sole slots) of all items this
  // workgroup has finished become visible device-wide with ONE release, then every item is counted in its M tile's
  // counter.  (A release per item costs an L2 write-back of the fp32 rows each time: measured 4 % of the launch.)
  // Counting late is safe: the items are in the hands of a running workgroup until they are counted.
  int n_pending = 0;  // finished, not yet counted (the same in every thread)
  auto flush_done = [&]() {
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // this wave's stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0 && n_pending > 0) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // the write-back is complete before the counters move
      for (int i = 0; i < n_pending; ++i)
        __hip_atomic_fetch_add(&tile_done[s_done[i]], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    n_pending = 0;
    __syncthreads();  // the list may be overwritten
  };
  // (Drawing the next ticket a whole item ahead, to hide the latency of the atomic, was measured slower: a workgroup
  // that holds a long item while it finishes another one keeps that item from an idle workgroup.  What is drawn
  // ahead here is drawn under the epilogue of the item that is being finished, a few microseconds before it is used.)
  if (threadIdx.x == 0) s_item[2] = -1;
  for (;;) {
    __syncthreads();  // the previous item is done with the LDS (and with *s_item)
    if (threadIdx.x == 0) {
      *s_item = draw(s_item[2]);
      s_item[2] = -1;
    }
    __syncthreads();
    const int q = *s_item;
    if (q < 0) break;  // nothing left in any queue
    const int4 item = g.work[q];
    const int tile = item.w >> kTileShift;
    int32_t *pre_ctr = tickets + ((home + qsel) & 7);  // (thread 0's value is the one that is used)
    if (GATED) {
      gemm_bf16_item<true, true, FP8, TRAIN>(g, smem, item, 0, pre_ctr, s_item + 2);
      // Release side of the hand-over.  Every wave first waits until its own h stores have been acknowledged, so that
      // the one write-back below cannot overtake any of them (a workgroup barrier alone does not wait for global
      // stores).
      __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
      __syncthreads();  // every thread's h stores happen before thread 0's release ...
      if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // ... which writes this XCD's L2 back: visible device-wide
        // The write-back has to be complete before the counter moves.  The compiler places no wait between the two
        // here (the wave has just waited for its stores, and the write-back is not counted as outstanding), so the
        // wait is spelled out.
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        __hip_atomic_fetch_add(&tile_ready[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ... then counted
      }
    } else {
      // Acquire side: thread 0 polls with relaxed device-scope loads (an acquire per poll would invalidate the L2
      // every time), then one acquire fence orders the loads of h after the counter; the barrier hands the result to
      // the workgroup.  A wait that gives up (corrupt lists; cannot happen otherwise) raises the error word and the
      // item runs with a NaN in place of the gate weight, so that nothing computed from incomplete h can pass as a
      // result.
      if (threadIdx.x == 0) {
        int polls = 0, gave_up = 0;
        while (__hip_atomic_load(&tile_ready[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < nt1) {
          __builtin_amdgcn_s_sleep(32);
          if (++polls > max_polls) {
            __hip_atomic_store(error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            gave_up = 1;
            break;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // the invalidate is complete before the barrier lets the others load
        s_item[1] = gave_up;
      }
      __syncthreads();
      gemm_bf16_item<false, true, FP8>(g, smem, item, s_item[1], pre_ctr, s_item + 2);
      if (tile_done) {
        // remembered, counted later (flush_done): one write-back for all the items of this workgroup
        if (threadIdx.x == 0) s_done[n_pending] = tile;
        // (every thread counts: a uniform decision.)  Counting every item at once towards the end of the launch, so
        // that idle workgroups can reduce tokens while the last items run, was measured: no gain, the rows of the
        // last items are what the reduction waits for.
        if (++n_pending == kDoneCap) flush_done();
      }
    }
  }
  if (!GATED && tile_done) flush_done();
}

// ------------------------------------------------------------------------------------------------
// Combine as the last stage of the resident kernel (readiness-gated issue of Sec. IV-C on one GPU): a workgroup
// that has seen every GEMM-2 queue empty turns to the tokens.  One wave per token, tokens dealt round-robin over all
// resident waves.  The wave resolves the token's local slots (one lane per slot), waits until the GEMM-2 items of
// every M tile that holds one of those rows have been counted in tile_done (all of them are in the hands of running
// workgroups by then, so the wait ends), and sums the rows in slot order in fp32, exactly as combine_kernel does:
// bit-identical y.  Tokens with one local slot were written by GEMM-2 itself; tokens with none get zeros.
// Acquire side as in the GEMM-2 wait: relaxed device-scope polls, one acquire fence, then the loads.
// A wait that gives up raises the error word and the token's row is written as NaN.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void resident_combine(const PipelineArgs &p) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int n_waves = gridDim.x * (kGemmThreads / 64);
  const int base = p.offsets[p.e_lo];
  const int P = min(p.header[1], p.P_cap);
  const int d = p.g2.N;
  const float *rows = static_cast<const float *>(p.g2.out);
  bf16_t *y = static_cast<bf16_t *>(p.g2.y);
  for (int t = blockIdx.x * (kGemmThreads / 64) + (tid >> 6); t < p.T; t += n_waves) {  // t is wave-uniform
    const int row = combine_slot_row(p.topk_idx, p.inv_perm, t, p.k, lane, p.e_lo, p.E_loc, base, P);
    const int tile = row >= 0 ? min(max(p.row_tile[row], 0), p.n_mtiles_cap - 1) : 0;
    const uint64_t slots = __ballot(row >= 0);
    const int n = __popcll(slots);
    if (n == 1) continue;  // GEMM-2 has written this token's row
    bf16_t *yrow = y + (size_t)t * d;
    int poison = 0;
    if (n > 1) {
      int polls = 0;
      for (;;) {
        const bool ok = row < 0 || __hip_atomic_load(&p.tile_done[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= p.nt2;
        if (__ballot(!ok) == 0) break;
        __builtin_amdgcn_s_sleep(32);
        if (++polls > p.max_polls) {
          if (lane == 0) __hip_atomic_store(p.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          poison = 1;
          break;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    combine_token_rows<bf16_t, true>(rows, row, slots, d, yrow, lane, poison);
  }
}

__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_pipeline_kernel(const PipelineArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  __shared__ int s_item[3];  // [0] list position drawn by thread 0, [1] its wait gave up, [2] ticket drawn ahead
  gemm_bf16_drain<true>(p.g1, smem, s_item, p.tickets, p.tile_ready, p.error, p.nt1, p.max_polls);
  gemm_bf16_drain<false>(p.g2, smem, s_item, p.tickets + 8, p.tile_ready, p.error, p.nt1, p.max_polls);
}

// The resident kernel with Combine as its third stage: the whole layer after the tile table in one launch.
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_combine_kernel(const PipelineArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  __shared__ int s_item[3];
  gemm_bf16_drain<true>(p.g1, smem, s_item, p.tickets, p.tile_ready, p.error, p.nt1, p.max_polls);
  __shared__ int s_done[kDoneCap];
  gemm_bf16_drain<false>(p.g2, smem, s_item, p.tickets + 8, p.tile_ready, p.error, p.nt1, p.max_polls, p.tile_done,
                         s_done);
  resident_combine(p);
}

// The same resident kernel for the training forward: GEMM-1 also keeps g and u.
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_train_pipeline_kernel(const PipelineArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  __shared__ int s_item[3];
  gemm_bf16_drain<true, false, true>(p.g1, smem, s_item, p.tickets, p.tile_ready, p.error, p.nt1, p.max_polls);
  gemm_bf16_drain<false>(p.g2, smem, s_item, p.tickets + 8, p.tile_ready, p.error, p.nt1, p.max_polls);
}

// The same resident kernel on E4M3 operands.
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_fp8_pipeline_kernel(const PipelineArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  __shared__ int s_item[3];
  gemm_bf16_drain<true, true>(p.g1, smem, s_item, p.tickets, p.tile_ready, p.error, p.nt1, p.max_polls);
  gemm_bf16_drain<false, true>(p.g2, smem, s_item, p.tickets + 8, p.tile_ready, p.error, p.nt1, p.max_polls);
}

}  // namespace moe355
