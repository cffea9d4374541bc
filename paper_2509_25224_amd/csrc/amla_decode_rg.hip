// Absorbed-MLA decode for gfx950 (MI355X): the decode kernels whose output accumulator is laid out query
// row by register.
//
// One workgroup (4 waves, one per SIMD, 512 registers each) owns 128 query rows of one sequence; wave w
// owns rows 32 w .. 32 w + 31 and keeps their Q fragment (144 VGPRs) and their 32 x 512 FP32 output
// accumulator (256 accumulator registers) resident for the whole loop over the 64-key cache blocks.
//
// Per block (one iteration of Algorithm 1 / Algorithm 2):
//   [C1]  S^T = K Q^T, v_mfma_f32_32x32x16_bf16 with A = K rows from LDS and B = the Q fragment: every
//         register of a lane then holds a score of query row lane % 32, so the row max and row sums are
//         in-lane reductions plus one exchange with lane ^ 32.
//   [V1]  online softmax in base 2; the weights are rounded to BF16 straight into MFMA operand layout.
//   [C2]  O += P V, the same MFMA with A = P (query rows) and B = V read from the same LDS tile through
//         the transposing LDS read: the result tile has value column lane % 32 in every lane and query
//         row 8 (i / 4) + 4 (lane / 32) + i % 4 in register i.
//   [V2]  Because a register of the accumulator belongs to two query rows only (one per half of the
//         wave), the rescale O <- O * 2^(m_old - m_new) -- FP32 multiply (Algorithm 1, Eq. (2)) or INT32
//         add on the exponent field (Lemma 3.1, Algorithm 2's N) -- touches just the 16 registers of the
//         rows whose reference moved in this block, typically one or two rows out of 32, instead of all
//         256 registers whenever any row of the wave moved.  That is what lets the accumulator live in
//         AccVGPRs, which VALU instructions reach only through copies.
// KV blocks come HBM -> LDS by direct-to-LDS loads, double buffered; operand reads of both products run a
// few MFMAs ahead of their use.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "amla.h"
#include "amla_device.h"
#include "amla_plan.h"

namespace {

// LDS tile of these kernels, two regions.
//   Region A, the first 64 16-byte chunks of every row (the 512 value columns; K and V operands): 64 rows of 68
//   chunks (64 of data, 4 unused), the chunks of a row permuted within aligned groups of four: chunk c of row r
//   sits at position (c & ~3) | ((c + (r >> 2)) & 3).  With 64 banks of 4 bytes, the 16 lanes a 128-bit read
//   serves per cycle (16 rows, one chunk column) and the 32 lanes a transposing 64-bit read serves per cycle
//   (4 rows x 4 chunk columns) then both touch every bank once; a plain padded row cannot do that for both (the
//   first needs an odd multiple of four banks between rows, the second a multiple of sixteen).
//   Region B, chunks 64 .. 71 of every row (the last 64 of the 576 columns, K operands only): 64 rows of 8 chunks,
//   chunk 64 + c of row r at position c ^ ((r >> 1) & 7).
// The direct-to-LDS loads place the chunks: a load writes one KiB, lane l at + 16 l, and fetches whatever chunk
// belongs there.  Region A takes one load per row, region B one per 8 rows; with rows aligned to loads the
// address of a lane is a shift, an add and a mask away (18 loads per wave and tile, a handful of
// instructions each: they are issued between the MFMAs of the first product and must not cost more issue
// time than an MFMA leaves).
constexpr int kRgRowA = 68 * 16;                      // 1088 bytes between rows of region A
constexpr int kRgRegionA = kBlock * kRgRowA;          // 69632
constexpr int kRgRowB = 8 * 16;
constexpr int kRgTileBytes = kRgRegionA + kBlock * kRgRowB;   // 77824 = 76 KiB
constexpr int kRgLoadsA = kBlock / 4;                 // per wave: rows wave, wave + 4, ...
constexpr int kRgLoadsB = 2;                          // per wave: row groups wave and wave + 4
constexpr int kRgLdsBytes = 2 * kRgTileBytes;         // double buffer, 155648 of the 163840 bytes

// One 16-byte-per-lane direct-to-LDS load from scalar base + per-lane 32-bit offset (lane l lands at lds + 16 l,
// lds wave-uniform), issued from inline assembly like AMLA_HIDDEN_LDS_LOAD and for the same reason.
#ifndef AMLA_TARGET_HOOKS
// Three instructions: the LDS address is lds (wave-uniform, in an SGPR) plus a compile-time constant, added
// straight into M0; the global address is base (SGPR pair) + off (per lane) + a compile-time constant, added by the
// vector instruction that also fills the wait state between the M0 write and the load.
#define AMLA_HIDDEN_LDS_LOAD_AT(base, off, off_const, lds, lds_const)                                         \
  do {                                                                                                       \
    unsigned amla_voff_;                                                                                     \
    asm volatile("s_add_u32 m0, %2, %4\n\tv_add_u32 %0, %5, %1\n\tglobal_load_lds_dwordx4 %0, %3"           \
                 : "=&v"(amla_voff_)                                                                         \
                 : "v"(off), "s"(__builtin_amdgcn_readfirstlane((unsigned)(__UINTPTR_TYPE__)(lds))),         \
                   "s"(base), "n"(lds_const), "n"(off_const)                                                 \
                 : "memory", "m0", "scc");                                                                   \
  } while (0)
#else
#define AMLA_HIDDEN_LDS_LOAD_AT(base, off, off_const, lds, lds_const) \
  AMLA_HIDDEN_LDS_LOAD((base) + (off) + (off_const), (lds) + (lds_const))
#endif

// Per-lane constants of the tile loads.  Everything wave-uniform in a load's global address goes into its scalar
// base, so that issuing a load takes no vector instruction: with one wave per SIMD every instruction costs
// issue time that an MFMA's 32 cycles have to cover.
struct TileLoadLane {
  unsigned c16[4];   // region A: byte offset within the row of the chunk that lives at position lane, for row permutation 0 .. 3
  unsigned off_b;    // region B: byte offset of this lane's chunk within an 8-row group
};
__device__ __forceinline__ TileLoadLane tile_load_lane(const int wave, const int lane) {
  TileLoadLane t;
  // region A, load k: row i = wave + 4 k, whose permutation is (i >> 2) & 3 = k & 3; position l holds chunk
  // (l & ~3) | ((l - k) & 3)
#pragma unroll
  for (int k = 0; k < 4; ++k) t.c16[k] = 16u * (unsigned)((lane & ~3) | ((lane - k) & 3));
  // region B, rows 8 m + (lane >> 3) of row group m = wave + 4 k: (4 m) & 7 = 4 (wave & 1) whatever k
  const int c8 = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
  t.off_b = (unsigned)((lane >> 3) * kRowBytes + 64 * 16 + c8 * 16);
  return t;
}
// load n (0 .. 17) of this wave's share of a tile: 16 rows of region A (i = wave + 4 n), then two 8-row groups of
// region B (m = wave + 4 (n - 16))
template <int N>
__device__ __forceinline__ void issue_tile_load(const uint8_t* block_base, LDS_PTR(uint8_t) buf, const int wave,
                                                const TileLoadLane& t) {
  if constexpr (N < kRgLoadsA) {
    AMLA_HIDDEN_LDS_LOAD_AT(block_base + wave * kRowBytes, t.c16[N & 3], 4 * N * kRowBytes, buf + wave * kRgRowA,
                            4 * N * kRgRowA);
  } else {
    AMLA_HIDDEN_LDS_LOAD_AT(block_base + wave * 8 * kRowBytes, t.off_b, 4 * (N - kRgLoadsA) * 8 * kRowBytes,
                            buf + wave * 1024, kRgRegionA + 4 * (N - kRgLoadsA) * 1024);
  }
}
constexpr int kRgLoadsPerWave = kRgLoadsA + kRgLoadsB;   // 18

constexpr int kKAhead = 4;   // [C1]: K operands read this many MFMAs ahead
constexpr int kVAhead = 4;   // [C2]: V operands read this many MFMAs ahead

// acc + the two BF16 values packed in w, in FP32: one dot-product instruction with a pair of ones
#ifndef AMLA_TARGET_HOOKS
__device__ __forceinline__ float bf16_pair_sum(const unsigned w, const float acc) {
  const unsigned ones = 0x3f803f80u;
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, ones), acc, false);
}
#endif

// max of x over the two lanes l and l ^ 32: one cross-half register swap, no LDS
#ifndef AMLA_TARGET_HOOKS
__device__ __forceinline__ float max_over_halves(const float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
#endif

__device__ __forceinline__ float lane_value(float x, int src_lane) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(4 * src_lane, __float_as_int(x)));
}

// ---- the output accumulator: a register file of its own ------------------------------------------------------
// The 32 x 512 FP32 accumulator of a wave is the wave's 256 AccVGPRs, addressed by name: tile dt (value columns
// 32 dt .. 32 dt + 31) is a[16 dt : 16 dt + 15], register i of it holds query row 8 (i / 4) + 4 (lane / 32) + i % 4.
// Every access goes through the few assembly statements below, so the compiler never sees the accumulator as
// a value: it cannot move it, split it or copy it, and it allocates no AccVGPR itself (the library is built
// with MFMA results of the first product in VGPRs; the build checks the compiled kernels for stray AccVGPR
// uses).  What the compiler cannot see it cannot protect either, so the wait states these instructions need
// are written out here:
//   * an MFMA's operands come from VALU-written VGPRs (the packed weights): two idle states lead the product;
//   * consecutive MFMAs of the second product use different tiles, a tile recurs after 16 MFMAs;
//   * a rescale reads registers last written by the previous block's second product, which lies a whole first
//     product and softmax back (the shift depends on them), and is followed by idle states before the next
//     MFMA reads what it wrote;
//   * the epilogue waits for the last MFMA to drain before it copies the accumulator out.
#ifndef AMLA_TARGET_HOOKS
// Every statement that writes the accumulator names all 256 AccVGPRs as clobbered: no value of the compiler's
// can then live in an AccVGPR across it (the register allocator would otherwise park loop-invariant values
// there, to be overwritten by the MFMAs it cannot see).
#define AMLA_ACC_A10(n) "a" #n "0", "a" #n "1", "a" #n "2", "a" #n "3", "a" #n "4", "a" #n "5", "a" #n "6", "a" #n "7", "a" #n "8", "a" #n "9"
#define AMLA_ACC_ALL                                                                                                  \
  "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", AMLA_ACC_A10(1), AMLA_ACC_A10(2), AMLA_ACC_A10(3),      \
      AMLA_ACC_A10(4), AMLA_ACC_A10(5), AMLA_ACC_A10(6), AMLA_ACC_A10(7), AMLA_ACC_A10(8), AMLA_ACC_A10(9),           \
      AMLA_ACC_A10(10), AMLA_ACC_A10(11), AMLA_ACC_A10(12), AMLA_ACC_A10(13), AMLA_ACC_A10(14), AMLA_ACC_A10(15),     \
      AMLA_ACC_A10(16), AMLA_ACC_A10(17), AMLA_ACC_A10(18), AMLA_ACC_A10(19), AMLA_ACC_A10(20), AMLA_ACC_A10(21),     \
      AMLA_ACC_A10(22), AMLA_ACC_A10(23), AMLA_ACC_A10(24), "a250", "a251", "a252", "a253", "a254", "a255"
template <int DT>
__device__ __forceinline__ void acc_mfma(const bf16x8 a, const bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 a[%2*16:%2*16+15], %0, %1, a[%2*16:%2*16+15]"
               :
               : "v"(a), "v"(b), "n"(DT)
               : AMLA_ACC_ALL);
}
// tile DT <- 0: one MFMA with a zero addend and zero operands instead of sixteen register writes
template <int DT>
__device__ __forceinline__ void acc_clear_tile() {
  const bf16x8 z = __builtin_bit_cast(bf16x8, i32x4{0, 0, 0, 0});
  // (two idle states first: the zero operand may have been written by the VALU instruction just before)
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 a[%1*16:%1*16+15], %0, %0, 0" : : "v"(z), "n"(DT) : AMLA_ACC_ALL);
}
template <int R>
__device__ __forceinline__ float acc_read() {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(R));
  return x;
}
// The rescale of register I of all 16 tiles (the two query rows that own it), one statement: FP32 multiply, or
// Lemma 3.1 with a guard.  Two forms of the guard:
//   * any n23 (ADD_COMP: the shift may carry a mantissa term of either sign): as in exponent_add(), saturating
//     INT32 add, then max with the sign bit;
//   * n23 <= 0 (ADD: the reference only rises): saturating INT32 add, then the UNSIGNED minimum with x itself.
//     Inside the lemma's range the sum is below x as an unsigned number for either sign and is kept.  A negative
//     x whose exponent would drop below zero saturates to 0x80000000 = -0.0, which is below x too; a positive
//     one wraps to a negative integer, above x as an unsigned number, and x stays as it is -- an element below
//     2^(|delta| - 127) <= 2^-97 (+0.0 among them) is left unscaled instead of flushed, the same to any tolerance,
//     and the guard is one instruction instead of two.
// Four tiles travel together through the statement, each in registers of its own, so that an instruction's
// operands were written four instructions earlier: one dependent chain per tile would run at the VALU's
// result latency instead of its issue rate.
#define AMLA_ACC_EACH_FOUR(M) M(0, 16, 32, 48) M(64, 80, 96, 112) M(128, 144, 160, 176) M(192, 208, 224, 240)
#define AMLA_ACC_RD(r, off) "v_accvgpr_read_b32 " r ", a[%[i]+" #off "]\n\t"
#define AMLA_ACC_WR(r, off) "v_accvgpr_write_b32 a[%[i]+" #off "], " r "\n\t"
#define AMLA_ACC_RD4(o0, o1, o2, o3) AMLA_ACC_RD("%[x0]", o0) AMLA_ACC_RD("%[x1]", o1) AMLA_ACC_RD("%[x2]", o2) AMLA_ACC_RD("%[x3]", o3)
#define AMLA_ACC_SCALE_FOUR(o0, o1, o2, o3)                                                                  \
  AMLA_ACC_RD4(o0, o1, o2, o3)                                                                               \
  "v_mul_f32 %[x0], %[x0], %[f]\n\tv_mul_f32 %[x1], %[x1], %[f]\n\tv_mul_f32 %[x2], %[x2], %[f]\n\tv_mul_f32 %[x3], %[x3], %[f]\n\t" \
  AMLA_ACC_WR("%[x0]", o0) AMLA_ACC_WR("%[x1]", o1) AMLA_ACC_WR("%[x2]", o2) AMLA_ACC_WR("%[x3]", o3)
#define AMLA_ACC_ADD_FOUR(o0, o1, o2, o3)                                                                    \
  AMLA_ACC_RD4(o0, o1, o2, o3)                                                                               \
  "v_and_b32 %[y0], 0x80000000, %[x0]\n\tv_and_b32 %[y1], 0x80000000, %[x1]\n\t"                             \
  "v_and_b32 %[y2], 0x80000000, %[x2]\n\tv_and_b32 %[y3], 0x80000000, %[x3]\n\t"                             \
  "v_add_i32 %[x0], %[x0], %[f] clamp\n\tv_add_i32 %[x1], %[x1], %[f] clamp\n\t"                             \
  "v_add_i32 %[x2], %[x2], %[f] clamp\n\tv_add_i32 %[x3], %[x3], %[f] clamp\n\t"                             \
  "v_max_i32 %[x0], %[x0], %[y0]\n\tv_max_i32 %[x1], %[x1], %[y1]\n\t"                                       \
  "v_max_i32 %[x2], %[x2], %[y2]\n\tv_max_i32 %[x3], %[x3], %[y3]\n\t"                                       \
  AMLA_ACC_WR("%[x0]", o0) AMLA_ACC_WR("%[x1]", o1) AMLA_ACC_WR("%[x2]", o2) AMLA_ACC_WR("%[x3]", o3)
#define AMLA_ACC_LOWER_FOUR(o0, o1, o2, o3)                                                                  \
  AMLA_ACC_RD4(o0, o1, o2, o3)                                                                               \
  "v_add_i32 %[y0], %[x0], %[f] clamp\n\tv_add_i32 %[y1], %[x1], %[f] clamp\n\t"                             \
  "v_add_i32 %[y2], %[x2], %[f] clamp\n\tv_add_i32 %[y3], %[x3], %[f] clamp\n\t"                             \
  "v_min_u32 %[y0], %[y0], %[x0]\n\tv_min_u32 %[y1], %[y1], %[x1]\n\t"                                       \
  "v_min_u32 %[y2], %[y2], %[x2]\n\tv_min_u32 %[y3], %[y3], %[x3]\n\t"                                       \
  AMLA_ACC_WR("%[y0]", o0) AMLA_ACC_WR("%[y1]", o1) AMLA_ACC_WR("%[y2]", o2) AMLA_ACC_WR("%[y3]", o3)
#define AMLA_ACC_X4 [x0] "=&v"(x0), [x1] "=&v"(x1), [x2] "=&v"(x2), [x3] "=&v"(x3)
#define AMLA_ACC_Y4 [y0] "=&v"(y0), [y1] "=&v"(y1), [y2] "=&v"(y2), [y3] "=&v"(y3)
template <int I>
__device__ __forceinline__ void acc_scale_rows(const float factor) {
  int x0, x1, x2, x3;
  asm volatile(AMLA_ACC_EACH_FOUR(AMLA_ACC_SCALE_FOUR) : AMLA_ACC_X4 : [f] "v"(factor), [i] "n"(I) : AMLA_ACC_ALL);
}
template <int I>
__device__ __forceinline__ void acc_exponent_add_rows(const int n23) {
  int x0, x1, x2, x3, y0, y1, y2, y3;
  asm volatile(AMLA_ACC_EACH_FOUR(AMLA_ACC_ADD_FOUR) : AMLA_ACC_X4, AMLA_ACC_Y4 : [f] "v"(n23), [i] "n"(I) : AMLA_ACC_ALL);
}
// the same for n23 <= 0
template <int I>
__device__ __forceinline__ void acc_exponent_lower_rows(const int n23) {
  int x0, x1, x2, x3, y0, y1, y2, y3;
  asm volatile(AMLA_ACC_EACH_FOUR(AMLA_ACC_LOWER_FOUR) : AMLA_ACC_X4, AMLA_ACC_Y4 : [f] "v"(n23), [i] "n"(I) : AMLA_ACC_ALL);
}
__device__ __forceinline__ void acc_idle(void) { asm volatile("s_nop 7"); }
// x stays where it is in the instruction stream, and nothing of the compiler's lives in an AccVGPR across this point
// (between two statements that name the accumulator it would otherwise be free to put short-lived operands there)
#define AMLA_PIN(x) asm volatile("" : "+v"(x) : : AMLA_ACC_ALL)
// the kernel owns every AccVGPR from here on
__device__ __forceinline__ void acc_claim(void) { asm volatile("" : : : AMLA_ACC_ALL); }
#endif

template <int N, class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl<N>(f, std::make_integer_sequence<int, N>{});
}

// One piece of the decode loop: blocks [j0, j1) of sequence b for the 128 rows of row tile `tile`, one
// softmax state per row, result written in final form (to_final) or as an FP32 partial row set starting at
// row part_row0 of the workspace.  causal_shift (per lane: keys between this lane's row limit and the
// sequence's end; kNoKeys for the row of a padding token) and mask_span (wave-uniform: the piece's largest
// shift) are 0 without a mask.
template <int VARIANT, bool MASKED, bool ITER512>
__device__ __forceinline__ void decode_piece(const DecodeParams& p, LDS_PTR(uint8_t) smem, const int lane,
                                             const int wave, const int b, const int kv_len, const int j0,
                                             const int j1, const int tile, const bool to_final,
                                             const size_t part_row0, const int causal_shift, const int mask_span,
                                             const bool first_piece, const bool have_entry = false,
                                             const int entry = 0) {
  const int l32 = lane & 31;
  const int h = lane >> 5;
  const int row = tile * kRowsPerWg + wave * 32 + l32;   // this lane's query row within the sequence
  const size_t grow = (size_t)b * p.rows + (row < p.rows ? row : 0);

  float m_run = -INFINITY;   // running row max of t = s * scale * log2 e
  float ref = 0.f;           // reference subtracted in the exponent: m_run (MUL), rint(m_run) (ADD),
                             // m_run - log2 S16 (ADD_COMP)
  float mu_run = 0.f;        // ADD_COMP: rint(m_run) = -n_i
  float c_run = 1.f;         // ADD_COMP: c_i = S16 / S32
  float l_f32 = 0.f;         // sum of 2^(t - ref) in FP32 (feeds lse), over this half-wave's keys
  float l_b16 = 0.f;         // sum of the BF16-rounded weights (normalises the output), over this half-wave's keys

  const int32_t* tab = p.table + (size_t)b * p.max_blocks;
  const uint8_t* kvb = reinterpret_cast<const uint8_t*>(p.kv);
  const size_t blk_bytes = (size_t)kBlock * kRowBytes;
  auto phys_of = [&](int j) {
    return min(max(__builtin_amdgcn_readfirstlane(AMLA_UNIFORM_LOAD_I32(tab, j)), 0), p.num_blocks - 1);
  };
  // The block-table entry of the first block is asked for first (a memory round trip of its own), then the
  // query rows; the first tile's loads follow as soon as the entry is there.  (have_entry: the caller already
  // holds table entry j0.)
  const int first_entry = have_entry ? entry : j0 < j1 ? AMLA_UNIFORM_LOAD_I32(tab, j0) : 0;
  __builtin_amdgcn_sched_barrier(0);

  // A wave none of whose 32 rows exists (fewer than 128 heads x tokens in the last row tile: 16 heads of a
  // tensor-parallel shard leave three of the four waves without a row) takes no part in the arithmetic.  Such
  // waves fetch the tiles instead, all 72 loads of each dealt among them, so the waves that work issue none;
  // they also clear the slots past the sequence's end and pass every barrier the working waves pass, in the
  // same order.  Their matrix and vector pipes stay idle, which on a chip that runs this loop at its power
  // limit is clock for the waves that work.
  const int working_waves = min(kThreads / 64, (p.rows - tile * kRowsPerWg + 31) / 32);   // workgroup-uniform, >= 1
  const bool fetch_own_share = working_waves == kThreads / 64;
  if (wave >= working_waves) {   // wave-uniform
    const int first_phys = min(max(__builtin_amdgcn_readfirstlane(first_entry), 0), p.num_blocks - 1);
    if (!first_piece) __syncthreads();
    const TileLoadLane tl_even = tile_load_lane(0, lane), tl_odd = tile_load_lane(1, lane);
    const int fetchers = kThreads / 64 - working_waves, me = wave - working_waves;
    auto fetch_tile = [&](const uint8_t* block, LDS_PTR(uint8_t) to) {
      // load n of wave w's share is slot 4 n + w; a fetching wave takes the slots congruent to its number
      static_for<kRgLoadsPerWave>([&](auto k) {
        for (int w = 0; w < kThreads / 64; ++w)
          if ((4 * k.value + w) % fetchers == me) issue_tile_load<k.value>(block, to, w, (w & 1) ? tl_odd : tl_even);
      });
    };
    if (j0 < j1) fetch_tile(kvb + (size_t)first_phys * blk_bytes, smem);
    for (int j = j0; j < j1; ++j) {
      LDS_PTR(uint8_t) buf = smem + ((j - j0) & 1) * kRgTileBytes;
      LDS_PTR(uint8_t) nxt = smem + ((j + 1 - j0) & 1) * kRgTileBytes;
      AMLA_WAIT_TILE_LOADS();
      __syncthreads();
      const int rem = kv_len - j * kBlock;
      if (rem < kBlock) {
        for (int c = (int)threadIdx.x; c < (kBlock - rem) * (kRowBytes / 16); c += kThreads) {
          const int r = rem + c / (kRowBytes / 16), cc = c % (kRowBytes / 16);
          LDS_PTR(uint8_t) at = cc < 64 ? buf + r * kRgRowA + cc * 16 : buf + kRgRegionA + r * kRgRowB + (cc - 64) * 16;
          *(LDS_PTR(i32x4))at = i32x4{0, 0, 0, 0};
        }
        __syncthreads();
      }
      if (j + 1 < j1) fetch_tile(kvb + (size_t)phys_of(j + 1) * blk_bytes, nxt);
    }
    return;
  }

  // Q fragment: B operand of S^T = K Q^T.  Lane holds q[row][16 ks + 8 h .. + 7].  Rows past the end of the
  // sequence's row range read row 0 (valid memory); their results are never stored.
  bf16x8 qf[kDqk / 16];
  const i32x4* qrow = reinterpret_cast<const i32x4*>(p.q + grow * kDqk) + h;
#pragma unroll
  for (int ks = 0; ks < kDqk / 16; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, qrow[2 * ks]);
  __builtin_amdgcn_sched_barrier(0);
  const int first_phys = min(max(__builtin_amdgcn_readfirstlane(first_entry), 0), p.num_blocks - 1);

  // the previous piece's last tile may still be read by a slower wave
  if (!first_piece) __syncthreads();
  const TileLoadLane tl = tile_load_lane(wave, lane);
  if (j0 < j1 && fetch_own_share) {
    const uint8_t* first = kvb + (size_t)first_phys * blk_bytes;
    static_for<kRgLoadsPerWave>([&](auto k) { issue_tile_load<k.value>(first, smem, wave, tl); });
  }

  // (The first tile and the query rows are on their way; the accumulator is cleared under their latency.)
  // accumulator register 16 dt + i: value column 32 dt + l32, query row 32 wave + 8 (i / 4) + 4 h + i % 4
  static_for<kDv / 32>([&](auto dt) { acc_clear_tile<dt.value>(); });

  // The query rows are waited for here: the tile loads are hidden from the compiler's wait counting, and a wait
  // for these loads left inside the loop would be a wait for the tile.
#pragma unroll
  for (int ks = 0; ks < kDqk / 16; ++ks) AMLA_ARRIVED(qf[ks]);

  // per-lane LDS offsets of the operand reads (see the tile layout above)
  // [C1] A operand, steps 0 .. 31 (region A): row l32 (+ 32 for the second key tile), chunk 2 ks + h; even and
  // odd steps differ in the chunk's low bits only, so two bases and immediate offsets cover these 64 reads
  const int k_even = l32 * kRgRowA + 16 * ((h + (l32 >> 2)) & 3);
  const int k_odd = l32 * kRgRowA + 16 * ((h + (l32 >> 2) + 2) & 3);
  // steps 32 .. 35 (region B): chunk 2 q + h of the row's last eight at position (2 q + h) ^ ((row >> 1) & 7)
  const int k_tail = kRgRegionA + l32 * kRgRowB + 16 * (h ^ ((l32 >> 1) & 1));
  const int k_tail_x = (l32 >> 2) & 3;                              // bits 1 .. 2 of the permutation: q ^ this
  // [C2] B operand through the transposing read: 16 lanes fetch 4 keys x 16 value columns; the second half
  // of a 16-key step lies 8 rows on, where the permutation is 2 further
  const int g16 = lane >> 4, i16 = lane & 15;
  const int v_row = 4 * (g16 >> 1) + (i16 >> 2);
  const int v_chk = 2 * (g16 & 1) + ((i16 & 3) >> 1);
  const int v_lo = v_row * kRgRowA + 16 * ((v_chk + (g16 >> 1)) & 3) + 8 * (i16 & 1);
  const int v_hi = (v_row + 8) * kRgRowA + 16 * ((v_chk + (g16 >> 1) + 2) & 3) + 8 * (i16 & 1);

  for (int j = j0; j < j1; ++j) {
    LDS_PTR(uint8_t) buf = smem + ((j - j0) & 1) * kRgTileBytes;
    LDS_PTR(uint8_t) nxt = smem + ((j + 1 - j0) & 1) * kRgTileBytes;
    // Block j has landed for this wave; the barrier makes that true for all waves and also guarantees that
    // everyone is done reading the other buffer, which is refilled next.
    AMLA_WAIT_TILE_LOADS();
    __syncthreads();
    // the next block streams in under the first product: its loads are issued between the MFMAs there
    const bool more = j + 1 < j1;
    const uint8_t* next_block = kvb + (size_t)(more ? phys_of(j + 1) : 0) * blk_bytes;

    const int rem = kv_len - j * kBlock;           // valid keys in this block (>= 1)
    if (rem < kBlock) {
      // Slots past the sequence's end belong to nobody: their weights are zero, but 0 * NaN would still
      // poison the value product, so the rows are cleared in LDS before anyone reads them.
      for (int c = (int)threadIdx.x; c < (kBlock - rem) * (kRowBytes / 16); c += kThreads) {
        const int r = rem + c / (kRowBytes / 16), cc = c % (kRowBytes / 16);
        LDS_PTR(uint8_t) at = cc < 64 ? buf + r * kRgRowA + cc * 16 : buf + kRgRegionA + r * kRgRowB + (cc - 64) * 16;
        *(LDS_PTR(i32x4))at = i32x4{0, 0, 0, 0};
      }
      __syncthreads();
    }

    // The block is worked as two sub-blocks of 32 keys, each one iteration of the online softmax, so that the
    // vector work of one sub-block runs while the matrix pipe is busy with the other's product (a wave issues
    // in order, but an MFMA keeps its pipe for 32 cycles and independent VALU instructions issue behind it):
    //   phase A  S0^T = K[0:32] Q^T                      | the next tile's loads
    //   phase B  S1^T = K[32:64] Q^T                     | softmax of sub-block 0
    //            rescale for sub-block 0
    //   phase C  O += P0 V[0:32]                         | softmax of sub-block 1
    //            rescale for sub-block 1
    //   phase D  O += P1 V[32:64]
    // The softmax is cut into chunks of at most about seven VALU issue slots, one chunk behind each MFMA.
    f32x16 s0 = f32x16{0}, s1 = f32x16{0};
    bf16x8 ka[kKAhead];
    auto k_addr = [&](int ks, int kt) {
      if (ks < 32) return buf + ((ks & 1) ? k_odd : k_even) + kt * 32 * kRgRowA + (ks >> 1) * 64;
      return buf + k_tail + 32 * ((ks - 32) ^ k_tail_x) + kt * 32 * kRgRowB;
    };
    constexpr int kSteps = kDqk / 16;   // 36 MFMAs per sub-block of the first product

    // softmax state of the sub-block in flight
    float mxp = 0.f;       // partial row max
    float alpha = 1.f;     // factor on the old row sums (MUL, ADD_COMP) and, for MUL, on the old accumulator
    int n23 = 0;           // ADD: (n_i - n_{i-1}) << 23, <= 0; ADD_COMP: plus the mantissa term
    float psum = 0.f, bsum = 0.f, p_even = 0.f;
    unsigned pk[16];
    const int rem_row = MASKED ? rem - causal_shift : rem;
    const bool masked_block = MASKED ? rem < kBlock + mask_span : rem < kBlock;

    // chunk C of the softmax of sub-block SB (scores T).  The empty assembly statements pin a chunk's inputs and
    // results to its place in the instruction stream (pure arithmetic would otherwise sink to its first use,
    // behind the MFMAs it is meant to run under).
    float m_new = 0.f, m_use = 0.f, p_odd = 0.f;
    auto softmax_chunk = [&](auto sbc, auto cc, f32x16& T, auto&& mid) {
      constexpr int SB = sbc.value, C = cc.value;
      constexpr bool pins_first = C == 0 || (C >= 5 && C < 5 + 24 && (C - 5) % 3 < 2);
      if constexpr (!pins_first) mid();
      if constexpr (C == 0) {
        if (masked_block) {
          // with the causal mask a row's own limit lies causal_shift keys before the sequence's end
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = 32 * SB + 4 * h + 8 * (r >> 2) + (r & 3);
            if (key >= rem_row) T[r] = -INFINITY;
          }
        }
        AMLA_OPAQUE(T);
        mid();
        mxp = fmaxf(fmaxf(T[0], T[1]), T[2]);
        mxp = fmaxf(fmaxf(mxp, T[3]), T[4]);
        mxp = fmaxf(fmaxf(mxp, T[5]), T[6]);
        mxp = fmaxf(fmaxf(mxp, T[7]), T[8]);
        AMLA_OPAQUE(mxp);
      } else if constexpr (C == 1) {
        mxp = fmaxf(fmaxf(mxp, T[9]), T[10]);
        mxp = fmaxf(fmaxf(mxp, T[11]), T[12]);
        mxp = fmaxf(fmaxf(mxp, T[13]), T[14]);
        mxp = fmaxf(mxp, T[15]);
        AMLA_OPAQUE(mxp);
      } else if constexpr (C == 2) {
        mxp = max_over_halves(mxp);
        AMLA_OPAQUE(mxp);
      } else if constexpr (C == 3) {
        m_new = fmaxf(m_run, mxp * p.scale_log2e);
        // Under a mask a row may have seen no key yet: it starts its recurrence at the first sub-block that holds
        // one, and until then keeps a finite reference so that its weights are 2^(-inf) = 0 and not NaN.
        m_use = MASKED ? (m_new == -INFINITY ? 0.f : m_new) : m_new;
        AMLA_OPAQUE(m_new);
        if (MASKED) AMLA_OPAQUE(m_use);
      } else if constexpr (C == 4) {
        if (!MASKED) m_use = m_new;
        const bool first = MASKED ? ((j == j0 && SB == 0) || m_run == -INFINITY) : (j == j0 && SB == 0);
        float ref_new;
        bool keep = false;   // wave-uniform; only ever true with ITER512
        alpha = 1.f;
        n23 = 0;
        if constexpr (SB == 0 && VARIANT != AMLA_RESCALE_ADD_COMP) {
          // The reference is brought up to the running maximum once per 64-key block, behind the second
          // sub-block (the block size of Algorithm 1 / Algorithm 2 stays the cache block).  The first sub-block
          // keeps the previous block's reference when no row's maximum has left it by more than 2^8: its
          // weights are then at most 2^8 instead of 1 -- the same relative precision in BF16 and FP32 -- and the
          // accumulator is rescaled once per block instead of twice.  Otherwise, and in a piece's first block,
          // the sub-block moves the reference itself.
          const bool far = first || m_new - ref > 8.f;
          if (j != j0 && __builtin_amdgcn_ballot_w64(far) == 0) {
            m_run = m_new;
            psum = 0.f;
            bsum = 0.f;
            AMLA_OPAQUE(m_run);
            return;
          }
        }
        if constexpr (SB == 1 && ITER512) {
          // AMLA_FLAG_ITERATION_512: the iteration of the recurrence is eight cache blocks (the KV block of
          // Section 4.2), so the second sub-block of every block but the iteration's last keeps the reference in the
          // same way -- here without a branch (the new reference is the old one, so the shift is 0 and the factor
          // 2^0): measured cheaper in this phase.
          const bool far = first || m_new - ref > 8.f;
          keep = ((j - j0) & 7) != 7 && __builtin_amdgcn_ballot_w64(far) == 0;
        }
        if (VARIANT == AMLA_RESCALE_ADD_COMP) {
          // Algorithm 2's compensation (S32, S16, c_i, eps, N) in base 2: S32 = 2^(m - mu) in [2^-1/2, 2^1/2], S16 its
          // BF16 rounding, weights 2^(t - m) S16 = 2^(t - (m - log2 S16)); the shift of the exponent field and the
          // mantissa nudge 1.5 eps 2^23 travel in one integer
          const float mu = __builtin_rintf(m_use);
          const float s32 = fast_exp2(m_use - mu);
          const float s16 = __uint_as_float(pack_bf16(s32, 0.f) << 16);
          const float c_new = s16 / s32;
          ref_new = m_use - fast_log2(s16);
          if (!first) {
            const float eps = 1.5f * (c_new / c_run - 1.f);
            n23 = max((int)(mu_run - mu), -30) * (1 << 23) + (int)__builtin_rintf(eps * 8388608.f);
            alpha = fast_exp2(ref - ref_new);
          }
          mu_run = mu;
          c_run = c_new;
        } else if (VARIANT == AMLA_RESCALE_MUL) {
          ref_new = ITER512 && keep ? ref : m_use;
          if (!first) alpha = fast_exp2(ref - ref_new);
        } else {
          ref_new = ITER512 && keep ? ref : __builtin_rintf(m_use);
          if (!first) n23 = max((int)(ref - ref_new), -30) * (1 << 23);
        }
        m_run = m_new;
        ref = ref_new;
        psum = 0.f;
        bsum = 0.f;
        AMLA_OPAQUE(ref);
        if (VARIANT == AMLA_RESCALE_MUL)
          AMLA_OPAQUE(alpha);
        else
          AMLA_OPAQUE(n23);
      } else if constexpr (C < 5 + 24) {
        // the 16 weights, a pair per three chunks: two exponentials, then the sums and the BF16 pair
        constexpr int q = (C - 5) / 3, part = (C - 5) % 3;
        if constexpr (part < 2) {
          float t = T[2 * q + part];
          AMLA_OPAQUE(t);
          mid();
          const float pv = fast_exp2(__builtin_fmaf(t, p.scale_log2e, -ref));
          if constexpr (part == 0) {
            p_even = pv;
            AMLA_OPAQUE(p_even);
          } else {
            p_odd = pv;
            AMLA_OPAQUE(p_odd);
          }
        } else {
          psum += p_even + p_odd;
          unsigned w = pack_bf16(p_even, p_odd);
          bsum = bf16_pair_sum(w, bsum);
          AMLA_OPAQUE(psum);
          AMLA_OPAQUE(w);
          AMLA_OPAQUE(bsum);
          pk[SB * 8 + q] = w;
        }
      } else if constexpr (C == 29) {
        // the row sums are kept per half of the wave (each half sums its own keys of every sub-block; both halves
        // apply the same factors) and added once at the end of the piece
        l_f32 = (VARIANT == AMLA_RESCALE_ADD ? exponent_add(l_f32, n23) : l_f32 * alpha) + psum;
        AMLA_OPAQUE(l_f32);
      } else if constexpr (C == 30) {
        l_b16 = (VARIANT == AMLA_RESCALE_ADD ? exponent_add(l_b16, n23) : l_b16 * alpha) + bsum;
        AMLA_OPAQUE(l_b16);
      }
    };
    constexpr int kSoftmaxChunks = 31;
    // the same work in 47 smaller chunks (a pair of weights in five: the two arguments, either exponential, the
    // sums, the BF16 pair), for the steps of the second product, which have less issue time to spare
    float t_even = 0.f, t_odd = 0.f;
    auto softmax_fine = [&](auto sbc, auto cc, f32x16& T, auto&& mid) {
      constexpr int SB = sbc.value, C = cc.value;
      if constexpr (C < 5) {
        softmax_chunk(sbc, cc, T, mid);
      } else if constexpr (C < 45) {
        constexpr int q = (C - 5) / 5, part = (C - 5) % 5;
        if constexpr (part == 0) {
          float a = T[2 * q], b = T[2 * q + 1];
          AMLA_OPAQUE(a);
          AMLA_OPAQUE(b);
          mid();
          t_even = __builtin_fmaf(a, p.scale_log2e, -ref);
          t_odd = __builtin_fmaf(b, p.scale_log2e, -ref);
          AMLA_OPAQUE(t_even);
          AMLA_OPAQUE(t_odd);
        } else if constexpr (part == 1) {
          AMLA_OPAQUE(t_even);
          mid();
          p_even = fast_exp2(t_even);
          AMLA_OPAQUE(p_even);
        } else if constexpr (part == 2) {
          AMLA_OPAQUE(t_odd);
          mid();
          p_odd = fast_exp2(t_odd);
          AMLA_OPAQUE(p_odd);
        } else if constexpr (part == 3) {
          AMLA_OPAQUE(p_even);
          mid();
          psum += p_even + p_odd;
          AMLA_OPAQUE(psum);
        } else {
          AMLA_OPAQUE(p_odd);
          mid();
          unsigned w = pack_bf16(p_even, p_odd);
          bsum = bf16_pair_sum(w, bsum);
          AMLA_OPAQUE(w);
          AMLA_OPAQUE(bsum);
          pk[SB * 8 + q] = w;
        }
      } else {
        softmax_chunk(sbc, std::integral_constant<int, C - 45 + 29>{}, T, mid);
      }
    };
    constexpr int kFineChunks = 47;

    // [V2] rescale the accumulator registers of the rows whose reference moved in the sub-block just finished.
    // `drain`: the second product's last MFMAs may still be in flight.
    auto rescale = [&](const bool not_first, const bool drain) {
      const bool moved = VARIANT == AMLA_RESCALE_MUL ? alpha != 1.f : n23 != 0;
      unsigned rows_moved = (unsigned)__builtin_amdgcn_ballot_w64(moved);   // bit r: row r of the wave (both halves agree)
      if ((p.flags & AMLA_FLAG_NO_SKIP) && not_first) rows_moved = 0xffffffffu;
      if (rows_moved != 0) {
        if (drain) {
          acc_idle();
          acc_idle();
          acc_idle();
        }
        const int bits = VARIANT == AMLA_RESCALE_MUL ? __float_as_int(alpha) : n23;
        static_for<4>([&](auto gc) {
          constexpr int g = gc.value;
          if (rows_moved & (0xffu << (8 * g))) {
            static_for<4>([&](auto ec) {
              constexpr int e = ec.value;
              // register 4 g + e of every tile holds row 8 g + e in lanes 0..31 and row 8 g + e + 4 in lanes 32..63
              if (rows_moved & (0x11u << (8 * g + e))) {
                const int lo = __builtin_amdgcn_readlane(bits, 8 * g + e);
                const int hi = __builtin_amdgcn_readlane(bits, 8 * g + e + 4);
                const int mine = h ? hi : lo;
                if (VARIANT == AMLA_RESCALE_MUL)
                  acc_scale_rows<4 * g + e>(__int_as_float(mine));
                else if (VARIANT == AMLA_RESCALE_ADD)
                  acc_exponent_lower_rows<4 * g + e>(mine);
                else
                  acc_exponent_add_rows<4 * g + e>(mine);
              }
            });
          }
        });
        acc_idle();
      }
    };

    // ---- phase A: [C1] for keys 0 .. 31; the next block streams in under it ----
#pragma unroll
    for (int d = 0; d < kKAhead; ++d) ka[d] = *(LDS_PTR(bf16x8))k_addr(d, 0);
    auto phase_a = [&](auto more_c) {
      static_for<kSteps>([&](auto ksc) {
        constexpr int ks = ksc.value;
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks % kKAhead], qf[ks], s0, 0, 0, 0);
        AMLA_PIN(s0);
        constexpr int nk = ks + kKAhead;
        ka[ks % kKAhead] = *(LDS_PTR(bf16x8))(nk < kSteps ? k_addr(nk, 0) : k_addr(nk - kSteps, 1));
        // the 18 loads of the next tile: one behind every second step
        if constexpr (more_c.value && (ks & 1)) issue_tile_load<(ks >> 1)>(next_block, nxt, wave, tl);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    if (more && fetch_own_share)
      phase_a(std::true_type{});
    else
      phase_a(std::false_type{});

    // ---- phase B: [C1] for keys 32 .. 63 | [V1] of sub-block 0 ----
    static_for<kSteps>([&](auto ksc) {
      constexpr int ks = ksc.value;
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[(kSteps + ks) % kKAhead], qf[ks], s1, 0, 0, 0);
      AMLA_PIN(s1);
      // (the operand read sits between a chunk's input pins and its arithmetic: an instruction that reads what an
      // assembly statement has just defined is given a wait state by the compiler)
      auto read_next = [&]() {
        if constexpr (ks + kKAhead < kSteps) ka[(kSteps + ks) % kKAhead] = *(LDS_PTR(bf16x8))k_addr(ks + kKAhead, 1);
      };
      if constexpr (ks < kSoftmaxChunks)
        softmax_chunk(std::integral_constant<int, 0>{}, ksc, s0, read_next);
      else
        read_next();
      __builtin_amdgcn_sched_barrier(0);
    });

    // the first V operands of [C2]
    s16x4 vr[kVAhead][2];
#pragma unroll
    for (int d = 0; d < kVAhead; ++d) {
      vr[d][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(buf + v_lo + d * 64));
      vr[d][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(buf + v_hi + d * 64));
    }
    __builtin_amdgcn_sched_barrier(0);
    rescale(j != j0, false);
    __builtin_amdgcn_sched_barrier(0);

    // ---- [C2] O[32 rows x 512] += P V, 16 keys x 32 columns per MFMA ----
    auto pv_mfma = [&](auto nc) {
      constexpr int n = nc.value, st = n / (kDv / 32), dt = n % (kDv / 32);
      const i32x4 pb = {(int)pk[4 * st], (int)pk[4 * st + 1], (int)pk[4 * st + 2], (int)pk[4 * st + 3]};
      const i32x2 lo2 = __builtin_bit_cast(i32x2, vr[n % kVAhead][0]), hi2 = __builtin_bit_cast(i32x2, vr[n % kVAhead][1]);
      const i32x4 vb = {lo2[0], lo2[1], hi2[0], hi2[1]};
      acc_mfma<dt>(__builtin_bit_cast(bf16x8, pb), __builtin_bit_cast(bf16x8, vb));
    };
    auto pv_reads = [&](auto nc) {
      constexpr int n = nc.value;
      constexpr int nx = n + kVAhead;
      if constexpr (nx < 4 * (kDv / 32)) {
        constexpr int step = (nx / (kDv / 32)) * 16 * kRgRowA + (nx % (kDv / 32)) * 64;
        vr[n % kVAhead][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(buf + v_lo + step));
        vr[n % kVAhead][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(buf + v_hi + step));
      }
    };
    // ---- phase C: keys 0 .. 31 | [V1] of sub-block 1 ----
    // (one fine chunk a step: maximum, reference, and the weights of keys 32 .. 53)
    static_for<2 * (kDv / 32)>([&](auto nc) {
      pv_mfma(nc);
      softmax_fine(std::integral_constant<int, 1>{}, nc, s1, [&]() { pv_reads(nc); });
      __builtin_amdgcn_sched_barrier(0);
    });
    rescale(true, true);
    __builtin_amdgcn_sched_barrier(0);
    // ---- phase D: keys 32 .. 63 | the remaining weights (keys 54 .. 63, needed from step 16 on) and the row sums ----
    static_for<2 * (kDv / 32)>([&](auto nc) {
      constexpr int n = nc.value;
      constexpr auto step = std::integral_constant<int, 2 * (kDv / 32) + n>{};
      pv_mfma(step);
      if constexpr (32 + n < kFineChunks)
        softmax_fine(std::integral_constant<int, 1>{}, std::integral_constant<int, 32 + n>{}, s1, [&]() { pv_reads(step); });
      else
        pv_reads(step);
      __builtin_amdgcn_sched_barrier(0);
    });
  }

  // ---- epilogue (the final division by the row sum of Algorithm 1 / Algorithm 2) ----
  l_b16 += __shfl_xor(l_b16, 32);
  l_f32 += __shfl_xor(l_f32, 32);
  const float inv = l_b16 > 0.f ? 1.f / l_b16 : 0.f;
  const float lse = l_f32 > 0.f ? (ref + fast_log2(l_f32)) * 0.6931471805599453f : -INFINITY;
  if (row < p.rows && h == 0) {
    if (to_final) {
      if (p.lse != nullptr) p.lse[grow] = lse;
    } else {
      p.part_lse[part_row0 + row] = lse;
    }
  }
  acc_idle();
  acc_idle();
  acc_idle();
  static_for<16>([&](auto ic) {
    constexpr int i = ic.value;
    const int rw = 8 * (i >> 2) + 4 * h + (i & 3);          // row of register i within the wave
    const float inv_i = lane_value(inv, rw);
    const int row_i = tile * kRowsPerWg + wave * 32 + rw;
    float o[kDv / 32];
    static_for<kDv / 32>([&](auto dt) { o[dt.value] = acc_read<16 * dt.value + i>() * inv_i; });
    if (row_i < p.rows) {
      if (to_final) {
        uint16_t* orow = p.out + ((size_t)b * p.rows + row_i) * kDv + l32;
#pragma unroll
        for (int dt = 0; dt < kDv / 32; ++dt) orow[32 * dt] = (uint16_t)pack_bf16(o[dt], 0.f);
      } else {
        // a partial row goes out in FP16 (the values are normalised, so of the value rows' magnitude; the merge
        // weights them in FP32), the lane's 16 columns side by side at position 16 l32: two 16-byte stores
        // instead of sixteen, and half the bytes that the combine kernel reads back
        unsigned hw[kDv / 64];
#pragma unroll
        for (int k = 0; k < kDv / 64; ++k) hw[k] = pack_f16(o[2 * k], o[2 * k + 1]);
        i32x4* prow = reinterpret_cast<i32x4*>(reinterpret_cast<uint16_t*>(p.part_o) + (part_row0 + row_i) * kDv + 16 * l32);
        prow[0] = i32x4{(int)hw[0], (int)hw[1], (int)hw[2], (int)hw[3]};
        prow[1] = i32x4{(int)hw[4], (int)hw[5], (int)hw[6], (int)hw[7]};
      }
    }
  });
}

// Equal-share decomposition: workgroup = (sequence, split, 128-row tile).
template <int VARIANT, bool ITER512>
__global__ __launch_bounds__(kThreads) AMLA_ONE_WAVE_PER_SIMD
void amla_decode_rg_kernel(const DecodeParams p) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem_raw[];
  LDS_PTR(uint8_t) smem = (LDS_PTR(uint8_t))smem_raw;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  acc_claim();

  // Workgroup -> (sequence, split, row tile).  Consecutive workgroup ids go round-robin over the 8 XCDs.  The row
  // tiles of one (sequence, split) get ids that differ by 8, so that they land on the same XCD next to each other
  // and share the KV blocks in that XCD's L2; so do the splits of one sequence, which all read the same query
  // rows (sequence = 8 * (group / splits) + xcd, split = group % splits: with four shares the query rows were
  // otherwise fetched from HBM four times, once per XCD).
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int group = slot / p.n_tiles;
  const int tile = slot % p.n_tiles;
  const int b = (group / p.n_splits) * 8 + xcd;
  const int split = group % p.n_splits;
  if (b >= p.batch) return;

  // The first 64 entries of the sequence's block-table row are asked for together with its length, one per lane:
  // a share that starts within them (any share of a sequence of up to 4096 keys, the first shares of a longer
  // one) then has its first entry without a second memory round trip before the first tile can be requested.
  const int32_t* table_row = p.table + (size_t)b * p.max_blocks;
  const int lane_entry = table_row[min(lane, p.max_blocks - 1)];
  const int kv_len = plan_len(__builtin_amdgcn_readfirstlane(p.seqlens[b]), p.max_blocks, kBlock);
  const int nb = plan_blocks_of(kv_len, kBlock);
  const int j0 = (int)(((long long)split * nb) / p.n_splits);
  const int j1 = (int)(((long long)(split + 1) * nb) / p.n_splits);
  const bool have_entry = j0 < 64;
  const int entry = __builtin_amdgcn_readlane(lane_entry, j0 & 63);
  decode_piece<VARIANT, false, ITER512>(p, smem, lane, wave, b, kv_len, j0, j1, tile, p.n_splits == 1,
                               (size_t)split * p.batch * p.rows + (size_t)b * p.rows, 0, 0, true, have_entry, entry);
}

// Balanced decomposition (ragged batches, causal mask among the s_q tokens, per-sequence query counts):
// workgroup = (worker, row tile).  The 64-key blocks of all sequences are laid end to end and cut into
// p.n_streams equal worker ranges (amla_plan.h); a worker walks its range sequence by sequence, every (worker,
// sequence) pair is a piece with its own softmax state.  A piece that covers its whole sequence writes the
// final result, any other writes a partial row set into slot worker + sequence of the workspace, which
// amla_combine_balanced_kernel merges.
template <int VARIANT, bool ITER512>
__global__ __launch_bounds__(kThreads) AMLA_ONE_WAVE_PER_SIMD
void amla_decode_rg_balanced_kernel(const DecodeParams p) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem_raw[];
  LDS_PTR(uint8_t) smem = (LDS_PTR(uint8_t))smem_raw;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  acc_claim();

  // workers go round-robin over the 8 XCDs; the row tiles of one worker sit next to each other on the same
  // XCD and share the worker's KV blocks in that XCD's L2
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int stream = (slot / p.n_tiles) * 8 + xcd;
  const int tile = slot % p.n_tiles;
  if (stream >= p.n_streams) return;

  // total number of blocks of the batch, then this worker's range of the concatenated list
  int total = 0;
  for (int c = 0; c < p.batch; c += 64) {
    const int i = c + lane;
    total += wave_sum(i < p.batch ? plan_blocks_of(plan_len(p.seqlens[i], p.max_blocks, kBlock), kBlock) : 0);
  }
  total = __builtin_amdgcn_readfirstlane(total);
  const long long g0 = plan_worker_begin(stream, total, p.n_streams);
  const long long g1 = plan_worker_begin(stream + 1, total, p.n_streams);
  if (g0 >= g1) return;
  // the sequence that holds global block g0, and g0's position in it
  int b0 = -1, jstart = 0, base = 0;
  for (int c = 0; c < p.batch && b0 < 0; c += 64) {
    const int i = c + lane;
    const int nbi = i < p.batch ? plan_blocks_of(plan_len(p.seqlens[i], p.max_blocks, kBlock), kBlock) : 0;
    const int incl = wave_inclusive_scan(nbi, lane);
    const int excl = incl - nbi;
    const bool hit = (long long)base + excl <= g0 && g0 < (long long)base + incl;
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(hit);
    if (mask != 0) {
      const int l = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask));
      b0 = c + l;
      jstart = (int)(g0 - ((long long)base + __builtin_amdgcn_readlane(excl, l)));
    }
    base += __builtin_amdgcn_readlane(incl, 63);
  }
  if (b0 < 0) return;   // unreachable when g0 < total

  const int row = tile * kRowsPerWg + wave * 32 + (lane & 31);   // this lane's query row within the sequence
  PlanWalk walk = {b0, jstart, g1 - g0};
  bool first_piece = true;
  while (walk.left > 0 && walk.b < p.batch) {
    const int kv_len = plan_len(__builtin_amdgcn_readfirstlane(p.seqlens[walk.b]), p.max_blocks, kBlock);
    PlanPiece piece;
    if (!plan_next(&walk, plan_blocks_of(kv_len, kBlock), &piece)) continue;
    // A row's limit lies causal_shift keys before the sequence's end.  Causal mask among the q_len query
    // tokens of the sequence: token t sits q_len - 1 - t positions before the end of the cache and sees the
    // keys up to and including its own, kv_len - (q_len - 1 - t) of them.  A padding token (t >= q_len) sees
    // none and ends as out = 0, lse = -inf like any row without keys.  mask_span is the largest shift of the
    // piece (wave-uniform): blocks closer than that to the end need the mask.
    int q_len = p.s_q;
    if (p.q_lens != nullptr) q_len = min(max(__builtin_amdgcn_readfirstlane(p.q_lens[piece.b]), 0), p.s_q);
    const int mask_span = q_len < p.s_q ? kNoKeys : p.causal_span;
    const int t_row = row / p.heads;
    const int causal_shift = t_row >= q_len ? kNoKeys : (p.causal_span != 0 ? q_len - 1 - t_row : 0);
    decode_piece<VARIANT, true, ITER512>(p, smem, lane, wave, piece.b, kv_len, piece.j0, piece.j1, tile, piece.full != 0,
                                ((size_t)stream + piece.b) * p.rows, causal_shift, mask_span, first_piece);
    first_piece = false;
  }
}

}  // namespace

// The kernels of this file for a rescale variant (AMLA_RESCALE_MUL, _ADD or _ADD_COMP), for amla_decode to
// launch with 256 threads and amla_row_rescale_lds_bytes() of dynamic LDS; iteration_512 = the build whose
// recurrence steps once per eight cache blocks (AMLA_FLAG_ITERATION_512).
int amla_row_rescale_lds_bytes() { return kRgLdsBytes; }
AmlaDecodeKernel amla_row_rescale_kernel(int variant, bool balanced, bool iteration_512) {
  if (iteration_512) {   // MUL and ADD only (amla_decode refuses the flag for the compensated variant)
    if (balanced)
      return variant == AMLA_RESCALE_ADD ? amla_decode_rg_balanced_kernel<AMLA_RESCALE_ADD, true>
                                         : amla_decode_rg_balanced_kernel<AMLA_RESCALE_MUL, true>;
    return variant == AMLA_RESCALE_ADD ? amla_decode_rg_kernel<AMLA_RESCALE_ADD, true>
                                       : amla_decode_rg_kernel<AMLA_RESCALE_MUL, true>;
  }
  if (balanced)
    return variant == AMLA_RESCALE_ADD_COMP ? amla_decode_rg_balanced_kernel<AMLA_RESCALE_ADD_COMP, false>
           : variant == AMLA_RESCALE_ADD    ? amla_decode_rg_balanced_kernel<AMLA_RESCALE_ADD, false>
                                            : amla_decode_rg_balanced_kernel<AMLA_RESCALE_MUL, false>;
  return variant == AMLA_RESCALE_ADD_COMP ? amla_decode_rg_kernel<AMLA_RESCALE_ADD_COMP, false>
         : variant == AMLA_RESCALE_ADD    ? amla_decode_rg_kernel<AMLA_RESCALE_ADD, false>
                                          : amla_decode_rg_kernel<AMLA_RESCALE_MUL, false>;
}
