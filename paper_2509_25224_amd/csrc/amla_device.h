// Device-side definitions shared by the translation units of the absorbed-MLA decode library: tile and
// layout constants, the kernel parameter block, and the small helpers every decode kernel uses (guarded
// exponent add of Lemma 3.1, bf16 packing, the direct-to-LDS tile loads).
#ifndef AMLA_DEVICE_H_
#define AMLA_DEVICE_H_

#include <stdint.h>

constexpr int kDqk = 576;
constexpr int kDv = 512;
constexpr int kBlock = 64;               // keys per cache block
constexpr int kRowBytes = kDqk * 2;      // 1152 bytes of bf16 per cached row
constexpr int kLdsRow = kRowBytes + 16;  // padded LDS row: 73 chunks of 16 B (odd -> no bank conflicts)
constexpr int kChunksPerRow = kLdsRow / 16;           // 73
constexpr int kTileBytes = kBlock * kLdsRow;          // 74752 = 73 * 1024
constexpr int kTileLoads = kTileBytes / 1024;         // 73 wave-wide 1 KiB direct-to-LDS loads
constexpr int kRowsPerWg = 128;
constexpr int kThreads = 256;
constexpr int kLdsBytes = 2 * kTileBytes;             // double buffer, 149504 B of the 160 KiB

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i32x2;

// Target hooks.  The definitions below are the gfx950 ones; a CPU build of these kernels (tests
// only: bounds-checked runs of the index logic) defines them beforehand.
#ifndef AMLA_TARGET_HOOKS
#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLB_PTR(T) __attribute__((address_space(1))) T*
// every direct-to-LDS load of this wave has landed
#define AMLA_WAIT_TILE_LOADS() asm volatile("s_waitcnt vmcnt(0)" ::: "memory")
// make x opaque to the optimiser at this point (stops hoisting of what is derived from it)
#define AMLA_OPAQUE(x) asm volatile("" : "+v"(x))
// one wave per SIMD: the whole 512-register file belongs to it
#define AMLA_ONE_WAVE_PER_SIMD __attribute__((amdgpu_waves_per_eu(1, 1)))
// One 16-byte-per-lane direct-to-LDS load (lane l lands at lds + 16 l, lds wave-uniform) issued from inline
// assembly, so that the compiler's wait-count pass does not know LDS is being written: it otherwise puts a
// full vmcnt(0) in front of the first transposing LDS read that follows, and the second product could never
// overlap the loads.  The kernels' own wait (AMLA_WAIT_TILE_LOADS, then the barrier) is what orders the tile's
// arrival before its readers.  The compiler's waits for its own vector-memory operations stay correct with
// loads it does not count: the counter is in-order and extra outstanding operations only make a wait longer.
#define AMLA_HIDDEN_LDS_LOAD(gptr, lds)                                                                      \
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"                              \
               :                                                                                             \
               : "v"(gptr), "s"(__builtin_amdgcn_readfirstlane((unsigned)(__UINTPTR_TYPE__)(lds)))           \
               : "memory", "m0")
// a use of x the compiler must honour here: whatever load produces x is waited for at this point
#define AMLA_ARRIVED(x) asm volatile("" : : "v"(x))
// element i of an int32 array that no kernel writes while this one runs, read through the scalar cache
// when i is wave-uniform (a load that counts in lgkmcnt, not in the vmcnt of the tile loads)
#define AMLA_UNIFORM_LOAD_I32(p, i) (((const __attribute__((address_space(4))) int32_t*)(uintptr_t)(p))[i])
#endif

struct DecodeParams {
  const uint16_t* q;        // [B, G, 576] bf16 bits (G = s_q * H rows per sequence)
  const uint16_t* kv;       // [num_blocks, 64, 576]
  const int32_t* table;     // [B, max_blocks]
  const int32_t* seqlens;   // [B]
  uint16_t* out;            // [B, G, 512] bf16 bits
  float* lse;               // [B, G] or null
  float* part_o;            // [n_splits, B, G, 512] f32 (n_splits > 1)
  float* part_lse;          // [n_splits, B, G]
  float scale_log2e;        // softmax_scale * log2(e)
  int32_t batch;
  int32_t rows;             // G
  int32_t n_tiles;          // ceil(G / 128)
  int32_t n_splits;
  int32_t max_blocks;
  int32_t n_streams;        // batch * n_splits; balanced decomposition: number of workers
  int32_t flags;
  int32_t num_blocks;       // physical blocks in the pool (the balanced kernel clamps table entries)
  int32_t heads;            // rows of a sequence are (t, h) flattened: t * heads + h
  int32_t causal_span;      // s_q - 1 under the causal mask among the s_q query tokens, else 0
  int32_t s_q;              // query tokens per sequence in the q array
  const int32_t* q_lens;    // [B] query tokens sequence b really has (<= s_q), or null: s_q everywhere
};

// A row's shift that puts its limit before every key: the row of a padding token.
constexpr int kNoKeys = 1 << 30;

// Lemma 3.1 with a guard: x * 2^delta as an integer add of n23 = delta << 23 (delta <= 0) on the
// bit pattern.  The saturating add pins a negative float whose exponent would go below zero at
// 0x80000000 (-0.0); the max with the sign bit turns a wrapped positive float into +0.0.
// n23 may also carry a small mantissa term of either sign (Algorithm 2's eps inside N): the guard
// only concerns sums that leave the float's own sign range.
__device__ __forceinline__ float exponent_add(float x, int n23) {
  const int i = __float_as_int(x);
  int r = __builtin_elementwise_add_sat(i, n23);
  r = max(r, i & (int)0x80000000);
  return __int_as_float(r);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);   // round to nearest even
  return __builtin_bit_cast(unsigned, b);
}

// two FP32 values as a pair of FP16 (round to nearest even), lo in the low half
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ unsigned pack_f16(float lo, float hi) {
  f32x2 v = {lo, hi};
  f16x2 b = __builtin_convertvector(v, f16x2);
  return __builtin_bit_cast(unsigned, b);
}

// Issue this wave's share (one of NWAVES) of the direct-to-LDS loads of one 64 x 576 bf16 block.
// LDS destination of load i is the 1 KiB range [i * 1024, (i + 1) * 1024) of the tile buffer,
// lane l landing at + 16 l; chunk c = 64 i + l of the padded tile is row c / 73, column chunk
// c % 73, the 73rd chunk of a row being padding (it receives 16 harmless bytes).
template <int NWAVES = 4, bool HIDDEN = false>
__device__ __forceinline__ void issue_tile_loads(const uint8_t* block_base, LDS_PTR(uint8_t) buf,
                                                 int wave, int lane) {
  // keep the per-lane offsets out of loop-invariant hoisting: 19 of them per lane would
  // cost more registers than recomputing them costs VALU slots
  AMLA_OPAQUE(lane);
#pragma unroll
  for (int k = 0; k < (kTileLoads + NWAVES - 1) / NWAVES; ++k) {
    const int i = wave + NWAVES * k;
    if (i < kTileLoads) {
      const int c = i * 64 + lane;
      const int row = (int)(((unsigned)c * 57457u) >> 22);      // c / 73 for c < 4672
      const int cc = c - row * kChunksPerRow;
      const int off = (cc < kChunksPerRow - 1) ? (c - row) * 16 : 0;
      if (HIDDEN) {
        AMLA_HIDDEN_LDS_LOAD(block_base + off, buf + i * 1024);
      } else {
        __builtin_amdgcn_global_load_lds((const GLB_PTR(void))(block_base + off),
                                         (LDS_PTR(void))(buf + i * 1024), 16, 0, 0);
      }
    }
  }
}

constexpr float kLazyThreshold = 8.f;   // base-2 units: the weights may grow to 2^8 before the reference moves

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(v, o);
    if (lane >= o) v += u;
  }
  return v;
}

// Kernels defined in other translation units of the library, looked up by amla_decode.
typedef void (*AmlaDecodeKernel)(const DecodeParams);
AmlaDecodeKernel amla_row_rescale_kernel(int variant, bool balanced, bool iteration_512);   // amla_decode_rg.hip
int amla_row_rescale_lds_bytes();

#endif  // AMLA_DEVICE_H_
