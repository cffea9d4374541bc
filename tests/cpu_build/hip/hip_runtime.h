// CPU stand-in for <hip/hip_runtime.h> (tests only): the HIP / gfx950 constructs the decode library uses,
// so that its source -- kernels and host code alike -- compiles for the host unmodified and runs under
// AddressSanitizer.  One OS thread per work-item;
// the 64 threads of a wave meet at a barrier for every wave-wide operation (shuffle, ballot, readlane,
// MFMA, transposing LDS read), the threads of a workgroup at __syncthreads().
//
// Semantics of the two matrix-pipeline operations are the ones measured on the hardware:
//   v_mfma_f32_32x32x16_bf16: A lane l holds row l%32, k = 8*(l/32)+0..7; B lane l holds column l%32,
//       same k; C/D register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//   ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives, for j = 0..3, element i%4 of
//       the 4 x b16 that lane (i/4 + 4j) of the group addressed.
// Direct-to-LDS loads are made deliberately strict: at issue the destination is filled with a NaN
// pattern, the data lands when the issuing wave waits for its loads.  A kernel that reads a tile
// before waiting, or refills a buffer another wave may still read, then produces NaNs.
#ifndef AMLA_TESTS_HIP_RUNTIME_SHIM_H_
#define AMLA_TESTS_HIP_RUNTIME_SHIM_H_

#include <algorithm>
#include <atomic>
#include <sched.h>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <string>
#include <thread>
#include <vector>

struct dim3 {
  unsigned x, y, z;
  dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
inline thread_local dim3 threadIdx, blockIdx, blockDim;

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __shared__
using std::max;
using std::min;

namespace shim {

// A yielding barrier: there are far more threads than cores, so a waiter gives up its time slice
// instead of spinning or sleeping on a futex (waking 63 sleepers per wave-wide operation is what
// costs the time otherwise).
class Barrier {
 public:
  explicit Barrier(unsigned n) : n_(n) {}
  void arrive_and_wait() {
    const unsigned gen = gen_.load(std::memory_order_acquire);
    if (count_.fetch_add(1, std::memory_order_acq_rel) + 1 == n_) {
      count_.store(0, std::memory_order_relaxed);
      gen_.store(gen + 1, std::memory_order_release);
    } else {
      while (gen_.load(std::memory_order_acquire) == gen) sched_yield();
    }
  }

 private:
  const unsigned n_;
  std::atomic<unsigned> count_{0}, gen_{0};
};

struct WaveCtx {
  Barrier bar{64};
  alignas(64) unsigned char slot[2][64][64];
};
struct PendingLoad {
  const void* src;
  void* dst;
};
inline thread_local WaveCtx* wave = nullptr;
inline thread_local Barrier* wg_bar = nullptr;
inline thread_local int lane = 0;
inline thread_local unsigned turn = 0;
inline thread_local std::vector<PendingLoad>* pending = nullptr;

// every lane contributes `mine`; returns a pointer to the 64 contributions (valid until the wave's
// next collective but one)
template <class T>
inline const unsigned char (*exchange(const T& mine))[64] {
  static_assert(sizeof(T) <= 64, "payload");
  const unsigned t = turn++ & 1u;
  std::memcpy(wave->slot[t][lane], &mine, sizeof(T));
  wave->bar.arrive_and_wait();
  return wave->slot[t];
}
template <class T>
inline T peer(const unsigned char (*all)[64], int l) {
  T v;
  std::memcpy(&v, all[l], sizeof(T));
  return v;
}

template <class T>
inline T shfl_xor(T v, int m) {
  return peer<T>(exchange(v), lane ^ m);
}
template <class T>
inline T shfl_up(T v, int d) {
  auto all = exchange(v);
  return lane >= d ? peer<T>(all, lane - d) : v;
}
template <class T>
inline T readfirstlane(T v) {
  return peer<T>(exchange(v), 0);
}
inline int readlane(int v, int l) { return peer<int>(exchange(v), l & 63); }
// ds_bpermute_b32: lane l receives the value of lane (addr / 4) % 64
inline int bpermute(int addr, int v) { return peer<int>(exchange(v), (addr >> 2) & 63); }
inline unsigned long long ballot(bool p) {
  auto all = exchange((int)p);
  unsigned long long m = 0;
  for (int l = 0; l < 64; ++l) m |= (unsigned long long)(peer<int>(all, l) != 0) << l;
  return m;
}

template <class AB, class C>
inline C mfma_32x32x16_bf16(AB a, AB b, C c, int, int, int) {
  struct Frag {
    AB a, b;
  } mine = {a, b};
  auto all = exchange(mine);
  const int col = lane & 31, half = lane >> 5;
  Frag colf[2];   // the two lanes that hold column `col` of B (k 0..7 and 8..15)
  colf[0] = peer<Frag>(all, col);
  colf[1] = peer<Frag>(all, col + 32);
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r / 4) + 4 * half + r % 4;
    const Frag r0 = peer<Frag>(all, row), r1 = peer<Frag>(all, row + 32);
    double acc = 0.0;
    for (int e = 0; e < 8; ++e) {
      acc += (double)(float)r0.a[e] * (double)(float)colf[0].b[e];
      acc += (double)(float)r1.a[e] * (double)(float)colf[1].b[e];
    }
    c[r] = (float)((double)c[r] + acc);
  }
  return c;
}

// v_mfma_f32_16x16x32_bf16 with the operand layouts the CDNA4 ISA documents (not measured by this
// build): A lane l holds row l%16, k = 8*(l/16)+0..7; B lane l holds column l%16, same k; C/D register
// r of lane l is row 4*(l/16) + r, column l%16.
template <class AB, class C>
inline C mfma_16x16x32_bf16(AB a, AB b, C c, int, int, int) {
  struct Frag {
    AB a, b;
  } mine = {a, b};
  auto all = exchange(mine);
  const int col = lane & 15, grp = lane >> 4;
  for (int r = 0; r < 4; ++r) {
    const int row = 4 * grp + r;
    double acc = 0.0;
    for (int kg = 0; kg < 4; ++kg) {
      const Frag fr = peer<Frag>(all, row + 16 * kg), fc = peer<Frag>(all, col + 16 * kg);
      for (int e = 0; e < 8; ++e) acc += (double)(float)fr.a[e] * (double)(float)fc.b[e];
    }
    c[r] = (float)((double)c[r] + acc);
  }
  return c;
}

template <class V4>
inline V4 ds_read_tr16_b64(V4* p) {
  V4 mine;
  std::memcpy(&mine, p, sizeof(V4));
  auto all = exchange(mine);
  const int g = lane / 16, i = lane % 16;
  V4 out;
  for (int j = 0; j < 4; ++j) out[j] = peer<V4>(all, g * 16 + i / 4 + 4 * j)[i % 4];
  return out;
}

inline void global_load_lds(const void* g, void* lds_base, int bytes, int, int) {
  if (bytes != 16) std::abort();
  unsigned char* dst = static_cast<unsigned char*>(lds_base) + 16 * lane;
  volatile unsigned char probe = *static_cast<const unsigned char*>(g);          // the read is checked at issue
  probe = static_cast<const unsigned char*>(g)[15];
  (void)probe;
  for (int i = 0; i < 8; ++i) reinterpret_cast<uint16_t*>(dst)[i] = 0x7FC0;      // bf16 NaN until it lands
  pending->push_back({g, dst});
}
inline void wait_tile_loads() {
  for (const PendingLoad& l : *pending) std::memcpy(l.dst, l.src, 16);
  pending->clear();
}
// all but the last n loads this wave issued have landed (they land in issue order)
inline void wait_tile_loads_but(int n) {
  const size_t keep = std::min<size_t>((size_t)std::max(n, 0), pending->size());
  const size_t land = pending->size() - keep;
  for (size_t i = 0; i < land; ++i) std::memcpy((*pending)[i].dst, (*pending)[i].src, 16);
  pending->erase(pending->begin(), pending->begin() + land);
}
inline void syncthreads() { wg_bar->arrive_and_wait(); }

// Runs kernel(args) for every workgroup of a 1-D or 2-D grid with `threads` work-items each (a
// multiple of 64).  Workgroups run one after another; the work-items of one run concurrently.
template <class F>
void launch(unsigned grid_x, unsigned grid_y, unsigned threads, F kernel) {
  const unsigned n_waves = threads / 64;
  std::vector<std::unique_ptr<WaveCtx>> waves;
  for (unsigned w = 0; w < n_waves; ++w) waves.emplace_back(new WaveCtx);
  Barrier wg(threads);
  std::vector<std::thread> pool;
  for (unsigned t = 0; t < threads; ++t) {
    pool.emplace_back([&, t] {
      std::vector<PendingLoad> my_pending;
      pending = &my_pending;
      wave = waves[t / 64].get();
      wg_bar = &wg;
      lane = (int)(t % 64);
      turn = 0;
      threadIdx.x = t;
      blockDim.x = threads;
      for (unsigned y = 0; y < grid_y; ++y)
        for (unsigned x = 0; x < grid_x; ++x) {
          blockIdx.x = x;
          blockIdx.y = y;
          kernel();
          if (!my_pending.empty()) {
            std::fprintf(stderr, "shim: a wave left the kernel with direct-to-LDS loads in flight\n");
            std::abort();
          }
          wg.arrive_and_wait();   // the next workgroup reuses the LDS buffer
        }
    });
  }
  for (auto& th : pool) th.join();
}

}  // namespace shim

// ---- the slice of the HIP runtime API the library's host code uses ---------------------------------
typedef int hipError_t;
typedef void* hipStream_t;
enum { hipSuccess = 0, hipErrorNotSupported = 801 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
enum { hipDeviceAttributeMultiprocessorCount = 63, hipDeviceAttributeClockRate = 5 };
// no device here: the query fails and the library falls back to its documented default of 256 compute units
inline hipError_t hipDeviceGetAttribute(int*, int, int) { return hipErrorNotSupported; }
// a __device__ variable is an ordinary host variable here, and its "device address" is its address
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))
inline hipError_t hipGetSymbolAddress(void** ptr, const void* symbol) {
  *ptr = const_cast<void*>(symbol);
  return hipSuccess;
}
#define hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, ...)                              \
  do {                                                                                             \
    const dim3 shim_grid = (grid), shim_block = (block);                                           \
    (void)(lds_bytes);                                                                             \
    (void)(stream);                                                                                \
    shim::launch(shim_grid.x, shim_grid.y, shim_block.x, [&] { kern(__VA_ARGS__); });              \
  } while (0)

#define __syncthreads() shim::syncthreads()
#define __shfl_xor(v, m) shim::shfl_xor((v), (m))
#define __shfl_up(v, d) shim::shfl_up((v), (d))
#define __builtin_amdgcn_readfirstlane(v) shim::readfirstlane((v))
#define __builtin_amdgcn_readlane(v, l) shim::readlane((v), (l))
#define __builtin_amdgcn_ballot_w64(p) shim::ballot((p))
#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) shim::mfma_32x32x16_bf16((a), (b), (c), (x), (y), (z))
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, x, y, z) shim::mfma_16x16x32_bf16((a), (b), (c), (x), (y), (z))
#define __builtin_amdgcn_ds_read_tr16_b64_v4i16(p) shim::ds_read_tr16_b64((p))
#define __builtin_amdgcn_global_load_lds(g, l, n, o, a) shim::global_load_lds((g), (l), (n), (o), (a))
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_ds_bpermute(addr, v) shim::bpermute((addr), (v))
#define __builtin_amdgcn_exp2f(x) exp2f((x))
#define __builtin_amdgcn_logf(x) log2f((x))
#define __expf(x) expf((x))
#define __logf(x) logf((x))

inline int __float_as_int(float f) { return __builtin_bit_cast(int, f); }
inline float __int_as_float(int i) { return __builtin_bit_cast(float, i); }
inline float __uint_as_float(unsigned u) { return __builtin_bit_cast(float, u); }

// target hooks of amla_decode_kernels.inc
#define AMLA_TARGET_HOOKS 1
#define LDS_PTR(T) T*
#define GLB_PTR(T) T*
#ifdef SHIM_PLANT_NO_WAIT
#define AMLA_WAIT_TILE_LOADS() ((void)0)   // planted mistake for the harness's own test: tiles are read before they land
#else
#define AMLA_WAIT_TILE_LOADS() shim::wait_tile_loads()
#endif
#define AMLA_OPAQUE(x) ((void)(x))
#define AMLA_PIN(x) ((void)(x))
#define AMLA_ONE_WAVE_PER_SIMD
#define AMLA_UNIFORM_LOAD_I32(p, i) ((p)[i])
#define AMLA_ARRIVED(x) ((void)(x))
#define AMLA_HIDDEN_LDS_LOAD(gptr, lds) shim::global_load_lds((gptr), (lds), 16, 0, 0)


// The accumulator file of the row-rescale kernels (256 AccVGPRs per lane, addressed by name from assembly
// statements on the GPU): here an array per work-item behind the same functions.  Tile dt is registers
// 16 dt .. 16 dt + 15 with the C/D layout of the MFMA.
#include <array>
namespace shim {
inline thread_local float acc_file[256];
}
template <int DT, class AB>
inline void acc_mfma(AB a, AB b) {
  std::array<float, 16> c;
  for (int r = 0; r < 16; ++r) c[r] = shim::acc_file[16 * DT + r];
  c = shim::mfma_32x32x16_bf16(a, b, c, 0, 0, 0);
  for (int r = 0; r < 16; ++r) shim::acc_file[16 * DT + r] = c[r];
}
template <int DT>
inline void acc_clear_tile() {
  for (int r = 0; r < 16; ++r) shim::acc_file[16 * DT + r] = 0.f;
}
template <int R>
inline float acc_read() { return shim::acc_file[R]; }
template <int I>
inline void acc_scale_rows(float factor) {
  for (int dt = 0; dt < 16; ++dt) shim::acc_file[16 * dt + I] *= factor;
}
template <int I>
inline void acc_exponent_add_rows(int n23) {
  // saturating INT32 add, then max with the sign bit (the instruction pair of the GPU build)
  for (int dt = 0; dt < 16; ++dt) {
    const int i = __builtin_bit_cast(int, shim::acc_file[16 * dt + I]);
    long long r = (long long)i + n23;
    r = r > 2147483647ll ? 2147483647ll : (r < -2147483648ll ? -2147483648ll : r);
    const int guard = i & (int)0x80000000;
    shim::acc_file[16 * dt + I] = __builtin_bit_cast(float, std::max((int)r, guard));
  }
}
template <int I>
inline void acc_exponent_lower_rows(int n23) {
  // n23 <= 0: saturating INT32 add, then the unsigned minimum with the operand (the instruction pair of the GPU build)
  for (int dt = 0; dt < 16; ++dt) {
    const int i = __builtin_bit_cast(int, shim::acc_file[16 * dt + I]);
    long long r = (long long)i + n23;
    r = r > 2147483647ll ? 2147483647ll : (r < -2147483648ll ? -2147483648ll : r);
    const unsigned u = std::min((unsigned)(int)r, (unsigned)i);
    shim::acc_file[16 * dt + I] = __builtin_bit_cast(float, u);
  }
}
inline void wait_tile_loads_but(int n) { shim::wait_tile_loads_but(n); }
// v_dot2_f32_bf16 with a pair of ones: the two BF16 values of w added to acc in FP32
inline float bf16_pair_sum(unsigned w, float acc) {
  return acc + (__builtin_bit_cast(float, w << 16) + __builtin_bit_cast(float, w & 0xffff0000u));
}
// v_permlane32_swap + max: the larger of x in lanes l and l ^ 32
inline float max_over_halves(float x) { return std::fmax(x, shim::shfl_xor(x, 32)); }
inline void acc_idle() {}
inline void acc_claim() {}

#endif  // AMLA_TESTS_HIP_RUNTIME_SHIM_H_
