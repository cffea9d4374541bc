// Absorbed-MLA decode attention for gfx950 (MI355X): the C-ABI entry points, the host side (argument checks,
// split choice, dispatch) and the kernels that keep the output accumulator transposed.
//
// Two kernel families run the same path (paged KV gather -> [C1] S = Q K^T -> [V1] online softmax -> [V2]
// rescale -> [C2] O += P V -> epilogue; Algorithm 1 / Algorithm 2 per 64-key block):
//   * the row-rescale kernels of amla_decode_rg.hip, the default: second product computed as O = P V, so a
//     register of the accumulator belongs to two query rows and the rescale touches only rows whose reference
//     moved;
//   * the kernels below (AMLA_FLAG_TRANSPOSED_ACC, and the lazy and ldexp variants, which exist here only):
//     both products transposed, S^T = K Q^T and O^T = V^T P^T, so every register of a lane belongs to query
//     row lane % 32, the rescale factor is a per-lane scalar, and a rescale passes over all 256 accumulator
//     registers whenever any of the wave's 32 rows moved -- the cost of the paper's [V2] stage as it appears on
//     this hardware, kept as the baseline the row-rescale kernels are measured against.
// Device code of this file: amla_decode_kernels.inc (kernels, included below), amla_decode_equal_share.inc
// (the equal-share kernel), amla_decode_piece.inc (the body of the decode loop, shared by the equal-share and
// the balanced kernels), amla_decode_balanced.inc (the balanced walk); amla_plan.h holds the balanced
// decomposition's integer arithmetic; amla_device.h what both families share.
//
// One workgroup (4 waves, one per SIMD, up to 512 registers each) owns 128 query rows of one sequence and a
// contiguous range of that sequence's 64-key cache blocks.  Wave w owns rows 32 w .. 32 w + 31 and keeps, for
// those rows, the whole Q fragment (144 VGPRs) and the whole 32 x 512 FP32 output accumulator (256 registers)
// resident for the entire loop, so the accumulator never leaves the register file (the data movement that the
// paper's Section 3.1 identifies as the bottleneck of the [V2] stage does not exist here).  The KV block is
// brought HBM -> LDS by direct-to-LDS loads (global_load_lds_dwordx4), double buffered.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "amla.h"
#include "amla_device.h"
#include "amla_plan.h"

namespace {

#include "amla_decode_kernels.inc"

constexpr int kMaxDevices = 64;

// The decode kernels use more dynamic LDS than a launch may ask for by default; the attribute that
// allows it is set once per kernel and device, on the first call, so that later calls (for instance
// under stream capture) consist of launches only.
constexpr int kMaxDecodeKernels = 64;
const void* g_lds_ok[kMaxDevices][kMaxDecodeKernels];
std::mutex g_lds_ok_mutex;

bool allow_large_lds(const void* kernel, int lds_bytes = kLdsBytes) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  std::lock_guard<std::mutex> lock(g_lds_ok_mutex);
  int n = 0;
  for (; n < kMaxDecodeKernels && g_lds_ok[dev][n] != nullptr; ++n)
    if (g_lds_ok[dev][n] == kernel) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if (n < kMaxDecodeKernels) g_lds_ok[dev][n] = kernel;
  return true;
}

// Compute units of the current device, read once per device.
int g_cu_count[kMaxDevices];
std::mutex g_cu_count_mutex;
int device_cu_count() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  std::lock_guard<std::mutex> lock(g_cu_count_mutex);
  if (g_cu_count[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
      (void)hipGetLastError();
      n = 256;
    }
    g_cu_count[dev] = n;
  }
  return g_cu_count[dev];
}

// Workspace of amla_decode_static_workspace: one array per device, part of the loaded code object, held until
// the process ends.  In host code the array's name is only a stand-in for the symbol; its device address is
// asked for once per device, with that device current, and used from then on.
constexpr size_t kStaticWorkspaceBytes = (size_t)128 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

void* static_workspace() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// The causal mask and the per-sequence query counts live in the balanced kernels only, so they select them.
bool uses_balanced(const amla_desc* d) {
  return (d->flags & (AMLA_FLAG_BALANCED | AMLA_FLAG_CAUSAL)) != 0 || d->q_lens != nullptr;
}

// The lazy reference and the ldexp variant exist in the transposed-accumulator kernels only.
bool uses_transposed(const amla_desc* d) {
  return (d->flags & (AMLA_FLAG_TRANSPOSED_ACC | AMLA_FLAG_LAZY_RESCALE)) != 0 || d->variant == AMLA_RESCALE_ADD_LDEXP;
}

bool desc_supported(const amla_desc* d) {
  if (d == nullptr) return false;
  if (d->d_qk != kDqk || d->d_v != kDv || d->block_size != kBlock) return false;
  if (d->batch < 1 || d->s_q < 1 || d->num_heads < 1 || d->num_blocks < 1 || d->max_blocks_per_seq < 1) return false;
  if (d->variant != AMLA_RESCALE_MUL && d->variant != AMLA_RESCALE_ADD && d->variant != AMLA_RESCALE_ADD_COMP &&
      d->variant != AMLA_RESCALE_ADD_LDEXP)
    return false;
  if (d->num_splits < 0 || d->num_splits > 256 || d->reserved != 0) return false;
  if ((d->flags & ~(AMLA_FLAG_NO_SKIP | AMLA_FLAG_LAZY_RESCALE | AMLA_FLAG_BALANCED | AMLA_FLAG_CAUSAL |
                    AMLA_FLAG_ITERATION_512 | AMLA_FLAG_TRANSPOSED_ACC)) != 0)
    return false;
  // the 512-key iteration exists in the row-rescale kernels, for the variants whose reference may lag
  if ((d->flags & AMLA_FLAG_ITERATION_512) &&
      (uses_transposed(d) || (d->variant != AMLA_RESCALE_MUL && d->variant != AMLA_RESCALE_ADD)))
    return false;
  // ldexp rescale with the balanced decomposition does not exist (the compiler's AGPR-copy rewrite pass
  // crashes on that instantiation of the transposed-accumulator kernels)
  if (d->variant == AMLA_RESCALE_ADD_LDEXP && uses_balanced(d)) return false;
  // the compensated reference follows the row max by construction: no lazy form
  if (d->variant == AMLA_RESCALE_ADD_COMP && (d->flags & AMLA_FLAG_LAZY_RESCALE)) return false;
  if ((long long)d->batch * d->max_blocks_per_seq > (1ll << 31) - 1) return false;
  const long long rows = (long long)d->s_q * d->num_heads;
  if (rows > (1 << 20) || (long long)d->batch * rows > (1ll << 31) - 1) return false;
  return true;
}

int choose_splits(const amla_desc* d) {
  if (d->num_splits > 0) return d->num_splits;
  const long long rows = (long long)d->s_q * d->num_heads;
  const long long tiles = (rows + kRowsPerWg - 1) / kRowsPerWg;
  const long long cus = device_cu_count();
  if (uses_balanced(d)) {
    // workers: one workgroup per CU over all row tiles, never more workers than blocks can exist
    long long w = cus / tiles > 0 ? cus / tiles : 1;
    const long long most = (long long)d->batch * d->max_blocks_per_seq;
    if (w > most) w = most;
    if (w > 256) w = 256;
    return (int)w;
  }
  // Equal shares: the split factor that a small cost model likes best, in units of one 64-key block of one
  // workgroup.  A workgroup costs its share of the longest possible sequence plus a fixed part (prologue,
  // epilogue; more when it writes FP32 partial rows); the workgroups run in rounds of one per compute unit; the
  // combine kernel costs a little per split.  At least four blocks per share, at most 64 shares.  (Measured at
  // batch 96, two tokens, 4096 keys: 281 us unsplit, 320 us in two shares, 343 us in four -- 192 workgroups
  // on 256 compute units are better left alone than cut into one and a half rounds.)
  const long long base = (long long)d->batch * tiles;       // workgroups without splitting
  if (base >= cus) return 1;
  const long long blocks = d->max_blocks_per_seq > 0 ? d->max_blocks_per_seq : 1;
  long long cap = blocks / 4 > 0 ? blocks / 4 : 1;
  if (cap > 64) cap = 64;
  long long best = 1, best_cost = 0;
  for (long long ns = 1; ns <= cap; ++ns) {
    const long long rounds = (base * ns + cus - 1) / cus;
    const long long share = (blocks + ns - 1) / ns;
    // tenths of a block: fixed part 4.0 (6.0 with partial rows), combine 1.0 + 0.6 per share
    const long long cost = rounds * (10 * share + (ns > 1 ? 60 : 40)) + (ns > 1 ? 10 + 6 * ns : 0);
    if (ns == 1 || cost < best_cost) {
      best = ns;
      best_cost = cost;
    }
  }
  return (int)best;
}

// Everything a call enqueues, shared by amla_decode and its variants: the decode kernel of the selected
// family and decomposition, then the combine kernel where pieces have to be merged.  `workspace` holds
// amla_workspace_bytes(desc) bytes (checked by the caller).
int enqueue_decode(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* seqlens,
                   float softmax_scale, void* out, float* lse, const amla_desc* desc, void* workspace, int ns) {
  const bool balanced = uses_balanced(desc);
  DecodeParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.kv = static_cast<const uint16_t*>(kv_cache);
  p.table = block_table;
  p.seqlens = seqlens;
  p.out = static_cast<uint16_t*>(out);
  p.lse = lse;
  p.batch = desc->batch;
  p.rows = desc->s_q * desc->num_heads;
  p.n_tiles = (p.rows + kRowsPerWg - 1) / kRowsPerWg;
  p.n_splits = ns;
  p.max_blocks = desc->max_blocks_per_seq;
  p.n_streams = balanced ? ns : desc->batch * ns;
  p.flags = desc->flags;
  p.num_blocks = desc->num_blocks;
  p.heads = desc->num_heads;
  p.causal_span = (desc->flags & AMLA_FLAG_CAUSAL) ? desc->s_q - 1 : 0;
  p.s_q = desc->s_q;
  p.q_lens = desc->q_lens;
  p.scale_log2e = softmax_scale * 1.4426950408889634f;
  const size_t n_rows = (size_t)desc->batch * p.rows;
  p.part_o = (ns > 1 || balanced) ? static_cast<float*>(workspace) : nullptr;
  p.part_lse = ns > 1 ? p.part_o + (size_t)ns * n_rows * kDv : nullptr;
  if (balanced) p.part_lse = p.part_o + ((size_t)ns + desc->batch - 1) * p.rows * kDv;

  hipStream_t stream = static_cast<hipStream_t>(desc->stream);
  const long long streams_pad = ((long long)p.n_streams + 7) / 8 * 8;
  // (the equal-share row-rescale kernels deal sequences, not streams, over the 8 XCDs: the batch is padded)
  const long long grid = (!uses_transposed(desc) && !balanced ? ((long long)desc->batch + 7) / 8 * 8 * ns : streams_pad) * p.n_tiles;
  if (grid > 0x7fffffffll) return AMLA_ERR_UNSUPPORTED;
  const bool lazy = (desc->flags & AMLA_FLAG_LAZY_RESCALE) != 0;
  AmlaDecodeKernel kern = nullptr;
  int lds_bytes = kLdsBytes;
  if (!uses_transposed(desc)) {
    kern = amla_row_rescale_kernel(desc->variant, balanced, (desc->flags & AMLA_FLAG_ITERATION_512) != 0);
    lds_bytes = amla_row_rescale_lds_bytes();
  } else if (!balanced) {
    kern = desc->variant == AMLA_RESCALE_ADD_COMP ? amla_decode_kernel<AMLA_RESCALE_ADD_COMP, false>
           : desc->variant == AMLA_RESCALE_ADD_LDEXP
               ? (lazy ? amla_decode_kernel<AMLA_RESCALE_ADD_LDEXP, true> : amla_decode_kernel<AMLA_RESCALE_ADD_LDEXP, false>)
           : desc->variant == AMLA_RESCALE_ADD
               ? (lazy ? amla_decode_kernel<AMLA_RESCALE_ADD, true> : amla_decode_kernel<AMLA_RESCALE_ADD, false>)
               : (lazy ? amla_decode_kernel<AMLA_RESCALE_MUL, true> : amla_decode_kernel<AMLA_RESCALE_MUL, false>);
  } else {
    kern = desc->variant == AMLA_RESCALE_ADD_COMP ? amla_decode_balanced_kernel<AMLA_RESCALE_ADD_COMP, false>
           : desc->variant == AMLA_RESCALE_ADD     ? (lazy ? amla_decode_balanced_kernel<AMLA_RESCALE_ADD, true>
                                                             : amla_decode_balanced_kernel<AMLA_RESCALE_ADD, false>)
                                                   : (lazy ? amla_decode_balanced_kernel<AMLA_RESCALE_MUL, true>
                                                           : amla_decode_balanced_kernel<AMLA_RESCALE_MUL, false>);
  }
  if (!allow_large_lds(reinterpret_cast<const void*>(kern), lds_bytes)) return AMLA_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds_bytes, stream, p);
  if (hipGetLastError() != hipSuccess) return AMLA_ERR_LAUNCH;
  if (balanced) {
    // (the row-rescale kernels leave their partial rows in FP16, the transposed-accumulator kernels in FP32)
    const auto combine = uses_transposed(desc) ? amla_combine_balanced_kernel<false> : amla_combine_balanced_kernel<true>;
    hipLaunchKernelGGL(combine, dim3((unsigned)n_rows), dim3(128), 0, stream, p.part_o,
                       p.part_lse, p.seqlens, p.out, p.lse, p.batch, p.rows, ns, p.max_blocks);
    if (hipGetLastError() != hipSuccess) return AMLA_ERR_LAUNCH;
  } else if (ns > 1) {
    const auto combine = uses_transposed(desc) ? amla_combine_kernel<false> : amla_combine_kernel<true>;
    hipLaunchKernelGGL(combine, dim3((unsigned)n_rows), dim3(128), 0, stream, p.part_o, p.part_lse,
                       p.out, p.lse, (int)n_rows, ns);
    if (hipGetLastError() != hipSuccess) return AMLA_ERR_LAUNCH;
  }
  return AMLA_OK;
}

// the argument checks every decode entry point makes
int check_decode_args(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* seqlens,
                      float softmax_scale, void* out, const amla_desc* desc) {
  if (q == nullptr || kv_cache == nullptr || block_table == nullptr || seqlens == nullptr || out == nullptr ||
      desc == nullptr)
    return AMLA_ERR_NULL_ARG;
  if (!desc_supported(desc)) return AMLA_ERR_UNSUPPORTED;
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale)) return AMLA_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(kv_cache) | reinterpret_cast<uintptr_t>(out)) & 15)
    return AMLA_ERR_UNSUPPORTED;
  return AMLA_OK;
}

}  // namespace

extern "C" {

int amla_effective_splits(const amla_desc* desc) {
  if (!desc_supported(desc)) return 0;
  return choose_splits(desc);
}

size_t amla_workspace_bytes(const amla_desc* desc) {
  if (!desc_supported(desc)) return 0;
  const int ns = choose_splits(desc);
  if (uses_balanced(desc)) {
    // one slot of s_q * num_heads partial rows per (worker, sequence) piece: slot ids < workers + batch - 1
    const size_t slots = (size_t)ns + desc->batch - 1;
    return slots * desc->s_q * desc->num_heads * (kDv + 1) * sizeof(float);
  }
  if (ns <= 1) return 0;
  const size_t rows = (size_t)desc->batch * desc->s_q * desc->num_heads;
  return (size_t)ns * rows * (kDv + 1) * sizeof(float);
}

int amla_decode(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* seqlens,
                float softmax_scale, void* out, float* lse, const amla_desc* desc) {
  const int bad = check_decode_args(q, kv_cache, block_table, seqlens, softmax_scale, out, desc);
  if (bad != AMLA_OK) return bad;
  const int ns = choose_splits(desc);
  const size_t need = amla_workspace_bytes(desc);
  if (need > 0) {
    if (desc->workspace == nullptr || desc->workspace_bytes < need) return AMLA_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(desc->workspace) & 15) return AMLA_ERR_WORKSPACE;
  }
  return enqueue_decode(q, kv_cache, block_table, seqlens, softmax_scale, out, lse, desc, desc->workspace, ns);
}

int amla_decode_static_workspace(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* seqlens,
                                 float softmax_scale, void* out, float* lse, const amla_desc* desc) {
  const int bad = check_decode_args(q, kv_cache, block_table, seqlens, softmax_scale, out, desc);
  if (bad != AMLA_OK) return bad;
  const int ns = choose_splits(desc);
  const size_t need = amla_workspace_bytes(desc);
  if (need > kStaticWorkspaceBytes) return AMLA_ERR_WORKSPACE;
  void* base = nullptr;
  if (need > 0) {
    base = static_workspace();
    if (base == nullptr) return AMLA_ERR_LAUNCH;
  }
  return enqueue_decode(q, kv_cache, block_table, seqlens, softmax_scale, out, lse, desc, base, ns);
}

size_t amla_static_workspace_limit(void) { return kStaticWorkspaceBytes; }

int amla_exponent_add(const float* x, float* y, size_t n, int32_t delta, void* stream) {
  if (x == nullptr || y == nullptr) return AMLA_ERR_NULL_ARG;
  if (delta > 0 || delta < -126) return AMLA_ERR_UNSUPPORTED;
  if (n == 0) return AMLA_OK;
  const size_t blocks = (n + 255) / 256;
  if (blocks > 0x7fffffffull) return AMLA_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(amla_exponent_add_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), x, y, n, delta * (1 << 23));
  return hipGetLastError() == hipSuccess ? AMLA_OK : AMLA_ERR_LAUNCH;
}

int amla_mfma_probe(int32_t iters, int32_t workgroups, double* flops, void* stream) {
  if (flops == nullptr) return AMLA_ERR_NULL_ARG;
  if (iters < 1 || iters > (1 << 22) || workgroups < 1 || workgroups > 65535) return AMLA_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(amla_mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(nullptr), iters);
  if (hipGetLastError() != hipSuccess) return AMLA_ERR_LAUNCH;
  // 4 waves per workgroup, 4 MFMAs of 32 x 32 x 16 multiply-adds per iteration and wave
  *flops = (double)iters * 4.0 * 4.0 * (2.0 * 32 * 32 * 16) * (double)workgroups;
  return AMLA_OK;
}

int amla_device_info(int32_t* compute_units, int32_t* clock_khz) {
  if (compute_units == nullptr || clock_khz == nullptr) return AMLA_ERR_NULL_ARG;
  int dev = -1, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) {
    (void)hipGetLastError();
    return AMLA_ERR_LAUNCH;
  }
  *compute_units = cus;
  *clock_khz = khz;
  return AMLA_OK;
}

int amla_plan_segments(const int32_t* seqlens, int32_t batch, int32_t workers, int32_t* pieces, int32_t capacity,
                       int32_t* n_pieces, int32_t* seq_workers) {
  if (seqlens == nullptr || pieces == nullptr || n_pieces == nullptr || seq_workers == nullptr) return AMLA_ERR_NULL_ARG;
  if (batch < 1 || workers < 1 || capacity < 0) return AMLA_ERR_UNSUPPORTED;
  long long total = 0;
  for (int b = 0; b < batch; ++b) {
    if (seqlens[b] < 0) return AMLA_ERR_UNSUPPORTED;
    total += plan_blocks_of(seqlens[b], kBlock);
  }
  if (total > (1ll << 31) - 1) return AMLA_ERR_UNSUPPORTED;
  int n = 0;
  for (int w = 0; w < workers; ++w) {
    const long long g0 = plan_worker_begin(w, total, workers), g1 = plan_worker_begin(w + 1, total, workers);
    if (g0 >= g1) continue;
    // the sequence that holds global block g0 (the kernel finds it with a wave-wide scan)
    long long base = 0;
    int b0 = 0;
    while (base + plan_blocks_of(seqlens[b0], kBlock) <= g0) base += plan_blocks_of(seqlens[b0++], kBlock);
    PlanWalk walk = {b0, (int32_t)(g0 - base), g1 - g0};
    while (walk.left > 0 && walk.b < batch) {
      PlanPiece piece;
      if (!plan_next(&walk, plan_blocks_of(seqlens[walk.b], kBlock), &piece)) continue;
      if (n < capacity) {
        int32_t* row = pieces + 6 * (size_t)n;
        row[0] = w; row[1] = piece.b; row[2] = piece.j0; row[3] = piece.j1; row[4] = w + piece.b; row[5] = piece.full;
      }
      ++n;
    }
  }
  *n_pieces = n;
  // what the combine kernel derives for each sequence: first and last worker that meet it (-1, -1 if empty)
  long long before = 0;
  for (int b = 0; b < batch; ++b) {
    const int nb = plan_blocks_of(seqlens[b], kBlock);
    seq_workers[2 * b] = nb > 0 ? (int32_t)plan_worker_of_block(before, total, workers) : -1;
    seq_workers[2 * b + 1] = nb > 0 ? (int32_t)plan_worker_of_block(before + nb - 1, total, workers) : -1;
    before += nb;
  }
  return n <= capacity ? AMLA_OK : AMLA_ERR_WORKSPACE;
}

// Theorem B.3's construction: the rotation sits at the minimum of the partial sums of
// a_i = V_i - C_{i+1}.
int amla_preload_rotation(const int64_t* cube, const int64_t* vec, int32_t n, int32_t* first_stage,
                          int32_t* external_pair, int32_t* preload_count) {
  if (cube == nullptr || vec == nullptr || first_stage == nullptr || external_pair == nullptr ||
      preload_count == nullptr)
    return AMLA_ERR_NULL_ARG;
  if (n < 1 || n > 4096) return AMLA_ERR_UNSUPPORTED;
  const int64_t limit = (int64_t)1 << 62;
  int64_t sum_c = 0, sum_v = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (cube[i] < 0 || vec[i] < 0 || cube[i] >= limit - sum_c || vec[i] >= limit - sum_v) return AMLA_ERR_UNSUPPORTED;
    sum_c += cube[i];
    sum_v += vec[i];
  }
  if (sum_v > sum_c) return AMLA_ERR_UNSUPPORTED;
  int64_t f = 0, best = 0;
  int32_t arg = 0;
  for (int32_t l = 1; l <= n; ++l) {
    f += vec[l - 1] - cube[l % n];  // a_l
    if (arg == 0 || f < best) {
      best = f;
      arg = l;
    }
  }
  const int32_t last = arg % n + 1;  // C_{l+1}
  *external_pair = last;
  *first_stage = last % n + 1;
  *preload_count = n;
  return AMLA_OK;
}

const char* amla_status_string(int status) {
  switch (status) {
    case AMLA_OK: return "ok";
    case AMLA_ERR_NULL_ARG: return "a required pointer is NULL";
    case AMLA_ERR_UNSUPPORTED: return "unsupported shape, option, scale or pointer alignment";
    case AMLA_ERR_WORKSPACE: return "split-KV workspace missing, misaligned or too small";
    case AMLA_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
