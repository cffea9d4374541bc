/*
 * amla.h -- C ABI of the absorbed-MLA decode attention library for MI355X (gfx950).
 *
 * The operation (Section 2.1 Eq. (1), Section 2.2, Section 3.1 of the AMLA paper): for every
 * query row (b, t, h) -- sequence b, query token t of s_q, head h of num_heads --
 *
 *     s_j   = softmax_scale * sum_{d<576} q[b,t,h,d] * K_b[j,d]          j = 0 .. kv_len[b]-1
 *     out   = sum_j softmax(s)_j * K_b[j, 0:512]
 *     lse   = ln sum_j exp(s_j)
 *
 * where K_b[j,:] is the 576-wide latent+RoPE row of cached token j of sequence b and the
 * value row is its first 512 columns (one shared KV head for all query heads).  All s_q query
 * tokens of a sequence attend to the whole cached prefix; there is no mask among them.
 *
 * The kernels run the FlashAttention recurrence (Algorithm 1) over 64-key cache blocks with
 * the output accumulator held in MFMA accumulator registers.  Rescale variants:
 *   AMLA_RESCALE_MUL  O <- O * 2^(m_old - m_new)            FP32 multiply (Algorithm 1, Eq. (2))
 *   AMLA_RESCALE_ADD  O <- AS_FP32(AS_INT32(O) + (n_new - n_old) * 2^23)
 *                     with the running reference quantised to an integer power of two
 *                     (Eq. (4), Lemma 3.1, Algorithm 2's n_i, N and AtomicAdd<INT32>), the INT32 add
 *                     guarded so that an exponent that would drop to or below zero never yields
 *                     a wrapped bit pattern: such an element (magnitude below 2^-97) becomes a
 *                     signed zero or keeps its value, whichever the kernel's form of the guard gives.
 *   AMLA_RESCALE_ADD_COMP  the ADD variant with the BF16 scale compensation of Algorithm 2
 *                     (S32, S16, c_i, eps) and Appendix A: the weights are 2^(t - m) * S16 with S16 the
 *                     BF16 rounding of S32 = 2^(m - rint(m)), so the largest weight of a row is
 *                     BF16-exact as in Algorithm 1; the same INT32 add then also carries
 *                     rint(2^23 * 1.5 * (c_i / c_{i-1} - 1)), c_i = S16 / S32, which multiplies
 *                     the old accumulator by approximately c_i / c_{i-1} (Appendix A's reading
 *                     of c_i; Algorithm 2 prints the reciprocal).
 *   AMLA_RESCALE_ADD_LDEXP  the ADD variant with the exponent add done by the FP32 ldexp
 *                     instruction (v_ldexp_f32) instead of an INT32 add on the bit pattern: the
 *                     same product x * 2^n wherever Lemma 3.1 applies, zeros, signs and underflow
 *                     handled by the instruction itself.  Transposed-accumulator kernels only.
 *
 * Two kernel families run the path.  The default lays the accumulator out query row by register
 * (second product computed as O = P V): a register then belongs to two query rows, and the rescale
 * touches only the 16 registers of each row whose reference moved in the block.  It works a block as two
 * 32-key halves so that the softmax of one half runs under the MFMAs of the other; the reference follows
 * the running maximum once per 64-key block (MUL, ADD; the first half keeps the previous block's
 * reference while no row has left it by more than 2^8) or per half (ADD_COMP).  The other
 * (AMLA_FLAG_TRANSPOSED_ACC) computes both products transposed, so the rescale factor is a per-lane
 * scalar and every rescale passes over all 256 accumulator registers of the wave; it is kept as the
 * baseline in which the cost of the paper's [V2] stage shows, and carries the lazy and ldexp forms.
 *
 * Every pointer below is a DEVICE pointer unless it says host.  amla_decode allocates no device
 * memory, never synchronises the device, reads no environment variable, and enqueues all work on
 * desc->stream.  The caller owns every buffer.  The only state kept between calls is per device and
 * set up by the first call that needs it: the number of compute units, and the record of which
 * kernels have been allowed their dynamic LDS size.  After that first call a call consists of kernel
 * launches only, so it may be recorded under stream capture (make the first call of a kind outside it).
 */
#ifndef AMLA_H_
#define AMLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  AMLA_OK = 0,
  AMLA_ERR_NULL_ARG = -1,     /* a required pointer is NULL */
  AMLA_ERR_UNSUPPORTED = -2,  /* shape or option outside what the kernels support */
  AMLA_ERR_WORKSPACE = -3,    /* split-KV needs a workspace and it is missing or too small */
  AMLA_ERR_LAUNCH = -4        /* the HIP runtime refused a launch */
};

enum { AMLA_RESCALE_MUL = 0, AMLA_RESCALE_ADD = 1, AMLA_RESCALE_ADD_COMP = 2, AMLA_RESCALE_ADD_LDEXP = 3 };

/* desc->flags */
enum {
  AMLA_FLAG_NO_SKIP = 1,        /* rescale the accumulator on every block even when the factor is 1
                                   (measurement aid: exposes the raw cost of the MUL / ADD rescale) */
  AMLA_FLAG_LAZY_RESCALE = 2,   /* move the reference of the exponent only when the running row max
                                   exceeds it by more than 2^8; in between the softmax weights may
                                   grow up to 2^8 (same relative precision in bf16 and FP32), so the
                                   accumulator rescale becomes a rare event.  Same result up to
                                   rounding.  Transposed-accumulator kernels only (selects them); not
                                   with AMLA_RESCALE_ADD_COMP, whose reference follows the row max by
                                   construction. */
  AMLA_FLAG_BALANCED = 8,       /* decomposition for ragged batches: the 64-key
                                   blocks of all sequences are laid end to end and cut into equal
                                   ranges, one per worker workgroup; a worker walks its range sequence
                                   by sequence, and the pieces of a sequence are merged like split-KV
                                   partials.  desc->num_splits then means the number of workers
                                   (0 = library chooses: one workgroup per compute unit), and the
                                   workspace holds one slot per piece (amla_workspace_bytes answers for
                                   this flag too).  Both kernel families. */
  AMLA_FLAG_CAUSAL = 16,        /* causal mask among the s_q query tokens of a sequence (multi-token
                                   prediction: the s_q tokens are the last s_q positions of the cache):
                                   token t attends to keys 0 .. kv_len - s_q + t, i.e. to
                                   kv_len - (s_q - 1 - t) keys; a token whose limit is <= 0 gets
                                   out = 0, lse = -inf.  Without the flag every token attends to all
                                   kv_len keys.  Runs in the balanced kernels (implies
                                   AMLA_FLAG_BALANCED). */
  AMLA_FLAG_ITERATION_512 = 32, /* one iteration of the recurrence = eight 64-key cache blocks, the 512-key
                                   KV block of Section 4.2: the reference (and with it the accumulator
                                   rescale) moves once per 512 keys of a workgroup's range instead of once
                                   per cache block.  The eight blocks are worked one after the other under
                                   the reference the iteration started with (their weights may exceed 1;
                                   a row whose maximum leaves that reference by more than 2^8 moves it at
                                   once).  Same result up to rounding.  Default (row-rescale) kernels with
                                   AMLA_RESCALE_MUL or AMLA_RESCALE_ADD only. */
  AMLA_FLAG_TRANSPOSED_ACC = 128 /* run the kernels that compute both products transposed (S^T = K Q^T,
                                   O^T = V^T P^T): the accumulator's rescale factor is then a per-lane
                                   scalar and a rescale passes over all 256 accumulator registers of the
                                   wave whenever any of its 32 rows moved.  Same method and roundings as
                                   the default kernels.  These kernels read block-table entries and (in
                                   the equal-share decomposition) lengths as they are, and need finite
                                   values in the cache slots past a sequence's end. */
};

typedef struct amla_desc {
  int32_t batch;               /* B >= 1 */
  int32_t s_q;                 /* query tokens per sequence, >= 1 */
  int32_t num_heads;           /* H >= 1; rows of one sequence are (t, h) flattened: t*H + h */
  int32_t d_qk;                /* must be 576 */
  int32_t d_v;                 /* must be 512 */
  int32_t block_size;          /* keys per cache block, must be 64 */
  int32_t num_blocks;          /* physical blocks in kv_cache */
  int32_t max_blocks_per_seq;  /* row stride of block_table */
  int32_t variant;             /* one of AMLA_RESCALE_* */
  int32_t num_splits;          /* split-KV factor: each sequence's blocks are cut into this many
                                  contiguous ranges processed by separate workgroups and merged
                                  by a combine kernel.  0 = library chooses from the shape; at
                                  most 256. */
  int32_t flags;               /* AMLA_FLAG_* */
  int32_t reserved;            /* must be 0 */
  void* workspace;             /* device scratch for split-KV partials; may be NULL when the
                                  effective split factor is 1 */
  size_t workspace_bytes;      /* size of workspace */
  void* stream;                /* hipStream_t; NULL = the default stream */
  const int32_t* q_lens;       /* device int32 [batch] or NULL.  Not NULL: sequence b has only its first
                                  q_lens[b] (0 .. s_q, clamped into that range) of the s_q query tokens
                                  of the padded q array -- a batch whose sequences carry different
                                  numbers of new tokens.  Sequence b is then the problem with
                                  s_q = q_lens[b] (also for AMLA_FLAG_CAUSAL: token t attends to
                                  kv_len - (q_lens[b] - 1 - t) keys); the rows of its padding tokens are
                                  written as out = 0, lse = -inf.  Runs in the balanced kernels (implies
                                  AMLA_FLAG_BALANCED). */
} amla_desc;

/*
 * amla_decode -- decode attention over a paged latent KV cache (operation above; the loop is
 * Algorithm 1 / Algorithm 2 of the paper per 64-key block, Section 3).
 *
 *   q            bf16 [batch, s_q, num_heads, 576], contiguous, read only
 *   kv_cache     bf16 [num_blocks, 64, 576], contiguous, read only.  Slots past a sequence's end
 *                inside its last block may hold anything (the default kernels clear them on chip
 *                before the value product); with AMLA_FLAG_TRANSPOSED_ACC they must hold finite
 *                values (they are masked, but a NaN there would still poison the value product).
 *   block_table  int32 [batch, max_blocks_per_seq]; entry j of row b is the physical block of
 *                keys 64j .. 64j+63 of sequence b.  Entries j >= ceil(kv_len[b]/64) are never
 *                read.  Entries that are read must lie in [0, num_blocks).  The default kernels
 *                clamp them into that range and lengths into [0, 64 * max_blocks_per_seq] (a wrong
 *                entry then gives a wrong result, not a wild access).
 *   seqlens      int32 [batch], 0 <= kv_len[b] <= 64 * max_blocks_per_seq
 *   softmax_scale  multiplies q.k before the softmax (the paper's 1/sqrt(D_k) generalised);
 *                finite and > 0
 *   out          bf16 [batch, s_q, num_heads, 512], fully overwritten; rows of a sequence with
 *                kv_len 0 are written as 0
 *   lse          f32 [batch, s_q, num_heads] natural-log sum of exponentials, -inf for kv_len 0;
 *                may be NULL when not wanted
 *   desc         host pointer; see amla_desc
 *
 * Returns AMLA_OK or a negative AMLA_ERR_*; never throws, never aborts.  On error nothing
 * has been enqueued.
 *
 * Concurrency: the function may be called from several host threads; calls whose work may run at
 * the same time (different streams) need different `out`, `lse` and `desc->workspace` buffers.
 * The workspace need not be cleared between calls: every partial row that is read has been
 * written by the same call.
 */
int amla_decode(const void* q, const void* kv_cache, const int32_t* block_table,
                const int32_t* seqlens, float softmax_scale, void* out, float* lse,
                const amla_desc* desc);

/*
 * amla_decode_static_workspace -- amla_decode for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels,
 * same result, but the split-KV / balanced partial results go to a fixed array of
 * amla_static_workspace_limit() bytes (128 MiB) that is part of the library's device image -- one per GPU
 * the library runs on, held until the process ends.  desc->workspace and desc->workspace_bytes are
 * ignored.  The call allocates and frees nothing, on the device or through any library; like amla_decode
 * it only enqueues kernels on desc->stream.
 * Returns AMLA_ERR_WORKSPACE, with nothing enqueued, when amla_workspace_bytes(desc) exceeds the limit;
 * AMLA_ERR_LAUNCH when the array's device address cannot be obtained; otherwise what amla_decode returns.
 * All calls on one GPU share that GPU's array: two calls whose kernels overlap in time (different
 * streams, different host threads) race on it; calls on one stream are safe.  The array keeps the last
 * call's contents and nothing in it has to be cleared: every partial row a call reads was written by
 * that same call.
 */
int amla_decode_static_workspace(const void* q, const void* kv_cache, const int32_t* block_table,
                                 const int32_t* seqlens, float softmax_scale, void* out, float* lse,
                                 const amla_desc* desc);

/* Size in bytes of the array amla_decode_static_workspace uses. */
size_t amla_static_workspace_limit(void);

/*
 * amla_workspace_bytes -- bytes of desc->workspace that amla_decode needs for this desc
 * (0 when the effective split factor is 1).  Only shape fields, num_splits and flags are
 * read.  Returns 0 for a NULL or unsupported desc.  The figure is 512 FP32 values and a log-sum-exp
 * per partial row whichever kernels run; the default kernels store their partial rows as FP16 (the
 * rows are normalised, so of the value rows' magnitude, and the merge weights them in FP32) and
 * leave the rest of the range untouched.
 */
size_t amla_workspace_bytes(const amla_desc* desc);

/*
 * amla_effective_splits -- the split-KV factor amla_decode will use for this desc
 * (desc->num_splits if > 0, else the library's choice from batch, rows and
 * max_blocks_per_seq).  Returns 0 for a NULL or unsupported desc.
 */
int amla_effective_splits(const amla_desc* desc);

/*
 * amla_exponent_add -- Lemma 3.1 as the kernels apply it: for each of the n device floats
 * x[i], writes AS_FP32(AS_INT32(x[i]) + delta * 2^23) to y[i] when the biased exponent stays
 * positive and a zero with x[i]'s sign otherwise.  Requires -126 <= delta <= 0.  Runs the
 * same device helper the ADD variant uses on the accumulator registers (test entry point).
 * `stream` is a hipStream_t or NULL.  x and y may alias.
 */
int amla_exponent_add(const float* x, float* y, size_t n, int32_t delta, void* stream);

/*
 * amla_mfma_probe -- measurement support: enqueues `workgroups` workgroups of 4 waves that each run
 * `iters` iterations of four independent register-resident v_mfma_f32_32x32x16_bf16 (no memory
 * traffic), and writes the number of floating-point operations that launch performs to *flops
 * (host).  Timing the launch gives the sustained MFMA rate of the device under its power limit,
 * the measured counterpart of the datasheet peak that utilisation is quoted against (the paper
 * quotes both a theoretical and a throttled peak).  1 <= iters <= 2^22, 1 <= workgroups <= 65535.
 */
int amla_mfma_probe(int32_t iters, int32_t workgroups, double* flops, void* stream);

/*
 * amla_device_info -- measurement support: the number of compute units and the maximum engine clock (kHz) of
 * the current device as the HIP runtime reports them (host pointers).  The datasheet MFMA peak that utilisation
 * is quoted against is compute units x 4096 FLOP per clock x this clock.  AMLA_ERR_LAUNCH when the runtime
 * refuses the query.
 */
int amla_device_info(int32_t* compute_units, int32_t* clock_khz);

/*
 * amla_plan_segments -- host-only view of the balanced decomposition (AMLA_FLAG_BALANCED), computed
 * with the same integer routines the kernels use; for tests and for sizing.  `seqlens` is a HOST
 * array of `batch` lengths.  Writes up to `capacity` pieces as rows of six int32
 * (worker, sequence, first block, end block, workspace slot, covers-whole-sequence) to `pieces`
 * (host) in the order the workers produce them, the number of pieces to *n_pieces, and for every
 * sequence the first and last worker that meet it (as the combine kernel derives them; -1, -1 for
 * an empty sequence) to seq_workers[2 * batch] (host).  Returns AMLA_ERR_WORKSPACE when
 * `capacity` was too small (*n_pieces is still the full count).
 */
int amla_plan_segments(const int32_t* seqlens, int32_t batch, int32_t workers, int32_t* pieces, int32_t capacity,
                       int32_t* n_pieces, int32_t* seq_workers);

/*
 * amla_preload_rotation -- the Cycle of the Preload Pipeline (Section 4.1, Theorem 4.1; Appendix B,
 * Theorem B.3), host only.  For the dependency chain C_1 -> V_1 -> C_2 -> ... -> C_n -> V_n of n
 * matrix ("Cube") and n vector stages with durations cube[i-1], vec[i-1] >= 0 (HOST arrays, any one
 * unit, e.g. cycles; sums below 2^62), finds the cyclic order of the matrix stages in one Cycle of
 * the steady loop under which n - 1 of the C_i -> V_i dependencies stay inside the Cycle and their
 * vector stages still end with it, so that only n stages have to be preloaded.  The rule is the
 * one of the proof: with a_i = V_i - C_{i+1} (C_{n+1} = C_1) and F(l) = a_1 + ... + a_l, take the
 * first l in 1..n that minimises F; the Cycle ends with C_{l+1} and starts with C_{l+2} (cyclic).
 * Writes the 1-based number of the Cycle's first matrix stage to *first_stage, the pair whose
 * C -> V dependency crosses Cycles (the last matrix stage) to *external_pair and the Preload count
 * (= n) to *preload_count.  Requires sum(vec) <= sum(cube) -- the matrix-bound case the theorem is
 * proved for -- and 1 <= n <= 4096; otherwise AMLA_ERR_UNSUPPORTED.  For the chain of this library
 * (n = 2, V_2 = 0) the answer is first_stage 2, external_pair 1, count 2 for any durations: the Cycle
 * [C1, C2, V1] of Section 4.1 in which V1 consumes the previous Cycle's C1.
 */
int amla_preload_rotation(const int64_t* cube, const int64_t* vec, int32_t n, int32_t* first_stage,
                          int32_t* external_pair, int32_t* preload_count);

/* amla_status_string -- static, NUL-terminated description of a status code (host). */
const char* amla_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* AMLA_H_ */
