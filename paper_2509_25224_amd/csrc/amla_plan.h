// Work decomposition for ragged batches: the 64-key cache blocks of all sequences of a batch are
// laid end to end (sequence 0's blocks, then sequence 1's, ...) and cut into W contiguous worker
// ranges of equal length.  A worker walks its range sequence by sequence; every (worker, sequence)
// pair it touches is a *piece* with its own softmax state, and pieces of one sequence are merged
// afterwards exactly like split-KV partials (the merge rule of Algorithm 1's update).  This file
// holds the integer arithmetic shared by the decode kernel, the combine kernel and the host-side
// test entry point, so that all three agree on who owns which block and which slot.
//
// Facts used by the callers (checked by the CPU tests through amla_plan_segments):
//   * worker w owns global blocks [plan_worker_begin(w), plan_worker_begin(w + 1));
//   * plan_worker_of_block(g) is the one worker whose range holds g;
//   * the pieces of a batch, taken in (worker, sequence) order, have strictly increasing slot
//     ids w + b (from one piece to the next either the worker or the sequence advances), so
//     slots are unique and < W + B - 1;
//   * a piece is *full* when it covers its whole sequence; then and only then the sequence has a
//     single piece, which writes the final result itself.
#ifndef AMLA_PLAN_H_
#define AMLA_PLAN_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define AMLA_PLAN_FN __host__ __device__ inline
#else
#define AMLA_PLAN_FN inline
#endif

// first global block of worker w (w may be W: one past the last worker's range), T blocks in total
AMLA_PLAN_FN int64_t plan_worker_begin(int64_t w, int64_t T, int64_t W) { return w * T / W; }

// the worker whose range holds global block g, 0 <= g < T: the largest w with w T / W <= g
AMLA_PLAN_FN int64_t plan_worker_of_block(int64_t g, int64_t T, int64_t W) { return ((g + 1) * W - 1) / T; }

AMLA_PLAN_FN int32_t plan_blocks_of(int32_t kv_len, int32_t block) { return (kv_len + block - 1) / block; }

// a length as the balanced kernels read it: inside the documented range [0, block * max_blocks] even
// if the caller's array is not, so that no block-table entry outside a sequence's row is touched
AMLA_PLAN_FN int32_t plan_len(int32_t kv_len, int32_t max_blocks, int32_t block) {
  const int64_t most = (int64_t)max_blocks * block;
  return kv_len < 0 ? 0 : (kv_len > most ? (int32_t)(most > 0x7fffffff ? 0x7fffffff : most) : kv_len);
}

// One piece of a worker's walk.
struct PlanPiece {
  int32_t b;       // sequence
  int32_t j0, j1;  // its blocks [j0, j1) of the sequence, j0 < j1
  int32_t full;    // covers the whole sequence
};

// State of a worker's walk over its range.  `b` is the current sequence, `j` the next block of it,
// `left` the blocks still to process.  plan_next() returns the next piece and advances, skipping
// sequences without blocks; it must only be called while left > 0.  `nb_of(b)` is supplied by the
// caller as the array of block counts would cost registers on the device: the caller passes the
// block count of sequence `b` and is asked again (return value 0, b advanced) when that
// sequence is exhausted or empty.
struct PlanWalk {
  int32_t b, j;
  int64_t left;
};

// Tries to take a piece from sequence w->b which has nb blocks.  Returns 1 and fills *piece when one
// was taken; returns 0 when the sequence has nothing left (w->b was advanced, ask again with the
// next sequence's block count).
AMLA_PLAN_FN int plan_next(PlanWalk* w, int32_t nb, PlanPiece* piece) {
  if (w->j >= nb) {
    w->b += 1;
    w->j = 0;
    return 0;
  }
  const int64_t avail = (int64_t)nb - w->j;
  const int64_t take = avail < w->left ? avail : w->left;
  piece->b = w->b;
  piece->j0 = w->j;
  piece->j1 = (int32_t)(w->j + take);
  piece->full = (piece->j0 == 0 && piece->j1 == nb) ? 1 : 0;
  w->left -= take;
  w->j = piece->j1;
  return 1;
}

#endif  // AMLA_PLAN_H_
