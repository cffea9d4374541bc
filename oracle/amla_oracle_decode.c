/*
 * amla_oracle_decode -- the CPU oracle's definition of absorbed-MLA decode attention as plain C with host
 * pointers, in the argument order of the library's decode entry point.  TEST INFRASTRUCTURE ONLY: it shares no
 * code, header or constant with the HIP path, and only tests, the smoke check and the benchmark's CPU-baseline
 * leg may load it.
 *
 * What it computes is Eq. (1): out = softmax(scale * q K^T) V per query row, with K the 576-wide cached row and
 * V its first 512 columns (Section 2.2, Section 3.1: D_k = 576, D_v = 512), over the exact values of the BF16
 * inputs, in double precision, as the two-pass safe softmax (row maximum first, then exponentials and sums;
 * no blocking, no recurrence), plus lse = max + ln(sum).  Conventions outside the paper: logical key j of
 * sequence b lives in physical block block_table[b][j / 64], slot j % 64; a row without keys is out = 0,
 * lse = -inf; with `causal` the s_q (or q_lens[b]) query tokens are the last positions of the cache and token t
 * sees the first kv_len - (count - 1 - t) keys; tokens t >= q_lens[b] are padding: out = 0, lse = -inf.
 *
 * Arguments (all HOST memory, caller-owned):
 *   q            uint16 BF16 bit patterns [batch, s_q, num_heads, 576]
 *   kv_cache     uint16 BF16 bit patterns [num_blocks, 64, 576]
 *   block_table  int32 [batch, max_blocks_per_seq]; entries past a sequence's last block are not read
 *   seqlens      int32 [batch], 0 <= seqlens[b] <= 64 * max_blocks_per_seq
 *   out          double [batch, s_q, num_heads, 512], not rounded
 *   lse          double [batch, s_q, num_heads], natural logarithm
 * Returns 0, or -1 for a null pointer or non-positive size, -2 for a length outside its range, -3 for a block
 * id that is read and lies outside [0, num_blocks), -4 for a q_lens entry outside [0, s_q].  Nothing is
 * written after an error is found in a sequence; sequences before it are complete.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t batch, s_q, num_heads;
  int32_t num_blocks, max_blocks_per_seq;
  int32_t causal;          /* 0: every token sees all kv_len keys */
  const int32_t* q_lens;   /* int32 [batch] or NULL = s_q tokens everywhere */
} amla_oracle_shape;

enum { D_QK = 576, D_V = 512, BLOCK = 64 };

static double bf16_value(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

int amla_oracle_decode(const uint16_t* q, const uint16_t* kv_cache, const int32_t* block_table,
                       const int32_t* seqlens, float softmax_scale, double* out, double* lse,
                       const amla_oracle_shape* shape) {
  if (!q || !kv_cache || !block_table || !seqlens || !out || !lse || !shape) return -1;
  const int B = shape->batch, T = shape->s_q, H = shape->num_heads;
  if (B <= 0 || T <= 0 || H <= 0 || shape->num_blocks <= 0 || shape->max_blocks_per_seq <= 0) return -1;
  const double scale = (double)softmax_scale;
  for (int b = 0; b < B; ++b) {
    const int L = seqlens[b];
    if (L < 0 || (int64_t)L > (int64_t)BLOCK * shape->max_blocks_per_seq) return -2;
    const int Tb = shape->q_lens ? shape->q_lens[b] : T;
    if (Tb < 0 || Tb > T) return -4;
    for (int j = 0; j < L; j += BLOCK) {
      const int32_t id = block_table[(size_t)b * shape->max_blocks_per_seq + j / BLOCK];
      if (id < 0 || id >= shape->num_blocks) return -3;
    }
    double* s = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    if (!s) return -1;
    for (int t = 0; t < T; ++t) {
      for (int h = 0; h < H; ++h) {
        const size_t row = ((size_t)b * T + t) * H + h;
        double* o = out + row * D_V;
        for (int d = 0; d < D_V; ++d) o[d] = 0.0;
        int keys = 0;
        if (t < Tb) {
          keys = shape->causal ? L - (Tb - 1 - t) : L;
          if (keys < 0) keys = 0;
        }
        if (keys == 0) {
          lse[row] = -INFINITY;
          continue;
        }
        const uint16_t* qr = q + row * D_QK;
        /* pass 1: logits and their maximum */
        double m = -INFINITY;
        for (int j = 0; j < keys; ++j) {
          const int32_t id = block_table[(size_t)b * shape->max_blocks_per_seq + j / BLOCK];
          const uint16_t* kr = kv_cache + ((size_t)id * BLOCK + j % BLOCK) * D_QK;
          double dot = 0.0;
          for (int d = 0; d < D_QK; ++d) dot += bf16_value(qr[d]) * bf16_value(kr[d]);
          s[j] = dot * scale;
          if (s[j] > m) m = s[j];
        }
        /* pass 2: weights, their sum, the weighted sum of the value rows */
        double z = 0.0;
        for (int j = 0; j < keys; ++j) {
          const int32_t id = block_table[(size_t)b * shape->max_blocks_per_seq + j / BLOCK];
          const uint16_t* vr = kv_cache + ((size_t)id * BLOCK + j % BLOCK) * D_QK;   /* V = first 512 columns */
          const double p = exp(s[j] - m);
          z += p;
          for (int d = 0; d < D_V; ++d) o[d] += p * bf16_value(vr[d]);
        }
        for (int d = 0; d < D_V; ++d) o[d] /= z;
        lse[row] = m + log(z);
      }
    }
    free(s);
  }
  return 0;
}
