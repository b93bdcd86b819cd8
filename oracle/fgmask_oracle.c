/*
 * ORACLE -- test infrastructure, not product.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call this; the product path never does.
 *
 * Plain CPU version of the mean-query/key top-p mask (paper Sec. 4.3 "Determining the
 * Fine-grain Sparse Mask with Top-p Masking"), taking the steps in the paper's order:
 *
 *   1. q_avg(i) = mean of the rows of query block i (M rows; the last block may be short),
 *      k_avg(j) = mean of the rows of key block j   (N rows; the last block may be short).
 *   2. A_hat(i, :) = softmax_j( scale * <q_avg(i), k_avg(j)> )     (paper: scale = 1/sqrt(D)).
 *   3. For each query block i: sort the key blocks by A_hat(i, j), largest first, and keep
 *      the smallest prefix whose cumulative probability is at least p.
 *
 * Readings (the paper is silent): the two pooled tensors are stored in the tensors' own
 * type, bf16 -- the sum of a block is taken in fp32 in row order, divided by the number of
 * rows in fp32 and rounded once to bf16 (nearest even); this fixes, bit for bit, the
 * inputs of step 2 on any implementation.  Steps 2 and 3 are fp64 here.  Equal
 * probabilities are ordered by ascending key-block index.
 *
 * Per query block the oracle reports the kept set and the whole ranking with its
 * cumulative probabilities, so a test can tell an exact match from a set that differs
 * only where the cumulative sum is within rounding of p.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round to nearest even; the inputs here are finite */
static inline uint16_t f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/*
 * Step 1 for one tensor: x [slices, L, d] bf16 bits, blocks of `rows_per_block` rows.
 * pooled [slices, ceil(L/rows_per_block), d] bf16 bits.
 */
void fgmask_oracle_pool(const uint16_t* x, int32_t slices, int32_t L, int32_t d, int32_t rows_per_block,
                        uint16_t* pooled) {
  const int64_t nb = ((int64_t)L + rows_per_block - 1) / rows_per_block;
  for (int64_t s = 0; s < slices; s++)
    for (int64_t b = 0; b < nb; b++) {
      const int64_t r0 = b * rows_per_block;
      const int64_t r1 = r0 + rows_per_block < L ? r0 + rows_per_block : L;
      for (int32_t c = 0; c < d; c++) {
        volatile float acc = 0.0f; /* volatile: every partial sum is rounded to fp32 */
        for (int64_t r = r0; r < r1; r++) acc = acc + bf16_to_f32(x[(s * L + r) * d + c]);
        volatile float mean = acc / (float)(r1 - r0);
        pooled[(s * nb + b) * d + c] = f32_to_bf16(mean);
      }
    }
}

typedef struct {
  double p;
  int32_t j;
} ranked;

static int by_prob_then_index(const void* a, const void* b) {
  const ranked* x = (const ranked*)a;
  const ranked* y = (const ranked*)b;
  if (x->p > y->p) return -1;
  if (x->p < y->p) return 1;
  return (x->j > y->j) - (x->j < y->j);
}

/*
 * Steps 2 and 3 for one query block.
 * q_avg [d], k_avg [G, d]: bf16 bits of the pooled tensors of one slice.
 * order [G]  : key-block ids, most probable first (ties: ascending id).
 * cum   [G]  : cumulative probability along `order` (sequential fp64 sum).
 * returns the number kept: the smallest n with cum[n-1] >= p (G if the sum never reaches p).
 */
int32_t fgmask_oracle_row(const uint16_t* q_avg, const uint16_t* k_avg, int32_t G, int32_t d, double scale, double p,
                          int32_t* order, double* cum) {
  double* s = (double*)malloc(sizeof(double) * (size_t)G);
  ranked* rk = (ranked*)malloc(sizeof(ranked) * (size_t)G);
  if (!s || !rk) {
    free(s);
    free(rk);
    return -1;
  }
  double m = -INFINITY;
  for (int32_t j = 0; j < G; j++) {
    double dot = 0.0;
    for (int32_t c = 0; c < d; c++) dot += (double)bf16_to_f32(q_avg[c]) * (double)bf16_to_f32(k_avg[(int64_t)j * d + c]);
    s[j] = scale * dot;
    if (s[j] > m) m = s[j];
  }
  double z = 0.0;
  for (int32_t j = 0; j < G; j++) z += exp(s[j] - m);
  for (int32_t j = 0; j < G; j++) {
    rk[j].p = exp(s[j] - m) / z;
    rk[j].j = j;
  }
  qsort(rk, (size_t)G, sizeof(ranked), by_prob_then_index);
  int32_t kept = G;
  double c = 0.0;
  for (int32_t t = 0; t < G; t++) {
    c += rk[t].p;
    order[t] = rk[t].j;
    cum[t] = c;
    if (kept == G && c >= p) kept = t + 1;
  }
  free(s);
  free(rk);
  return kept;
}
