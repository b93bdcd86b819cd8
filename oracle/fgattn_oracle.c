/*
 * ORACLE -- test infrastructure, not product.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call this; the product path never does.
 *
 * Plain fp64 CPU definition of what the fine-grained sparse attention forward pass
 * computes.  The method is exact (the approximation lives in the choice of mask, which
 * is an input here), so the oracle is the definition written out:
 *
 *   - Sec. 2 "Efficient dense attention": P = softmax(Q K^T / sqrt(D)), O = P V, with the
 *     sum of exponentials as the normaliser; here the factor 1/sqrt(D) is the argument
 *     `scale`.
 *   - Sec. 2 "Efficient block sparse attention" and Sec. 1: an M x N block of scores is
 *     either computed entirely or skipped entirely; a skipped key takes no part in the
 *     softmax of that query block (equivalent to a score of -infinity).
 *   - Fig. 1b / Sec. 4.1: for each group of M queries only the keys whose indices appear
 *     in the sparse index mask of that group are loaded; the values use the same indices.
 *
 * For work item w = (slice s, query block i), rows r in [i*M, min((i+1)*M, L)):
 *     A      = union over g in indices[indptr[w] : indptr[w+1]] of keys [g*N, min((g+1)*N, L))
 *     s_k    = scale * <q_r, k_k>                      for k in A
 *     lse_r  = m + ln sum_k exp(s_k - m),  m = max_k s_k
 *     out_r  = sum_k exp(s_k - lse_r) * v_k
 * An empty A gives out_r = 0 and lse_r = -infinity.
 *
 * No tiling, no online rescaling, no blocking: per row a two-pass softmax over the whole
 * active set.  bf16 inputs are widened exactly to double.  OpenMP over work items only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_f64(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

int fgattn_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * q, k, v : bf16 bit patterns, [slices, L, d] contiguous (slices = B*H).
 * indptr  : [slices*ceil(L/M) + 1]; indices: key-GROUP ids in [0, ceil(L/N)), no duplicates per item.
 * items   : n_items work-item ids to evaluate (w = slice*ceil(L/M) + i).
 * out     : [n_items, M, d] double; lse: [n_items, M] double.  Rows past L are left untouched.
 * returns 0, or -1 for an out-of-range group id / item id or a failed allocation.
 */
int fgattn_oracle_items(const uint16_t* q, const uint16_t* k, const uint16_t* v, int32_t slices, int32_t L, int32_t d,
                        int32_t M, int32_t N, double scale, const int64_t* indptr, const int32_t* indices,
                        const int64_t* items, int64_t n_items, double* out, double* lse) {
  const int64_t QB = ((int64_t)L + M - 1) / M;
  const int64_t G = ((int64_t)L + N - 1) / N;
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(G * N > 0 ? G * N : 1));
    int64_t* keys = (int64_t*)malloc(sizeof(int64_t) * (size_t)(G * N > 0 ? G * N : 1));
    double* qrow = (double*)malloc(sizeof(double) * (size_t)d);
    if (!s || !keys || !qrow) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int64_t t = 0; t < n_items; t++) {
        int64_t w = items[t];
        if (w < 0 || w >= (int64_t)slices * QB) {
#pragma omp atomic write
          err = 1;
          continue;
        }
        int64_t sl = w / QB, i = w % QB;
        /* active key set A, in list order */
        int64_t na = 0;
        int bad = 0;
        for (int64_t e = indptr[w]; e < indptr[w + 1]; e++) {
          int64_t g = indices[e];
          if (g < 0 || g >= G) { bad = 1; break; }
          for (int64_t key = g * N; key < (g + 1) * N && key < L; key++) keys[na++] = key;
        }
        if (bad) {
#pragma omp atomic write
          err = 1;
          continue;
        }
        const uint16_t* Kb = k + sl * (int64_t)L * d;
        const uint16_t* Vb = v + sl * (int64_t)L * d;
        for (int64_t r = i * M; r < (i + 1) * M && r < L; r++) {
          const uint16_t* qr = q + (sl * (int64_t)L + r) * d;
          double* o = out + (t * M + (r - i * M)) * d;
          for (int c = 0; c < d; c++) { qrow[c] = bf16_to_f64(qr[c]); o[c] = 0.0; }
          if (na == 0) { lse[t * M + (r - i * M)] = -INFINITY; continue; }
          double m = -INFINITY;
          for (int64_t a = 0; a < na; a++) {
            const uint16_t* kr = Kb + keys[a] * d;
            double dot = 0.0;
            for (int c = 0; c < d; c++) dot += qrow[c] * bf16_to_f64(kr[c]);
            s[a] = scale * dot;
            if (s[a] > m) m = s[a];
          }
          double sum = 0.0;
          for (int64_t a = 0; a < na; a++) sum += exp(s[a] - m);
          double l = m + log(sum);
          lse[t * M + (r - i * M)] = l;
          for (int64_t a = 0; a < na; a++) {
            double p = exp(s[a] - l);
            const uint16_t* vr = Vb + keys[a] * d;
            for (int c = 0; c < d; c++) o[c] += p * bf16_to_f64(vr[c]);
          }
        }
      }
    }
    free(s);
    free(keys);
    free(qrow);
  }
  return err ? -1 : 0;
}
