/*
 * Host-only driver for a -fsanitize=address,undefined build of the C files that tests and benchmarks rely on:
 * the input generator (fgw_gen.c), the attention oracle (fgattn_oracle.c) and the top-p mask oracle
 * (fgmask_oracle.c).  It is compiled together with them (they are #included so that one gcc line builds
 * everything with the sanitizers on) and walks every exported function over small shapes with ragged tails:
 * short last query block, short last key group, every mask kind.  The sanitizers abort on any out-of-bounds
 * access, use of uninitialised heap, signed overflow or misaligned access; the driver itself only checks
 * return codes and that results are finite.
 */
#include <stdio.h>

#include "../paper_2509_16518_amd/workloads/fgw_gen.c"
#define bf16_to_f64 oracle_bf16_to_f64
#include "../oracle/fgattn_oracle.c"
#define bf16_to_f32 mask_bf16_to_f32
#define f32_to_bf16 mask_f32_to_bf16
#include "../oracle/fgmask_oracle.c"

static int run_case(int kind, int heads, int L, int M, int N, int d, int gt, int gh, int gw) {
  fgw_mask_spec s;
  memset(&s, 0, sizeof(s));
  s.kind = kind; s.heads = heads; s.L = L; s.M = M; s.N = N;
  s.gt = gt; s.gh = gh; s.gw = gw; s.dt = 1; s.dh = 2; s.dw = 2;
  s.density = 0.3; s.sigma = 0.6; s.skew = 0.5; s.seed = 77 + kind;
  const int64_t QB = ((int64_t)L + M - 1) / M, G = ((int64_t)L + N - 1) / N, items = heads * QB;
  int64_t* indptr = (int64_t*)malloc(sizeof(int64_t) * (size_t)(items + 1));
  int64_t nnz = fgw_mask_count(&s, indptr);
  if (nnz < 0 || indptr[items] != nnz) return 1;
  int32_t* indices = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
  if (fgw_mask_fill(&s, indptr, indices) != 0) return 2;
  for (int64_t e = 0; e < nnz; e++)
    if (indices[e] < 0 || indices[e] >= G) return 3;
  const int64_t n = (int64_t)heads * L * d;
  uint16_t* q = (uint16_t*)malloc(2 * (size_t)n);
  uint16_t* k = (uint16_t*)malloc(2 * (size_t)n);
  uint16_t* v = (uint16_t*)malloc(2 * (size_t)n);
  fgw_normal_bf16(s.seed, 1, q, n);
  fgw_normal_bf16(s.seed, 2, k, n);
  fgw_normal_bf16(s.seed, 3, v, n);
  int64_t* it = (int64_t*)malloc(sizeof(int64_t) * (size_t)items);
  for (int64_t w = 0; w < items; w++) it[w] = items - 1 - w;
  double* out = (double*)calloc((size_t)(items * M * d), sizeof(double));
  double* lse = (double*)calloc((size_t)(items * M), sizeof(double));
  if (fgattn_oracle_items(q, k, v, heads, L, d, M, N, 0.125, indptr, indices, it, items, out, lse) != 0) return 4;
  for (int64_t x = 0; x < items * M * d; x++)
    if (!isfinite(out[x])) return 5;
  /* an out-of-range id must be refused, not followed */
  if (nnz > 0) {
    const int32_t keep = indices[nnz - 1];
    indices[nnz - 1] = (int32_t)G;
    if (fgattn_oracle_items(q, k, v, heads, L, d, M, N, 0.125, indptr, indices, it, items, out, lse) == 0) return 6;
    indices[nnz - 1] = keep;
  }
  /* top-p mask oracle: block means, then every query block of slice 0 */
  uint16_t* qa = (uint16_t*)malloc(2 * (size_t)(heads * QB * d));
  uint16_t* ka = (uint16_t*)malloc(2 * (size_t)(heads * G * d));
  fgmask_oracle_pool(q, heads, L, d, M, qa);
  fgmask_oracle_pool(k, heads, L, d, N, ka);
  int32_t* order = (int32_t*)malloc(sizeof(int32_t) * (size_t)G);
  double* cum = (double*)malloc(sizeof(double) * (size_t)G);
  for (int64_t i = 0; i < QB; i++) {
    const int32_t kept = fgmask_oracle_row(qa + i * d, ka, (int32_t)G, d, 0.125, 0.9, order, cum);
    if (kept < 1 || kept > G || !(cum[G - 1] > 0.999 && cum[G - 1] < 1.001)) return 7;
  }
  free(indptr); free(indices); free(q); free(k); free(v); free(it); free(out); free(lse);
  free(qa); free(ka); free(order); free(cum);
  return 0;
}

int main(void) {
  int bad = 0;
  for (int kind = 0; kind <= 4; kind++) {
    bad |= run_case(kind, 2, 1000, 16, 1, 64, 10, 10, 10) << 0;   /* short last query block (1000 = 62*16 + 8) */
    bad |= run_case(kind, 1, 1000, 64, 24, 64, 10, 10, 10) << 4;  /* short last key group (1000 = 41*24 + 16) */
    bad |= run_case(kind, 3, 96, 128, 7, 128, 4, 4, 6) << 8;      /* one query block, larger than L */
  }
  bad |= fgattn_oracle_threads() < 1;
  printf(bad ? "sanitize driver: FAILED %d\n" : "sanitize driver: ok\n", bad);
  return bad ? 1 : 0;
}
