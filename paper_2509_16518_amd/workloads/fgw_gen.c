/*
 * Seeded synthetic inputs for the fine-grained sparse attention path: bf16 N(0,1)
 * tensors and CSR masks of active key groups per (head, query block).
 *
 * This file holds input generation only.  It contains no attention arithmetic and is
 * shared by the CPU oracle's tests and the GPU path's tests/benchmarks so both see the
 * same bits.  Everything is a pure function of (seed, coordinates): a counter-based
 * generator, so any element or any mask row can be regenerated on its own.
 *
 * Mask kinds (the synthetic stand-ins for video-DiT attention masks, which are local in
 * space-time yet irregular -- paper Sec. 4.3 first paragraph and Fig. 2a caption -- and
 * for the random masks of the micro-benchmark in Sec. 5.1):
 *   FGW_MASK_WINDOW_FILL : locality window around the query block's centre token on a
 *                          T x Hg x Wg token grid, plus hashed random fill up to a target
 *                          density (the fill probability is chosen per block so the
 *                          expected density equals the target; blocks whose window
 *                          already exceeds it get no fill).
 *   FGW_MASK_RANDOM      : every key group active with probability `density`.
 *   FGW_MASK_ALL         : every key group active (0% sparsity).
 *   FGW_MASK_SKEW_HEADS  : WINDOW_FILL whose target density varies per head
 *                          (lognormal, clipped) and per block (+-50% around the head's).
 *   FGW_MASK_SKEW_LEN    : the skew generator of Sec. 5.1 "Ablation": per block a list
 *                          length drawn uniformly in [(1-skew)*Lmax, Lmax] and that many
 *                          key groups chosen at random.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FGW_MASK_WINDOW_FILL = 0, FGW_MASK_RANDOM = 1, FGW_MASK_ALL = 2, FGW_MASK_SKEW_HEADS = 3,
       FGW_MASK_SKEW_LEN = 4 };

typedef struct {
  int32_t kind;
  int32_t heads;            /* B*H: number of (batch, head) slices */
  int32_t L, M, N;          /* tokens, query-block rows, keys per key group */
  int32_t gt, gh, gw;       /* token grid T x Hg x Wg, W fastest; gt*gh*gw == L for window kinds */
  int32_t dt, dh, dw;       /* window half-widths */
  double density;           /* target density (1 - sparsity) */
  double sigma;             /* SKEW_HEADS: sigma of ln(head density) */
  double skew;              /* SKEW_LEN: (Lmax - Lmin) / Lmax */
  uint64_t seed;
} fgw_mask_spec;

static inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
static inline uint64_t hash4(uint64_t seed, uint64_t a, uint64_t b, uint64_t c) {
  uint64_t h = mix64(seed ^ 0xD1B54A32D192ED03ull);
  h = mix64(h ^ a);
  h = mix64(h ^ (b + 0x632BE59BD9B4E019ull));
  h = mix64(h ^ (c + 0xA0761D6478BD642Full));
  return h;
}
/* uniform in (0,1) with 53 bits */
static inline double u01(uint64_t h) { return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0); }

static inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

/* out[i] = bf16(N(0,1)) for i in [0,n); pair (2j, 2j+1) comes from one Box-Muller draw of counter j. */
void fgw_normal_bf16(uint64_t seed, uint64_t stream, uint16_t* out, int64_t n) {
  int64_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < pairs; j++) {
    double u1 = u01(hash4(seed, stream, (uint64_t)j, 1));
    double u2 = u01(hash4(seed, stream, (uint64_t)j, 2));
    double r = sqrt(-2.0 * log(u1));
    double a = 6.283185307179586476925 * u2;
    out[2 * j] = f32_to_bf16_rne((float)(r * cos(a)));
    if (2 * j + 1 < n) out[2 * j + 1] = f32_to_bf16_rne((float)(r * sin(a)));
  }
}

static inline int64_t n_qblocks(const fgw_mask_spec* s) { return ((int64_t)s->L + s->M - 1) / s->M; }
static inline int64_t n_groups(const fgw_mask_spec* s) { return ((int64_t)s->L + s->N - 1) / s->N; }

/* marks win[g] = 1 for every key group holding a key inside the window of block i; returns the count */
static int64_t window_groups(const fgw_mask_spec* s, int64_t i, uint8_t* win) {
  int64_t G = n_groups(s);
  memset(win, 0, (size_t)G);
  int64_t row0 = i * s->M;
  int64_t rows = s->L - row0 < s->M ? s->L - row0 : s->M;
  int64_t c = row0 + rows / 2;
  int64_t ct = c / ((int64_t)s->gh * s->gw), ch = (c / s->gw) % s->gh, cw = c % s->gw;
  int64_t cnt = 0;
  for (int64_t t = ct - s->dt; t <= ct + s->dt; t++) {
    if (t < 0 || t >= s->gt) continue;
    for (int64_t h = ch - s->dh; h <= ch + s->dh; h++) {
      if (h < 0 || h >= s->gh) continue;
      for (int64_t w = cw - s->dw; w <= cw + s->dw; w++) {
        if (w < 0 || w >= s->gw) continue;
        int64_t key = (t * s->gh + h) * s->gw + w;
        if (key >= s->L) continue;
        int64_t g = key / s->N;
        if (!win[g]) { win[g] = 1; cnt++; }
      }
    }
  }
  return cnt;
}

/* per-head target density for SKEW_HEADS: lognormal with mean `density`, clipped to [0.05, 0.95] */
static double head_density(const fgw_mask_spec* s, int64_t head) {
  double u1 = u01(hash4(s->seed, 0x68656164ull, (uint64_t)head, 1));
  double u2 = u01(hash4(s->seed, 0x68656164ull, (uint64_t)head, 2));
  double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
  double rho = exp(log(s->density) - 0.5 * s->sigma * s->sigma + s->sigma * z);
  if (rho < 0.05) rho = 0.05;
  if (rho > 0.95) rho = 0.95;
  return rho;
}

/* decides the active key groups of work item (head, i); writes them ascending into dst if dst != NULL */
static int64_t build_row(const fgw_mask_spec* s, int64_t head, int64_t i, uint8_t* win, uint64_t* keys, int32_t* dst) {
  int64_t G = n_groups(s);
  int64_t n = 0;
  if (s->kind == FGW_MASK_ALL) {
    if (dst) for (int64_t g = 0; g < G; g++) dst[g] = (int32_t)g;
    return G;
  }
  if (s->kind == FGW_MASK_RANDOM) {
    for (int64_t g = 0; g < G; g++)
      if (u01(hash4(s->seed, (uint64_t)head, (uint64_t)i, (uint64_t)g)) < s->density) {
        if (dst) dst[n] = (int32_t)g;
        n++;
      }
    return n;
  }
  if (s->kind == FGW_MASK_SKEW_LEN) {
    /* list length uniform in [Lmin, Lmax], Lmax chosen so the mean density is `density` */
    double lmax = 2.0 * s->density * (double)G / (2.0 - s->skew);
    if (lmax > (double)G) lmax = (double)G;
    double lmin = (1.0 - s->skew) * lmax;
    double u = u01(hash4(s->seed, 0x6C656Eull, (uint64_t)head, (uint64_t)i));
    int64_t len = (int64_t)floor(lmin + u * (lmax - lmin) + 0.5);
    if (len < 1) len = 1;
    if (len > G) len = G;
    /* the `len` groups with the smallest hash: a uniformly random subset of that size */
    for (int64_t g = 0; g < G; g++) keys[g] = (hash4(s->seed, (uint64_t)head, (uint64_t)i, (uint64_t)g) & ~0xFFFFFFFFull) | (uint64_t)g;
    /* selection by threshold: find the len-th smallest with a copy + qsort-free nth_element */
    uint64_t* tmp = keys + G;
    memcpy(tmp, keys, (size_t)G * 8);
    int64_t lo = 0, hi = G - 1, kth = len - 1;
    while (lo < hi) {
      uint64_t p = tmp[(lo + hi) / 2];
      int64_t a = lo, b = hi;
      while (a <= b) {
        while (tmp[a] < p) a++;
        while (tmp[b] > p) b--;
        if (a <= b) { uint64_t t = tmp[a]; tmp[a] = tmp[b]; tmp[b] = t; a++; b--; }
      }
      if (kth <= b) hi = b; else if (kth >= a) lo = a; else break;
    }
    uint64_t thr = tmp[kth];
    for (int64_t g = 0; g < G; g++)
      if (keys[g] <= thr) { if (dst) dst[n] = (int32_t)g; n++; }
    return n;
  }
  /* window kinds */
  int64_t wcnt = window_groups(s, i, win);
  double rho = s->density;
  if (s->kind == FGW_MASK_SKEW_HEADS) {
    double f = 0.5 + u01(hash4(s->seed, 0x626C6B00ull, (uint64_t)head, (uint64_t)i));
    rho = head_density(s, head) * f;
    if (rho > 0.98) rho = 0.98;
  }
  double p = G > wcnt ? (rho * (double)G - (double)wcnt) / (double)(G - wcnt) : 0.0;
  if (p < 0.0) p = 0.0;
  if (p > 1.0) p = 1.0;
  for (int64_t g = 0; g < G; g++) {
    int on = win[g] || (p > 0.0 && u01(hash4(s->seed, (uint64_t)head, (uint64_t)i, (uint64_t)g)) < p);
    if (on) { if (dst) dst[n] = (int32_t)g; n++; }
  }
  return n;
}

/* Pass 1: indptr[0..items] (items = heads * ceil(L/M)); returns nnz, or -1 on a bad spec. */
int64_t fgw_mask_count(const fgw_mask_spec* s, int64_t* indptr) {
  if (s->heads < 1 || s->L < 1 || s->M < 1 || s->N < 1) return -1;
  int windowed = s->kind == FGW_MASK_WINDOW_FILL || s->kind == FGW_MASK_SKEW_HEADS;
  if (windowed && (int64_t)s->gt * s->gh * s->gw != s->L) return -1;
  int64_t QB = n_qblocks(s), G = n_groups(s), items = (int64_t)s->heads * QB;
  int fail = 0;
#pragma omp parallel
  {
    uint8_t* win = (uint8_t*)malloc((size_t)G);
    uint64_t* keys = (uint64_t*)malloc((size_t)G * 16);
    if (!win || !keys) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t w = 0; w < items; w++) indptr[w + 1] = build_row(s, w / QB, w % QB, win, keys, NULL);
    }
    free(win);
    free(keys);
  }
  if (fail) return -1;
  indptr[0] = 0;
  for (int64_t w = 0; w < items; w++) indptr[w + 1] += indptr[w];
  return indptr[items];
}

/* Pass 2: indices[indptr[w] .. indptr[w+1]) = ascending active key groups of item w. */
int fgw_mask_fill(const fgw_mask_spec* s, const int64_t* indptr, int32_t* indices) {
  int64_t QB = n_qblocks(s), G = n_groups(s), items = (int64_t)s->heads * QB;
  int fail = 0;
#pragma omp parallel
  {
    uint8_t* win = (uint8_t*)malloc((size_t)G);
    uint64_t* keys = (uint64_t*)malloc((size_t)G * 16);
    if (!win || !keys) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t w = 0; w < items; w++) {
        int64_t n = build_row(s, w / QB, w % QB, win, keys, indices + indptr[w]);
        if (n != indptr[w + 1] - indptr[w]) {
#pragma omp atomic write
          fail = 2;
        }
      }
    }
    free(win);
    free(keys);
  }
  return fail ? -1 : 0;
}
