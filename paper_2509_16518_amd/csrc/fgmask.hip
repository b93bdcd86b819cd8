// Mean-query/key top-p mask (paper Sec. 4.3 "Determining the Fine-grain Sparse Mask with Top-p
// Masking") for CDNA4: block means of Q and K, approximate attention between the block means,
// and per query block the smallest set of key blocks, most probable first, whose probability
// mass reaches p -- written straight into the CSR form the forward kernel reads.
//
// Kernels (all on the caller's stream):
//   pool_kernel     block means (fp32 running sum in row order, fp32 divide, one bf16 rounding)
//   scores_kernel   S = scale * Q_avg K_avg^T with bf16 MFMA, fp32 scores to the workspace
//   select_kernel   one workgroup per query block: finds the CUT, the 64-bit key (score, then
//                   lower id first) of the last kept key block, without sorting the row
//   scan_kernel     counts -> indptr
//   emit_kernel     ids whose key is >= the cut, ascending, into indices
//
// Selection works on integers so that it does not depend on the order of additions: the weight
// of a key block is exp2((s - max) * log2 e) in 2^-40 fixed point, the row's mass Z is the integer
// sum, and the kept set is the smallest prefix of the ranking whose integer mass reaches
// ceil(p * Z).  The ranking is never materialised: a histogram over the score range locates the
// bin in which the running mass crosses the target, only that bin's members are sorted.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include "fgattn.h"

namespace fgm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kSelThreads = 256;
constexpr int kBins = 2048;
constexpr int kCap = 2048;          // members of the crossing bin that are sorted in LDS
constexpr float kLog2e = 1.44269504088896340736f;

__device__ __forceinline__ unsigned ordered_bits(float s) {   // monotone: larger score, larger unsigned
  const unsigned u = __float_as_uint(s);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float from_ordered(unsigned o) {
  const unsigned u = o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu);
  return __uint_as_float(u);
}
// ---------------------------------------------------------------------------------------------
// Step 1: block means.  One thread per (block, column): the additions run in row order, so every
// implementation of this reading produces the same bits.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128) pool_kernel(const uint16_t* x, int64_t sb, int64_t sh, int64_t sl, int H, int L,
                                                    int d, int rows_per_block, int nblocks, uint16_t* pooled,
                                                    unsigned* range_init) {
  const int c = threadIdx.x;
  const int blk = blockIdx.x;
  const int slice = blockIdx.y;
  if (c >= d) return;
  // the Q pass also resets the (max, min) pair of the score row this query block will own
  if (range_init != nullptr && c == 0) {
    range_init[2 * ((int64_t)slice * nblocks + blk)] = 0u;
    range_init[2 * ((int64_t)slice * nblocks + blk) + 1] = 0xFFFFFFFFu;
  }
  const int b = slice / H, h = slice - b * H;
  const int r0 = blk * rows_per_block;
  const int r1 = min(r0 + rows_per_block, L);
  const uint16_t* p = x + b * sb + h * sh + (int64_t)r0 * sl + c;
  float acc = 0.0f;
  for (int r = r0; r < r1; r++, p += sl) acc = acc + __uint_as_float((unsigned)(*p) << 16);
  const float mean = __fdiv_rn(acc, (float)(r1 - r0));
  unsigned u = __float_as_uint(mean);
  u += 0x7FFFu + ((u >> 16) & 1u);   // nearest even; the inputs are finite
  pooled[((int64_t)slice * nblocks + blk) * d + c] = (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------------------
// Step 2a: scores.  A wave owns 32 query blocks (A operand, kept in registers) and walks over
// tiles of 32 key blocks (B operand, read straight from global memory: 16 bytes per lane and
// step); in the accumulator a register holds one query block and 32 consecutive key blocks across
// lanes, so every store covers whole 128-byte lines.
// ---------------------------------------------------------------------------------------------
constexpr int kTilesPerWave = 16;

template <int D>
__global__ void __launch_bounds__(256) scores_kernel(const uint16_t* qp, const uint16_t* kp, int64_t k_slice_stride,
                                                      int64_t k_row_stride, int QB, int G, int Gs, float scale,
                                                      float* scores, unsigned* range) {
  constexpr int STEPS = D / 16;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int ln = lane & 31, g = lane >> 5;
  const int slice = blockIdx.z;
  const int q0 = blockIdx.y * 32;
  const int tile0 = (blockIdx.x * 4 + wv) * kTilesPerWave;
  if (tile0 * 32 >= G) return;
  bf16x8 qf[STEPS];
  {
    const int qrow = min(q0 + ln, QB - 1);
    const char* src = reinterpret_cast<const char*>(qp + ((int64_t)slice * QB + qrow) * D);
#pragma unroll
    for (int s = 0; s < STEPS; s++) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(src + (2 * s + g) * 16));
  }
  const char* kbase = reinterpret_cast<const char*>(kp + slice * k_slice_stride);
  auto load_tile = [&](int tile, bf16x8 (&kf)[STEPS]) {
    const int krow = min(tile * 32 + ln, G - 1);
    const char* src = kbase + (int64_t)krow * k_row_stride * 2;
#pragma unroll
    for (int s = 0; s < STEPS; s++) kf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(src + (2 * s + g) * 16));
  };
  // running range of the scores this lane produced, per accumulator register (= per query block)
  float vmax[16], vmin[16];
#pragma unroll
  for (int r = 0; r < 16; r++) {
    vmax[r] = -INFINITY;
    vmin[r] = INFINITY;
  }
  const int ntiles = min(kTilesPerWave, (G - tile0 * 32 + 31) / 32);
  bf16x8 kf[STEPS], kn[STEPS];
  load_tile(tile0, kf);
  for (int t = 0; t < ntiles; t++) {
    if (t + 1 < ntiles) load_tile(tile0 + t + 1, kn);   // next tile's operand in flight during this tile's MFMAs
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0.0f;
#pragma unroll
    for (int s = 0; s < STEPS; s++) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[s], kf[s], acc, 0, 0, 0);
    const int col = (tile0 + t) * 32 + ln;
    if (col < G) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int qrow = q0 + 8 * (r / 4) + 4 * g + (r % 4);
        const float v = acc[r] * scale;
        vmax[r] = fmaxf(vmax[r], v);
        vmin[r] = fminf(vmin[r], v);
        if (qrow < QB) scores[((int64_t)slice * QB + qrow) * Gs + col] = v;
      }
    }
#pragma unroll
    for (int s = 0; s < STEPS; s++) kf[s] = kn[s];
  }
  // one (max, min) update per query block and wave: reduce over the 32 lanes that share the block
#pragma unroll
  for (int r = 0; r < 16; r++) {
    float a = vmax[r], b = vmin[r];
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) {
      a = fmaxf(a, __shfl_xor(a, off));
      b = fminf(b, __shfl_xor(b, off));
    }
    const int qrow = q0 + 8 * (r / 4) + 4 * g + (r % 4);
    if (ln == 0 && qrow < QB && a >= b) {
      unsigned* rr = range + 2 * ((int64_t)slice * QB + qrow);
      atomicMax(rr, ordered_bits(a));
      atomicMin(rr + 1, ordered_bits(b));
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Step 2b + 3: selection.
// ---------------------------------------------------------------------------------------------
// rank key of key block j with score s: higher score first, then lower id first
__device__ __forceinline__ unsigned long long rank_key(float s, int j) {
  return ((unsigned long long)ordered_bits(s) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)j);
}
__device__ __forceinline__ unsigned long long weight_of(float s, float rmax) {
  const float e = exp2f((s - rmax) * kLog2e);          // in (0, 1]
  return (unsigned long long)(e * 1099511627776.0f);   // 2^40 fixed point, truncated
}

// Visits every score of a row: four consecutive scores per thread and step (16-byte loads; rows start 16-byte
// aligned and their stride is a multiple of four floats), four steps in flight.
template <typename Fn>
__device__ __forceinline__ void for_each_score(const float* s, int G, Fn&& fn) {
  constexpr int STEP = kSelThreads * 4;
  auto visit = [&](const float4& v, int j4) {
    fn(v.x, j4);
    if (j4 + 1 < G) fn(v.y, j4 + 1);
    if (j4 + 2 < G) fn(v.z, j4 + 2);
    if (j4 + 3 < G) fn(v.w, j4 + 3);
  };
  int j4 = threadIdx.x * 4;
  for (; j4 + 3 * STEP < G; j4 += 4 * STEP) {
    const float4 a = *reinterpret_cast<const float4*>(s + j4);
    const float4 b = *reinterpret_cast<const float4*>(s + j4 + STEP);
    const float4 c = *reinterpret_cast<const float4*>(s + j4 + 2 * STEP);
    const float4 d = *reinterpret_cast<const float4*>(s + j4 + 3 * STEP);
    visit(a, j4);
    visit(b, j4 + STEP);
    visit(c, j4 + 2 * STEP);
    visit(d, j4 + 3 * STEP);
  }
  for (; j4 < G; j4 += STEP) visit(*reinterpret_cast<const float4*>(s + j4), j4);
}

// Exclusive prefix of `n` over the threads of the workgroup in thread order; *total gets the sum.
// wave_tot: four words of shared memory.  Contains two barriers.
__device__ __forceinline__ unsigned block_exclusive(unsigned n, unsigned* wave_tot, unsigned* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned incl = n;
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  unsigned before = 0;
  for (int w2 = 0; w2 < wv; w2++) before += wave_tot[w2];
  *total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
  __syncthreads();
  return before + incl - n;
}

struct SelShared {
  unsigned long long mass[kBins];
  unsigned cnt[kBins];
  unsigned long long cand[kCap];
  unsigned long long red64[kSelThreads];
  unsigned long long mass_above, target, cut;
  unsigned n_above, bin, bin_cnt, ncand, klo, khi, run;
  int done;
};

__device__ __forceinline__ unsigned long long block_sum_u64(SelShared& sh, unsigned long long v) {
  const int tid = threadIdx.x;
  sh.red64[tid] = v;
  __syncthreads();
  for (int off = kSelThreads / 2; off > 0; off >>= 1) {
    if (tid < off) sh.red64[tid] += sh.red64[tid + off];
    __syncthreads();
  }
  const unsigned long long r = sh.red64[0];
  __syncthreads();
  return r;
}

// Finds, in the histogram just built, the bin where the running mass (starting from mass_above) reaches the
// target; updates mass_above / n_above to exclude that bin and stores bin / bin_cnt.
__device__ __forceinline__ void locate_bin(SelShared& sh) {
  const int tid = threadIdx.x;
  constexpr int PER = kBins / kSelThreads;
  unsigned long long local = 0;
  for (int i = 0; i < PER; i++) local += sh.mass[tid * PER + i];
  sh.red64[tid] = local;
  __syncthreads();
  if (tid == 0) {
    // the caller guarantees mass_above < target <= mass_above + (mass of this histogram)
    unsigned long long run = sh.mass_above;
    int t = 0;
    while (t < kSelThreads - 1 && run + sh.red64[t] < sh.target) run += sh.red64[t++];
    int b = t * PER;
    while (b < kBins - 1 && run + sh.mass[b] < sh.target) run += sh.mass[b++];
    unsigned n = sh.n_above;
    for (int i = 0; i < b; i++) n += sh.cnt[i];
    sh.mass_above = run;
    sh.n_above = n;
    sh.bin = (unsigned)b;
    sh.bin_cnt = sh.cnt[b];
  }
  __syncthreads();
}

__global__ void __launch_bounds__(kSelThreads) select_kernel(const float* scores, const unsigned* range, int G, int Gs,
                                                             float top_p, unsigned long long* cut, unsigned* count) {
  __shared__ SelShared sh;
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const float* s = scores + row * Gs;

  // range of the scores (collected by the scores kernel)
  const float rmax = from_ordered(range[2 * row]), rmin = from_ordered(range[2 * row + 1]);
  const float width = rmax - rmin;
  const float inv = width > 0.0f ? (float)kBins / width : 0.0f;
  auto value_bin = [&](float v) -> int {   // bin 0 holds the largest scores
    const int b = (int)((rmax - v) * inv);
    return b < 0 ? 0 : (b > kBins - 1 ? kBins - 1 : b);
  };

  // pass 2: mass of the row and its histogram over the score range
  for (int i = tid; i < kBins; i += kSelThreads) {
    sh.mass[i] = 0;
    sh.cnt[i] = 0;
  }
  __syncthreads();
  unsigned long long zl = 0;
  for_each_score(s, G, [&](float v, int) {
    const unsigned long long w = weight_of(v, rmax);
    zl += w;
    const int b = value_bin(v);
    atomicAdd(&sh.mass[b], w);
    atomicAdd(&sh.cnt[b], 1u);
  });
  const unsigned long long Z = block_sum_u64(sh, zl);
  if (tid == 0) {
    double t = ceil((double)top_p * (double)Z);
    unsigned long long T = t < 1.0 ? 1ull : (unsigned long long)t;
    if (T > Z) T = Z;
    sh.target = T;
    sh.mass_above = 0;
    sh.n_above = 0;
    sh.done = 0;
  }
  __syncthreads();
  locate_bin(sh);

  // The members of the crossing bin form a contiguous stretch of the ranking.  While there are too many to
  // sort, narrow the stretch: take the range [klo, khi] of their ordered score bits and histogram it again,
  // now linearly in those bits (every round divides the range by kBins, so a few rounds reach a single value).
  bool by_value = true;     // how the current bin is defined: value_bin() == bin, or key range [klo, khi]
  unsigned klo = 0, khi = 0;
  for (int round = 0; round < 6; round++) {
    const unsigned bin = sh.bin;
    if (sh.bin_cnt <= (unsigned)kCap) break;
    // range of ordered bits inside the current bin
    if (tid == 0) {
      sh.klo = 0xFFFFFFFFu;
      sh.khi = 0u;
    }
    __syncthreads();
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
    for_each_score(s, G, [&](float v, int) {
      const unsigned o = ordered_bits(v);
      const bool in = by_value ? (value_bin(v) == (int)bin) : (o >= klo && o <= khi);
      if (in) {
        lo = min(lo, o);
        hi = max(hi, o);
      }
    });
    atomicMin(&sh.klo, lo);
    atomicMax(&sh.khi, hi);
    __syncthreads();
    klo = sh.klo;
    khi = sh.khi;
    by_value = false;
    if (klo == khi) break;   // one score value left: a run of equal scores, handled by id below
    const unsigned long long R = (unsigned long long)(khi - klo) + 1ull;
    for (int i = tid; i < kBins; i += kSelThreads) {
      sh.mass[i] = 0;
      sh.cnt[i] = 0;
    }
    __syncthreads();
    for_each_score(s, G, [&](float v, int) {
      const unsigned o = ordered_bits(v);
      if (o >= klo && o <= khi) {
        const int b = (int)(((unsigned long long)(khi - o) * kBins) / R);
        atomicAdd(&sh.mass[b], weight_of(v, rmax));
        atomicAdd(&sh.cnt[b], 1u);
      }
    });
    __syncthreads();
    locate_bin(sh);
    // ordered bits of the new bin b: khi - o in [ceil(b*R/kBins), ceil((b+1)*R/kBins) - 1]
    const unsigned long long b = sh.bin;
    const unsigned long long d_lo = (b * R + kBins - 1) / kBins;
    const unsigned long long d_hi = ((b + 1) * R + kBins - 1) / kBins - 1;
    const unsigned nkhi = khi - (unsigned)d_lo;
    const unsigned nklo = khi - (unsigned)(d_hi > (unsigned long long)(khi - klo) ? (khi - klo) : d_hi);
    khi = nkhi;
    klo = nklo;
    __syncthreads();
  }

  const unsigned bin = sh.bin;
  const unsigned bin_cnt = sh.bin_cnt;
  if (bin_cnt == 0) {   // unreachable (the crossing bin has mass, hence members); kept so that no path leaves the outputs unset
    if (tid == 0) {
      cut[row] = ~0ull;
      count[row] = sh.n_above;
    }
    return;
  }
  if (bin_cnt <= (unsigned)kCap) {
    // sort the members of the crossing bin by rank key (descending) and walk their masses
    if (tid == 0) sh.ncand = 0;
    int n2 = 1;
    while (n2 < (int)bin_cnt) n2 <<= 1;
    for (int i = tid; i < n2; i += kSelThreads) sh.cand[i] = 0ull;
    __syncthreads();
    for_each_score(s, G, [&](float v, int j) {
      const unsigned o = ordered_bits(v);
      const bool in = by_value ? (value_bin(v) == (int)bin) : (o >= klo && o <= khi);
      if (in) {
        const unsigned pos = atomicAdd(&sh.ncand, 1u);
        if (pos < (unsigned)kCap) sh.cand[pos] = rank_key(v, j);
      }
    });
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1)
      for (int jj = k >> 1; jj > 0; jj >>= 1) {
        for (int i = tid; i < n2; i += kSelThreads) {
          const int l = i ^ jj;
          if (l > i) {
            const unsigned long long a = sh.cand[i], b = sh.cand[l];
            const bool desc = (i & k) == 0;
            if (desc ? (a < b) : (a > b)) {
              sh.cand[i] = b;
              sh.cand[l] = a;
            }
          }
        }
        __syncthreads();
      }
    // first position t where mass_above + (masses of cand[0..t]) reaches the target
    constexpr int PER = kCap / kSelThreads;
    unsigned long long local = 0;
    for (int i = 0; i < PER; i++) {
      const int idx = tid * PER + i;
      if (idx < (int)bin_cnt) local += weight_of(from_ordered((unsigned)(sh.cand[idx] >> 32)), rmax);
    }
    sh.red64[tid] = local;
    __syncthreads();
    if (tid == 0) {
      unsigned long long run = sh.mass_above;
      int t = 0;
      while (t < kSelThreads - 1 && run + sh.red64[t] < sh.target) run += sh.red64[t++];
      int idx = t * PER;
      const int lastc = (int)bin_cnt - 1;
      if (idx > lastc) idx = lastc;
      while (idx < lastc) {
        run += weight_of(from_ordered((unsigned)(sh.cand[idx] >> 32)), rmax);
        if (run >= sh.target) break;
        idx++;
      }
      cut[row] = sh.cand[idx];
      count[row] = sh.n_above + (unsigned)idx + 1u;
    }
    return;
  }

  // A run of more than kCap equal scores contains the crossing: all of them weigh the same, so the number
  // to keep follows by division, and they are taken in ascending id.
  const float v_eq = from_ordered(klo);
  const unsigned long long w_eq = weight_of(v_eq, rmax);
  unsigned long long need = sh.target > sh.mass_above ? sh.target - sh.mass_above : 1ull;
  unsigned long long t_keep = w_eq > 0 ? (need + w_eq - 1) / w_eq : (unsigned long long)bin_cnt;
  if (t_keep < 1) t_keep = 1;
  if (t_keep > bin_cnt) t_keep = bin_cnt;
  unsigned run = 0;   // members seen in the chunks before this one (the same in every thread)
  for (int base = 0; base < G && (unsigned long long)run < t_keep; base += kSelThreads * 4) {
    const int j4 = base + tid * 4;
    bool in[4] = {false, false, false, false};
    if (j4 < G) {
      const float4 v = *reinterpret_cast<const float4*>(s + j4);
      in[0] = ordered_bits(v.x) == klo;
      in[1] = j4 + 1 < G && ordered_bits(v.y) == klo;
      in[2] = j4 + 2 < G && ordered_bits(v.z) == klo;
      in[3] = j4 + 3 < G && ordered_bits(v.w) == klo;
    }
    unsigned total;
    unsigned pos = run + block_exclusive((unsigned)in[0] + in[1] + in[2] + in[3], sh.cnt, &total);
    for (int e = 0; e < 4; e++)
      if (in[e] && (unsigned long long)(++pos) == t_keep) {
        cut[row] = rank_key(v_eq, j4 + e);
        count[row] = sh.n_above + (unsigned)t_keep;
      }
    run += total;
  }
}

// counts -> indptr (one workgroup; rows are at most a few tens of thousands)
__global__ void __launch_bounds__(1024) scan_kernel(const unsigned* count, int64_t rows, int64_t* indptr) {
  __shared__ long long part[1024];
  __shared__ long long carry;
  const int tid = threadIdx.x;
  if (tid == 0) {
    carry = 0;
    indptr[0] = 0;
  }
  __syncthreads();
  for (int64_t base = 0; base < rows; base += 1024) {
    const int64_t r = base + tid;
    part[tid] = r < rows ? (long long)count[r] : 0;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const long long add = tid >= off ? part[tid - off] : 0;
      __syncthreads();
      part[tid] += add;
      __syncthreads();
    }
    if (r < rows) indptr[r + 1] = carry + part[tid];
    __syncthreads();
    if (tid == 0) carry += part[1023];
    __syncthreads();
  }
}

// ids whose rank key is not below the cut, in ascending order
__global__ void __launch_bounds__(kSelThreads) emit_kernel(const float* scores, int G, int Gs,
                                                           const unsigned long long* cut, const int64_t* indptr,
                                                           int32_t* indices, int64_t capacity) {
  __shared__ unsigned wave_tot[4];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const float* s = scores + row * Gs;
  const unsigned long long c = cut[row];
  const int64_t out0 = indptr[row];
  unsigned run = 0;
  constexpr int STEP = kSelThreads * 4;
  const float4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
  float4 nxt[3];   // the next three chunks are in flight while this one is ranked and written
#pragma unroll
  for (int i = 0; i < 3; i++) nxt[i] = i * STEP + tid * 4 < G ? *reinterpret_cast<const float4*>(s + i * STEP + tid * 4) : zero4;
  for (int base = 0; base < G; base += STEP) {
    const int j4 = base + tid * 4;
    const float4 v = nxt[0];
    nxt[0] = nxt[1];
    nxt[1] = nxt[2];
    nxt[2] = j4 + 3 * STEP < G ? *reinterpret_cast<const float4*>(s + j4 + 3 * STEP) : zero4;
    bool keep[4] = {false, false, false, false};
    if (j4 < G) {
      keep[0] = rank_key(v.x, j4) >= c;
      keep[1] = j4 + 1 < G && rank_key(v.y, j4 + 1) >= c;
      keep[2] = j4 + 2 < G && rank_key(v.z, j4 + 2) >= c;
      keep[3] = j4 + 3 < G && rank_key(v.w, j4 + 3) >= c;
    }
    unsigned total;
    int64_t pos = out0 + run + block_exclusive((unsigned)keep[0] + keep[1] + keep[2] + keep[3], wave_tot, &total);
    for (int e = 0; e < 4; e++)
      if (keep[e]) {
        if (pos < capacity) indices[pos] = j4 + e;
        pos++;
      }
    run += total;
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct Layout {
  int64_t rows, QB, G, Gs, slices;
  size_t qp_off, kp_off, scores_off, cut_off, count_off, range_off, total;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int layout_of(const fgattn_params* p, Layout* lo) {
  if (p == nullptr) return FGATTN_E_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1 || p->N < 1) return FGATTN_E_SHAPE;
  if (p->d != 64 && p->d != 128) return FGATTN_E_SHAPE;
  if (p->M != 16 && p->M != 32 && p->M != 64 && p->M != 128) return FGATTN_E_SHAPE;
  if (p->L > (1 << 24)) return FGATTN_E_SHAPE;
  lo->slices = (int64_t)p->B * p->H;
  lo->QB = ((int64_t)p->L + p->M - 1) / p->M;
  lo->G = ((int64_t)p->L + p->N - 1) / p->N;
  lo->Gs = (lo->G + 3) & ~(int64_t)3;
  lo->rows = lo->slices * lo->QB;
  if (lo->rows > 0x7fffffffLL || lo->slices > 65535) return FGATTN_E_SHAPE;
  size_t off = 0;
  lo->qp_off = off;
  off = align256(off + (size_t)lo->rows * p->d * 2);
  lo->kp_off = off;
  if (p->N > 1 || p->B > 1) off = align256(off + (size_t)lo->slices * lo->G * p->d * 2);   // else K is read in place
  lo->scores_off = off;
  off = align256(off + (size_t)lo->rows * lo->Gs * 4);
  lo->cut_off = off;
  off = align256(off + (size_t)lo->rows * 8);
  lo->count_off = off;
  off = align256(off + (size_t)lo->rows * 4);
  lo->range_off = off;
  off = align256(off + (size_t)lo->rows * 8);
  lo->total = off;
  return FGATTN_OK;
}

static int device_ok() {
  static int known[64];   // 0 unknown, 1 gfx950, 2 other
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FGATTN_E_DEVICE;
  if (known[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return FGATTN_E_DEVICE;
    known[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
  }
  return known[dev] == 1 ? FGATTN_OK : FGATTN_E_DEVICE;
}

static bool launched() { return hipGetLastError() == hipSuccess; }

}  // namespace fgm

extern "C" {

size_t fgattn_mask_workspace_bytes(const fgattn_params* p) {
  fgm::Layout lo;
  if (fgm::layout_of(p, &lo) != FGATTN_OK) return 0;
  return lo.total;
}

int fgattn_mask_select(const void* q, const void* k, const fgattn_params* p, float top_p, int64_t* mask_indptr,
                       void* workspace, size_t workspace_bytes, void* stream_v) {
  using namespace fgm;
  Layout lo;
  int rc = layout_of(p, &lo);
  if (rc) return rc;
  if (!q || !k || !mask_indptr || !workspace) return FGATTN_E_NULL;
  if (!(top_p > 0.0f) || !(top_p <= 1.0f) || !isfinite(p->scale)) return FGATTN_E_SCALE;
  if ((reinterpret_cast<uintptr_t>(q) & 15) || (reinterpret_cast<uintptr_t>(k) & 15) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(mask_indptr) & 7))
    return FGATTN_E_ALIGN;
  const int64_t strides[6] = {p->q_stride_b, p->q_stride_h, p->q_stride_l, p->k_stride_b, p->k_stride_h, p->k_stride_l};
  for (int i = 0; i < 6; i++)
    if (strides[i] < 0 || (strides[i] % 8) != 0) return FGATTN_E_STRIDE;
  if (p->q_stride_l < p->d || p->k_stride_l < p->d) return FGATTN_E_STRIDE;
  if (workspace_bytes < lo.total) return FGATTN_E_WORKSPACE;
  rc = device_ok();
  if (rc) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  char* ws = static_cast<char*>(workspace);
  uint16_t* qp = reinterpret_cast<uint16_t*>(ws + lo.qp_off);
  uint16_t* kp = reinterpret_cast<uint16_t*>(ws + lo.kp_off);
  float* scores = reinterpret_cast<float*>(ws + lo.scores_off);
  unsigned long long* cut = reinterpret_cast<unsigned long long*>(ws + lo.cut_off);
  unsigned* count = reinterpret_cast<unsigned*>(ws + lo.count_off);
  unsigned* range = reinterpret_cast<unsigned*>(ws + lo.range_off);
  const uint16_t* qx = static_cast<const uint16_t*>(q);
  const uint16_t* kx = static_cast<const uint16_t*>(k);

  hipLaunchKernelGGL(pool_kernel, dim3((unsigned)lo.QB, (unsigned)lo.slices), dim3(128), 0, stream, qx, p->q_stride_b,
                     p->q_stride_h, p->q_stride_l, p->H, p->L, p->d, p->M, (int)lo.QB, qp, range);
  if (!launched()) return FGATTN_E_DEVICE;
  const uint16_t* kmat = kx;
  int64_t k_slice_stride = 0, k_row_stride = p->k_stride_l;
  bool k_in_place = p->N == 1 && p->B == 1;   // a block of one row is the row itself; slices are then heads
  if (k_in_place) {
    k_slice_stride = p->k_stride_h;
  } else {
    hipLaunchKernelGGL(pool_kernel, dim3((unsigned)lo.G, (unsigned)lo.slices), dim3(128), 0, stream, kx, p->k_stride_b,
                       p->k_stride_h, p->k_stride_l, p->H, p->L, p->d, p->N, (int)lo.G, kp, static_cast<unsigned*>(nullptr));
    if (!launched()) return FGATTN_E_DEVICE;
    kmat = kp;
    k_slice_stride = lo.G * p->d;
    k_row_stride = p->d;
  }
  const dim3 sgrid((unsigned)((lo.G + 4 * kTilesPerWave * 32 - 1) / (4 * kTilesPerWave * 32)), (unsigned)((lo.QB + 31) / 32),
                   (unsigned)lo.slices);
  if (p->d == 128)
    hipLaunchKernelGGL(scores_kernel<128>, sgrid, dim3(256), 0, stream, qp, kmat, k_slice_stride, k_row_stride, (int)lo.QB,
                       (int)lo.G, (int)lo.Gs, p->scale, scores, range);
  else
    hipLaunchKernelGGL(scores_kernel<64>, sgrid, dim3(256), 0, stream, qp, kmat, k_slice_stride, k_row_stride, (int)lo.QB,
                       (int)lo.G, (int)lo.Gs, p->scale, scores, range);
  if (!launched()) return FGATTN_E_DEVICE;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)lo.rows), dim3(kSelThreads), 0, stream, scores, range, (int)lo.G,
                     (int)lo.Gs, top_p, cut, count);
  if (!launched()) return FGATTN_E_DEVICE;
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, count, lo.rows, mask_indptr);
  return launched() ? FGATTN_OK : FGATTN_E_DEVICE;
}

int fgattn_mask_emit(const fgattn_params* p, const int64_t* mask_indptr, int32_t* mask_indices, int64_t indices_capacity,
                     const void* workspace, size_t workspace_bytes, void* stream_v) {
  using namespace fgm;
  Layout lo;
  int rc = layout_of(p, &lo);
  if (rc) return rc;
  if (!mask_indptr || !workspace || (!mask_indices && indices_capacity > 0)) return FGATTN_E_NULL;
  if (indices_capacity < 0) return FGATTN_E_SHAPE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(mask_indices) & 3)) return FGATTN_E_ALIGN;
  if (workspace_bytes < lo.total) return FGATTN_E_WORKSPACE;
  rc = device_ok();
  if (rc) return rc;
  const char* ws = static_cast<const char*>(workspace);
  const float* scores = reinterpret_cast<const float*>(ws + lo.scores_off);
  const unsigned long long* cut = reinterpret_cast<const unsigned long long*>(ws + lo.cut_off);
  hipLaunchKernelGGL(emit_kernel, dim3((unsigned)lo.rows), dim3(kSelThreads), 0, static_cast<hipStream_t>(stream_v), scores,
                     (int)lo.G, (int)lo.Gs, cut, mask_indptr, mask_indices, indices_capacity);
  return launched() ? FGATTN_OK : FGATTN_E_DEVICE;
}

}  // extern "C"
