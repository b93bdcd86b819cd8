// Mean-query/key top-p mask (paper Sec. 4.3 "Determining the Fine-grain Sparse Mask with Top-p
// Masking") for CDNA4: block means of Q and K, approximate attention between the block means,
// and per query block the smallest set of key blocks, most probable first, whose probability
// mass reaches p -- written straight into the CSR form the forward kernel reads.
//
// Kernels (all on the caller's stream):
//   pool_kernel        block means (fp32 running sum in row order, fp32 divide, one bf16 rounding)
//   scores_kernel      S = scale * Q_avg K_avg^T with bf16 MFMA, fp32 scores to the workspace
//   select_bins_kernel rows of up to 32768 scores: persistent 512-thread workgroups, two per compute unit; the
//                      row is read once, the bin of every score stays in LDS as 16 bits; finds the CUT, the 64-bit
//                      key (score, then lower id first) of the last kept key block, without sorting the row, and
//                      leaves the kept set as one bit per key block
//   select_kernel      longer rows (or on request): the same selection, one workgroup per query block,
//                      every pass reading the row from device memory; leaves the same outputs
//   scan_kernel        counts -> indptr
//   emit_bits_kernel   kept ids, ascending, into indices (from the bit rows)
//
// The scores are the only large intermediate (4 bytes per pair of query block and key block).  They are
// produced and consumed in chunks of whole score tiles (128 query blocks of one slice), scores_kernel and
// the selection kernel alternating over one buffer of bounded size; what outlives a chunk is one bit per pair.
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

#include <type_traits>

#include "fgattn.h"

namespace fgm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kSelThreads = 256;
constexpr int kBins = 2048;
constexpr int kCap = 2048;          // members of the crossing bin that are sorted in LDS
// Rows of up to kRowBinsMax scores are selected by 512-thread workgroups that read the row once and keep the bin
// of every score in LDS.
constexpr int kRowThreads = 512;
constexpr int kRowBins = 1024;
constexpr int kRowCap = 512;
constexpr int kRowBinsMax = 32768;
constexpr float kLog2e = 1.44269504088896340736f;

__device__ __forceinline__ unsigned ordered_bits(float s) {   // monotone: larger score, larger unsigned
  const unsigned u = __float_as_uint(s);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
// lane-wise arithmetic on the two 16-bit halves of a word
typedef __attribute__((ext_vector_type(2))) unsigned short u16x2;
__device__ __forceinline__ unsigned pk_sub_u16(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, (u16x2)(__builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ unsigned pk_min_u16(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ float from_ordered(unsigned o) {
  const unsigned u = o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu);
  return __uint_as_float(u);
}
// ---------------------------------------------------------------------------------------------
// Step 1: block means.  One thread per (block, pair of columns): the additions of a column run in
// row order, so every implementation of this reading produces the same bits.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint16_t mean_bf16(float acc, int n) {
  const float mean = __fdiv_rn(acc, (float)n);
  unsigned u = __float_as_uint(mean);
  u += 0x7FFFu + ((u >> 16) & 1u);   // nearest even; the inputs are finite
  return (uint16_t)(u >> 16);
}

__global__ void __launch_bounds__(64) pool_kernel(const uint16_t* x, int64_t sb, int64_t sh, int64_t sl, int H, int L,
                                                   int d, int rows_per_block, int nblocks, uint16_t* pooled,
                                                   unsigned* range_init) {
  const int c = threadIdx.x * 2;
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
  const uint16_t* p = x + b * sb + h * sh + (int64_t)r0 * sl + c;   // 4-byte aligned: strides are multiples of 8 elements
  float acc0 = 0.0f, acc1 = 0.0f;
  int r = r0;
  for (; r + 8 <= r1; r += 8, p += 8 * sl) {
    unsigned w[8];
#pragma unroll
    for (int i = 0; i < 8; i++) w[i] = *reinterpret_cast<const unsigned*>(p + i * sl);
#pragma unroll
    for (int i = 0; i < 8; i++) {
      acc0 = acc0 + __uint_as_float(w[i] << 16);
      acc1 = acc1 + __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  for (; r < r1; r++, p += sl) {
    const unsigned w = *reinterpret_cast<const unsigned*>(p);
    acc0 = acc0 + __uint_as_float(w << 16);
    acc1 = acc1 + __uint_as_float(w & 0xFFFF0000u);
  }
  const unsigned out = (unsigned)mean_bf16(acc0, r1 - r0) | ((unsigned)mean_bf16(acc1, r1 - r0) << 16);
  *reinterpret_cast<unsigned*>(pooled + ((int64_t)slice * nblocks + blk) * d + c) = out;
}

// ---------------------------------------------------------------------------------------------
// Step 2a: scores.  A workgroup owns 128 query blocks (32 per wave, A operand, kept in registers)
// and walks over tiles of 32 key blocks.  A tile is read from global memory once per workgroup,
// whole rows at a time (16 bytes per thread, next tile in flight during this tile's MFMAs), and
// passed through LDS, from where every wave takes it as its B operand; the 16-byte chunks of a row
// are XOR-swizzled so that both the row-wise writes and the column-wise operand reads are free of
// bank conflicts.  In the accumulator a register holds one query block and 32 consecutive key
// blocks across lanes, so every store covers whole 128-byte lines.
// ---------------------------------------------------------------------------------------------
constexpr int kTilesPerGroup = 16;

template <int D>
__global__ void __launch_bounds__(256) scores_kernel(const uint16_t* qp, const uint16_t* kp, int64_t k_slice_stride,
                                                      int64_t k_row_stride, int QB, int G, int Gs, float scale,
                                                      int unit0, int YT, float* scores, unsigned* range) {
  constexpr int STEPS = D / 16;
  constexpr int ROWB = D * 2;                 // bytes of a row of K
  constexpr int CHUNKS = ROWB / 16;           // 16-byte chunks per row
  constexpr int TILEB = 32 * ROWB;
  constexpr int LPT = TILEB / 16 / 256;       // chunks per thread and tile
  static_assert(LPT >= 1, "a tile is at least one chunk per thread");
  __shared__ __attribute__((aligned(16))) unsigned char ktile[2][TILEB];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int ln = lane & 31, g = lane >> 5;
  // blockIdx.y names a score tile of this chunk: unit = slice * YT + (tile of 128 query blocks inside the slice)
  const int unit = unit0 + blockIdx.y;
  const int slice = unit / YT;
  const int qtile0 = (unit - slice * YT) * 128;
  const int q0 = qtile0 + wv * 32;   // (a wave past the last query block still helps with the tiles)
  const int tile0 = blockIdx.x * kTilesPerGroup;
  auto swz = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
  bf16x8 qf[STEPS];
  {
    const int qrow = min(q0 + ln, QB - 1);
    const char* src = reinterpret_cast<const char*>(qp + ((int64_t)slice * QB + qrow) * D);
#pragma unroll
    for (int s = 0; s < STEPS; s++) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(src + (2 * s + g) * 16));
  }
  const char* kbase = reinterpret_cast<const char*>(kp + slice * k_slice_stride);
  i32x4 stage[LPT];
  auto fetch_tile = [&](int tile) {
#pragma unroll
    for (int i = 0; i < LPT; i++) {
      const int ci = i * 256 + tid, row = ci / CHUNKS, c = ci % CHUNKS;
      const int krow = min(tile * 32 + row, G - 1);
      stage[i] = *reinterpret_cast<const i32x4*>(kbase + (int64_t)krow * k_row_stride * 2 + c * 16);
    }
  };
  auto stash_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LPT; i++) {
      const int ci = i * 256 + tid, row = ci / CHUNKS, c = ci % CHUNKS;
      *reinterpret_cast<i32x4*>(&ktile[buf][row * ROWB + ((c ^ swz(row)) * 16)]) = stage[i];
    }
  };
  // running range of the scores this lane produced, per accumulator register (= per query block)
  float vmax[16], vmin[16];
#pragma unroll
  for (int r = 0; r < 16; r++) {
    vmax[r] = -INFINITY;
    vmin[r] = INFINITY;
  }
  const int ntiles = min(kTilesPerGroup, (G - tile0 * 32 + 31) / 32);   // >= 1 by the grid
  fetch_tile(tile0);
  stash_tile(0);
  __syncthreads();
  for (int t = 0; t < ntiles; t++) {
    if (t + 1 < ntiles) fetch_tile(tile0 + t + 1);
    const unsigned char* kt = ktile[t & 1];
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0.0f;
#pragma unroll
    for (int s = 0; s < STEPS; s++) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(kt + ln * ROWB + (((2 * s + g) ^ swz(ln)) * 16)));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[s], kf, acc, 0, 0, 0);
    }
    const int col = (tile0 + t) * 32 + ln;
    if (col < G) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int qrow = q0 + 8 * (r / 4) + 4 * g + (r % 4);
        const float v = acc[r] * scale;
        vmax[r] = fmaxf(vmax[r], v);
        vmin[r] = fminf(vmin[r], v);
        if (qrow < QB) scores[((int64_t)blockIdx.y * 128 + (qrow - qtile0)) * Gs + col] = v;
      }
    }
    if (t + 1 < ntiles) stash_tile((t + 1) & 1);   // (the buffer that was read in step t - 1, before the last barrier)
    __syncthreads();
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
// Weight of a score relative to the row maximum: trunc(2^40 * 2^((s - rmax) * log2 e)), 2^-40 fixed point.
// The bare exponential instruction differs from exp2f only below 2^-126, where the weight is zero either way.
// The product with 2^40 is exact, and so is its split into a multiple of 2^16 and a remainder (the hardware
// has no float -> 64-bit integer conversion).
__device__ __forceinline__ unsigned long long weight_of(float s, float rmax) {
  const float x = __builtin_amdgcn_exp2f((s - rmax) * kLog2e) * 1099511627776.0f;   // in [0, 2^40]
  const unsigned hi = (unsigned)(x * (1.0f / 65536.0f));
  const unsigned lo = (unsigned)__builtin_fmaf(-(float)hi, 65536.0f, x);
  return ((unsigned long long)hi << 16) + lo;
}

// Visits every score of a row: four consecutive scores per thread and step (16-byte loads; rows start 16-byte
// aligned and their stride is a multiple of four floats), four steps in flight.
template <int THREADS, typename Fn>
__device__ __forceinline__ void for_each_score(const float* s, int G, Fn&& fn) {
  constexpr int STEP = THREADS * 4;
  auto whole = [&](const float4& v, int j4) {
    fn(v.x, j4);
    fn(v.y, j4 + 1);
    fn(v.z, j4 + 2);
    fn(v.w, j4 + 3);
  };
  auto ragged = [&](const float4& v, int j4) {
    fn(v.x, j4);
    if (j4 + 1 < G) fn(v.y, j4 + 1);
    if (j4 + 2 < G) fn(v.z, j4 + 2);
    if (j4 + 3 < G) fn(v.w, j4 + 3);
  };
  int j4 = threadIdx.x * 4;
  for (; j4 + 3 * STEP + 3 < G; j4 += 4 * STEP) {
    const float4 a = *reinterpret_cast<const float4*>(s + j4);
    const float4 b = *reinterpret_cast<const float4*>(s + j4 + STEP);
    const float4 c = *reinterpret_cast<const float4*>(s + j4 + 2 * STEP);
    const float4 d = *reinterpret_cast<const float4*>(s + j4 + 3 * STEP);
    whole(a, j4);
    whole(b, j4 + STEP);
    whole(c, j4 + 2 * STEP);
    whole(d, j4 + 3 * STEP);
  }
  for (; j4 < G; j4 += STEP) ragged(*reinterpret_cast<const float4*>(s + j4), j4);
}

// Exclusive prefix of `n` over the threads of the workgroup in thread order; *total gets the sum.
// wave_tot: THREADS / 64 words of shared memory.  Contains two barriers.
template <int THREADS>
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
  unsigned all = 0;
  for (int w2 = 0; w2 < THREADS / 64; w2++) all += wave_tot[w2];
  *total = all;
  __syncthreads();
  return before + incl - n;
}

template <int THREADS, int BINS, int CAP>
struct SelShared {
  unsigned long long mass[BINS];
  unsigned wave_tot[THREADS / 64];
  alignas(16) unsigned long long cand[CAP];
  unsigned long long wave_m[THREADS / 64];
  unsigned wave_n[THREADS / 64];
  unsigned long long mass_above, target, cut;
  unsigned n_above, bin, bin_cnt, ncand, klo, khi;
};

template <int THREADS, int BINS, int CAP>
__device__ __forceinline__ unsigned long long block_sum_u64(SelShared<THREADS, BINS, CAP>& sh, unsigned long long v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  if ((threadIdx.x & 63) == 0) sh.wave_m[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long r = 0;
  for (int w2 = 0; w2 < THREADS / 64; w2++) r += sh.wave_m[w2];
  __syncthreads();
  return r;
}

// Exclusive prefix, in thread order, of a mass; *tm gets the mass of all threads.  Contains two barriers.
template <int THREADS, int BINS, int CAP>
__device__ __forceinline__ void block_exclusive_mass(SelShared<THREADS, BINS, CAP>& sh, unsigned long long m,
                                                     unsigned long long* em, unsigned long long* tm) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned long long im = m;
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long um = __shfl_up(im, off);
    if (lane >= off) im += um;
  }
  if (lane == 63) sh.wave_m[wv] = im;
  __syncthreads();
  unsigned long long bm = 0;
  for (int w2 = 0; w2 < wv; w2++) bm += sh.wave_m[w2];
  unsigned long long all = bm;
  for (int w2 = wv; w2 < THREADS / 64; w2++) all += sh.wave_m[w2];
  *tm = all;
  __syncthreads();
  *em = bm + im - m;
}

// Finds, in the histogram just built, the bin where the running mass (starting from mass_above) reaches the
// target; updates mass_above to exclude that bin and stores the bin.  Every thread owns BINS / THREADS consecutive
// bins; a prefix over the threads names the one owner whose bins contain the crossing.  FIRST: the histogram is
// that of the whole row; its mass Z sets the target ceil(top_p * Z) (at least 1, at most Z), and nothing lies above
// it yet.
template <bool FIRST, int THREADS, int BINS, int CAP>
__device__ __forceinline__ void locate_bin(SelShared<THREADS, BINS, CAP>& sh, float top_p) {
  const int tid = threadIdx.x;
  constexpr int PER = BINS / THREADS;
  const unsigned long long base = FIRST ? 0ull : sh.mass_above;
  unsigned long long target = FIRST ? 0ull : sh.target;
  unsigned long long local = 0;
  for (int i = 0; i < PER; i++) local += sh.mass[tid * PER + i];
  unsigned long long em, Z;
  block_exclusive_mass(sh, local, &em, &Z);
  if constexpr (FIRST) {   // every thread computes the same target
    const double t = ceil((double)top_p * (double)Z);
    target = t < 1.0 ? 1ull : (unsigned long long)t;
    if (target > Z) target = Z;
  }
  // the caller guarantees base < target <= base + (mass of this histogram); the two extra clauses only make sure
  // that some bin is named if that did not hold
  const unsigned long long lo = base + em;
  const bool mine = (lo < target && (target <= lo + local || tid == THREADS - 1)) || (tid == 0 && target <= lo);
  if (mine) {
    unsigned long long run = lo;
    int b = tid * PER;
    while (b < tid * PER + PER - 1 && run + sh.mass[b] < target) {
      run += sh.mass[b];
      b++;
    }
    sh.mass_above = run;
    sh.bin = (unsigned)b;
    if constexpr (FIRST) {
      sh.target = target;
      sh.n_above = 0;
    }
  }
  __syncthreads();
}

// Sorts cand[0 .. n2) (n2 a power of two above 64, unused entries zero) by descending key in LDS.  All threads call
// it; it ends with a barrier.
template <int THREADS, typename SH>
__device__ __forceinline__ void sort_candidates(SH& sh, int n2) {
  const int tid = threadIdx.x;
  for (int k = 2; k <= n2; k <<= 1)
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
      for (int i = tid; i < n2; i += THREADS) {
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
}

// Selection for one query block (row of scores `s`, in device memory or in LDS); called by all threads of the
// workgroup.  Writes the cut, the count and the kept set as one bit per key block (`keep_bits`, Gw words per row).
//
// Passes over the row: (1) histogram of mass over the score range; (2) the scores ranked above the crossing bin
// are counted and written as bits straight away, the bin's members are collected; then the members are ranked,
// and the bits of those at or above the cut are added.  Only a crossing bin
// with more members than the sort holds takes further passes, and a last one that writes all bits from the cut.
template <int THREADS, int BINS, int CAP, typename SH>
__device__ __forceinline__ void select_row(SH& sh, const float* s, int64_t row, float rmax, float rmin, int G, float top_p,
                                           unsigned long long* cut, unsigned* count, uint32_t* keep_bits, int Gw) {
  const int tid = threadIdx.x, lane = tid & 63;
  uint32_t* const bits_row = keep_bits + row * Gw;
  // All bits of the row from the cut (in sh.cut): set where the rank key is not below it.  A thread ranks four
  // consecutive key blocks, eight lanes make a word.
  auto write_all_bits = [&]() {
    __syncthreads();
    const unsigned long long c = sh.cut;
    for (int base = 0; base < Gw * 32; base += THREADS * 4) {
      const int j4 = base + tid * 4;
      unsigned nib = 0;
      if (j4 < G) {
        const float4 v = *reinterpret_cast<const float4*>(s + j4);
        nib = (rank_key(v.x, j4) >= c ? 1u : 0u) | (j4 + 1 < G && rank_key(v.y, j4 + 1) >= c ? 2u : 0u) |
              (j4 + 2 < G && rank_key(v.z, j4 + 2) >= c ? 4u : 0u) | (j4 + 3 < G && rank_key(v.w, j4 + 3) >= c ? 8u : 0u);
      }
      unsigned word = nib << (4 * (tid & 7));
      word |= __shfl_xor(word, 1);
      word |= __shfl_xor(word, 2);
      word |= __shfl_xor(word, 4);
      if ((tid & 7) == 0 && (j4 >> 5) < Gw) bits_row[j4 >> 5] = word;
    }
  };
  // The bits of everything above the crossing bin are in memory already (pass 2): add those of the collected
  // members cand[0 .. n) that are at or above the cut.  Those stores were made by other waves of this workgroup:
  // every wave waits until its own have completed before the barrier, so the atomics on the same words, which go to
  // the same L2, come after them (a device-wide fence would do too, but writes back the whole L2 on this chip).
  auto add_member_bits = [&](unsigned n) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const unsigned long long c = sh.cut;
    for (unsigned i = tid; i < n; i += THREADS) {
      const unsigned long long key = sh.cand[i];
      if (key >= c) {
        const unsigned id = 0xFFFFFFFFu - (unsigned)key;
        atomicOr(&bits_row[id >> 5], 1u << (id & 31));
      }
    }
  };

  // [rmin, rmax]: range of the scores (collected by the scores kernel)
  const float width = rmax - rmin;
  const float inv = width > 0.0f ? (float)BINS / width : 0.0f;
  auto value_bin = [&](float v) -> int {   // bin 0 holds the largest scores
    const int b = (int)((rmax - v) * inv);
    return b < 0 ? 0 : (b > BINS - 1 ? BINS - 1 : b);
  };

  // pass 1: mass of the row and its histogram over the score range
  for (int i = tid; i < BINS; i += THREADS) sh.mass[i] = 0;
  __syncthreads();
  for_each_score<THREADS>(s, G, [&](float v, int) { atomicAdd(&sh.mass[value_bin(v)], weight_of(v, rmax)); });
  __syncthreads();
  locate_bin<true>(sh, top_p);

  // One pass: counts the scores ranked above the crossing bin and collects the rank keys of its members, as many
  // as fit the sort.  cls(v): -1 above the bin, 0 inside, +1 below or outside what was the bin before.  WITH_BITS:
  // "above" of a thread's four consecutive key blocks is a nibble of the row's bits, eight lanes make a word (every
  // word of the row is written once).  Four 16-byte loads are in flight.
  auto count_and_collect = [&](auto&& cls, auto with_bits) {
    if (tid == 0) sh.ncand = 0;
    __syncthreads();
    unsigned na = 0;
    constexpr int STEP = THREADS * 4;
    const float4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int base = 0; base < Gw * 32; base += 4 * STEP) {   // (the same trip count for all threads: they vote below)
      float4 v[4];
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int j4 = base + e * STEP + tid * 4;
        v[e] = j4 < G ? *reinterpret_cast<const float4*>(s + j4) : zero4;
      }
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int j4 = base + e * STEP + tid * 4;
        const float x[4] = {v[e].x, v[e].y, v[e].z, v[e].w};
        unsigned nib = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int c = j4 + i < G ? cls(x[i]) : 1;
          nib |= c < 0 ? 1u << i : 0u;
          if (c == 0) {
            const unsigned pos = atomicAdd(&sh.ncand, 1u);
            if (pos < (unsigned)CAP) sh.cand[pos] = rank_key(x[i], j4 + i);
          }
        }
        na += (unsigned)__popc(nib);
        if constexpr (decltype(with_bits)::value) {
          unsigned word = nib << (4 * (tid & 7));
          word |= __shfl_xor(word, 1);
          word |= __shfl_xor(word, 2);
          word |= __shfl_xor(word, 4);
          if ((tid & 7) == 0 && (j4 >> 5) < Gw) bits_row[j4 >> 5] = word;
        }
      }
    }
    const unsigned long long na_all = block_sum_u64(sh, (unsigned long long)na);   // (its barriers also order the atomics before the read of ncand)
    if (tid == 0) {
      sh.n_above += (unsigned)na_all;
      sh.bin_cnt = sh.ncand;
    }
    __syncthreads();
  };
  {
    const int b0 = (int)sh.bin;
    count_and_collect(
        [&](float v) {
          const int b = value_bin(v);
          return b < b0 ? -1 : (b == b0 ? 0 : 1);
        },
        std::true_type{});
  }

  // The members of the crossing bin form a contiguous stretch of the ranking.  While there are too many to
  // sort, narrow the stretch: take the range [klo, khi] of their ordered score bits and histogram it again,
  // now linearly in those bits (every round divides the range by BINS, so a few rounds reach a single value).
  bool by_value = true;     // how the current bin is defined: value_bin() == bin, or key range [klo, khi]
  bool bits_partial = true; // the bits in memory are those of pass 2 (everything above the first crossing bin)
  unsigned klo = 0, khi = 0;
  for (int round = 0; round < 6; round++) {
    const unsigned bin = sh.bin;
    if (sh.bin_cnt <= (unsigned)CAP) break;
    bits_partial = false;   // members of the first bin get ranked above the final one: all bits are rewritten at the end
    // range of ordered bits inside the current bin
    if (tid == 0) {
      sh.klo = 0xFFFFFFFFu;
      sh.khi = 0u;
    }
    __syncthreads();
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
    for_each_score<THREADS>(s, G, [&, bin, by_value, klo, khi](float v, int) {
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
    for (int i = tid; i < BINS; i += THREADS) sh.mass[i] = 0;
    __syncthreads();
    for_each_score<THREADS>(s, G, [&](float v, int) {
      const unsigned o = ordered_bits(v);
      if (o >= klo && o <= khi) {
        const int b = (int)(((unsigned long long)(khi - o) * BINS) / R);
        atomicAdd(&sh.mass[b], weight_of(v, rmax));
      }
    });
    __syncthreads();
    locate_bin<false>(sh, top_p);
    // ordered bits of the new bin b: khi - o in [ceil(b*R/BINS), ceil((b+1)*R/BINS) - 1]
    const unsigned long long b = sh.bin;
    const unsigned long long d_lo = (b * R + BINS - 1) / BINS;
    const unsigned long long d_hi = ((b + 1) * R + BINS - 1) / BINS - 1;
    const unsigned nkhi = khi - (unsigned)d_lo;
    const unsigned nklo = khi - (unsigned)(d_hi > (unsigned long long)(khi - klo) ? (khi - klo) : d_hi);
    const unsigned old_hi = khi;
    count_and_collect(
        [&](float v) {
          const unsigned o = ordered_bits(v);
          return (o > nkhi && o <= old_hi) ? -1 : ((o >= nklo && o <= nkhi) ? 0 : 1);
        },
        std::false_type{});
    khi = nkhi;
    klo = nklo;
    __syncthreads();
  }

  const unsigned bin_cnt = sh.bin_cnt;
  auto finish_bits = [&]() {
    if (bits_partial)
      add_member_bits(bin_cnt);
    else
      write_all_bits();
  };
  if (bin_cnt == 0) {   // unreachable (the crossing bin has mass, hence members); kept so that no path leaves the outputs unset
    if (tid == 0) {
      sh.cut = ~0ull;
      cut[row] = ~0ull;
      count[row] = sh.n_above;
    }
    finish_bits();
    return;
  }
  if (bin_cnt <= (unsigned)CAP) {
    // rank the members of the crossing bin (they are in cand[0 .. bin_cnt)) and walk their masses
    if (bin_cnt <= 64u) {
      // few members (the usual case): the first wave holds one each, ranks them by counting (the keys are
      // distinct), orders their masses by rank through LDS and finds the crossing with a prefix over its lanes
      if (tid < 64) {
        const int n = (int)bin_cnt;
        const unsigned long long key = tid < n ? sh.cand[tid] : 0ull;
        const unsigned key_lo = (unsigned)key, key_hi = (unsigned)(key >> 32);
        int rank = 0;
        for (int j = 0; j < n; j++) {
          const unsigned long long other = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)key_hi, j) << 32) |
                                           (unsigned)__builtin_amdgcn_readlane((int)key_lo, j);
          rank += other > key ? 1 : 0;
        }
        if (tid < n) {
          sh.mass[rank] = weight_of(from_ordered(key_hi), rmax);
          sh.mass[64 + rank] = key;
        }
        unsigned long long inc = tid < n ? sh.mass[tid] : 0ull;   // (same wave: LDS accesses complete in order)
        for (int off = 1; off < 64; off <<= 1) {
          const unsigned long long up = __shfl_up(inc, off);
          if (tid >= off) inc += up;
        }
        const unsigned long long reached = __ballot(tid < n && sh.mass_above + inc >= sh.target);
        const int idx = reached ? __ffsll((long long)reached) - 1 : n - 1;   // (the last one if the masses fell short)
        if (tid == idx) {
          const unsigned long long c = sh.mass[64 + idx];
          sh.cut = c;
          cut[row] = c;
          count[row] = sh.n_above + (unsigned)idx + 1u;
        }
      }
      finish_bits();
      return;
    }
    int n2 = 128;
    while (n2 < (int)bin_cnt) n2 <<= 1;
    for (int i = (int)bin_cnt + tid; i < n2; i += THREADS) sh.cand[i] = 0ull;
    __syncthreads();
    sort_candidates<THREADS>(sh, n2);
    // first position where mass_above + (masses of cand[0..position]) reaches the target: every thread owns
    // CAP / THREADS consecutive candidates, a prefix over the threads names the owner of the crossing
    constexpr int PER = CAP / THREADS;
    const unsigned long long target = sh.target, base = sh.mass_above;
    const int lastc = (int)bin_cnt - 1;
    unsigned long long local = 0;
    for (int i = 0; i < PER; i++) {
      const int idx = tid * PER + i;
      if (idx <= lastc) local += weight_of(from_ordered((unsigned)(sh.cand[idx] >> 32)), rmax);
    }
    unsigned long long em;
    unsigned long long all;
    block_exclusive_mass(sh, local, &em, &all);
    const unsigned long long lo = base + em;
    // (the second clause names the last candidate if the masses fell short of the target, the third the first
    // one if the target was already reached; neither happens with a consistent histogram)
    const bool mine = (lo < target && (target <= lo + local || tid == lastc / PER)) || (tid == 0 && target <= lo);
    if (mine && tid * PER <= lastc) {
      unsigned long long run = lo;
      int idx = tid * PER;
      const int stop = min(lastc, tid * PER + PER - 1);
      while (idx < stop) {
        run += weight_of(from_ordered((unsigned)(sh.cand[idx] >> 32)), rmax);
        if (run >= target) break;
        idx++;
      }
      sh.cut = sh.cand[idx];
      cut[row] = sh.cand[idx];
      count[row] = sh.n_above + (unsigned)idx + 1u;
    }
    finish_bits();
    return;
  }

  // A run of more than CAP equal scores contains the crossing: all of them weigh the same, so the number
  // to keep follows by division, and they are taken in ascending id.
  const float v_eq = from_ordered(klo);
  const unsigned long long w_eq = weight_of(v_eq, rmax);
  unsigned long long need = sh.target > sh.mass_above ? sh.target - sh.mass_above : 1ull;
  unsigned long long t_keep = w_eq > 0 ? (need + w_eq - 1) / w_eq : (unsigned long long)bin_cnt;
  if (t_keep < 1) t_keep = 1;
  if (t_keep > bin_cnt) t_keep = bin_cnt;
  unsigned run = 0;   // members seen in the chunks before this one (the same in every thread)
  for (int base = 0; base < G && (unsigned long long)run < t_keep; base += THREADS * 4) {
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
    unsigned pos = run + block_exclusive<THREADS>((unsigned)in[0] + in[1] + in[2] + in[3], sh.wave_tot, &total);
#pragma unroll
    for (int e = 0; e < 4; e++)
      if (in[e] && (unsigned long long)(++pos) == t_keep) {
        sh.cut = rank_key(v_eq, j4 + e);
        cut[row] = rank_key(v_eq, j4 + e);
        count[row] = sh.n_above + (unsigned)t_keep;
      }
    run += total;
  }
  write_all_bits();   // (this path is only reached through the narrowing rounds)
}

// Row `local` of a chunk's score buffer that starts at score tile unit0: the (slice, query block) row it holds, or
// -1 for the unused rows of a slice's last tile.
__device__ __forceinline__ int64_t chunk_row(int64_t local, int unit0, int YT, int QB) {
  const int unit = unit0 + (int)(local >> 7);
  const int slice = unit / YT;
  const int qb = (unit - slice * YT) * 128 + (int)(local & 127);
  return qb < QB ? (int64_t)slice * QB + qb : -1;
}

// One workgroup per query block, rows read from device memory in every pass.
template <int THREADS, int BINS, int CAP>
__global__ void __launch_bounds__(THREADS) select_kernel(const float* scores, const unsigned* range, int unit0, int YT, int QB,
                                                         int G, int Gs, float top_p, unsigned long long* cut, unsigned* count,
                                                         uint32_t* keep_bits, int Gw) {
  __shared__ SelShared<THREADS, BINS, CAP> sh;
  const int64_t local = blockIdx.x;
  const int64_t row = chunk_row(local, unit0, YT, QB);
  if (row < 0) return;
  select_row<THREADS, BINS, CAP>(sh, scores + local * Gs, row, from_ordered(range[2 * row]),
                                        from_ordered(range[2 * row + 1]), G, top_p, cut, count, keep_bits, Gw);
}

// Rows of at most kRowBinsMax scores: the row is read from device memory ONCE.  That pass builds the mass histogram
// and leaves, in LDS, the bin of every score as 16 bits; the second pass then works on those alone (eight per lane
// and step: bin < crossing bin -> the key block is kept, eight such bits are a byte of the bit row; bin == crossing
// bin -> a member, whose score is fetched again by id).  64 KB of bins + the histogram + the members let two 512-thread
// workgroups share a compute unit, so the short barrier-separated phases of one row hide under the passes of
// another; the workgroups are persistent and take rows in turn.  A crossing bin with more members than fit is
// rare and handed to select_row, which starts that row over from device memory.
template <int THREADS, int BINS, int CAP>
struct alignas(16) BinsShared {
  SelShared<THREADS, BINS, CAP> sel;
  // the same memory serves the general path when a row is handed over (it needs no 16-bit bins)
  union {
    uint16_t bins[kRowBinsMax];
    SelShared<THREADS, kBins, kCap> general;
  };
};

template <int THREADS, int BINS, int CAP>
__global__ void __launch_bounds__(THREADS) select_bins_kernel(const float* scores, const unsigned* range, int64_t chunk_rows,
                                                              int unit0, int YT, int QB, int G, int Gs, float top_p,
                                                              unsigned long long* cut, unsigned* count, uint32_t* keep_bits,
                                                              int Gw) {
  static_assert(CAP == THREADS, "one member per thread in the ranking");
  static_assert(BINS >= 128 && BINS % THREADS == 0 && BINS < 0x7FFF, "bins (16 bits each in LDS, one value set aside)");
  __shared__ BinsShared<THREADS, BINS, CAP> shm;
  auto& sh = shm.sel;
  const int tid = threadIdx.x, lane = tid & 63;
  for (int64_t local = blockIdx.x; local < chunk_rows; local += gridDim.x) {
    const int64_t row = chunk_row(local, unit0, YT, QB);
    if (row < 0) continue;   // (the same for all threads)
    const float* s = scores + local * Gs;
    const float rmax = from_ordered(range[2 * row]), rmin = from_ordered(range[2 * row + 1]);
    uint32_t* const bits_row = keep_bits + row * Gw;
    const float width = rmax - rmin;
    const float inv = width > 0.0f ? (float)BINS / width : 0.0f;
    auto value_bin = [&](float v) -> int {   // bin 0 holds the largest scores
      const int b = (int)((rmax - v) * inv);
      return b < 0 ? 0 : (b > BINS - 1 ? BINS - 1 : b);
    };
    __syncthreads();   // the row before this one is done with the shared state
    for (int i = tid; i < BINS; i += THREADS) sh.mass[i] = 0;
    if (tid == 0) sh.ncand = 0;
    __syncthreads();

    // pass 1: four consecutive scores per thread and step, four steps in flight while four are processed; the bins go
    // to LDS in the order of the key blocks; positions past the end get kPastEnd (no bin is as large)
    constexpr unsigned kPastEnd = 0x7FFFu;
    {
      constexpr int STEP = THREADS * 4;
      auto one = [&](float v) -> unsigned {
        const int b = value_bin(v);
        atomicAdd(&sh.mass[b], weight_of(v, rmax));
        return (unsigned)b;
      };
      auto four = [&](const float4& v, int j4) {
        unsigned b0, b1, b2, b3;
        if (j4 + 3 < G) {   // (all but the last four of a row whose length is not a multiple of four)
          b0 = one(v.x);
          b1 = one(v.y);
          b2 = one(v.z);
          b3 = one(v.w);
        } else {
          b0 = one(v.x);
          b1 = j4 + 1 < G ? one(v.y) : kPastEnd;
          b2 = j4 + 2 < G ? one(v.z) : kPastEnd;
          b3 = kPastEnd;
        }
        *reinterpret_cast<uint2*>(&shm.bins[j4]) = uint2{b0 | (b1 << 16), b2 | (b3 << 16)};
      };
      const float4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
      auto load4 = [&](float4 (&x)[4], int j0) {
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] = j0 + e * STEP < G ? *reinterpret_cast<const float4*>(s + j0 + e * STEP) : zero4;
      };
      float4 cur[4], nxt[4];
      int j4 = tid * 4;
      load4(cur, j4);
      for (; j4 < G; j4 += 4 * STEP) {   // (no barrier inside: threads may leave at different trip counts)
        load4(nxt, j4 + 4 * STEP);
#pragma unroll
        for (int e = 0; e < 4; e++)
          if (j4 + e * STEP < G) four(cur[e], j4 + e * STEP);
#pragma unroll
        for (int e = 0; e < 4; e++) cur[e] = nxt[e];
      }
    }
    __syncthreads();
    locate_bin<true>(sh, top_p);

    // pass 2 on the bins, eight per lane and step with 16-bit arithmetic on pairs: bin - crossing bin is negative
    // for a key block ranked above the crossing bin (it is kept) and zero for a member of it.  The eight sign bits of
    // a lane make a byte of the row's bits, four lanes a word.  A wave owns a contiguous stretch of the row
    // (a multiple of 512 key blocks).
    {
      const unsigned b0 = sh.bin;
      const unsigned b0b0 = b0 | (b0 << 16);
      const int wv = tid >> 6;
      const int per_wave = ((G + THREADS * 8 - 1) / (THREADS * 8)) * 512;   // key blocks per wave
      const int k0 = wv * per_wave;                                            // first key block of this wave
      const int steps = min(per_wave >> 9, max(0, (G - k0 + 511) >> 9));       // of this wave (the same in all lanes)
      unsigned na = 0;
      for (int i = 0; i < steps; i++) {
        const int j8 = k0 + i * 512 + lane * 8;   // (below kRowBinsMax: at most G rounded up to 512)
        const uint4 w = *reinterpret_cast<const uint4*>(&shm.bins[j8]);
        const unsigned d0 = pk_sub_u16(w.x, b0b0), d1 = pk_sub_u16(w.y, b0b0), d2 = pk_sub_u16(w.z, b0b0), d3 = pk_sub_u16(w.w, b0b0);
        // word r holds key blocks j8 + 2r (low half) and j8 + 2r + 1: their sign bits go to bits 2r and 16 + 2r
        unsigned y = (d0 >> 15) & 0x00010001u;
        y |= (d1 >> 13) & 0x00040004u;
        y |= (d2 >> 11) & 0x00100010u;
        y |= (d3 >> 9) & 0x00400040u;
        unsigned byte = (y & 0x55u) | ((y >> 15) & 0xAAu);         // bit e: key block j8 + e is above the crossing bin
        const int left = G - j8;                                   // key blocks of this lane inside the row
        byte = left >= 8 ? byte : (left > 0 ? byte & ((1u << left) - 1u) : 0u);
        na += (unsigned)__popc(byte);
        unsigned word = byte << (8 * (lane & 3));
        word |= __shfl_xor(word, 1);
        word |= __shfl_xor(word, 2);
        const int wi = ((k0 + i * 512) >> 5) + (lane >> 2);
        if ((lane & 3) == 0 && wi < Gw) bits_row[wi] = word;
        // members: some half of the differences is zero
        const unsigned m01 = pk_min_u16(d0, d1), m23 = pk_min_u16(d2, d3);
        const unsigned m = pk_min_u16(m01, m23);
        if (min(m & 0xFFFFu, m >> 16) == 0u) {
          const unsigned dd[4] = {d0, d1, d2, d3};
#pragma unroll
          for (int e = 0; e < 8; e++) {
            const unsigned half = (e & 1 ? dd[e >> 1] >> 16 : dd[e >> 1]) & 0xFFFFu;
            if (half == 0u && e < left) {
              const unsigned pos = atomicAdd(&sh.ncand, 1u);
              if (pos < (unsigned)CAP) sh.cand[pos] = (unsigned long long)(unsigned)(j8 + e);
            }
          }
        }
      }
      const unsigned long long na_all = block_sum_u64(sh, (unsigned long long)na);   // (its barriers also order the atomics before the read of ncand)
      if (tid == 0) sh.n_above = (unsigned)na_all;
    }
    const unsigned n = sh.ncand;   // (read by all threads after the barriers of the sum)
    if (n > (unsigned)CAP) {
      // too many members for one ranking: the general path takes the row from the start (it rewrites all outputs)
      __syncthreads();
      select_row<THREADS, kBins, kCap>(shm.general, s, row, rmax, rmin, G, top_p, cut, count, keep_bits, Gw);
      continue;
    }
    // the members: thread i holds member i -- rank key from the score, fetched again by id
    unsigned long long key = 0ull;
    if (tid < (int)n) {
      const unsigned id = (unsigned)sh.cand[tid];
      key = rank_key(s[id], (int)id);
    }
    __syncthreads();   // all ids read
    if (tid < (((int)n + 7) & ~7)) sh.cand[tid] = key;   // (zeros up to a multiple of eight: they rank below every key)
    __syncthreads();
    // rank by counting (the keys are distinct), masses ordered by rank through LDS, crossing by a prefix over the threads
    int rank = 0;
    if (tid < (int)n)
      for (unsigned j = 0; j < n; j += 8) {   // eight keys per step: four 16-byte reads in flight
        unsigned long long o[8];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const ulonglong2 two = *reinterpret_cast<const ulonglong2*>(&sh.cand[j + e]);
          o[e] = two.x;
          o[e + 1] = two.y;
        }
#pragma unroll
        for (int e = 0; e < 8; e++) rank += o[e] > key ? 1 : 0;
      }
    __syncthreads();   // all of cand read: the ordered keys go back into it
    if (tid < (int)n) {
      sh.cand[rank] = key;
      sh.mass[rank] = weight_of(from_ordered((unsigned)(key >> 32)), rmax);
    }
    __syncthreads();
    {
      const unsigned long long w = tid < (int)n ? sh.mass[tid] : 0ull;
      unsigned long long before, all;
      block_exclusive_mass(sh, w, &before, &all);
      const unsigned long long target = sh.target, base = sh.mass_above;
      // the first member at which the running mass reaches the target; the last one if the masses fell short (they do
      // not with a consistent histogram)
      const bool here = tid < (int)n && ((base + before < target && base + before + w >= target) ||
                                         (tid == (int)n - 1 && base + before + w < target) || (tid == 0 && base >= target));
      if (here) {
        sh.cut = sh.cand[tid];
        cut[row] = sh.cand[tid];
        count[row] = sh.n_above + (unsigned)tid + 1u;
      }
      if (n == 0 && tid == 0) {   // unreachable (the crossing bin has mass, hence members); no output is left unset
        sh.cut = ~0ull;
        cut[row] = ~0ull;
        count[row] = sh.n_above;
      }
    }
    // The bits of everything above the crossing bin are in memory (pass 2), stored by other waves of this workgroup:
    // every wave waits until its own stores have completed before the barrier, so the atomics on the same words,
    // which go to the same L2, come after them.  Members at or above the cut are kept too.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid < (int)n && key >= sh.cut) {
      const unsigned id = 0xFFFFFFFFu - (unsigned)key;
      atomicOr(&bits_row[id >> 5], 1u << (id & 31));
    }
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

// Kept ids in ascending order, from the bit rows that the selection leaves: 256 words (8192 key blocks) per step, ids
// collected in LDS in ascending order and written out as one contiguous stretch.
__global__ void __launch_bounds__(kSelThreads) emit_bits_kernel(const uint32_t* keep_bits, int Gw, const int64_t* indptr,
                                                                int32_t* indices, int64_t capacity) {
  __shared__ unsigned wave_tot[4];
  __shared__ int32_t stage[kSelThreads * 32];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const uint32_t* bits = keep_bits + row * Gw;
  int64_t out = indptr[row];
  uint32_t nxt = tid < Gw ? bits[tid] : 0u;
  for (int base = 0; base < Gw; base += kSelThreads) {
    const int wd = base + tid;
    uint32_t word = nxt;
    nxt = wd + kSelThreads < Gw ? bits[wd + kSelThreads] : 0u;
    unsigned total;
    unsigned pos = block_exclusive<kSelThreads>((unsigned)__popc(word), wave_tot, &total);
    while (word) {
      stage[pos++] = wd * 32 + (__ffs(word) - 1);
      word &= word - 1;
    }
    __syncthreads();
    for (unsigned i = tid; i < total; i += kSelThreads)
      if (out + i < capacity) indices[out + i] = stage[i];
    out += total;
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
// The score buffer takes whole tiles of 128 query-block rows; as many tiles as fit kScoreBudget, at least one.
constexpr size_t kScoreBudget = (size_t)1 << 30;

struct Layout {
  int64_t rows, QB, G, Gs, Gw, slices;
  int64_t YT, units, chunk_units;   // score tiles per slice, in all, and per chunk
  bool row_in_lds;   // rows of scores fit the LDS-row selection kernel
  size_t qp_off, kp_off, scores_off, cut_off, count_off, range_off, bits_off, total;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int layout_of(const fgattn_params* p, Layout* lo) {
  if (p == nullptr) return FGATTN_E_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1 || p->N < 1) return FGATTN_E_SHAPE;
  if (p->d != 64 && p->d != 128) return FGATTN_E_SHAPE;
  if (p->M != 16 && p->M != 32 && p->M != 64 && p->M != 128) return FGATTN_E_SHAPE;
  if (p->L > (1 << 24)) return FGATTN_E_SHAPE;
  if (p->flags & ~31) return FGATTN_E_FLAGS;
  lo->slices = (int64_t)p->B * p->H;
  lo->QB = ((int64_t)p->L + p->M - 1) / p->M;
  lo->G = ((int64_t)p->L + p->N - 1) / p->N;
  lo->Gs = (lo->G + 31) & ~(int64_t)31;   // rows start on 128-byte lines
  lo->Gw = (lo->G + 31) / 32;
  lo->row_in_lds = lo->Gs <= kRowBinsMax && !(p->flags & FGATTN_FLAG_MASK_ROWS_IN_HBM);
  lo->rows = lo->slices * lo->QB;
  if (lo->rows > 0x7fffffffLL || lo->slices > 65535) return FGATTN_E_SHAPE;
  lo->YT = (lo->QB + 127) / 128;
  lo->units = lo->slices * lo->YT;
  const size_t tile_bytes = (size_t)128 * lo->Gs * 4;
  lo->chunk_units = (p->flags & FGATTN_FLAG_MASK_ONE_TILE_CHUNKS) ? 1 : (int64_t)(kScoreBudget / tile_bytes);
  if (lo->chunk_units < 1) lo->chunk_units = 1;
  if (lo->chunk_units > 65535) lo->chunk_units = 65535;   // (a chunk's tiles are the y dimension of a grid)
  if (lo->chunk_units > lo->units) lo->chunk_units = lo->units;
  size_t off = 0;
  lo->qp_off = off;
  off = align256(off + (size_t)lo->rows * p->d * 2);
  lo->kp_off = off;
  if (p->N > 1 || p->B > 1) off = align256(off + (size_t)lo->slices * lo->G * p->d * 2);   // else K is read in place
  lo->scores_off = off;
  off = align256(off + (size_t)lo->chunk_units * tile_bytes);
  lo->cut_off = off;
  off = align256(off + (size_t)lo->rows * 8);
  lo->count_off = off;
  off = align256(off + (size_t)lo->rows * 4);
  lo->range_off = off;
  off = align256(off + (size_t)lo->rows * 8);
  lo->bits_off = off;
  off = align256(off + (size_t)lo->rows * lo->Gw * 4);
  lo->total = off;
  return FGATTN_OK;
}

// gfx950 or an error; *cus (if given) gets the number of compute units
static int device_ok(int* cus = nullptr) {
  static int known[64];   // 0 unknown, 1 gfx950, 2 other
  static int units[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FGATTN_E_DEVICE;
  if (known[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return FGATTN_E_DEVICE;
    units[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    known[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 2;
  }
  if (cus) *cus = units[dev];
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
  int cus = 1;
  rc = device_ok(&cus);
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

  hipLaunchKernelGGL(pool_kernel, dim3((unsigned)lo.QB, (unsigned)lo.slices), dim3(64), 0, stream, qx, p->q_stride_b,
                     p->q_stride_h, p->q_stride_l, p->H, p->L, p->d, p->M, (int)lo.QB, qp, range);
  if (!launched()) return FGATTN_E_DEVICE;
  const uint16_t* kmat = kx;
  int64_t k_slice_stride = 0, k_row_stride = p->k_stride_l;
  bool k_in_place = p->N == 1 && p->B == 1;   // a block of one row is the row itself; slices are then heads
  if (k_in_place) {
    k_slice_stride = p->k_stride_h;
  } else {
    hipLaunchKernelGGL(pool_kernel, dim3((unsigned)lo.G, (unsigned)lo.slices), dim3(64), 0, stream, kx, p->k_stride_b,
                       p->k_stride_h, p->k_stride_l, p->H, p->L, p->d, p->N, (int)lo.G, kp, static_cast<unsigned*>(nullptr));
    if (!launched()) return FGATTN_E_DEVICE;
    kmat = kp;
    k_slice_stride = lo.G * p->d;
    k_row_stride = p->d;
  }
  uint32_t* keep_bits = reinterpret_cast<uint32_t*>(ws + lo.bits_off);
  const unsigned gx = (unsigned)((lo.G + kTilesPerGroup * 32 - 1) / (kTilesPerGroup * 32));
  for (int64_t unit0 = 0; unit0 < lo.units; unit0 += lo.chunk_units) {
    const int64_t nunits = lo.units - unit0 < lo.chunk_units ? lo.units - unit0 : lo.chunk_units;
    const int64_t chunk_rows = nunits * 128;
    const dim3 sgrid(gx, (unsigned)nunits);
    if (p->d == 128)
      hipLaunchKernelGGL(scores_kernel<128>, sgrid, dim3(256), 0, stream, qp, kmat, k_slice_stride, k_row_stride, (int)lo.QB,
                         (int)lo.G, (int)lo.Gs, p->scale, (int)unit0, (int)lo.YT, scores, range);
    else
      hipLaunchKernelGGL(scores_kernel<64>, sgrid, dim3(256), 0, stream, qp, kmat, k_slice_stride, k_row_stride, (int)lo.QB,
                         (int)lo.G, (int)lo.Gs, p->scale, (int)unit0, (int)lo.YT, scores, range);
    if (!launched()) return FGATTN_E_DEVICE;
    if (lo.row_in_lds) {
      const unsigned wgs = (unsigned)(chunk_rows < 2 * cus ? chunk_rows : 2 * cus);   // two fit a compute unit
      hipLaunchKernelGGL((select_bins_kernel<kRowThreads, kRowBins, kRowCap>), dim3(wgs), dim3(kRowThreads), 0, stream, scores, range, chunk_rows,
                         (int)unit0, (int)lo.YT, (int)lo.QB, (int)lo.G, (int)lo.Gs, top_p, cut, count, keep_bits, (int)lo.Gw);
    } else {
      hipLaunchKernelGGL((select_kernel<kSelThreads, kBins, kCap>), dim3((unsigned)chunk_rows), dim3(kSelThreads), 0, stream,
                         scores, range, (int)unit0, (int)lo.YT, (int)lo.QB, (int)lo.G, (int)lo.Gs, top_p, cut, count, keep_bits,
                         (int)lo.Gw);
    }
    if (!launched()) return FGATTN_E_DEVICE;
  }
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
  hipLaunchKernelGGL(emit_bits_kernel, dim3((unsigned)lo.rows), dim3(kSelThreads), 0, static_cast<hipStream_t>(stream_v),
                     reinterpret_cast<const uint32_t*>(ws + lo.bits_off), (int)lo.Gw, mask_indptr, mask_indices,
                     indices_capacity);
  return launched() ? FGATTN_OK : FGATTN_E_DEVICE;
}

}  // extern "C"
