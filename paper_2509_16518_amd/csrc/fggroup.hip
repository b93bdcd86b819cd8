// Grouping of query tiles that attend to similar sets of key blocks (paper Sec. 4.2), on the device.
//
//   bitmap_kernel     CSR mask -> one bit row per query tile
//   distance_kernel   d(i, j) = popcount(row_i XOR row_j) for all tile pairs of a slice (Sec. 4.2's distance)
//   greedy_kernel     the section's heuristic: the first ungrouped tile becomes a representative and takes the
//                     R - 1 ungrouped tiles closest to it (equal distances: lower tile index first)
//   consecutive_kernel  "merge-consecutive": R consecutive tiles per group
//   union_kernel      per group: OR of the members' rows, its popcount
//   scan_kernel       counts -> union_indptr
//   emit_kernel       per group: the union's key-block ids in ascending order and, per id, the bit mask of the
//                     members that selected it
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <type_traits>

#include "fgattn.h"

namespace fgg {

constexpr int kThreads = 256;

// one workgroup per query tile: its bit row is built in LDS and written out whole
__global__ void __launch_bounds__(kThreads) bitmap_kernel(const int64_t* indptr, const int32_t* indices, int Gw,
                                                          uint32_t* bits) {
  extern __shared__ uint32_t row[];
  const int tid = threadIdx.x;
  const int64_t w = blockIdx.x;
  for (int i = tid; i < Gw; i += kThreads) row[i] = 0u;
  __syncthreads();
  const int64_t beg = indptr[w], end = indptr[w + 1];
  for (int64_t e = beg + tid; e < end; e += kThreads) {
    const int g = indices[e];
    atomicOr(&row[g >> 5], 1u << (g & 31));
  }
  __syncthreads();
  for (int i = tid; i < Gw; i += kThreads) bits[w * Gw + i] = row[i];
}

// 64 x 64 block of the distance matrix of one slice per workgroup; a thread owns a 4 x 4 patch
__global__ void __launch_bounds__(kThreads) distance_kernel(const uint32_t* bits, int QB, int Gw, uint32_t* dist) {
  __shared__ uint32_t A[64][33], B[64][33];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int slice = blockIdx.z;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const uint32_t* base = bits + (int64_t)slice * QB * Gw;
  uint32_t acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++) acc[a][b] = 0;
  for (int w0 = 0; w0 < Gw; w0 += 32) {
    for (int t = tid; t < 64 * 32; t += kThreads) {
      const int r = t >> 5, c = t & 31;
      const bool inw = w0 + c < Gw;
      A[r][c] = (inw && i0 + r < QB) ? base[(int64_t)(i0 + r) * Gw + w0 + c] : 0u;
      B[r][c] = (inw && j0 + r < QB) ? base[(int64_t)(j0 + r) * Gw + w0 + c] : 0u;
    }
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < 32; c++) {
      uint32_t av[4], bv[4];
#pragma unroll
      for (int a = 0; a < 4; a++) av[a] = A[ty * 4 + a][c];
#pragma unroll
      for (int b = 0; b < 4; b++) bv[b] = B[tx * 4 + b][c];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) acc[a][b] += (uint32_t)__popc(av[a] ^ bv[b]);
    }
    __syncthreads();
  }
  uint32_t* out = dist + (int64_t)slice * QB * QB;
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int i = i0 + ty * 4 + a, j = j0 + tx * 4 + b;
      if (i < QB && j < QB) out[(int64_t)i * QB + j] = acc[a][b];
    }
}

__global__ void __launch_bounds__(kThreads) consecutive_kernel(int QB, int R, int NG, int32_t* group_tiles) {
  const int local = blockIdx.x * kThreads + threadIdx.x;   // position g*R + r inside the slice = the tile index
  if (local < NG * R) group_tiles[(int64_t)blockIdx.y * NG * R + local] = local < QB ? local : -1;
}

// one workgroup per slice; `used` lives in LDS (one byte per tile)
__global__ void __launch_bounds__(kThreads) greedy_kernel(const uint32_t* dist, int QB, int R, int NG,
                                                          int32_t* group_tiles) {
  extern __shared__ unsigned char used[];
  __shared__ unsigned long long best[kThreads];
  __shared__ int seed_s;
  const int tid = threadIdx.x;
  const int slice = blockIdx.x;
  const uint32_t* D = dist + (int64_t)slice * QB * QB;
  int32_t* out = group_tiles + (int64_t)slice * NG * R;
  for (int i = tid; i < QB; i += kThreads) used[i] = 0;
  __syncthreads();
  int next = 0;   // every tile below `next` is used (the same value in all threads)
  for (int g = 0; g < NG; g++) {
    if (tid == 0) {
      int s = next;
      while (s < QB && used[s]) s++;
      seed_s = s;
      if (s < QB) used[s] = 1;
    }
    __syncthreads();
    const int seed = seed_s;
    next = seed + 1;
    if (tid == 0) out[g * R] = seed < QB ? seed : -1;
    const uint32_t* drow = D + (int64_t)(seed < QB ? seed : 0) * QB;
    for (int r = 1; r < R; r++) {
      // smallest (distance, index) among the unused tiles
      unsigned long long mine = ~0ull;
      if (seed < QB)
        for (int j = tid; j < QB; j += kThreads)
          if (!used[j]) {
            const unsigned long long key = ((unsigned long long)drow[j] << 32) | (unsigned)j;
            mine = key < mine ? key : mine;
          }
      best[tid] = mine;
      __syncthreads();
      for (int off = kThreads / 2; off > 0; off >>= 1) {
        if (tid < off) best[tid] = best[tid + off] < best[tid] ? best[tid + off] : best[tid];
        __syncthreads();
      }
      const unsigned long long win = best[0];
      __syncthreads();
      if (tid == 0) {
        if (win != ~0ull) {
          const int j = (int)(win & 0xFFFFFFFFu);
          used[j] = 1;
          out[g * R + r] = j;
        } else {
          out[g * R + r] = -1;
        }
      }
      __syncthreads();
    }
    if (R == 1) __syncthreads();   // no pick, hence no barrier since seed_s was read
  }
}

// Minimum of a 32-bit value over the 64 lanes of a wave, returned in every lane: shifts within rows of 16
// lanes, then the last lane of a row broadcast into the next row(s); lanes without a source keep the identity.
__device__ __forceinline__ unsigned wave_min_u32(unsigned x) {
  constexpr unsigned ID = 0xFFFFFFFFu;
  auto shifted = [&](unsigned v, auto ctrl, auto row_mask, auto bank_mask) {
    return (unsigned)__builtin_amdgcn_update_dpp((int)ID, (int)v, decltype(ctrl)::value, decltype(row_mask)::value,
                                                 decltype(bank_mask)::value, false);
  };
  using std::integral_constant;
  unsigned y = min(x, shifted(x, integral_constant<int, 0x111>(), integral_constant<int, 0xf>(), integral_constant<int, 0xf>()));   // row_shr:1
  y = min(y, shifted(x, integral_constant<int, 0x112>(), integral_constant<int, 0xf>(), integral_constant<int, 0xf>()));            // row_shr:2
  y = min(y, shifted(x, integral_constant<int, 0x113>(), integral_constant<int, 0xf>(), integral_constant<int, 0xf>()));            // row_shr:3
  y = min(y, shifted(y, integral_constant<int, 0x114>(), integral_constant<int, 0xf>(), integral_constant<int, 0xe>()));            // row_shr:4
  y = min(y, shifted(y, integral_constant<int, 0x118>(), integral_constant<int, 0xf>(), integral_constant<int, 0xc>()));            // row_shr:8
  y = min(y, shifted(y, integral_constant<int, 0x142>(), integral_constant<int, 0xa>(), integral_constant<int, 0xf>()));            // row_bcast:15
  y = min(y, shifted(y, integral_constant<int, 0x143>(), integral_constant<int, 0xc>(), integral_constant<int, 0xf>()));            // row_bcast:31
  return (unsigned)__builtin_amdgcn_readlane((int)y, 63);
}

// The same heuristic for slices of at most KPT * kThreads tiles whose (distance, index) pairs fit 32 bits
// (`jbits` for the index): the representative's row of distances is read once per group into registers, KPT
// keys per thread, and every pick is a register minimum, a wave minimum and one barrier.
template <int KPT>
__global__ void __launch_bounds__(kThreads) greedy_small_kernel(const uint32_t* dist, int QB, int R, int NG, int jbits,
                                                                int32_t* group_tiles) {
  extern __shared__ unsigned char used[];
  __shared__ unsigned best[2][kThreads / 64];
  __shared__ int seed_s, spec_s;
  const int tid = threadIdx.x, wv = tid >> 6;
  const int slice = blockIdx.x;
  const uint32_t* D = dist + (int64_t)slice * QB * QB;
  int32_t* out = group_tiles + (int64_t)slice * NG * R;
  const unsigned jmask = (1u << jbits) - 1u;
  for (int i = tid; i < QB; i += kThreads) used[i] = 0;
  __syncthreads();
  int next = 0;        // every tile below `next` is used (the same value in all threads)
  unsigned round = 0;  // picks so far: selects the half of best[] in use
  // distances of row `ahead_row`, read one group early: the first unused tile after the representative becomes
  // the next representative unless this group picks it
  unsigned ahead[KPT] = {};
  int ahead_row = -1;
  for (int g = 0; g < NG; g++) {
    if (tid == 0) {
      int s = next;
      while (s < QB && used[s]) s++;
      seed_s = s;
      if (s < QB) used[s] = 1;
      int c = s + 1;
      while (c < QB && used[c]) c++;
      spec_s = c;
    }
    __syncthreads();
    const int seed = seed_s, spec = spec_s;
    next = seed + 1;
    if (tid == 0) out[g * R] = seed < QB ? seed : -1;
    unsigned key[KPT];   // (distance, index) of the unused tiles this thread owns, all ones otherwise
    const uint32_t* drow = D + (int64_t)(seed < QB ? seed : 0) * QB;
    // (all loads unconditional, with clamped indices: they are issued back to back, and the rows read ahead stay
    // in flight while this group picks)
    unsigned now[KPT];
#pragma unroll
    for (int i = 0; i < KPT; i++) now[i] = drow[min(i * kThreads + tid, QB - 1)];
    const bool have = seed == ahead_row;
#pragma unroll
    for (int i = 0; i < KPT; i++) {
      const int j = i * kThreads + tid;
      const bool cand = seed < QB && j < QB && !used[j];
      const unsigned dv = have ? ahead[i] : now[i];
      key[i] = cand ? ((dv << jbits) | (unsigned)j) : 0xFFFFFFFFu;
    }
    ahead_row = spec < QB ? spec : -1;
    {
      const uint32_t* srow = D + (int64_t)(spec < QB ? spec : 0) * QB;
#pragma unroll
      for (int i = 0; i < KPT; i++) ahead[i] = srow[min(i * kThreads + tid, QB - 1)];
    }
    for (int r = 1; r < R; r++, round++) {
      unsigned mine = key[0];
#pragma unroll
      for (int i = 1; i < KPT; i++) mine = min(mine, key[i]);
      const unsigned w = wave_min_u32(mine);
      if ((tid & 63) == 0) best[round & 1][wv] = w;
      __syncthreads();
      unsigned win = best[round & 1][0];
#pragma unroll
      for (int k = 1; k < kThreads / 64; k++) win = min(win, best[round & 1][k]);
      if (win != 0xFFFFFFFFu) {
        const int j = (int)(win & jmask);
#pragma unroll
        for (int i = 0; i < KPT; i++)
          if (j == i * kThreads + tid) key[i] = 0xFFFFFFFFu;
        if (tid == 0) {
          used[j] = 1;
          out[g * R + r] = j;
        }
      } else if (tid == 0) {
        out[g * R + r] = -1;
      }
    }
    __syncthreads();   // seed_s is rewritten for the next group (also orders groups without picks, R = 1)
  }
}

// one workgroup per group: OR of the members' rows into `ubits`, number of set bits into `count`
__global__ void __launch_bounds__(kThreads) union_kernel(const uint32_t* bits, const int32_t* group_tiles, int QB, int Gw,
                                                         int R, int NG, uint32_t* ubits, unsigned* count) {
  __shared__ unsigned red[kThreads];
  const int tid = threadIdx.x;
  const int64_t grp = blockIdx.x;
  const int slice = (int)(grp / NG);
  const uint32_t* base = bits + (int64_t)slice * QB * Gw;
  int tiles[8];
  for (int r = 0; r < 8; r++) tiles[r] = r < R ? group_tiles[grp * R + r] : -1;
  unsigned n = 0;
  for (int i = tid; i < Gw; i += kThreads) {
    uint32_t u = 0;
    for (int r = 0; r < 8; r++)
      if (tiles[r] >= 0) u |= base[(int64_t)tiles[r] * Gw + i];
    ubits[grp * Gw + i] = u;
    n += (unsigned)__popc(u);
  }
  red[tid] = n;
  __syncthreads();
  for (int off = kThreads / 2; off > 0; off >>= 1) {
    if (tid < off) red[tid] += red[tid + off];
    __syncthreads();
  }
  if (tid == 0) count[grp] = red[0];
}

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

// one workgroup per group: ids of the union in ascending order with their member masks
__global__ void __launch_bounds__(kThreads) emit_kernel(const uint32_t* bits, const uint32_t* ubits,
                                                        const int32_t* group_tiles, const int64_t* uindptr, int QB,
                                                        int Gw, int R, int NG, int32_t* uindices, uint8_t* umemb,
                                                        int64_t capacity) {
  __shared__ unsigned wave_tot[4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t grp = blockIdx.x;
  const int slice = (int)(grp / NG);
  const uint32_t* base = bits + (int64_t)slice * QB * Gw;
  int tiles[8];
  for (int r = 0; r < 8; r++) tiles[r] = r < R ? group_tiles[grp * R + r] : -1;
  const int64_t out0 = uindptr[grp];
  unsigned run = 0;
  for (int w0 = 0; w0 < Gw; w0 += kThreads) {
    const int i = w0 + tid;
    const uint32_t u = i < Gw ? ubits[grp * Gw + i] : 0u;
    const unsigned n = (unsigned)__popc(u);
    unsigned incl = n;
    for (int off = 1; off < 64; off <<= 1) {
      const unsigned up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    unsigned before = run;
    for (int w2 = 0; w2 < wv; w2++) before += wave_tot[w2];
    const unsigned total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
    if (u != 0u) {
      uint32_t m[8];
      for (int r = 0; r < 8; r++) m[r] = tiles[r] >= 0 ? base[(int64_t)tiles[r] * Gw + i] : 0u;
      int64_t pos = out0 + before + incl - n;
      uint32_t rest = u;
      while (rest) {
        const int b = __ffs(rest) - 1;
        rest &= rest - 1;
        unsigned mask = 0;
        for (int r = 0; r < 8; r++) mask |= ((m[r] >> b) & 1u) << r;
        if (pos < capacity) {
          uindices[pos] = i * 32 + b;
          umemb[pos] = (uint8_t)mask;
        }
        pos++;
      }
    }
    run += total;
  }
}

struct Layout {
  int64_t slices, QB, G, Gw, R, NG, groups;
  size_t bits_off, ubits_off, count_off, dist_off, total;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int layout_of(const fgattn_params* p, int mode, Layout* lo) {
  if (p == nullptr) return FGATTN_E_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1 || p->N < 1) return FGATTN_E_SHAPE;
  if (p->M != 16 && p->M != 32 && p->M != 64 && p->M != 128) return FGATTN_E_SHAPE;
  if (mode != FGATTN_GROUP_CONSECUTIVE && mode != FGATTN_GROUP_XOR) return FGATTN_E_FLAGS;
  if (p->L > (1 << 24)) return FGATTN_E_SHAPE;
  lo->slices = (int64_t)p->B * p->H;
  lo->QB = ((int64_t)p->L + p->M - 1) / p->M;
  lo->G = ((int64_t)p->L + p->N - 1) / p->N;
  lo->Gw = (lo->G + 31) / 32;
  lo->R = 128 / p->M;
  lo->NG = (lo->QB + lo->R - 1) / lo->R;
  lo->groups = lo->slices * lo->NG;
  if (lo->slices > 65535 || lo->slices * lo->QB > 0x7fffffffLL || lo->Gw * 4 > 60 * 1024 || lo->QB > 48 * 1024)
    return FGATTN_E_SHAPE;
  size_t off = 0;
  lo->bits_off = off;
  off = align256(off + (size_t)lo->slices * lo->QB * lo->Gw * 4);
  lo->ubits_off = off;
  off = align256(off + (size_t)lo->groups * lo->Gw * 4);
  lo->count_off = off;
  off = align256(off + (size_t)lo->groups * 4);
  lo->dist_off = off;
  if (mode == FGATTN_GROUP_XOR) off = align256(off + (size_t)lo->slices * lo->QB * lo->QB * 4);
  lo->total = off;
  return FGATTN_OK;
}

static int device_ok() {
  static int known[64];
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

}  // namespace fgg

extern "C" {

size_t fgattn_group_workspace_bytes(const fgattn_params* p, int mode) {
  fgg::Layout lo;
  if (fgg::layout_of(p, mode, &lo) != FGATTN_OK) return 0;
  return lo.total;
}

int fgattn_group_select(const int64_t* mask_indptr, const int32_t* mask_indices, const fgattn_params* p, int mode,
                        int32_t* group_tiles, int64_t* union_indptr, void* workspace, size_t workspace_bytes,
                        void* stream_v) {
  using namespace fgg;
  Layout lo;
  int rc = layout_of(p, mode, &lo);
  if (rc) return rc;
  if (!mask_indptr || !mask_indices || !group_tiles || !union_indptr || !workspace) return FGATTN_E_NULL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(union_indptr) & 7) ||
      (reinterpret_cast<uintptr_t>(group_tiles) & 3))
    return FGATTN_E_ALIGN;
  if (workspace_bytes < lo.total) return FGATTN_E_WORKSPACE;
  rc = device_ok();
  if (rc) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  char* ws = static_cast<char*>(workspace);
  uint32_t* bits = reinterpret_cast<uint32_t*>(ws + lo.bits_off);
  uint32_t* ubits = reinterpret_cast<uint32_t*>(ws + lo.ubits_off);
  unsigned* count = reinterpret_cast<unsigned*>(ws + lo.count_off);
  uint32_t* dist = reinterpret_cast<uint32_t*>(ws + lo.dist_off);
  const int QB = (int)lo.QB, Gw = (int)lo.Gw, R = (int)lo.R, NG = (int)lo.NG;

  hipLaunchKernelGGL(bitmap_kernel, dim3((unsigned)(lo.slices * lo.QB)), dim3(kThreads), (size_t)Gw * 4, stream, mask_indptr,
                     mask_indices, Gw, bits);
  if (!launched()) return FGATTN_E_DEVICE;
  if (mode == FGATTN_GROUP_CONSECUTIVE) {
    hipLaunchKernelGGL(consecutive_kernel, dim3((unsigned)((NG * R + kThreads - 1) / kThreads), (unsigned)lo.slices),
                       dim3(kThreads), 0, stream, QB, R, NG, group_tiles);
  } else {
    hipLaunchKernelGGL(distance_kernel, dim3((unsigned)((QB + 63) / 64), (unsigned)((QB + 63) / 64), (unsigned)lo.slices),
                       dim3(kThreads), 0, stream, bits, QB, Gw, dist);
    if (!launched()) return FGATTN_E_DEVICE;
    // a distance is at most twice the number of key blocks; with the tile index below it in 32 bits where it fits
    int jbits = 1;
    while ((1 << jbits) < QB) jbits++;
    const bool small = QB <= 16 * kThreads && (2 * lo.G + 1) < ((int64_t)1 << (32 - jbits));
    if (small && QB <= 4 * kThreads)
      hipLaunchKernelGGL(greedy_small_kernel<4>, dim3((unsigned)lo.slices), dim3(kThreads), (size_t)QB, stream, dist, QB, R,
                         NG, jbits, group_tiles);
    else if (small && QB <= 8 * kThreads)
      hipLaunchKernelGGL(greedy_small_kernel<8>, dim3((unsigned)lo.slices), dim3(kThreads), (size_t)QB, stream, dist, QB, R,
                         NG, jbits, group_tiles);
    else if (small)
      hipLaunchKernelGGL(greedy_small_kernel<16>, dim3((unsigned)lo.slices), dim3(kThreads), (size_t)QB, stream, dist, QB, R,
                         NG, jbits, group_tiles);
    else
      hipLaunchKernelGGL(greedy_kernel, dim3((unsigned)lo.slices), dim3(kThreads), (size_t)QB, stream, dist, QB, R, NG,
                         group_tiles);
  }
  if (!launched()) return FGATTN_E_DEVICE;
  hipLaunchKernelGGL(union_kernel, dim3((unsigned)lo.groups), dim3(kThreads), 0, stream, bits, group_tiles, QB, Gw, R, NG,
                     ubits, count);
  if (!launched()) return FGATTN_E_DEVICE;
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, count, lo.groups, union_indptr);
  return launched() ? FGATTN_OK : FGATTN_E_DEVICE;
}

int fgattn_group_emit(const fgattn_params* p, int mode, const int32_t* group_tiles, const int64_t* union_indptr,
                      int32_t* union_indices, uint8_t* union_members, int64_t capacity, const void* workspace,
                      size_t workspace_bytes, void* stream_v) {
  using namespace fgg;
  Layout lo;
  int rc = layout_of(p, mode, &lo);
  if (rc) return rc;
  if (!group_tiles || !union_indptr || !workspace || ((!union_indices || !union_members) && capacity > 0))
    return FGATTN_E_NULL;
  if (capacity < 0) return FGATTN_E_SHAPE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(union_indices) & 3))
    return FGATTN_E_ALIGN;
  if (workspace_bytes < lo.total) return FGATTN_E_WORKSPACE;
  rc = device_ok();
  if (rc) return rc;
  const char* ws = static_cast<const char*>(workspace);
  const uint32_t* bits = reinterpret_cast<const uint32_t*>(ws + lo.bits_off);
  const uint32_t* ubits = reinterpret_cast<const uint32_t*>(ws + lo.ubits_off);
  hipLaunchKernelGGL(emit_kernel, dim3((unsigned)lo.groups), dim3(kThreads), 0, static_cast<hipStream_t>(stream_v), bits,
                     ubits, group_tiles, union_indptr, (int)lo.QB, (int)lo.Gw, (int)lo.R, (int)lo.NG, union_indices,
                     union_members, capacity);
  return launched() ? FGATTN_OK : FGATTN_E_DEVICE;
}

}  // extern "C"
