// Forward kernel of fine-grained sparse attention for CDNA4 (gfx950, wave64).
//
// One persistent workgroup (4 waves) processes one work item at a time: a block of M query
// rows of one head against the compacted list of its active keys (paper Sec. 4.1, Fig. 1b).
// Per item: the query fragment stays in registers; the active K/V rows are gathered straight
// from global memory into LDS tiles with per-lane-address LDS-DMA loads (the gather-load of
// Sec. 4.1, re-designed for CDNA4), double-buffered so the gather of tile t+1 overlaps the
// matrix work on tile t (Sec. 4.1 "Overlapped indirect key/value load latency"); bf16 MFMA
// computes S^T = K_rel Q^T and O^T = V_rel^T P^T with fp32 online-softmax state in registers
// (Sec. 2 "Efficient dense attention").  Work items are fetched from a device-side queue in
// the order a pre-pass wrote (Sec. 4.2 "Load balancing", Appendix B).
//
// Transposed formulation: scores are produced as S^T (keys x queries) so that, in the MFMA
// accumulator layout, one lane owns one query column.  Row statistics (max, sum) are then
// per-lane scalars plus one exchange between lanes l and l^32, and the probabilities are
// already laid out as the B operand of the second MFMA: P never moves between lanes.
//
// Every wave owns a 32-query x 32-key piece of each tile.  A workgroup covers MT = 32, 64 or
// 128 query rows with RW = MT/32 waves along the rows and KW = 4/RW waves along the keys of a
// tile (NT = 32*KW keys); waves that split the keys keep private (max, sum, O) and merge once
// per work item.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fgattn_args.hpp"

namespace fg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

#define FG_LDS __attribute__((address_space(3)))
#define FG_CONST __attribute__((address_space(4)))

__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

// Gather-load primitive: every lane names its own 16-byte global source (base + 32-bit byte
// offset); the wave's 64 chunks land lane-linearly in LDS at lds_base + 16*lane (LDS-DMA, no
// VGPR staging).  Written as inline assembly so that the compiler does not track the transfer:
// the kernel orders these loads against LDS reads itself (vmcnt(0) + workgroup barrier once per
// tile), which lets the gather of tile t+1 stay in flight during all of tile t's matrix work.
__device__ __forceinline__ void gather16_to_lds(const void* base, unsigned byte_off, unsigned lds_base) {
  // base and lds_base are wave-uniform by construction; readfirstlane pins them to scalar registers
  // (it folds away when the value already lives in one)
  const uint64_t b64 = (uint64_t)(uintptr_t)base;
  base = (const void*)(uintptr_t)(((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b64 >> 32)) << 32) |
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)(b64 & 0xffffffffu)));
  lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base), "s"(lds_base)
      : "memory");   // m0 is a reserved register: no compiler-generated instruction of this kernel reads it
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(uintptr_t)((FG_LDS const unsigned char*)p);
}

__device__ __forceinline__ float lane_pair_max(float x) {
  // lanes l and l^32 hold the two halves of one query's key set
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane_pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int MT, int D>
struct FwdCfg {
  static constexpr int RW = MT / 32;            // waves along query rows (32 rows each)
  static constexpr int KW = 4 / RW;             // waves along keys within a tile (32 keys each)
  static constexpr int NT = 32 * KW;            // keys per LDS tile
  static constexpr int CH = D / 8;              // 16-byte chunks per row
  static constexpr int ROWB = D * 2;            // bytes per K or V row
  static constexpr int RPI = 64 / CH;           // rows fetched by one wave-wide 16 B/lane load
  static constexpr int RPW = NT / 4;            // rows of a tile each wave fetches
  static constexpr int IPW = RPW / RPI;         // load instructions per wave, per tile, per tensor
  static constexpr int SSTEPS = D / 16;         // MFMA steps along d for S^T
  static constexpr int DBLK = D / 32;           // 32-row blocks of O^T
  static constexpr int TENSOR_BYTES = NT * ROWB;
  static constexpr int STAGE_BYTES = 2 * TENSOR_BYTES;
  static constexpr int NSTAGE = 2;
  static constexpr int BIAS_OFF = NSTAGE * STAGE_BYTES;
  static constexpr int MERGE_REGS = DBLK * 16 + 2;
  static constexpr int MERGE_BYTES = (KW - 1) * RW * MERGE_REGS * 256;
  static constexpr int LDS_BYTES = BIAS_OFF + NSTAGE * NT * 4 + 16;
  static_assert(MT == 32 || MT == 64 || MT == 128, "query tile");
  static_assert(D == 64 || D == 128, "head dim");
  static_assert(IPW >= 1 && RPW % RPI == 0 && RPW % 8 == 0, "loader shape");
  static_assert(MERGE_BYTES <= NSTAGE * STAGE_BYTES, "merge scratch must fit in the tile buffers");
};

// Online softmax of one 32-key x 32-query score block held as an MFMA accumulator: one query per
// lane (registers 8c..8c+7 of the accumulator are the keys 16c + 8*(e/4) + 4*(lane/32) + e%4).
// First half: mask padded keys, new running max of this lane's query.
template <bool MASKED>
__device__ __forceinline__ void softmax_max(f32x16& S, const float* bias_keys, int g, float m_run, float& m_new) {
  if (MASKED) {
    // bias is 0 for a real key and -inf for a padded / out-of-range one
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      f32x4 bv = *reinterpret_cast<const f32x4*>(bias_keys + 8 * r4 + 4 * g);
#pragma unroll
      for (int e = 0; e < 4; e++) S[4 * r4 + e] = bv[e] < 0.0f ? -INFINITY : S[4 * r4 + e];
    }
  }
  float mx = fmaxf(S[0], S[1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(S[r], S[r + 1]));
  mx = lane_pair_max(mx);
  m_new = fmaxf(m_run, mx);
}

// Second half: p = exp2(c * (s - m)), partial row sum, P^T packed as the two B operands of the second MFMA.
template <bool MASKED>
__device__ __forceinline__ void softmax_exp(f32x16& S, float c_log2, float m_run, float& l_run, bf16x8 (&P)[2]) {
  const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;
  const float neg_mc = -m_safe * c_log2;
  float psum0 = 0.0f, psum1 = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[r], c_log2, neg_mc));
    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[r + 1], c_log2, neg_mc));
    if (MASKED) {   // needed when c_log2 == 0: exp2(-inf * 0) is NaN, not 0
      p0 = (S[r] == -INFINITY) ? 0.0f : p0;
      p1 = (S[r + 1] == -INFINITY) ? 0.0f : p1;
    }
    S[r] = p0;
    S[r + 1] = p1;
    psum0 += p0;
    psum1 += p1;
  }
  l_run += psum0 + psum1;
#pragma unroll
  for (int c = 0; c < 2; c++) {
    f32x8 f;
#pragma unroll
    for (int e = 0; e < 8; e++) f[e] = S[8 * c + e];
    P[c] = __builtin_convertvector(f, bf16x8);
  }
}

// NMODE selects how a compacted key position maps to a key row:
//   NMODE_DENSE   position == key (0% sparsity, no index list);
//   NMODE_N1      one key per group: key = indices[position];
//   NMODE_GROUPS  N >= 1 keys per group: key = indices[position / N] * N + position % N.
enum { NMODE_DENSE = 0, NMODE_N1 = 1, NMODE_GROUPS = 2 };

template <int MT, int D, int NMODE, int OCC>
__global__ void __launch_bounds__(256, OCC) fgattn_fwd_kernel(const FwdArgs a) {
  using C = FwdCfg<MT, D>;
  constexpr bool DENSE = NMODE == NMODE_DENSE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  __shared__ int s_item;

  const int tid = threadIdx.x;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int rw = wv / C::KW, kw = wv % C::KW;
  const int g = lane >> 5, ln = lane & 31;
  // loader role: this lane fetches 16-byte chunk `pc` of row `lrow` of each 1 KiB load
  const int lrow = lane / C::CH, pc = lane % C::CH;
  // transposed-read role for V: 16-lane group (g,u); lane n = 4*kq + q addresses key kq, d offset 4q
  const int u = (lane >> 4) & 1, kq = (lane & 15) >> 2, qq = lane & 3;

  float* bias = reinterpret_cast<float*>(smem + C::BIAS_OFF);
  const unsigned lds0 = lds_address(smem);

  // ---- LDS layout: rows of ROWB bytes, 16-byte chunks XOR-swizzled so that reads are bank-conflict free ----
  // The LDS of gfx950 serves 256 bytes per clock (64 banks): 16 lanes of a 16-byte read or 32 lanes of an
  // 8-byte read.  K (read as the A operand of S^T: lane -> row ln, chunk 2s+g) stores logical chunk c of row
  // r at chunk c ^ kswz(r), which spreads any 16 consecutive rows over 16 distinct 16-byte bank groups.
  // V (read through the transposing 8-byte read: 4 consecutive keys x 64 bytes per 32 lanes) stores chunk c
  // at c ^ vswz(r), which puts 4 consecutive rows into 4 distinct 64-byte bank groups.
  //   d = 128 (256-byte rows): kswz(r) = r & 15,       vswz(r) = (r & 3) << 2
  //   d =  64 (128-byte rows): kswz(r) = (r >> 1) & 7, vswz(r) = ((r >> 1) & 1) << 2
  // The gather writes LDS lane-linearly, so the swizzle is applied to the global source address: the lane
  // that lands on (row r, chunk pc) fetches logical chunk pc ^ swz(r).
  // reader, K: byte offset of step s is krow + ((32*s) ^ kxor)
  const int krow = (kw * 32 + ln) * C::ROWB;
  const int kxor = (g ^ (D == 128 ? (ln & 15) : ((ln >> 1) & 7))) << 4;
  // reader, V: lane n = 4*kq + qq of 16-lane group (g,u) addresses key row 4g+kq, d offset 16u + 4qq
  const int vrow = (kw * 32 + 4 * g + kq) * C::ROWB + ((qq & 1) << 3);
  const int vlp = 2 * u + (qq >> 1);                                    // chunk within the 4-chunk d block
  const int vsw = D == 128 ? (kq << 2) : (((kq >> 1) & 1) << 2);        // vswz of this lane's rows
  // loader: rows r0 + lrow with r0 a multiple of RPI; the lane-dependent part of the swizzled source chunk
  const unsigned kx = (unsigned)((pc ^ (D == 128 ? lrow : (lrow >> 1))) << 4);
  const unsigned vx = (unsigned)((pc ^ (D == 128 ? (lrow << 2) : (((lrow >> 1) & 1) << 2))) << 4);

  const unsigned k_rowb = (unsigned)(a.k_sl * 2), v_rowb = (unsigned)(a.v_sl * 2);
  const int N = DENSE ? 1 : a.N;
  const bool short_group = !DENSE && (a.L % N) != 0;

  int iter = 0;
  for (;;) {
    // ---------------- fetch the next work item ----------------
    if (a.static_assign) {
      int j = blockIdx.x + iter * gridDim.x;
      if (tid == 0) s_item = j < a.n_items ? a.order[j] : -1;
    } else {
      if (tid == 0) {
        int j = atomicAdd(a.counter, 1);
        s_item = j < a.n_items ? a.order[j] : -1;
      }
    }
    iter++;
    __syncthreads();
    const int w = __builtin_amdgcn_readfirstlane(s_item);
    if (w < 0) break;

    const int slice = w / a.QB, qi = w - slice * a.QB;
    const int b = slice / a.H, h = slice - b * a.H;
    const int row0 = qi * a.M;
    const int row_end = min(row0 + a.M, a.L);
    int64_t beg = 0;
    int cnt;  // active key groups of this item
    if (DENSE) {
      cnt = a.L;
    } else {
      beg = a.indptr[w];
      cnt = (int)(a.indptr[w + 1] - beg);
    }
    const int total = cnt * N;  // compacted key positions (a short last group leaves invalid ones)
    const int ntiles = (total + C::NT - 1) / C::NT;
    const int32_t* idx = DENSE ? nullptr : a.indices + beg;
    const uint16_t* kbase = a.k + b * a.k_sb + h * a.k_sh;
    const uint16_t* vbase = a.v + b * a.v_sb + h * a.v_sh;

    // ---------------- Q fragment (B operand of S^T), once per item ----------------
    bf16x8 qf[C::SSTEPS];
    {
      int qrow = min(row0 + rw * 32 + ln, a.L - 1);
      const char* qp = reinterpret_cast<const char*>(a.q + b * a.q_sb + h * a.q_sh + (int64_t)qrow * a.q_sl);
#pragma unroll
      for (int s = 0; s < C::SSTEPS; s++) {
        i32x4 raw = *reinterpret_cast<const i32x4*>(qp + (2 * s + g) * 16);
        raw ^= (int)a.q_sign;
        qf[s] = __builtin_bit_cast(bf16x8, raw);
      }
    }

    // ---------------- loader ----------------
    // Position p = t*NT + wv*RPW + i*RPI + lrow of the compacted list is fetched by this lane with load
    // instruction i of tile t.  Group ids are fetched one tile ahead of the rows they address.
    int gi[C::IPW];       // group id per load instruction, for the next tile to issue
    int wi[C::IPW];       // offset of the key inside its group (NMODE_GROUPS)
    int widx = 0;         // lane j: id of row j % RPW of this wave's share of the next tile but one
    int tq = 0, tr = 0;   // (t*NT) / N and (t*NT) % N for the next tile to prefetch, advanced without divisions
    const int lpos = wv * C::RPW + lrow;
    auto tile_needs_check = [&](int t) { return short_group || (t + 1) * C::NT > total; };
    // full tiles with one key per group: one coalesced load per wave brings the RPW ids of its rows
    // (lane j holds the id of row j % RPW); a cross-lane permute hands each lane the id of its own row
    auto coalesced_ids = [&](int t) { return NMODE == NMODE_N1 && !tile_needs_check(t); };
    auto fetch_ids_coalesced = [&](int t) { widx = idx[t * C::NT + wv * C::RPW + (lane & (C::RPW - 1))]; };
    auto select_ids = [&]() {
#pragma unroll
      for (int i = 0; i < C::IPW; i++) gi[i] = __builtin_amdgcn_ds_bpermute((i * C::RPI + lrow) << 2, widx);
    };
    auto fetch_ids_vector = [&](int t) {
      if (NMODE == NMODE_DENSE) return;
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        int grp;
        if (NMODE == NMODE_N1) {
          grp = t * C::NT + lpos + i * C::RPI;
        } else {
          const int x = tr + lpos + i * C::RPI;          // < N + NT
          const int q = N >= C::NT ? (x >= N ? 1 : 0) : (int)(((unsigned)x * a.n_recip16) >> 16);
          grp = tq + q;
          wi[i] = x - q * N;
        }
        gi[i] = idx[min(grp, cnt - 1)];
      }
      if (NMODE == NMODE_GROUPS) {
        tq += a.nt_div_n;
        tr += a.nt_mod_n;
        if (tr >= N) {
          tr -= N;
          tq += 1;
        }
      }
    };
    // One of the 2*IPW gather instructions of tile t: j = 2*i + (0: K rows, 1: V rows).
    // checked == false: every position of the tile is a real key (no bias writes, no range checks).
    auto issue_one = [&](int j, int t, int stage, bool checked) {
      const int i = j >> 1;
      const unsigned kst = lds0 + stage * C::STAGE_BYTES;
      const int r0 = wv * C::RPW + i * C::RPI;   // wave-uniform first row of this 1 KiB load
      const int p = t * C::NT + lpos + i * C::RPI;
      int key = NMODE == NMODE_DENSE ? p : NMODE == NMODE_N1 ? gi[i] : gi[i] * N + wi[i];
      if (checked) {
        const bool ok = p < total && key < a.L;
        key = ok ? key : 0;
        if ((j & 1) == 0 && pc == 0) bias[stage * C::NT + r0 + lrow] = ok ? 0.0f : -INFINITY;
      }
      if ((j & 1) == 0) {
        // uniform part of kswz(r0 + lrow): (r0 & 12) for d = 128, (r0 >> 1) & 4 for d = 64; vswz has none
        const unsigned ku = (unsigned)((D == 128 ? (r0 & 12) : ((r0 >> 1) & 4)) << 4);
        gather16_to_lds(kbase, __umul24((unsigned)key, k_rowb) + (kx ^ ku), kst + r0 * C::ROWB);
      } else {
        gather16_to_lds(vbase, __umul24((unsigned)key, v_rowb) + vx, kst + C::TENSOR_BYTES + r0 * C::ROWB);
      }
    };
    auto issue_tile = [&](int t, int stage, bool checked) {
#pragma unroll
      for (int j = 0; j < 2 * C::IPW; j++) issue_one(j, t, stage, checked);
    };

    // ---------------- accumulators ----------------
    f32x16 O[C::DBLK];
#pragma unroll
    for (int db = 0; db < C::DBLK; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) O[db][r] = 0.0f;
    float m_run = -INFINITY;   // running max of raw (unscaled) scores of this lane's query
    float l_run = 0.0f;        // this lane's partial sum of exponentials

    if (ntiles > 0) {
      if (coalesced_ids(0)) {
        fetch_ids_coalesced(0);
        select_ids();
      } else {
        fetch_ids_vector(0);
      }
      if (tile_needs_check(0)) issue_tile(0, 0, true); else issue_tile(0, 0, false);
      if (ntiles > 1) {
        if (coalesced_ids(1)) fetch_ids_coalesced(1); else fetch_ids_vector(1);
      }
    }

    for (int t = 0; t < ntiles; t++) {
      const int stage = t & 1;
      wait_vmem_all();
      __syncthreads();
      const unsigned char* kst = smem + stage * C::STAGE_BYTES;
      const unsigned char* vst = kst + C::TENSOR_BYTES;

      // ---- group ids: those of tile t+1 move into place, those of tile t+2 start their fetch ----
      const bool has_next = t + 1 < ntiles;
      const bool next_checked = has_next && tile_needs_check(t + 1);
      if (has_next && coalesced_ids(t + 1)) select_ids();
      if (t + 2 < ntiles && coalesced_ids(t + 2)) fetch_ids_coalesced(t + 2);

      // ---- K fragments of this wave's 32 keys: the first half is read up front ----
      auto read_kf = [&](int s) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(kst + krow + ((32 * s) ^ kxor)));
      };
      constexpr int KPRE = C::SSTEPS / 2;
      bf16x8 kf[C::SSTEPS];
#pragma unroll
      for (int s = 0; s < KPRE; s++) kf[s] = read_kf(s);
      __builtin_amdgcn_sched_barrier(0);

      // ---- the gather of the next tile goes out while the K fragments arrive ----
      if (has_next) {
        if (next_checked) issue_tile(t + 1, stage ^ 1, true); else issue_tile(t + 1, stage ^ 1, false);
      }
      __builtin_amdgcn_sched_barrier(0);

      // ---- S^T = K_rel Q^T; the first half of the V^T fragment reads rides behind the last MFMAs ----
      auto read_vf = [&](int db, int c, s16x4 (&dst)[2]) {
        const unsigned char* p0 = vst + vrow + ((((4 * db) ^ vsw) + vlp) << 4) + (16 * c) * C::ROWB;
        dst[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0));
        dst[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0 + 8 * C::ROWB));
      };
      f32x16 S;
#pragma unroll
      for (int r = 0; r < 16; r++) S[r] = 0.0f;
      s16x4 vf[C::DBLK][2][2];
#pragma unroll
      for (int s = 0; s < C::SSTEPS; s++) {
        if (s + KPRE < C::SSTEPS) kf[s + KPRE] = read_kf(s + KPRE);   // second half, one read per MFMA
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], S, 0, 0, 0);
        if (s >= C::SSTEPS / 2) {   // kf[0 .. SSTEPS/2) are dead by now: their registers take these fragments
          const int j = s - C::SSTEPS / 2;
          read_vf(j / 2, j % 2, vf[j / 2][j % 2]);
        }
      }
      if (t + 2 < ntiles && !coalesced_ids(t + 2)) fetch_ids_vector(t + 2);
      __builtin_amdgcn_sched_barrier(0);

      // ---- online softmax: one query per lane; O is rescaled only when some lane's max moved ----
      bf16x8 P[2];
      const bool masked = tile_needs_check(t);
      float m_new;
      if (masked) softmax_max<true>(S, bias + stage * C::NT + kw * 32, g, m_run, m_new);
      else softmax_max<false>(S, nullptr, g, m_run, m_new);
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_run - m_new) * a.c_log2);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) O[db][r] *= alpha;
        m_run = m_new;
      }
      if (masked) softmax_exp<true>(S, a.c_log2, m_run, l_run, P);
      else softmax_exp<false>(S, a.c_log2, m_run, l_run, P);
      __builtin_amdgcn_sched_barrier(0);
      // ---- O^T += V_rel^T P^T; the second half of the V^T fragments is read while the first half multiplies ----
#pragma unroll
      for (int db = C::DBLK / 2; db < C::DBLK; db++)
#pragma unroll
        for (int c = 0; c < 2; c++) read_vf(db, c, vf[db][c]);
#pragma unroll
      for (int db = 0; db < C::DBLK; db++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          s16x8 both = __builtin_shufflevector(vf[db][c][0], vf[db][c][1], 0, 1, 2, 3, 4, 5, 6, 7);
          O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), P[c], O[db], 0, 0, 0);
        }
    }

    // ---------------- epilogue ----------------
    float l_tot = lane_pair_sum(l_run);
    if (C::KW > 1) {
      __syncthreads();   // every wave is done with the tile buffers
      float* scratch = reinterpret_cast<float*>(smem);
      if (kw > 0) {
        float* dst = scratch + ((rw * (C::KW - 1) + kw - 1) * C::MERGE_REGS) * 64 + lane;
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) dst[(db * 16 + r) * 64] = O[db][r];
        dst[(C::DBLK * 16) * 64] = m_run;
        dst[(C::DBLK * 16 + 1) * 64] = l_tot;
      }
      __syncthreads();
      if (kw == 0) {
#pragma unroll
        for (int pw = 0; pw < C::KW - 1; pw++) {
          const float* src = scratch + ((rw * (C::KW - 1) + pw) * C::MERGE_REGS) * 64 + lane;
          const float m_o = src[(C::DBLK * 16) * 64];
          const float l_o = src[(C::DBLK * 16 + 1) * 64];
          const float m_new = fmaxf(m_run, m_o);
          const float a_me = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_run - m_new) * a.c_log2);
          const float a_ot = (m_o == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_o - m_new) * a.c_log2);
#pragma unroll
          for (int db = 0; db < C::DBLK; db++)
#pragma unroll
            for (int r = 0; r < 16; r++) O[db][r] = O[db][r] * a_me + src[(db * 16 + r) * 64] * a_ot;
          l_tot = l_tot * a_me + l_o * a_ot;
          m_run = m_new;
        }
      }
    }
    if (kw == 0) {
      const int row = row0 + rw * 32 + ln;
      if (row < row_end) {
        const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
        uint16_t* op = a.out + b * a.o_sb + h * a.o_sh + (int64_t)row * a.o_sl;
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++) {
            f32x4 f;
#pragma unroll
            for (int e = 0; e < 4; e++) f[e] = O[db][4 * r4 + e] * inv;
            bf16x4 o4 = __builtin_convertvector(f, bf16x4);
            *reinterpret_cast<i32x2*>(op + 32 * db + 8 * r4 + 4 * g) = __builtin_bit_cast(i32x2, o4);
          }
        if (g == 0) {
          const float lse = l_tot > 0.0f ? a.scale_abs * m_run + __logf(l_tot) : -INFINITY;
          a.lse[(int64_t)slice * a.L + row] = lse;
        }
      }
    }
    // the barrier at the top of the loop (after the queue pop) separates this item's LDS use from the next
    __syncthreads();
  }
  // The last workgroup to leave rewinds the queue, so a later launch can reuse the stored order
  // without a pre-pass.  Every workgroup reaches this point exactly once.
  if (!a.static_assign && tid == 0) {
    __threadfence();
    const int done = atomicAdd(a.counter + 1, 1);
    if (done == (int)gridDim.x - 1) {
      atomicExch(a.counter + 1, 0);
      atomicExch(a.counter, 0);
    }
  }
}

}  // namespace fg
