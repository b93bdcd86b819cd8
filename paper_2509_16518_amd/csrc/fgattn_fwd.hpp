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
#define FG_GLOBAL __attribute__((address_space(1)))


__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

// Gather-load primitive: every lane names its own 16-byte global source; the wave's 64 chunks
// land lane-linearly in LDS at lds_base + 16*lane (LDS-DMA, no VGPR staging).  Written as
// inline assembly so that the compiler does not track the transfer: the kernel orders these
// loads against LDS reads itself (vmcnt(0) + workgroup barrier once per tile), which lets the
// gather of tile t+1 stay in flight during all of tile t's matrix work.
__device__ __forceinline__ void gather16_to_lds(const void* gsrc, unsigned lds_base) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off"
      :
      : "v"(gsrc), "s"(lds_base)
      : "memory");   // m0 is a reserved register: no compiler-generated instruction of this kernel reads it
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(uintptr_t)((FG_LDS const unsigned char*)p);
}

__device__ __forceinline__ float lane_pair_exchange_max(float x) {
  // lanes l and l^32 hold the two halves of one query's key set
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane_pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int MT, int D, int KPW>
struct FwdCfg {
  static constexpr int RW = MT / 32;            // waves along query rows (32 rows each)
  static constexpr int KW = 4 / RW;             // waves along keys within a tile
  static constexpr int NT = KPW * KW;           // keys per LDS tile
  static constexpr int CH = D / 8;              // 16-byte chunks per row
  static constexpr int ROWB = D * 2;            // bytes per K or V row
  static constexpr int RPI = 64 / CH;           // rows fetched by one wave-wide 16 B/lane load
  static constexpr int RPW = NT / 4;            // rows of a tile each wave fetches
  static constexpr int IPW = RPW / RPI;         // load instructions per wave, per tile, per tensor
  static constexpr int KBLK = KPW / 32;         // 32-key MFMA blocks per wave per tile
  static constexpr int SSTEPS = D / 16;         // MFMA steps along d for S^T
  static constexpr int DBLK = D / 32;           // 32-row blocks of O^T
  static constexpr int TENSOR_BYTES = NT * ROWB;
  static constexpr int STAGE_BYTES = 2 * TENSOR_BYTES;
  static constexpr int BIAS_OFF = 2 * STAGE_BYTES;
  static constexpr int MERGE_REGS = DBLK * 16 + 2;
  static constexpr int MERGE_BYTES = (KW - 1) * RW * MERGE_REGS * 256;
  static constexpr int LDS_BYTES = BIAS_OFF + 2 * NT * 4 + 16;
  static_assert(MT == 32 || MT == 64 || MT == 128, "query tile");
  static_assert(D == 64 || D == 128, "head dim");
  static_assert(KPW == 32 || KPW == 64, "keys per wave per tile");
  static_assert(IPW >= 1 && RPW % RPI == 0 && RPW % 8 == 0, "loader shape");
  static_assert(MERGE_BYTES <= 2 * STAGE_BYTES, "merge scratch must fit in the tile buffers");
};

template <int MT, int D, int KPW, int OCC>
__global__ void __launch_bounds__(256, OCC) fgattn_fwd_kernel(const FwdArgs a) {
  using C = FwdCfg<MT, D, KPW>;
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

  // ---- per-lane LDS read offsets (loop invariant) ----
  // K as the A operand of S^T: lane reads row (ln), 16-byte chunk (2s+g), XOR-swizzled by row&7
  int koff[4];
#pragma unroll
  for (int s4 = 0; s4 < 4; s4++) koff[s4] = (kw * KPW + ln) * C::ROWB + (((2 * s4 + g) ^ (ln & 7)) << 4);
  // V^T through the transposing LDS read: swizzle (row&3)<<1 on the chunk index
  const int vlane_part = ((2 * u + (qq >> 1)) ^ (kq << 1));
  const int voff_even = (kw * KPW + 4 * g + kq) * C::ROWB + (vlane_part << 4) + ((qq & 1) << 3);
  const int voff_odd = (kw * KPW + 4 * g + kq) * C::ROWB + ((vlane_part ^ 4) << 4) + ((qq & 1) << 3);

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
    const bool dense = a.indptr == nullptr;
    int64_t beg = 0;
    int cnt;  // active key groups of this item
    if (dense) {
      cnt = a.L;
    } else {
      beg = a.indptr[w];
      cnt = (int)(a.indptr[w + 1] - beg);
    }
    const int gN = dense ? 1 : a.N;
    const int total = cnt * gN;  // compacted key positions (a short last group leaves invalid ones)
    const int ntiles = (total + C::NT - 1) / C::NT;
    const bool short_group = !dense && (a.L % a.N) != 0;
    const int32_t* idx = dense ? nullptr : a.indices + beg;
    const char* kbase = reinterpret_cast<const char*>(a.k + b * a.k_sb + h * a.k_sh);
    const char* vbase = reinterpret_cast<const char*>(a.v + b * a.v_sb + h * a.v_sh);
    const int64_t k_rowb = a.k_sl * 2, v_rowb = a.v_sl * 2;

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

    // ---------------- loader state ----------------
    int gi[C::IPW];   // group ids (sparse) fetched one tile ahead
    auto prefetch_idx = [&](int t) {
      if (dense) return;
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        int p = t * C::NT + wv * C::RPW + i * C::RPI + lrow;
        int grp = a.nshift >= 0 ? (p >> a.nshift) : (int)((unsigned)p / (unsigned)a.N);
        gi[i] = idx[min(grp, cnt - 1)];
      }
    };
    auto issue_tile = [&](int t, int stage) {
      unsigned char* kst = smem + stage * C::STAGE_BYTES;
      unsigned char* vst = kst + C::TENSOR_BYTES;
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        const int r0 = wv * C::RPW + i * C::RPI;   // wave-uniform first row of this 1 KiB load
        const int r = r0 + lrow;
        const int p = t * C::NT + r;
        int key;
        bool ok;
        if (dense) {
          key = p;
          ok = p < a.L;
        } else {
          int grp = a.nshift >= 0 ? (p >> a.nshift) : (int)((unsigned)p / (unsigned)a.N);
          key = gi[i] * a.N + (p - grp * a.N);
          ok = grp < cnt && key < a.L;
        }
        key = ok ? key : 0;
        const char* gk = kbase + (int64_t)key * k_rowb + ((pc ^ (r & 7)) << 4);
        const char* gv = vbase + (int64_t)key * v_rowb + ((pc ^ ((r & 3) << 1)) << 4);
        gather16_to_lds(gk, lds_address(kst + r0 * C::ROWB));
        gather16_to_lds(gv, lds_address(vst + r0 * C::ROWB));
        if (pc == 0) bias[stage * C::NT + r] = ok ? 0.0f : -INFINITY;
      }
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
      prefetch_idx(0);
      issue_tile(0, 0);
      if (ntiles > 1) prefetch_idx(1);
    }

    for (int t = 0; t < ntiles; t++) {
      const int stage = t & 1;
      wait_vmem_all();
      __syncthreads();
      if (t + 1 < ntiles) {
        issue_tile(t + 1, stage ^ 1);
        if (t + 2 < ntiles) prefetch_idx(t + 2);
      }
      const unsigned char* kst = smem + stage * C::STAGE_BYTES;
      const unsigned char* vst = kst + C::TENSOR_BYTES;

      // ---- S^T = K_rel Q^T ----
      f32x16 S[C::KBLK];
#pragma unroll
      for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) S[kb][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::SSTEPS; s++) {
#pragma unroll
        for (int kb = 0; kb < C::KBLK; kb++) {
          const unsigned char* p = kst + koff[s & 3] + (s >> 2) * 128 + kb * 32 * C::ROWB;
          bf16x8 ka = __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(p));
          S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[s], S[kb], 0, 0, 0);
        }
      }

      // ---- mask padded / invalid keys (last tile, or a short last key group anywhere) ----
      const bool mask_tile = short_group || (t == ntiles - 1 && (total % C::NT) != 0);
      if (mask_tile) {
#pragma unroll
        for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++) {
            f32x4 bv = *reinterpret_cast<const f32x4*>(bias + stage * C::NT + kw * KPW + kb * 32 + 8 * r4 + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; e++) S[kb][4 * r4 + e] = bv[e] < 0.0f ? -INFINITY : S[kb][4 * r4 + e];
          }
      }

      // ---- online softmax: one query per lane ----
      float mx = S[0][0];
#pragma unroll
      for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) mx = fmaxf(mx, S[kb][r]);
      mx = lane_pair_exchange_max(mx);
      const float m_new = fmaxf(m_run, mx);
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_run - m_new) * a.c_log2);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) O[db][r] *= alpha;
        m_run = m_new;
      }
      const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;
      const float neg_mc = -m_safe * a.c_log2;
      float psum = 0.0f;
#pragma unroll
      for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][r], a.c_log2, neg_mc));
          if (mask_tile) pv = (S[kb][r] == -INFINITY) ? 0.0f : pv;
          S[kb][r] = pv;
          psum += pv;
        }
      l_run += psum;

      // ---- P^T as the B operand: registers 8c..8c+7 of block kb are exactly keys(c, g, 0..7) ----
      bf16x8 P[C::KBLK][2];
#pragma unroll
      for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          f32x8 f;
#pragma unroll
          for (int e = 0; e < 8; e++) f[e] = S[kb][8 * c + e];
          P[kb][c] = __builtin_convertvector(f, bf16x8);
        }

      // ---- O^T += V_rel^T P^T ----
#pragma unroll
      for (int db = 0; db < C::DBLK; db++) {
        const int vlane = (db & 1) ? voff_odd : voff_even;
        const int chunk_base = ((4 * db) & ~4) << 4;   // chunk index bits above the swizzled ones
#pragma unroll
        for (int kb = 0; kb < C::KBLK; kb++)
#pragma unroll
          for (int c = 0; c < 2; c++) {
            const unsigned char* p0 = vst + vlane + chunk_base + (kb * 32 + 16 * c) * C::ROWB;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0 + 8 * C::ROWB));
            s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), P[kb][c], O[db], 0, 0, 0);
          }
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
