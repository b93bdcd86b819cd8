// Forward kernel of fine-grained sparse attention for CDNA4 (gfx950, wave64).
//
// One persistent workgroup (4 waves) processes one work item at a time: a block of M query
// rows of one head against the compacted list of its active keys (paper Sec. 4.1, Fig. 1b).
// Per item: the query fragment stays in registers; the active K/V rows are gathered straight
// from global memory into rings of LDS tiles with per-lane-address LDS-DMA loads (the
// gather-load of Sec. 4.1, re-designed for CDNA4), one or two tiles ahead of their use
// (Sec. 4.1 "Overlapped indirect key/value load latency"); bf16 MFMA computes
// S^T = K_rel Q^T and O^T = V_rel^T P^T with fp32 online-softmax state in registers (Sec. 2
// "Efficient dense attention").  A gather instruction holds the wave that issues it until the
// vector-memory path has taken it (~170 clocks under load); MFMAs issued before it keep
// executing meanwhile, so each tile's key loop interleaves one gather with one MFMA of each
// contraction, and keeps the softmax arithmetic in a separate vector-ALU phase.  Work items are
// fetched from a device-side queue in the order a pre-pass wrote (Sec. 4.2 "Load balancing",
// Appendix B).
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

#include <type_traits>

#include "fgattn_args.hpp"

namespace fg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
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
// tile), which lets the gathers of later tiles stay in flight during all of a tile's matrix work.
__device__ __forceinline__ void gather16_to_lds(const void* base, unsigned byte_off, unsigned lds_base) {
  // base and lds_base are wave-uniform by construction; readfirstlane pins them to scalar registers
  // (it folds away when the value already lives in one)
  const uint64_t b64 = (uint64_t)(uintptr_t)base;
  base = (const void*)(uintptr_t)(((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b64 >> 32)) << 32) |
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)(b64 & 0xffffffffu)));
  lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile(
      "s_mov_b32 m0, %2 ; fg_m0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base), "s"(lds_base)
      : "memory", "m0");
}
// The same transfer for a run of up to four 1 KiB loads that land back to back in LDS: M0 is written once
// (gather16_first) and the following loads (gather16_next<K>) add K KiB through the instruction offset.  That
// offset also enters the global address, so `base_m4k` is the true base minus 4096 and the byte offset carries
// +4096 - 1024*K (kept non-negative: the 32-bit offset is zero-extended).
// gather16_next relies on M0 still holding what the preceding gather16_first wrote.  The statements in between are
// MFMAs, LDS reads and vector arithmetic, none of which the compiler implements through M0 on gfx950; the build
// enforces it: it scans the generated assembly of every kernel and fails if any instruction other than the
// `s_mov_b32 m0` lines marked fg_m0 above writes M0.
__device__ __forceinline__ const void* pin_scalar(const void* p) {
  // wave-uniform by construction; readfirstlane pins it to scalar registers (it folds away when already there)
  const uint64_t b64 = (uint64_t)(uintptr_t)p;
  return (const void*)(uintptr_t)(((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(b64 >> 32)) << 32) |
                                  (unsigned)__builtin_amdgcn_readfirstlane((int)(b64 & 0xffffffffu)));
}
__device__ __forceinline__ void gather16_first(const void* base_m4k, unsigned byte_off, unsigned lds_base) {
  base_m4k = pin_scalar(base_m4k);
  lds_base = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile(
      "s_mov_b32 m0, %2 ; fg_m0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(byte_off), "s"(base_m4k), "s"(lds_base)
      : "memory", "m0");
}
template <int K>
__device__ __forceinline__ void gather16_next(const void* base_m4k, unsigned byte_off) {
  static_assert(K >= 1 && K <= 3, "the instruction offset is 13-bit signed");
  base_m4k = pin_scalar(base_m4k);
  if (K == 1) asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" : : "v"(byte_off), "s"(base_m4k) : "memory");
  if (K == 2) asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" : : "v"(byte_off), "s"(base_m4k) : "memory");
  if (K == 3) asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" : : "v"(byte_off), "s"(base_m4k) : "memory");
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

constexpr float kLazyLog2 = 8.0f;   // how far (log2 units) the exponent base may lag behind the running max

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
// MEMBER >= 0 (grouped query tiles): the row holds, per key, the bit mask of the group members that selected it;
// a query of member MEMBER keeps only the keys whose bit is set.
template <bool MASKED>
__device__ __forceinline__ void softmax_max(f32x16& S, const float* bias_keys, int g, float m_run, float& m_new,
                                            int member = -1) {
  if (MASKED && member >= 0) {
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      i32x4 bv = *reinterpret_cast<const i32x4*>(bias_keys + 8 * r4 + 4 * g);
#pragma unroll
      for (int e = 0; e < 4; e++) S[4 * r4 + e] = ((bv[e] >> member) & 1) ? S[4 * r4 + e] : -INFINITY;
    }
  } else if (MASKED) {
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

// NMODE selects how a compacted key position maps to a key row:
//   NMODE_DENSE   position == key (0% sparsity, no index list);
//   NMODE_N1      one key per group: key = indices[position];
//   NMODE_GROUPS  N >= 1 keys per group: key = indices[position / N] * N + position % N, L a multiple of N;
//   NMODE_GROUPS_SHORT  the same with a short last group (L not a multiple of N): any tile may then hold
//                 positions past the end of the sequence, which are masked out.
enum { NMODE_DENSE = 0, NMODE_N1 = 1, NMODE_GROUPS = 2, NMODE_GROUPS_SHORT = 3 };

// PART selects what is executed: PART_ALL is the forward pass; PART_GATHER keeps only the index translation and
// the row gathers, PART_COMPUTE everything but the row gathers (both leave meaningless results and exist so that
// the two halves of the kernel can be timed apart on the same launch shape).
enum { PART_ALL = 0, PART_GATHER = 1, PART_COMPUTE = 2 };

// GROUPED (paper Sec. 4.2): a work item is a GROUP of query tiles (a.tile_rows rows each, R = MT / tile_rows of
// them, listed in a.group_tiles) that shares one gathered key list -- the union of the members' lists -- while
// every member attends only to its own key blocks: a.memb holds, per entry of the union list, the bit mask of the
// members that selected it, and scores of the others are set to -inf before the softmax.
template <int MT, int D, int NMODE, int OCC, int PART = PART_ALL, bool GROUPED = false>
__global__ void __launch_bounds__(256, OCC) fgattn_fwd_kernel(const FwdArgs a) {
  using C = FwdCfg<MT, D>;
  constexpr bool DENSE = NMODE == NMODE_DENSE;
  constexpr bool WAVE_PRIO = NMODE == NMODE_DENSE || NMODE == NMODE_N1;
  static_assert(!GROUPED || (MT == 128 && (NMODE == NMODE_N1 || NMODE == NMODE_GROUPS_SHORT)),
                "groups are 128 query rows with a sparse list (any L: the variant that masks positions past the end)");
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
  // per bias-ring slot: tile number + 1 of the last tile that put a key to be masked out into the slot
  int* masked_tile = reinterpret_cast<int*>(smem + C::BIAS_OFF + C::NSTAGE * C::NT * 4);
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
  // reader, K: byte offset of step s is kor ^ (32*s): the row base has its low 8 bits clear and the swizzle term
  // ((g ^ kswz) << 4) only touches bits 4..7, so the sum folds into one XOR with the step constant
  const int kor = ((kw * 32 + ln) * C::ROWB) | ((g ^ (D == 128 ? (ln & 15) : ((ln >> 1) & 7))) << 4);
  // reader, V: lane n = 4*kq + qq of 16-lane group (g,u) addresses key row 4g+kq, d offset 16u + 4qq
  const int vrow = (kw * 32 + 4 * g + kq) * C::ROWB + ((qq & 1) << 3);
  const int vlp = 2 * u + (qq >> 1);                                    // chunk within the 4-chunk d block
  const int vsw = D == 128 ? (kq << 2) : (((kq >> 1) & 1) << 2);        // vswz of this lane's rows
  int voff[C::DBLK];                                                    // per-lane byte offset of d block db
#pragma unroll
  for (int db = 0; db < C::DBLK; db++) voff[db] = vrow + ((((4 * db) ^ vsw) + vlp) << 4);
  // loader: rows r0 + lrow with r0 a multiple of RPI; the lane-dependent part of the swizzled source chunk
  const unsigned kx = (unsigned)((pc ^ (D == 128 ? lrow : (lrow >> 1))) << 4);
  const unsigned vx = (unsigned)((pc ^ (D == 128 ? (lrow << 2) : (((lrow >> 1) & 1) << 2))) << 4);

  const unsigned k_rowb = (unsigned)(a.k_sl * 2), v_rowb = (unsigned)(a.v_sl * 2);
  const int N = DENSE ? 1 : a.N;
  constexpr bool short_group = NMODE == NMODE_GROUPS_SHORT;   // (the host picks the variant from L % N)

  // Per bias-ring slot: the tile that was last consumed from it had masked keys, so its row holds entries other
  // than zero and the next tile's loaders must rewrite it whole (true at the start: LDS holds anything).
  bool slot_dirty[2] = {true, true};
  // (this bookkeeping is used only where a short last group can put masked keys into any tile: N keys per group
  // with L not a multiple of N; elsewhere only a ragged last tile has them, and every checked tile writes its
  // whole row)
  constexpr bool LAZY_BIAS = NMODE == NMODE_GROUPS_SHORT && !GROUPED;
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
    // this lane's query row; in a group the 32 rows of a wave come from the member tiles' own positions
    int my_row = row0 + rw * 32 + ln;
    bool my_row_valid = my_row < row_end;
    int my_member = 0;   // which member of the group this lane's query belongs to
    if constexpr (GROUPED) {
      const int qg = rw * 32 + ln;
      my_member = qg / a.tile_rows;
      const int tile = a.group_tiles[(int64_t)w * a.R + my_member];
      my_row = tile * a.tile_rows + (qg - my_member * a.tile_rows);
      my_row_valid = tile >= 0 && my_row < a.L;
    }
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
    // Row that padded / out-of-range positions of a tile fetch (their scores are masked out): the item's first
    // active key, so that only rows of the active set are ever multiplied, even by zero (0 x Inf would be NaN).
    int pad_key = 0;
    if (!DENSE && cnt > 0) pad_key = __builtin_amdgcn_readfirstlane(idx[0]) * N;
    const uint16_t* kbase = a.k + b * a.k_sb + h * a.k_sh;
    const uint16_t* vbase = a.v + b * a.v_sb + h * a.v_sh;

    // ---------------- Q fragment (B operand of S^T), once per item ----------------
    bf16x8 qf[C::SSTEPS];
    {
      int qrow = GROUPED ? (my_row_valid ? my_row : 0) : min(my_row, a.L - 1);
      const char* qp = reinterpret_cast<const char*>(a.q + b * a.q_sb + h * a.q_sh + (int64_t)qrow * a.q_sl);
#pragma unroll
      for (int s = 0; s < C::SSTEPS; s++) {
        i32x4 raw = *reinterpret_cast<const i32x4*>(qp + (2 * s + g) * 16);
        raw ^= (int)a.q_sign;
        qf[s] = __builtin_bit_cast(bf16x8, raw);
      }
    }

    // ---------------- loader ----------------
    // Position p = T*NT + wv*RPW + i*RPI + lrow of the compacted list is fetched by this lane with load
    // instruction i of tile T.  Pipeline per tile T (one iteration per tile, one barrier each):
    //   iteration T-3: group ids fetched          iteration T-2: ids -> key rows, K(T) gathered
    //   iteration T-1: S(T) = K(T) Q^T, row max   iteration T  : V(T) gathered; P(T) = exp(S(T) - m)
    //   iteration T+1: O += V(T)^T P(T)^T
    // Past the end of the list the pipeline keeps running on the last tile again (clamped tile index): a few
    // redundant, in-bounds gathers per work item instead of existence checks in every iteration.
    int gi[C::IPW];       // group ids being fetched (next tile to convert)
    int gm[C::IPW];       // GROUPED: their membership masks
    int wi[C::IPW];       // offset of the key inside its group (NMODE_GROUPS)
    int widx = 0;         // coalesced id fetch: lane j holds the id of row j % RPW of this wave's rows
    int keyA[C::IPW], keyB[C::IPW], keyC[C::IPW];   // key rows of tiles t, t+1, t+2 in iteration t
    int tq = 0, tr = 0;   // (T*NT) / N and (T*NT) % N for the next tile to fetch ids for, advanced without divisions
    const int lpos = wv * C::RPW + lrow;
    const int last = ntiles - 1;
    const uint8_t* memb = GROUPED ? a.memb + beg : nullptr;
    // a tile whose positions need a per-key entry in the bias row: short last group, ragged last tile, or (GROUPED)
    // always, since the row then carries the membership masks
    auto tile_needs_check = [&](int T) { return GROUPED || short_group || (T + 1) * C::NT > total; };
    // ... and whether the scores of tile T need the bias row at all: with a short last group only the tiles that
    // contain it do, and the lanes that loaded its missing keys have said so in masked_tile (a stale entry of an
    // earlier work item can only make a tile take the bias row needlessly: the row is written for every tile)
    // (`entry` is masked_tile[T & 1], read by the caller early enough that its latency is hidden)
    auto tile_has_masked_keys = [&](int T, int entry) {
      if (GROUPED || (T + 1) * C::NT > total) return true;
      if (!short_group) return false;
      return __builtin_amdgcn_readfirstlane(entry) == T + 1;
    };
    // full tiles with one key per group: one coalesced load per wave brings the RPW ids of its rows;
    // a cross-lane permute then hands each lane the id of its own row
    auto coalesced_ids = [&](int T) { return NMODE == NMODE_N1 && !tile_needs_check(T); };
    auto fetch_ids = [&](int T) {
      if (NMODE == NMODE_DENSE) return;
      if (__builtin_expect(coalesced_ids(T), 1)) {
        widx = idx[T * C::NT + wv * C::RPW + (lane & (C::RPW - 1))];
        return;
      }
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        int grp;
        if (NMODE == NMODE_N1) {
          grp = T * C::NT + lpos + i * C::RPI;
        } else {
          const int x = tr + lpos + i * C::RPI;          // < N + NT
          // (24-bit multiplies, which run at full rate: x < 2 NT and the reciprocal has 17 bits; below, q N <= x)
          const int q = N >= C::NT ? (x >= N ? 1 : 0) : (int)(__umul24((unsigned)x, a.n_recip16) >> 16);
          grp = tq + q;
          wi[i] = x - (int)__umul24((unsigned)q, (unsigned)N);
        }
        gi[i] = idx[min(grp, cnt - 1)];
        if constexpr (GROUPED) gm[i] = memb[min(grp, cnt - 1)];
      }
      if ((NMODE == NMODE_GROUPS || NMODE == NMODE_GROUPS_SHORT) && T < last) {   // a repeated (clamped) last tile must see the same tq, tr again
        tq += a.nt_div_n;
        tr += a.nt_mod_n;
        if (tr >= N) {
          tr -= N;
          tq += 1;
        }
      }
    };
    // ids of tile T (fetched earlier) -> key rows in keyC; padded / out-of-range positions of a checked tile
    // read the item's first active row and get a -inf score bias
    auto make_keys = [&](int T) {
      if (NMODE == NMODE_N1 && __builtin_expect(coalesced_ids(T), 1)) {
#pragma unroll
        for (int i = 0; i < C::IPW; i++) keyC[i] = __builtin_amdgcn_ds_bpermute((i * C::RPI + lrow) << 2, widx);
        return;
      }
      const bool checked = tile_needs_check(T);
      if constexpr (!LAZY_BIAS) {
        // a checked tile writes its whole row (GROUPED: the membership masks, every tile)
#pragma unroll
        for (int i = 0; i < C::IPW; i++) {
          const int p = T * C::NT + lpos + i * C::RPI;
          // (group id and N are below 2^24 and so is their product, a key row)
          int key = NMODE == NMODE_DENSE ? p : NMODE == NMODE_N1 ? gi[i] : (int)__umul24((unsigned)gi[i], (unsigned)N) + wi[i];
          if (__builtin_expect(checked, 0)) {
            const bool ok = p < total && key < a.L;
            key = ok ? key : pad_key;
            if (pc == 0) {
              if constexpr (GROUPED)
                reinterpret_cast<int*>(bias)[(T & 1) * C::NT + lpos + i * C::RPI] = ok ? gm[i] : 0;
              else
                bias[(T & 1) * C::NT + lpos + i * C::RPI] = ok ? 0.0f : -INFINITY;
            }
          }
          keyC[i] = key;
        }
        return;
      }
      // Bias row of the slot: 0 for a real key, -inf for a padded / out-of-range one.  A row is all zeros unless its
      // tile had such keys; then the tile's consumers mark the slot dirty and the loaders of the next tile in it
      // write every entry.  Otherwise only the (rare) -inf entries are written, and the tile is announced in
      // masked_tile so that the consumers look at the row at all.
      const bool rewrite = slot_dirty[T & 1];
      bool ok[C::IPW];
      bool any_bad = false;
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        const int p = T * C::NT + lpos + i * C::RPI;
        int key = (int)__umul24((unsigned)gi[i], (unsigned)N) + wi[i];
        ok[i] = !checked || (p < total && key < a.L);
        any_bad |= !ok[i];
        keyC[i] = ok[i] ? key : pad_key;
      }
      if (__builtin_expect(rewrite || __builtin_amdgcn_ballot_w64(any_bad) != 0, 0)) {
        if (pc == 0) {
#pragma unroll
          for (int i = 0; i < C::IPW; i++)
            if (rewrite || !ok[i]) bias[(T & 1) * C::NT + lpos + i * C::RPI] = ok[i] ? 0.0f : -INFINITY;
        }
        if (any_bad) masked_tile[T & 1] = T + 1;
        slot_dirty[T & 1] = false;   // (a row left alone by unchecked tiles stays dirty until a tile rewrites it)
      }
    };
    // LDS: K ring slots 0,1 then V ring slots 0,1, TENSOR_BYTES each.  A run of up to four gathers of one wave
    // lands back to back, so only the first writes M0 and the others use the instruction offset (which also
    // enters the global address: base - 4096 and a per-lane constant + 4096 - 1024*(i%4) compensate).
    unsigned kcon[C::IPW], vcon[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; i++) {
      const int r0 = wv * C::RPW + i * C::RPI;
      // uniform part of kswz(r0 + lrow): (r0 & 12) for d = 128, (r0 >> 1) & 4 for d = 64; vswz has none
      const unsigned ku = (unsigned)((D == 128 ? (r0 & 12) : ((r0 >> 1) & 4)) << 4);
      kcon[i] = (kx ^ ku) + 4096u - 1024u * (i & 3);
      vcon[i] = vx + 4096u - 1024u * (i & 3);
    }
    const char* kbase_m4k = reinterpret_cast<const char*>(kbase) - 4096;
    const char* vbase_m4k = reinterpret_cast<const char*>(vbase) - 4096;
    auto gather_k = [&](auto ic, int slot, const int (&keys)[C::IPW]) {
      constexpr int i = decltype(ic)::value;
      if constexpr (PART == PART_COMPUTE) return;
      const unsigned off = __umul24((unsigned)keys[i], k_rowb) + kcon[i];
      if constexpr ((i & 3) == 0)
        gather16_first(kbase_m4k, off, lds0 + slot * C::TENSOR_BYTES + (wv * C::RPW + i * C::RPI) * C::ROWB);
      else
        gather16_next<(i & 3)>(kbase_m4k, off);
    };
    auto gather_v = [&](auto ic, int slot, const int (&keys)[C::IPW]) {
      constexpr int i = decltype(ic)::value;
      if constexpr (PART == PART_COMPUTE) return;
      const unsigned off = __umul24((unsigned)keys[i], v_rowb) + vcon[i];
      if constexpr ((i & 3) == 0)
        gather16_first(vbase_m4k, off, lds0 + (2 + slot) * C::TENSOR_BYTES + (wv * C::RPW + i * C::RPI) * C::ROWB);
      else
        gather16_next<(i & 3)>(vbase_m4k, off);
    };

    // ---------------- accumulators ----------------
    f32x16 O[C::DBLK];
#pragma unroll
    for (int db = 0; db < C::DBLK; db++)
#pragma unroll
      for (int r = 0; r < 16; r++) O[db][r] = 0.0f;
    f32x16 SA, SB;             // S^T of even / odd tiles (one is turned into P while the other accumulates)
    i32x4 PA[2], PB[2];        // P^T (packed bf16 pairs) of even / odd tiles: B operands of the second MFMA
    float m_run = -INFINITY;   // exponent base (raw score units) of this lane's query; lags the true max lazily
    float l_run = 0.0f;        // this lane's partial sum of exponentials
    float m_pend = -INFINITY;  // running max including the tile in S
    bool resc = false;         // wave-uniform: the tile in S moves the exponent base (O, l must be rescaled)

    constexpr int NE = C::SSTEPS;          // MFMA slots per phase: PV slot e = (d block e/2, key half e%2); QK slot e = d chunk e
    constexpr int AHEAD = 3;               // LDS fragment reads run this many slots ahead of their MFMA
    constexpr int VPS = 16 / NE;           // score values handled per slot
    // gathers per iteration and wave: IPW of V then IPW of K, spread over the NE slots of phase X
    constexpr int NDMA = 2 * C::IPW;
    constexpr int DMA_PER = (NDMA + NE - 1) / NE;
    constexpr int DMA_EVERY = NDMA >= NE ? 1 : NE / NDMA;
    auto read_vf = [&](const unsigned char* vst, int e) {
      const int db = e >> 1, c = e & 1;
      const unsigned char* p0 = vst + voff[db] + (16 * c) * C::ROWB;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS s16x4*)(p0 + 8 * C::ROWB));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // Phase X.  O^T += V^T P^T with V in slot `vslot` (a constant) and, with QK, Sn = K Q^T with K in the same
    // slot number of the K ring: one MFMA of each per slot.  With GATHER, every slot also issues one of this
    // iteration's gathers: V rows of the current tile (keys in keyA) -> the V slot this phase does not read, then
    // K rows of the tile after next (keys in keyC) -> the K slot this phase does not read.  The gather holds the
    // wave; the two MFMAs just issued execute underneath it.
    auto x_phase = [&](auto vslot, const i32x4 (&Pin)[2], auto with_gather, auto with_qk, f32x16& Sn) {
      constexpr bool GATHER = decltype(with_gather)::value;
      constexpr bool QK = decltype(with_qk)::value && PART != PART_GATHER;   // also Sn = K(slot vslot) Q^T
      const unsigned char* vst = smem + (2 + vslot) * C::TENSOR_BYTES;
      const unsigned char* kst = smem + vslot * C::TENSOR_BYTES;
      auto read_kf = [&](int s) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(kst + (kor ^ (32 * s))));
      };
      bf16x8 kf[NE];
      if constexpr (QK) {
#pragma unroll
        for (int e = 0; e < AHEAD; e++) kf[e] = read_kf(e);
#pragma unroll
        for (int r = 0; r < 16; r++) Sn[r] = 0.0f;
      }
      const bf16x8 pin[2] = {__builtin_bit_cast(bf16x8, Pin[0]), __builtin_bit_cast(bf16x8, Pin[1])};
      bf16x8 vf[NE];
#pragma unroll
      for (int e = 0; e < AHEAD; e++)
        if constexpr (PART != PART_GATHER) vf[e] = read_vf(vst, e);
      auto slot = [&](auto ec) {
        constexpr int e = decltype(ec)::value;
        if constexpr (PART != PART_GATHER) {
          if constexpr (e + AHEAD < NE) vf[e + AHEAD] = read_vf(vst, e + AHEAD);
          O[e >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[e], pin[e & 1], O[e >> 1], 0, 0, 0);
        }
        if constexpr (QK) {
          if constexpr (e + AHEAD < NE) kf[e + AHEAD] = read_kf(e + AHEAD);
          Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[e], qf[e], Sn, 0, 0, 0);
        }
        if constexpr (GATHER) {
          if constexpr (e % DMA_EVERY == 0) {
            constexpr int j0 = (e / DMA_EVERY) * DMA_PER;
            if constexpr (j0 < C::IPW) gather_v(std::integral_constant<int, j0>(), 1 - vslot, keyA);
            else if constexpr (j0 < NDMA) gather_k(std::integral_constant<int, j0 - C::IPW>(), 1 - vslot, keyC);
            if constexpr (DMA_PER > 1) {
              constexpr int j1 = j0 + 1;
              if constexpr (j1 < C::IPW) gather_v(std::integral_constant<int, j1>(), 1 - vslot, keyA);
              else if constexpr (j1 < NDMA) gather_k(std::integral_constant<int, j1 - C::IPW>(), 1 - vslot, keyC);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      slot(std::integral_constant<int, 0>());
      slot(std::integral_constant<int, 1>());
      slot(std::integral_constant<int, 2>());
      slot(std::integral_constant<int, 3>());
      if constexpr (NE > 4) {
        slot(std::integral_constant<int, 4>());
        slot(std::integral_constant<int, 5>());
        slot(std::integral_constant<int, 6>());
        slot(std::integral_constant<int, 7>());
      }
    };
    // Phase Y, vector ALU only in the key loop.  With EXP: P = exp2(c*(So - m)) of the previous tile's scores So,
    // row sum, bf16 pack into Pout.  Then the row max of the new scores Sn (tile Tm) and the rare decision to
    // move the exponent base (see kLazyLog2).  Also rotates the key-row sets (t+1 -> t, t+2 -> t+1).  With MFMA
    // (prologue only) it first computes Sn = K Q^T with K in slot `kslot`.
    auto y_phase = [&](auto kslot, int Tm, f32x16& Sn, const f32x16& So, i32x4 (&Pout)[2], auto with_exp,
                        auto with_mfma) {
      constexpr bool EXP = decltype(with_exp)::value;
      constexpr bool MFMA = decltype(with_mfma)::value;
      // written before the barrier that precedes this phase; consumed at its end
      const int masked_entry = LAZY_BIAS ? masked_tile[Tm & 1] : 0;
      if constexpr (PART == PART_GATHER) {   // only the bookkeeping the gathers depend on
#pragma unroll
        for (int i = 0; i < C::IPW; i++) {
          keyA[i] = keyB[i];
          keyB[i] = keyC[i];
        }
        return;
      }
      const unsigned char* kst = smem + kslot * C::TENSOR_BYTES;
      auto read_kf = [&](int s) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(kst + (kor ^ (32 * s))));
      };
      const float m_safe = (m_run == -INFINITY) ? 0.0f : m_run;   // a wave that has seen no valid key yet
      const float neg_mc = -m_safe * a.c_log2;
      float psum0 = 0.0f, psum1 = 0.0f;
      bf16x8 kf[NE];
      if constexpr (MFMA) {
#pragma unroll
        for (int e = 0; e < AHEAD; e++) kf[e] = read_kf(e);
#pragma unroll
        for (int r = 0; r < 16; r++) Sn[r] = 0.0f;
      }
      auto slot = [&](auto ec) {
        constexpr int e = decltype(ec)::value;
        if constexpr (MFMA) {
          if constexpr (e + AHEAD < NE) kf[e + AHEAD] = read_kf(e + AHEAD);
          Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[e], qf[e], Sn, 0, 0, 0);
        }
        if constexpr (EXP) {
#pragma unroll
          for (int x = 0; x < VPS; x += 2) {
            const int r = e * VPS + x;
            // masked keys hold S = -inf and c_log2 > 0 (the host substitutes a tiny positive value for
            // scale = 0), so their p is exactly 0 without a select
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(So[r], a.c_log2, neg_mc));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(So[r + 1], a.c_log2, neg_mc));
            psum0 += p0;
            psum1 += p1;
            f32x2 pp = {p0, p1};
            int pk = __builtin_bit_cast(int, __builtin_convertvector(pp, bf16x2));
            // the packed pair is consumed only after the next barrier; the pin keeps the compiler from sinking the
            // exponentials there, into the phase whose issue slots belong to the gathers
            asm volatile("" : "+v"(pk));
            Pout[r >> 3][(r & 7) >> 1] = pk;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      slot(std::integral_constant<int, 0>());
      slot(std::integral_constant<int, 1>());
      slot(std::integral_constant<int, 2>());
      slot(std::integral_constant<int, 3>());
      if constexpr (NE > 4) {
        slot(std::integral_constant<int, 4>());
        slot(std::integral_constant<int, 5>());
        slot(std::integral_constant<int, 6>());
        slot(std::integral_constant<int, 7>());
      }
      if (EXP) l_run += psum0 + psum1;
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        keyA[i] = keyB[i];
        keyB[i] = keyC[i];
      }
      float m_new;
      // (the same in every wave of the workgroup)
      const bool masked = LAZY_BIAS ? tile_has_masked_keys(Tm, masked_entry) : tile_needs_check(Tm);
      if (__builtin_expect(masked, 0))
        softmax_max<true>(Sn, bias + (Tm & 1) * C::NT + kw * 32, g, m_pend, m_new, GROUPED ? my_member : -1);
      else
        softmax_max<false>(Sn, nullptr, g, m_pend, m_new);
      if constexpr (LAZY_BIAS) slot_dirty[Tm & 1] |= masked;
      m_pend = m_new;
      const bool lane_moves = (m_run == -INFINITY) ? (m_new > m_run) : ((m_new - m_run) * a.c_log2 > kLazyLog2);
      resc = __builtin_amdgcn_ballot_w64(lane_moves) != 0;
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    // Iteration t, PAR = t & 1 (a constant, so every LDS slot is an immediate):
    //   X: O += V(t-1)^T P(t-1)^T (V slot PAR^1)  ||  S(t+1) = K(t+1) Q^T (K slot PAR^1)  ||  gathers V(t) -> V slot
    //      PAR and K(t+2) -> K slot PAR
    //   Y: P(t) = exp(S(t) - m) and the row max of S(t+1), on the vector ALU
    // Every gathered tile thus has phase Y and the barrier's wait to arrive before it is published.
    auto iteration = [&](int t, auto parc, const i32x4 (&Pin)[2], i32x4 (&Pout)[2], f32x16& Sn, const f32x16& So) {
      constexpr int PAR = decltype(parc)::value;
      // K(t+1) and V(t-1), gathered during the previous iteration, become visible to every wave; every wave is
      // done reading K(t) and V(t-2), whose slots this iteration refills
      wait_vmem_all();
      __syncthreads();
      float alpha = 1.0f;
      if (__builtin_expect(resc, 0)) {   // the exponent base moves: l now, O after the MFMAs of the old base
        alpha = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_run - m_pend) * a.c_log2);
        l_run *= alpha;
        m_run = m_pend;
      }
      make_keys(min(t + 2, last));        // ids fetched during the previous iteration -> keyC
      fetch_ids(min(t + 3, last));
      // wave priority: the gather phase above the vector-ALU phase above everything outside the key loop, so that
      // the waves that feed the memory pipe are issued first and a neighbour's prologue or epilogue never delays them
      // (measured: 1-3% faster with one key per group, 6% for the dense kernel at 128 rows; slower with N keys per
      // group, whose loaders do more vector-ALU work, so not used there)
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(3);
      x_phase(std::integral_constant<int, PAR ^ 1>(), Pin, yes(), yes(), Sn);
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(1);
      if (__builtin_expect(resc, 0)) {
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) O[db][r] *= alpha;
      }
      y_phase(std::integral_constant<int, PAR ^ 1>(), min(t + 1, last), Sn, So, Pout, yes(), no());
    };

    if (ntiles > 0) {
      // prologue: K(0) -> K slot 0; V(0) -> V slot 1, only so that the first iteration's O += V^T P^T (with
      // P = 0) multiplies finite numbers; then S(0) = K(0) Q^T while K(1) loads
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int e = 0; e < 4; e++) PB[c][e] = 0;
      fetch_ids(0);
      make_keys(0);
#pragma unroll
      for (int i = 0; i < C::IPW; i++) keyA[i] = keyB[i] = keyC[i];
      auto burst = [&](auto ic) {
        gather_k(ic, 0, keyC);
      };
      auto burst_v = [&](auto ic) {
        gather_v(ic, 1, keyC);
      };
      burst(std::integral_constant<int, 0>());
      if constexpr (C::IPW > 1) burst(std::integral_constant<int, 1>());
      if constexpr (C::IPW > 2) { burst(std::integral_constant<int, 2>()); burst(std::integral_constant<int, 3>()); }
      if constexpr (C::IPW > 4) {
        burst(std::integral_constant<int, 4>()); burst(std::integral_constant<int, 5>());
        burst(std::integral_constant<int, 6>()); burst(std::integral_constant<int, 7>());
      }
      burst_v(std::integral_constant<int, 0>());
      if constexpr (C::IPW > 1) burst_v(std::integral_constant<int, 1>());
      if constexpr (C::IPW > 2) { burst_v(std::integral_constant<int, 2>()); burst_v(std::integral_constant<int, 3>()); }
      if constexpr (C::IPW > 4) {
        burst_v(std::integral_constant<int, 4>()); burst_v(std::integral_constant<int, 5>());
        burst_v(std::integral_constant<int, 6>()); burst_v(std::integral_constant<int, 7>());
      }
      fetch_ids(min(1, last));
      wait_vmem_all();      // ids of tile 1
      make_keys(min(1, last));
      auto burst1 = [&](auto ic) { gather_k(ic, 1, keyC); };
      burst1(std::integral_constant<int, 0>());
      if constexpr (C::IPW > 1) burst1(std::integral_constant<int, 1>());
      if constexpr (C::IPW > 2) { burst1(std::integral_constant<int, 2>()); burst1(std::integral_constant<int, 3>()); }
      if constexpr (C::IPW > 4) {
        burst1(std::integral_constant<int, 4>()); burst1(std::integral_constant<int, 5>());
        burst1(std::integral_constant<int, 6>()); burst1(std::integral_constant<int, 7>());
      }
      fetch_ids(min(2, last));
      wait_vmem_all();
      __syncthreads();
      // S(0) from K slot 0; keyA/keyB end up as keys(0)/keys(1)
      y_phase(std::integral_constant<int, 0>(), 0, SA, SA, PA, no(), yes());
      m_run = m_pend;   // O = 0 and l = 0 so far: the first exponent base needs no rescale
      resc = false;
      int t = 0;
      for (; t + 1 < ntiles; t += 2) {
        iteration(t, std::integral_constant<int, 0>(), PB, PA, SB, SA);
        iteration(t + 1, std::integral_constant<int, 1>(), PA, PB, SA, SB);
      }
      if (t < ntiles) iteration(t, std::integral_constant<int, 0>(), PB, PA, SB, SA);
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(0);
      wait_vmem_all();
      __syncthreads();
      if ((ntiles & 1) == 0) x_phase(std::integral_constant<int, 1>(), PB, no(), no(), SA);
      else x_phase(std::integral_constant<int, 0>(), PA, no(), no(), SA);
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
      const int row = my_row;
      if (my_row_valid) {
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
