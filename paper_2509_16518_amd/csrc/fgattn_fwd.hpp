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
// contraction and a share of the previous tile's exponentials; the row max and the base decision
// follow in a short vector-ALU phase.  Work items are fetched from per-XCD device-side queues in the
// order a pre-pass wrote (Sec. 4.2 "Load balancing", Appendix B).
//
// Transposed formulation: scores are produced as S^T (keys x queries) so that, in the MFMA
// accumulator layout, one lane owns one query column.  Row statistics (max, sum) are then
// per-lane scalars plus one exchange between lanes l and l^32, and the probabilities are
// already laid out as the B operand of the second MFMA: P never moves between lanes.
//
// Every wave owns a 32-query x 32-key piece of each tile.  A workgroup of WV waves covers MT = 32, 64 or
// 128 query rows with RW = MT/32 waves along the rows and KW = WV/RW waves along the keys of a
// tile (NT = 32*KW keys); waves that split the keys keep private (max, sum, O) and merge once
// per work item.  WV is 4 except for the 32-row tile, which runs as single-wave workgroups: a wave's K and V
// slots take 32 KB at d = 128, so LDS admits five waves per compute unit, and five independent workgroups use
// them all (a four-wave workgroup would leave it at four).
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
// A run of up to four 1 KiB loads lands back to back in LDS: M0 is written once
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

// (three-input maximum, written so that the compiler selects v_max3_f32.  Not inline assembly: the compiler does not
// insert the wait states an MFMA result needs before a vector instruction reads it when that instruction is hidden
// in an asm statement)
__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
__device__ __forceinline__ float lane_pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr float kLazyLog2 = 8.0f;   // how far (log2 units) the exponent base may lag behind the running max

constexpr int cmin(int a, int b) { return a < b ? a : b; }
constexpr int cgcd(int a, int b) { return b == 0 ? a : cgcd(b, a % b); }
constexpr int clcm(int a, int b) { return a / cgcd(a, b) * b; }

// Tiling and LDS ring of one workgroup.  KS / VS = slots of the K ring / V ring (tiles of NT keys): in iteration t the
// workgroup reads K(t+1) and V(t-1) and gathers K(t+KS) and V(t+VS-2) into the slots that the previous iteration
// released, so KS-1 K tiles and VS-1 V tiles can be in flight.  The forward pass is instantiated with two slots each
// (deeper rings make the gather half alone faster -- a third K slot by 8% -- but not the whole kernel); the
// measurement aid also builds the gather half with a K ring of three.  WV = waves of a workgroup.
template <int MT, int D, int KS = 2, int VS = 2, int WV = 4>
struct FwdCfg {
  static constexpr int RW = MT / 32;            // waves along query rows (32 rows each)
  static constexpr int KW = WV / RW;            // waves along keys within a tile (32 keys each)
  static constexpr int NT = 32 * KW;            // keys per LDS tile
  static constexpr int CH = D / 8;              // 16-byte chunks per row
  static constexpr int ROWB = D * 2;            // bytes per K or V row
  static constexpr int RPI = 64 / CH;           // rows fetched by one wave-wide 16 B/lane load
  static constexpr int RPW = NT / WV;           // rows of a tile each wave fetches
  static constexpr int IPW = RPW / RPI;         // load instructions per wave, per tile, per tensor
  static constexpr int SSTEPS = D / 16;         // MFMA steps along d for S^T
  static constexpr int DBLK = D / 32;           // 32-row blocks of O^T
  static constexpr int TENSOR_BYTES = NT * ROWB;
  static constexpr int K_OFF = 0;
  static constexpr int V_OFF = KS * TENSOR_BYTES;
  static constexpr int RING_BYTES = (KS + VS) * TENSOR_BYTES;
  static constexpr int BIAS_OFF = RING_BYTES;   // (variants with a per-key bias row only)
  static constexpr int MERGE_REGS = DBLK * 16 + 2;
  static constexpr int MERGE_BYTES = (KW - 1) * RW * MERGE_REGS * 256;
  static constexpr int ITEM_OFF = RING_BYTES - 16;   // the work-item id is handed to the waves through the ring's last bytes
  static constexpr int LDS_BYTES_BIAS = BIAS_OFF + 2 * NT * 4 + 16;
  static constexpr int NKEYSETS = KS - VS + 3;  // key-row sets alive at once: tiles t+VS-2 (V gather) .. t+KS (K gather)
  static_assert(MT == 32 || MT == 64 || MT == 128, "query tile");
  static_assert(WV >= RW && WV % RW == 0 && (WV == 1 || WV == 2 || WV == 4), "waves of a workgroup");
  static_assert(D == 64 || D == 128, "head dim");
  static_assert(KS >= 2 && VS >= 2 && KS >= VS, "ring depths");
  static_assert(IPW >= 1 && RPW % RPI == 0 && (RPW & (RPW - 1)) == 0, "loader shape");
  static_assert(MERGE_BYTES <= ITEM_OFF, "merge scratch must fit in the tile buffers, below the work-item word");
};

// Online softmax of one 32-key x 32-query score block held as an MFMA accumulator: one query per
// lane (registers 8c..8c+7 of the accumulator are the keys 16c + 8*(e/4) + 4*(lane/32) + e%4).
// First half: mask padded keys, new running max of this lane's query.
// MASK_ROW: a row in LDS says which keys to mask out -- bias 0 for a real key and -inf for a padded / out-of-range
//   one, or, with member >= 0 (grouped query tiles), per key the bit mask of the group members that selected it (a
//   query of member MEMBER keeps only the keys whose bit is set).
// MASK_TAIL: only the tile's trailing positions are masked: accumulator row r of this lane is valid iff r < limit.
enum { MASK_NONE = 0, MASK_ROW = 1, MASK_TAIL = 2 };
template <int MASK>
__device__ __forceinline__ void softmax_max(f32x16& S, const float* bias_keys, int g, float m_run, float& m_new,
                                            int member = -1, int limit = 0) {
  if (MASK == MASK_ROW && member >= 0) {
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      i32x4 bv = *reinterpret_cast<const i32x4*>(bias_keys + 8 * r4 + 4 * g);
#pragma unroll
      for (int e = 0; e < 4; e++) S[4 * r4 + e] = ((bv[e] >> member) & 1) ? S[4 * r4 + e] : -INFINITY;
    }
  } else if (MASK == MASK_ROW) {
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      f32x4 bv = *reinterpret_cast<const f32x4*>(bias_keys + 8 * r4 + 4 * g);
#pragma unroll
      for (int e = 0; e < 4; e++) S[4 * r4 + e] = bv[e] < 0.0f ? -INFINITY : S[4 * r4 + e];
    }
  } else if (MASK == MASK_TAIL) {
    // register 4*r4 + e holds key row 8*r4 + 4*g + e of the wave's 32 keys; `limit` already has the 4*g taken off
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
      for (int e = 0; e < 4; e++) S[4 * r4 + e] = (8 * r4 + e) < limit ? S[4 * r4 + e] : -INFINITY;
  }
  // 16 scores -> 1 in eight three-input maxima, three levels deep (this phase is a serial dependency of the key loop)
  const float t0 = max3(S[0], S[1], S[2]), t1 = max3(S[3], S[4], S[5]), t2 = max3(S[6], S[7], S[8]);
  const float t3 = max3(S[9], S[10], S[11]), t4 = max3(S[12], S[13], S[14]);
  const float mx = fmaxf(max3(t0, t1, t2), max3(t3, t4, S[15]));
  // lanes l and l^32 hold the two halves of one query's key set
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
  m_new = max3(__uint_as_float(r[0]), __uint_as_float(r[1]), m_run);
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

// Which variants keep a per-key row in LDS (bias / membership): a short last key group and grouped query tiles.
// The others mask the ragged end of a list by position.
constexpr bool variant_has_mask_row(int nmode, bool grouped) {
  return grouped || nmode == NMODE_GROUPS_SHORT;
}
template <int MT, int D, int NMODE, bool GROUPED = false, int KS = 2, int VS = 2, int WV = 4>
constexpr int fwd_lds_bytes() {
  using C = FwdCfg<MT, D, KS, VS, WV>;
  return variant_has_mask_row(NMODE, GROUPED) ? C::LDS_BYTES_BIAS : C::RING_BYTES;
}

// id loads of the variants without a mask row: plain per-lane loads written as inline assembly so that the compiler
// does not track them.  (A tracked load makes the compiler wait with vmcnt(0) before the first use, which would also
// wait for every gather in flight: the counter is shared and the compiler cannot see the gathers.)  The kernel waits
// with the s_waitcnt that precedes each tile's barrier (wait_vmem_le(loaded) ties the register to that wait for the compiler);
// consumers clamp what they read to [0, L), so even a register read too early could never address out of bounds.
__device__ __forceinline__ void load_id_untracked(int& dst, const int32_t* base, unsigned byte_off) {
  // (scalar base + 32-bit per-lane offset: no 64-bit address arithmetic on the vector ALU)
  base = static_cast<const int32_t*>(pin_scalar(base));
  asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(byte_off), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmem_le() {   // s_waitcnt vmcnt(N): at most N vector-memory loads still in flight
  static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}
template <int N>
__device__ __forceinline__ void wait_vmem_le(int& loaded) {   // the same, and `loaded` (an untracked load's target) is valid after it
  static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(loaded) : "n"(N) : "memory");
}

// GROUPED (paper Sec. 4.2): a work item is a GROUP of query tiles (a.tile_rows rows each, R = MT / tile_rows of
// them, listed in a.group_tiles) that shares one gathered key list -- the union of the members' lists -- while
// every member attends only to its own key blocks: a.memb holds, per entry of the union list, the bit mask of the
// members that selected it, and scores of the others are set to -inf before the softmax.
template <int MT, int D, int NMODE, int OCC, int PART = PART_ALL, bool GROUPED = false, int KS = 2, int VS = 2, int WV = 4>
__global__ void __launch_bounds__(WV * 64, OCC) fgattn_fwd_kernel(const FwdArgs a) {
  using C = FwdCfg<MT, D, KS, VS, WV>;
  constexpr bool DENSE = NMODE == NMODE_DENSE;
  constexpr bool WAVE_PRIO = NMODE == NMODE_DENSE || NMODE == NMODE_N1;
  constexpr bool MASK_ROWS = variant_has_mask_row(NMODE, GROUPED);   // per-key bias / membership row in LDS
  constexpr bool ASM_IDS = NMODE == NMODE_N1 && !GROUPED;            // ids through untracked loads
  // ... whose cross-lane permute is issued before the barrier that precedes its use (measured on one box: 2.4% faster
  // at 128 query rows, 2.5% slower at 64 -- also when the ids are requested an iteration earlier, so that the wait
  // for them at the end of an iteration is free)
  constexpr bool EARLY_PERMUTE = ASM_IDS && MT == 128;
  static_assert(!GROUPED || (MT == 128 && (NMODE == NMODE_N1 || NMODE == NMODE_GROUPS_SHORT)),
                "groups are 128 query rows with a sparse list (any L: the variant that masks positions past the end)");
  static_assert(!MASK_ROWS || (KS == 2 && VS == 2), "the mask row is a two-slot ring and its id loads are tracked");
  // vector-memory operations per iteration and wave, in program order: [ids (ASM_IDS)] [V gathers] [K gathers]
  constexpr int PER = 2 * C::IPW + (ASM_IDS ? 1 : 0);
  // What may still be in flight at the barrier that opens iteration t+1: everything issued after V(t) (gathered in
  // iteration t+2-VS, first in its iteration) and after K(t+2) (gathered in iteration t+2-KS, last in its iteration)
  constexpr int WAITN = cmin(C::IPW + (VS - 2) * PER, (KS - 2) * PER);
  // ids are requested IDL iterations before they are turned into key rows; by then at least WAITN operations must
  // have followed them (the smallest such lead, rounded up to a power of two to keep the unrolled loop short)
  constexpr int IDL_MIN = ASM_IDS ? (WAITN <= 2 * C::IPW ? 1 : 1 + (WAITN - 2 * C::IPW + PER - 1) / PER) : 1;
  constexpr int IDL = IDL_MIN <= 1 ? 1 : IDL_MIN <= 2 ? 2 : 4;
  static_assert(IDL_MIN <= 4, "id lead");
  constexpr int AFTER_IDS = 2 * C::IPW + (IDL - 1) * PER;   // operations issued after an id load by the end of the iteration before its use
  static_assert(!ASM_IDS || (AFTER_IDS >= WAITN && AFTER_IDS <= 63), "id wait");
  constexpr int U = clcm(clcm(KS, VS), clcm(2, IDL));   // iterations per unrolled loop body: every slot is an immediate
  static_assert(U <= 12, "unroll");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

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
  int* masked_tile = reinterpret_cast<int*>(smem + C::BIAS_OFF + 2 * C::NT * 4);
  volatile int* s_item = reinterpret_cast<volatile int*>(smem + C::ITEM_OFF);
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
  // the XCD this workgroup runs on (hardware register XCC_ID, bits 3:0) picks its home queue
  const int my_xcd = __builtin_amdgcn_s_getreg((4 - 1) << 11 | 0 << 6 | 20) & 7;
  int queues_left = 8;
  for (;;) {
    // ---------------- fetch the next work item ----------------
    if (a.static_assign) {
      int j = blockIdx.x + iter * gridDim.x;
      if (tid == 0) *s_item = j < a.n_items ? a.order[j] : -1;
    } else {
      // One queue per XCD (each XCD has its own L2): queue q holds the work of a contiguous eighth of the (batch, head)
      // slices, in the order the pre-pass wrote, so that a head's K/V streams through one L2 instead of eight.  A
      // workgroup drains the queue of the XCD it runs on, then moves on to the next ones and helps there; a queue once
      // found empty stays empty, so `queues_left` only counts down.
      if (tid == 0) {
        int item = -1;
        const int slices = a.n_items / a.QB;
        while (queues_left > 0) {
          const int q = (my_xcd + 8 - queues_left) & 7;
          const int s0 = (q * slices) >> 3, s1 = ((q + 1) * slices) >> 3;
          const int len = (s1 - s0) * a.QB;
          if (len > 0) {
            const int j = atomicAdd(a.counter + 8 + q, 1);
            if (j < len) {
              item = a.order[s0 * a.QB + j];
              break;
            }
          }
          queues_left--;
        }
        *s_item = item;
      }
    }
    iter++;
    __syncthreads();
    const int w = __builtin_amdgcn_readfirstlane(*s_item);
    __syncthreads();   // the word lies inside the tile ring: every wave has read it before any gather may land there
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
    // (wave-uniform; pinned to scalar registers here, an item's set-up ahead of the first id load that uses it as its base)
    const int32_t* idx = DENSE ? nullptr : static_cast<const int32_t*>(pin_scalar(a.indices + beg));
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
    //   iteration T-KS-IDL: group ids requested     iteration T-KS : ids -> key rows, K(T) gathered
    //   iteration T-1     : S(T) = K(T) Q^T, row max iteration T-VS+2: V(T) gathered
    //   iteration T       : P(T) = exp(S(T) - m)     iteration T+1  : O += V(T)^T P(T)^T
    // Past the end of the list the pipeline keeps running on the last tile again (clamped tile index): a few
    // redundant, in-bounds gathers per work item instead of existence checks in every iteration.
    int gi[C::IPW];       // group ids being fetched (next tile to convert)
    int gm[C::IPW];       // GROUPED: their membership masks
    int wi[C::IPW];       // offset of the key inside its group (NMODE_GROUPS)
    int widx[IDL];        // coalesced id fetch: lane j holds the id of row j % RPW of this wave's rows; tile T in widx[T % IDL]
    // key rows of tiles t+VS-2 .. t+KS in iteration t (set 0 feeds the V gathers, the last set the K gathers)
    int keys[C::NKEYSETS][C::IPW];
    constexpr int KNEW = C::NKEYSETS - 1;
    int tq = 0, tr = 0;   // (T*NT) / N and (T*NT) % N for the next tile to fetch ids for, advanced without divisions
    const int lpos = wv * C::RPW + lrow;
    const unsigned id_lane4 = (unsigned)(wv * C::RPW + (lane & (C::RPW - 1))) * 4u;   // byte offset of this lane's id inside a tile's ids
    const int last = ntiles - 1;
    const uint8_t* memb = GROUPED ? a.memb + beg : nullptr;
    // a tile whose positions need checking: short last group, ragged last tile, or (GROUPED) always, since the mask
    // row then carries the membership masks
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
    auto coalesced_ids = [&](int T) { return NMODE == NMODE_N1 && (ASM_IDS || !tile_needs_check(T)); };
    auto fetch_ids = [&](int T, int& wdst) {
      if (NMODE == NMODE_DENSE) return;
      if constexpr (ASM_IDS) {
        // (the position is clamped into the list: a ragged last tile masks what lies past the end by position)
        load_id_untracked(wdst, idx, min((unsigned)(T * C::NT * 4) + id_lane4, (unsigned)(cnt - 1) * 4u));
        return;
      }
      if (__builtin_expect(coalesced_ids(T), 1)) {
        wdst = idx[T * C::NT + wv * C::RPW + (lane & (C::RPW - 1))];
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
    // Variants without a mask row turn ids into key rows in two steps, so that the cross-lane permute of the first has
    // the gather phase's first slots to complete before the second consumes it:
    //   keys_begin: ids of tile T (in wsrc) -> this lane's raw ids (one key per group: a permute is issued, nothing waits);
    //   keys_finish: raw ids -> key rows, clamped into the K/V slice; positions past the end of the list read the
    //   item's first active row (their scores are masked out by position).
    auto keys_begin = [&](int T, int wsrc, int (&kdst)[C::IPW]) {
#pragma unroll
      for (int i = 0; i < C::IPW; i++) {
        if constexpr (DENSE) kdst[i] = T * C::NT + lpos + i * C::RPI;
        else if constexpr (NMODE == NMODE_N1) kdst[i] = __builtin_amdgcn_ds_bpermute((i * C::RPI + lrow) << 2, wsrc);
        else kdst[i] = (int)__umul24((unsigned)gi[i], (unsigned)N) + wi[i];   // (group id and N are below 2^24, and so is their product)
      }
    };
    auto keys_finish = [&](int T, int (&kdst)[C::IPW]) {
      if constexpr (!DENSE) {   // clamped: whatever the register held, the gather stays inside the K/V slice
#pragma unroll
        for (int i = 0; i < C::IPW; i++) kdst[i] = (int)min((unsigned)kdst[i], (unsigned)(a.L - 1));
      }
      if (__builtin_expect(tile_needs_check(T), 0)) {
#pragma unroll
        for (int i = 0; i < C::IPW; i++) kdst[i] = T * C::NT + lpos + i * C::RPI < total ? kdst[i] : pad_key;
      }
    };
    // ids of tile T (fetched earlier, in wsrc) -> key rows in kdst; padded / out-of-range positions of a checked tile
    // read the item's first active row and have their scores masked out
    auto make_keys = [&](int T, int wsrc, int (&kdst)[C::IPW]) {
      if constexpr (!MASK_ROWS) {
        keys_begin(T, wsrc, kdst);
        keys_finish(T, kdst);
        return;
      }
      if (NMODE == NMODE_N1 && __builtin_expect(coalesced_ids(T), 1)) {
#pragma unroll
        for (int i = 0; i < C::IPW; i++) kdst[i] = __builtin_amdgcn_ds_bpermute((i * C::RPI + lrow) << 2, wsrc);
        return;
      }
      const bool checked = tile_needs_check(T);
      if constexpr (!LAZY_BIAS) {
        // a checked tile writes its whole row (GROUPED: the membership masks, every tile)
#pragma unroll
        for (int i = 0; i < C::IPW; i++) {
          const int p = T * C::NT + lpos + i * C::RPI;
          // (group id and N are below 2^24 and so is their product, a key row)
          int key = NMODE == NMODE_N1 ? gi[i] : (int)__umul24((unsigned)gi[i], (unsigned)N) + wi[i];
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
          kdst[i] = key;
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
        kdst[i] = ok[i] ? key : pad_key;
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
    // LDS: K ring slots 0..KS-1 then V ring slots 0..VS-1, TENSOR_BYTES each.  A run of up to four gathers of one
    // wave lands back to back, so only the first writes M0 and the others use the instruction offset (which also
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
    auto gather_k = [&](auto ic, int slot, const int (&kk)[C::IPW]) {
      constexpr int i = decltype(ic)::value;
      if constexpr (PART == PART_COMPUTE) return;
      const unsigned off = __umul24((unsigned)kk[i], k_rowb) + kcon[i];
      if constexpr ((i & 3) == 0)
        gather16_first(kbase_m4k, off, lds0 + C::K_OFF + slot * C::TENSOR_BYTES + (wv * C::RPW + i * C::RPI) * C::ROWB);
      else
        gather16_next<(i & 3)>(kbase_m4k, off);
    };
    auto gather_v = [&](auto ic, int slot, const int (&kk)[C::IPW]) {
      constexpr int i = decltype(ic)::value;
      if constexpr (PART == PART_COMPUTE) return;
      const unsigned off = __umul24((unsigned)kk[i], v_rowb) + vcon[i];
      if constexpr ((i & 3) == 0)
        gather16_first(vbase_m4k, off, lds0 + C::V_OFF + slot * C::TENSOR_BYTES + (wv * C::RPW + i * C::RPI) * C::ROWB);
      else
        gather16_next<(i & 3)>(vbase_m4k, off);
    };
    // all of one tile's K (or V) gathers of this wave, back to back (prologue)
    auto burst_k = [&](int slot, const int (&kk)[C::IPW]) {
      gather_k(std::integral_constant<int, 0>(), slot, kk);
      if constexpr (C::IPW > 1) gather_k(std::integral_constant<int, 1>(), slot, kk);
      if constexpr (C::IPW > 2) { gather_k(std::integral_constant<int, 2>(), slot, kk); gather_k(std::integral_constant<int, 3>(), slot, kk); }
      if constexpr (C::IPW > 4) {
        gather_k(std::integral_constant<int, 4>(), slot, kk); gather_k(std::integral_constant<int, 5>(), slot, kk);
        gather_k(std::integral_constant<int, 6>(), slot, kk); gather_k(std::integral_constant<int, 7>(), slot, kk);
      }
    };
    auto burst_v = [&](int slot, const int (&kk)[C::IPW]) {
      gather_v(std::integral_constant<int, 0>(), slot, kk);
      if constexpr (C::IPW > 1) gather_v(std::integral_constant<int, 1>(), slot, kk);
      if constexpr (C::IPW > 2) { gather_v(std::integral_constant<int, 2>(), slot, kk); gather_v(std::integral_constant<int, 3>(), slot, kk); }
      if constexpr (C::IPW > 4) {
        gather_v(std::integral_constant<int, 4>(), slot, kk); gather_v(std::integral_constant<int, 5>(), slot, kk);
        gather_v(std::integral_constant<int, 6>(), slot, kk); gather_v(std::integral_constant<int, 7>(), slot, kk);
      }
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
    float l_run = 0.0f, l_run2 = 0.0f;   // this lane's partial sum of exponentials, in two chains (even / odd scores)
    // derived from the exponent base whenever it moves (set_base), so that the key loop computes neither per tile:
    float neg_mc = 0.0f;           // -m_run * c_log2, 0 while m_run is -inf: the additive term of the exponent
    float m_move = -INFINITY;      // a running max above this moves the base: m_run + kLazyLog2 / c_log2 (-inf while m_run is)
    const float lazy_raw = kLazyLog2 / a.c_log2;
    auto set_base = [&](float m) {
      const bool none = m == -INFINITY;   // no valid key seen yet
      m_run = m;
      neg_mc = none ? 0.0f : -m * a.c_log2;
      m_move = none ? -INFINITY : m + lazy_raw;
    };
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
    // Phase X.  O^T += V^T P^T with V in slot `vrd` of the V ring and, with QK, Sn = K Q^T with K in slot `krd` of the K
    // ring: one MFMA of each per slot.  With EXP, every slot also takes its share of the exponentials of the previous
    // tile's scores So: P = exp2(c*(So - m)) packed to bf16 into Pout, and the row sum; they issue while the two matrix
    // instructions just issued execute.  With GATHER, every slot then issues one of this iteration's gathers: V rows
    // (keys in key set 0) -> V slot `vwr`, then K rows (keys in the newest key set) -> K slot `kwr`, both released by
    // the previous iteration.  The gather holds the wave; the matrix instructions execute underneath it.
    auto x_phase = [&](auto vrd_c, auto krd_c, auto vwr_c, auto kwr_c, const i32x4 (&Pin)[2], auto with_gather,
                       auto with_qk, f32x16& Sn, auto with_exp, const f32x16& So, i32x4 (&Pout)[2]) {
      constexpr int vrd = decltype(vrd_c)::value, krd = decltype(krd_c)::value;
      constexpr int vwr = decltype(vwr_c)::value, kwr = decltype(kwr_c)::value;
      constexpr bool GATHER = decltype(with_gather)::value;
      constexpr bool QK = decltype(with_qk)::value && PART != PART_GATHER;   // also Sn = K(slot krd) Q^T
      constexpr bool EXP = decltype(with_exp)::value && PART != PART_GATHER;  // also P = exp2(c*(So - m)) -> Pout, row sum
      const unsigned char* vst = smem + C::V_OFF + vrd * C::TENSOR_BYTES;
      const unsigned char* kst = smem + C::K_OFF + krd * C::TENSOR_BYTES;
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
        if constexpr (EXP) {
#pragma unroll
          for (int x = 0; x < VPS; x += 2) {
            const int r = e * VPS + x;
            // masked keys hold S = -inf and c_log2 > 0 (the host substitutes a tiny positive value for
            // scale = 0), so their p is exactly 0 without a select
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(So[r], a.c_log2, neg_mc));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(So[r + 1], a.c_log2, neg_mc));
            l_run += p0;
            l_run2 += p1;
            f32x2 pp = {p0, p1};
            int pk = __builtin_bit_cast(int, __builtin_convertvector(pp, bf16x2));
            asm volatile("" : "+v"(pk));   // keeps the compiler from sinking the conversion out of the slot
            Pout[r >> 3][(r & 7) >> 1] = pk;
          }
        }
        if constexpr (GATHER) {
          if constexpr (e % DMA_EVERY == 0) {
            constexpr int j0 = (e / DMA_EVERY) * DMA_PER;
            if constexpr (j0 < C::IPW) gather_v(std::integral_constant<int, j0>(), vwr, keys[0]);
            else if constexpr (j0 < NDMA) gather_k(std::integral_constant<int, j0 - C::IPW>(), kwr, keys[KNEW]);
            if constexpr (DMA_PER > 1) {
              constexpr int j1 = j0 + 1;
              if constexpr (j1 < C::IPW) gather_v(std::integral_constant<int, j1>(), vwr, keys[0]);
              else if constexpr (j1 < NDMA) gather_k(std::integral_constant<int, j1 - C::IPW>(), kwr, keys[KNEW]);
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
    // Phase Y, vector ALU only in the key loop: the row max of the new scores Sn (tile Tm) and the rare decision to
    // move the exponent base (see kLazyLog2).  With MFMA (prologue only) it first computes Sn = K Q^T with K in slot
    // `kslot` of the K ring.
    auto y_phase = [&](auto kslot, int Tm, f32x16& Sn, auto with_mfma) {
      constexpr bool MFMA = decltype(with_mfma)::value;
      // written before the barrier that precedes this phase; consumed at its end
      const int masked_entry = LAZY_BIAS ? masked_tile[Tm & 1] : 0;
      if constexpr (PART == PART_GATHER) return;
      if constexpr (MFMA) {
        const unsigned char* kst = smem + C::K_OFF + kslot * C::TENSOR_BYTES;
        auto read_kf = [&](int s) {
          return __builtin_bit_cast(bf16x8, *reinterpret_cast<const i32x4*>(kst + (kor ^ (32 * s))));
        };
        bf16x8 kf[NE];
#pragma unroll
        for (int e = 0; e < AHEAD; e++) kf[e] = read_kf(e);
#pragma unroll
        for (int r = 0; r < 16; r++) Sn[r] = 0.0f;
#pragma unroll
        for (int e = 0; e < NE; e++) {
          if (e + AHEAD < NE) kf[e + AHEAD] = read_kf(e + AHEAD);
          Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[e], qf[e], Sn, 0, 0, 0);
        }
      }
      float m_new;
      // (the same in every wave of the workgroup)
      const bool masked = LAZY_BIAS ? tile_has_masked_keys(Tm, masked_entry) : tile_needs_check(Tm);
      if (__builtin_expect(masked, 0)) {
        if constexpr (MASK_ROWS)
          softmax_max<MASK_ROW>(Sn, bias + (Tm & 1) * C::NT + kw * 32, g, m_pend, m_new, GROUPED ? my_member : -1);
        else   // positions of the tile at and past `total` are padding
          softmax_max<MASK_TAIL>(Sn, nullptr, g, m_pend, m_new, -1, total - Tm * C::NT - kw * 32 - 4 * g);
      } else {
        softmax_max<MASK_NONE>(Sn, nullptr, g, m_pend, m_new);
      }
      if constexpr (LAZY_BIAS) slot_dirty[Tm & 1] |= masked;
      m_pend = m_new;
      const bool lane_moves = m_new > m_move;   // (the first valid key of a lane also moves it: m_move = -inf until then)
      resc = __builtin_amdgcn_ballot_w64(lane_moves) != 0;
    };
    auto rotate_keys = [&]() {
#pragma unroll
      for (int s = 0; s + 1 < C::NKEYSETS; s++)
#pragma unroll
        for (int i = 0; i < C::IPW; i++) keys[s][i] = keys[s + 1][i];
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    // Iteration t, J = t mod U (a constant, so every LDS slot and register set is an immediate):
    //   X: O += V(t-1)^T P(t-1)^T  ||  S(t+1) = K(t+1) Q^T  ||  P(t) = exp(S(t) - m)  ||  gathers V(t+VS-2) and K(t+KS)
    //      into the slots that iteration t-1 read last
    //   Y: the row max of S(t+1), on the vector ALU
    // A gathered tile has at least phase Y and the barrier's wait to arrive before it is published, and whole
    // iterations more where the rings are deeper than two tiles.
    auto iteration = [&](auto jc, int t) {
      constexpr int J = decltype(jc)::value;
      constexpr int PAR = J & 1;
      i32x4 (&Pin)[2] = PAR ? PA : PB;
      i32x4 (&Pout)[2] = PAR ? PB : PA;
      f32x16& Sn = PAR ? SA : SB;
      const f32x16& So = PAR ? SB : SA;
      // K(t+1) and V(t-1) become visible to every wave: all but the WAITN most recent vector-memory operations of this
      // wave have completed (they complete in order), which covers its share of both tiles and the ids converted
      // below; every wave is done reading K(t) and V(t-2), whose slots this iteration refills
      if constexpr (ASM_IDS) wait_vmem_le<WAITN>(widx[(J + KS) % IDL]);
      else wait_vmem_le<WAITN>();
      __syncthreads();
      float alpha = 1.0f;
      if (__builtin_expect(resc, 0)) {   // the exponent base moves: l now, O after the MFMAs of the old base
        alpha = (m_run == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((m_run - m_pend) * a.c_log2);
        l_run *= alpha;
        l_run2 *= alpha;
        set_base(m_pend);
      }
      // ids requested IDL iterations ago -> key rows (with untracked id loads the cross-lane permute was already
      // issued before the barrier, at the end of the previous iteration, and only its result is consumed here)
      if constexpr (EARLY_PERMUTE) keys_finish(min(t + KS, last), keys[KNEW]);
      else make_keys(min(t + KS, last), widx[(J + KS) % IDL], keys[KNEW]);
      fetch_ids(min(t + KS + IDL, last), widx[(J + KS) % IDL]);
      // wave priority: the gather phase above the vector-ALU phase above everything outside the key loop, so that
      // the waves that feed the memory pipe are issued first and a neighbour's prologue or epilogue never delays them
      // (measured: 1-3% faster with one key per group, 6% for the dense kernel at 128 rows; slower with N keys per
      // group, whose loaders do more vector-ALU work, so not used there)
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(3);
      x_phase(std::integral_constant<int, (J + U - 1) % VS>(), std::integral_constant<int, (J + 1) % KS>(),
              std::integral_constant<int, (J + U - 2) % VS>(), std::integral_constant<int, J % KS>(), Pin, yes(), yes(), Sn,
              yes(), So, Pout);
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(1);
      if (__builtin_expect(resc, 0)) {
#pragma unroll
        for (int db = 0; db < C::DBLK; db++)
#pragma unroll
          for (int r = 0; r < 16; r++) O[db][r] *= alpha;
      }
      y_phase(std::integral_constant<int, 0>(), min(t + 1, last), Sn, no());
      rotate_keys();
      if constexpr (EARLY_PERMUTE) {
        // the ids of the tile whose K rows the next iteration gathers have arrived (their load was followed by
        // AFTER_IDS operations): hand them to the lanes now, so that the permute's latency passes in the barrier
        wait_vmem_le<AFTER_IDS>(widx[(J + 1 + KS) % IDL]);
        keys_begin(min(t + 1 + KS, last), widx[(J + 1 + KS) % IDL], keys[KNEW]);
      }
    };

    if (ntiles > 0) {
      // prologue: K(0) .. K(KS-1) -> their K slots; V(0) .. V(VS-3) -> their V slots; V(0) also -> the V slot that the
      // first iteration reads as "V(-1)", only so that its O += V^T P^T (with P = 0) multiplies finite numbers; then
      // S(0) = K(0) Q^T
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int e = 0; e < 4; e++) PB[c][e] = 0;
      int wpro[KS];   // ids of tiles 0 .. KS-1 (ASM_IDS: requested together)
      if constexpr (ASM_IDS) {
#pragma unroll
        for (int T = 0; T < KS; T++) fetch_ids(min(T, last), wpro[T]);
#pragma unroll
        for (int T = 0; T < IDL; T++) fetch_ids(min(KS + T, last), widx[(KS + T) % IDL]);
#pragma unroll
        for (int T = 0; T < KS; T++) wait_vmem_le<0>(wpro[T]);
      }
      int ktmp[C::IPW];
#pragma unroll
      for (int T = 0; T < KS; T++) {
        if constexpr (!ASM_IDS) fetch_ids(min(T, last), wpro[T]);
        make_keys(min(T, last), wpro[T], ktmp);
        burst_k(T, ktmp);
        if (T == 0) {
          burst_v(VS - 1, ktmp);
#pragma unroll
          for (int s = 0; s < C::NKEYSETS; s++)
#pragma unroll
            for (int i = 0; i < C::IPW; i++) keys[s][i] = ktmp[i];
        }
        if (T <= VS - 3) burst_v(T, ktmp);
        if (T >= VS - 2) {
#pragma unroll
          for (int i = 0; i < C::IPW; i++) keys[T - (VS - 2)][i] = ktmp[i];
        }
      }
      if constexpr (!ASM_IDS) fetch_ids(min(KS, last), widx[KS % IDL]);
      else if constexpr (EARLY_PERMUTE) {
        wait_vmem_le<0>(widx[KS % IDL]);   // (arrived with the wait above; this ties the register to a wait for the compiler)
        keys_begin(min(KS, last), widx[KS % IDL], keys[KNEW]);
      }
      wait_vmem_all();
      __syncthreads();
      // S(0) from K slot 0
      y_phase(std::integral_constant<int, 0>(), 0, SA, yes());
      set_base(m_pend);   // O = 0 and l = 0 so far: the first exponent base needs no rescale
      resc = false;
      int t = 0;
      for (;;) {
#define FG_STEP(J)                                             \
        if constexpr (U > J) {                                 \
          if (t >= ntiles) break;                              \
          iteration(std::integral_constant<int, J>(), t);      \
          t++;                                                 \
        }
        FG_STEP(0) FG_STEP(1) FG_STEP(2) FG_STEP(3) FG_STEP(4) FG_STEP(5)
        FG_STEP(6) FG_STEP(7) FG_STEP(8) FG_STEP(9) FG_STEP(10) FG_STEP(11)
#undef FG_STEP
      }
      if constexpr (WAVE_PRIO) __builtin_amdgcn_s_setprio(0);
      wait_vmem_all();
      __syncthreads();
      // O += V(ntiles-1)^T P(ntiles-1)^T: the slot and the register set depend on ntiles - 1 modulo lcm(VS, 2)
      constexpr int UD = clcm(VS, 2);
      const int jd = (ntiles - 1) % UD;
#define FG_DRAIN(J)                                                                                                   \
      if constexpr (UD > J) {                                                                                          \
        if (jd == J)                                                                                                   \
          x_phase(std::integral_constant<int, J % VS>(), std::integral_constant<int, 0>(), std::integral_constant<int, 0>(), \
                  std::integral_constant<int, 0>(), (J & 1) ? PB : PA, no(), no(), SA, no(), SA, PA);                 \
      }
      FG_DRAIN(0) FG_DRAIN(1) FG_DRAIN(2) FG_DRAIN(3) FG_DRAIN(4) FG_DRAIN(5) FG_DRAIN(6) FG_DRAIN(7)
#undef FG_DRAIN
    }

    // ---------------- epilogue ----------------
    float l_tot = lane_pair_sum(l_run + l_run2);
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
    // this item's LDS use (tile rings, merge scratch) ends here; the next item's begins with the work-item word
    __syncthreads();
  }
  // The last workgroup to leave rewinds the queue, so a later launch can reuse the stored order
  // without a pre-pass.  Every workgroup reaches this point exactly once.
  if (!a.static_assign && tid == 0) {
    __threadfence();
    const int done = atomicAdd(a.counter + 1, 1);
    if (done == (int)gridDim.x - 1) {
      atomicExch(a.counter + 1, 0);
      for (int q = 0; q < 8; q++) atomicExch(a.counter + 8 + q, 0);
    }
  }
}

}  // namespace fg
