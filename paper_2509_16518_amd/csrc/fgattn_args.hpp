// Kernel argument block shared by the host-side launcher and the forward kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fg {

struct FwdArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
  float* lse;
  const int64_t* indptr;   // null => dense: every key of [0, L) in order
  const int32_t* indices;
  const int32_t* order;    // work-item ids in processing order
  int32_t* counter;        // int32 ctrl[64]: [1] finished-workgroup count, [8 + q] head of the queue of XCD q (zeroed by the pre-pass)
  int64_t q_sb, q_sh, q_sl, k_sb, k_sh, k_sl, v_sb, v_sh, v_sl, o_sb, o_sh, o_sl;  // elements
  int32_t H, L, M, N, QB, n_items, static_assign;
  // group -> key expansion without divisions: NT = keys per LDS tile of the launched variant
  int32_t nt_div_n, nt_mod_n;
  uint32_t n_recip16;   // ceil(65536 / N), used only when N < NT
  float c_log2;      // |scale| * log2(e): exp(scale*s) == exp2(c_log2 * s')
  float scale_abs;   // |scale|
  uint32_t q_sign;   // 0x80008000 if scale < 0 (the sign is moved onto Q, exactly), else 0
  // grouped query tiles (Sec. 4.2): M is then the group's rows (128), QB the groups per slice, indptr / indices the
  // union lists; tile_rows = rows of one member tile, R = members per group
  const int32_t* group_tiles;   // [n_items * R] member tile ids inside the slice, -1 = no tile
  const uint8_t* memb;          // [nnz of the union lists] member bit masks
  int32_t tile_rows, R;
};

// Launches the forward kernel variant for (a.M, d) on `stream` with a persistent grid sized to
// the device (`cus` compute units).  If grid_only != nullptr nothing is launched and the grid
// size is stored there.  Returns an FGATTN_* code.
int launch_forward(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only);

// Gather-only (part = 1) or compute-only (part = 2) instantiation of the M = 64, d = 128, N = 1 variant.
int launch_part(const FwdArgs& a, int part, int cus, hipStream_t stream);

// Measurement aid: 16 MFMAs + 16 exponentials + `other` ordinary vector instructions per loop trip on 2 * cus workgroups
// of four waves; `out` takes 2 * cus * 256 floats.
int launch_issue_probe(int other, int iters, float* out, int cus, hipStream_t stream);

// Grouped query tiles: the 128-row variant with membership masks (d = 64 / 128; N = 1 or N > 1).
int launch_grouped(const FwdArgs& a, int d, int cus, hipStream_t stream);

// One translation unit per query-tile size keeps compile times parallel.
int launch_mt32(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only);
int launch_mt64(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only);
int launch_mt128(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only);

}  // namespace fg
