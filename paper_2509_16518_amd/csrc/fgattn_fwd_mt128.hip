// Forward-kernel instantiations for the 128-row query tile: d = 64 / 128; dense, one key per
// group, N keys per group.
#include "fgattn_fwd.hpp"
#include "fgattn_launch.hpp"

namespace fg {

static_assert(FwdCfg<128, 128>::NT == (128 <= 32 ? 128 : 128 == 64 ? 64 : 32), "host-side NT table out of date");

template <int D, int OCC>
static int launch_d(const FwdArgs& a, int cus, hipStream_t stream, int* grid_only) {
  static int occ[4][64];
  if (a.indptr == nullptr)
    return launch_variant(fgattn_fwd_kernel<128, D, NMODE_DENSE, OCC>, fwd_lds_bytes<128, D, NMODE_DENSE>(), a, cus, stream, grid_only, occ[0]);
  if (a.N == 1)
    return launch_variant(fgattn_fwd_kernel<128, D, NMODE_N1, OCC>, fwd_lds_bytes<128, D, NMODE_N1>(), a, cus, stream, grid_only, occ[1]);
  if (a.N > 0 && a.L % a.N == 0)
    return launch_variant(fgattn_fwd_kernel<128, D, NMODE_GROUPS, OCC>, fwd_lds_bytes<128, D, NMODE_GROUPS>(), a, cus, stream, grid_only, occ[2]);
  return launch_variant(fgattn_fwd_kernel<128, D, NMODE_GROUPS_SHORT, OCC>, fwd_lds_bytes<128, D, NMODE_GROUPS_SHORT>(), a, cus, stream, grid_only, occ[3]);
}

int launch_mt128(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only) {
  if (d == 64) return launch_d<64, 2>(a, cus, stream, grid_only);
  return launch_d<128, 2>(a, cus, stream, grid_only);
}

}  // namespace fg
