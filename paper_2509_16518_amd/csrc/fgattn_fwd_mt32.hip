// Forward-kernel instantiations for the 32-row query tile: d = 64 / 128; dense, one key per
// group, N keys per group.  Single-wave workgroups (32 keys per tile): see FwdCfg.
#include "fgattn_fwd.hpp"
#include "fgattn_launch.hpp"

namespace fg {

static_assert(FwdCfg<32, 128, 2, 2, 1>::NT == (32 <= 32 ? 32 : 32 == 64 ? 64 : 32), "host-side NT table out of date");

// WPS: waves per SIMD the register budget is set for.  d = 128: two (256 registers; LDS admits five waves per CU
// anyway).  d = 64 (16 KB of LDS per wave): three for the one-key-per-group variant (ten waves per CU, a few spilled
// registers) and two for the others, whose loaders need more registers -- as measured, 3-5% either way.
template <int D, int WPS_N1, int WPS>
static int launch_d(const FwdArgs& a, int cus, hipStream_t stream, int* grid_only) {
  static int occ[4][64];
  if (a.indptr == nullptr)
    return launch_variant(fgattn_fwd_kernel<32, D, NMODE_DENSE, WPS, PART_ALL, false, 2, 2, 1>,
                          fwd_lds_bytes<32, D, NMODE_DENSE, false, 2, 2, 1>(), a, cus, stream, grid_only, occ[0], 0, 64);
  if (a.N == 1)
    return launch_variant(fgattn_fwd_kernel<32, D, NMODE_N1, WPS_N1, PART_ALL, false, 2, 2, 1>,
                          fwd_lds_bytes<32, D, NMODE_N1, false, 2, 2, 1>(), a, cus, stream, grid_only, occ[1], 0, 64);
  if (a.N > 0 && a.L % a.N == 0)
    return launch_variant(fgattn_fwd_kernel<32, D, NMODE_GROUPS, WPS, PART_ALL, false, 2, 2, 1>,
                          fwd_lds_bytes<32, D, NMODE_GROUPS, false, 2, 2, 1>(), a, cus, stream, grid_only, occ[2], 0, 64);
  return launch_variant(fgattn_fwd_kernel<32, D, NMODE_GROUPS_SHORT, WPS, PART_ALL, false, 2, 2, 1>,
                        fwd_lds_bytes<32, D, NMODE_GROUPS_SHORT, false, 2, 2, 1>(), a, cus, stream, grid_only, occ[3], 0, 64);
}

int launch_mt32(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only) {
  if (d == 64) return launch_d<64, 3, 2>(a, cus, stream, grid_only);
  return launch_d<128, 2, 2>(a, cus, stream, grid_only);
}

}  // namespace fg
