// Forward-kernel instantiations for grouped query tiles (paper Sec. 4.2): 128 query rows per work item made of
// R member tiles that share one gathered key list and keep their own masks.
#include "fgattn_fwd.hpp"
#include "fgattn_launch.hpp"

namespace fg {

template <int D>
static int launch_d(const FwdArgs& a, int cus, hipStream_t stream) {
  static int occ[2][64];
  if (a.N == 1)
    return launch_variant(fgattn_fwd_kernel<128, D, NMODE_N1, 2, PART_ALL, true>, fwd_lds_bytes<128, D, NMODE_N1, true>(), a, cus, stream, nullptr, occ[0]);
  return launch_variant(fgattn_fwd_kernel<128, D, NMODE_GROUPS_SHORT, 2, PART_ALL, true>, fwd_lds_bytes<128, D, NMODE_GROUPS_SHORT, true>(), a, cus, stream, nullptr, occ[1]);
}

int launch_grouped(const FwdArgs& a, int d, int cus, hipStream_t stream) {
  if (d == 64) return launch_d<64>(a, cus, stream);
  return launch_d<128>(a, cus, stream);
}

}  // namespace fg
