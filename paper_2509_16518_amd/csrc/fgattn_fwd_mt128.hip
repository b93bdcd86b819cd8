// Forward-kernel instantiations for the 128-row query tile (d = 64 and d = 128).
#include "fgattn_fwd.hpp"
#include "fgattn_launch.hpp"

namespace fg {

int launch_mt128(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only) {
  static int occ64[64], occ128[64];
  if (d == 64)
    return launch_variant(fgattn_fwd_kernel<128, 64, 64, 2>, FwdCfg<128, 64, 64>::LDS_BYTES, a, cus, stream, grid_only, occ64);
  return launch_variant(fgattn_fwd_kernel<128, 128, 64, 2>, FwdCfg<128, 128, 64>::LDS_BYTES, a, cus, stream, grid_only,
                        occ128);
}

}  // namespace fg
