// Partial instantiations of the forward kernel (gather only / compute only) for the variant the headline
// workload runs (64-row query tile, d = 128, one key per group): they let a benchmark time the two halves of
// the kernel apart on the launch shape of the full kernel.
#include "fgattn_fwd.hpp"
#include "fgattn_launch.hpp"

namespace fg {

int launch_part(const FwdArgs& a, int part, int cus, hipStream_t stream) {
  static int occ[6][64];
  if (a.M == 128) {
    constexpr int lds = fwd_lds_bytes<128, 128, NMODE_N1>();
    if (part == PART_GATHER)
      return launch_variant(fgattn_fwd_kernel<128, 128, NMODE_N1, 2, PART_GATHER>, lds, a, cus, stream, nullptr, occ[2]);
    return launch_variant(fgattn_fwd_kernel<128, 128, NMODE_N1, 2, PART_COMPUTE>, lds, a, cus, stream, nullptr, occ[3]);
  }
  constexpr int lds = fwd_lds_bytes<64, 128, NMODE_N1>();
  if (part == 3)   // gathers only, K ring of three tiles, V ring of two: 80 KiB of LDS per workgroup, still two per compute unit
    return launch_variant(fgattn_fwd_kernel<64, 128, NMODE_N1, 2, PART_GATHER, false, 3, 2>,
                          fwd_lds_bytes<64, 128, NMODE_N1, false, 3, 2>(), a, cus, stream, nullptr, occ[4]);
  if (part == 4)   // gathers only, one workgroup per compute unit (four issuing waves instead of eight)
    return launch_variant(fgattn_fwd_kernel<64, 128, NMODE_N1, 2, PART_GATHER>, lds, a, cus, stream, nullptr, occ[5], 1);
  if (part == PART_GATHER)
    return launch_variant(fgattn_fwd_kernel<64, 128, NMODE_N1, 2, PART_GATHER>, lds, a, cus, stream, nullptr, occ[0]);
  return launch_variant(fgattn_fwd_kernel<64, 128, NMODE_N1, 2, PART_COMPUTE>, lds, a, cus, stream, nullptr, occ[1]);
}

}  // namespace fg
