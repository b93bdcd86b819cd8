// Host-side launcher template: occupancy-sized persistent grid, opt-in to large dynamic LDS.
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>

#include "fgattn.h"
#include "fgattn_args.hpp"

namespace fg {

template <typename Kernel>
int launch_variant(Kernel kernel, int lds_bytes, const FwdArgs& a, int cus, hipStream_t stream, int* grid_only,
                   int* occ_cache, int wgs_per_cu_cap = 0, int threads = 256) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FGATTN_E_DEVICE;
  static std::mutex cache_mutex;   // one per kernel variant: first calls from several host threads take turns
  std::unique_lock<std::mutex> lock(cache_mutex);
  if (occ_cache[dev] == 0) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds_bytes) != hipSuccess)
      return FGATTN_E_DEVICE;
    int occ = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, threads, lds_bytes) != hipSuccess || occ < 1)
      return FGATTN_E_DEVICE;
    occ_cache[dev] = occ;
  }
  long long want = (long long)cus * (wgs_per_cu_cap > 0 && wgs_per_cu_cap < occ_cache[dev] ? wgs_per_cu_cap : occ_cache[dev]);
  lock.unlock();
  int grid = (int)(a.n_items < want ? a.n_items : want);
  if (grid < 1) grid = 1;
  if (grid_only) {
    *grid_only = grid;
    return FGATTN_OK;
  }
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds_bytes, stream, a);
  return hipGetLastError() == hipSuccess ? FGATTN_OK : FGATTN_E_DEVICE;
}

}  // namespace fg
