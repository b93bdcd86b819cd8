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

// Issue-port probe: what a SIMD sustains on the forward kernel's instruction mix alone -- per 32x32x16 MFMA one
// exponential and OTHER / 16 ordinary vector instructions (OTHER = 0: the MFMAs alone), independent accumulators, no
// memory traffic, no barriers --
// with the forward kernel's occupancy (two 4-wave workgroups per compute unit, enforced by the LDS request).  The
// compute half of the kernel cannot run faster than this on the same mix.
template <int OTHER>
__global__ void __launch_bounds__(256, 2) issue_probe_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    a[i] = (__bf16)(float)(threadIdx.x % 3);
    b[i] = (__bf16)1.0f;
  }
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) c[j][r] = 0.0f;
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; i++) x[i] = threadIdx.x * 1e-3f + i * 0.125f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int m = 0; m < 16; m++) {
      c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[m & 3], 0, 0, 0);
      if constexpr (OTHER >= 16) {   // (the multiply-add that forms the exponent is one of the OTHER)
        x[m & 7] = __builtin_amdgcn_exp2f(x[m & 7] * 0.25f - 4.0f);
#pragma unroll
        for (int j = (m * (OTHER - 16)) / 16; j < ((m + 1) * (OTHER - 16)) / 16; j++)
          x[(j + 1) & 7] = __builtin_fmaf(x[(j + 1) & 7], 0.999f, 0.001f);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = c[0][0] + c[1][3] + c[2][5] + c[3][7];
#pragma unroll
  for (int i = 0; i < 8; i++) s += x[i];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

int launch_issue_probe(int other, int iters, float* out, int cus, hipStream_t stream) {
  const int grid = 2 * cus;
  auto go = [&](auto kernel) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess)
      return FGATTN_E_DEVICE;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 65536, stream, out, iters);
    return hipGetLastError() == hipSuccess ? FGATTN_OK : FGATTN_E_DEVICE;
  };
  if (other == 59) return go(issue_probe_kernel<59>);
  if (other == 61) return go(issue_probe_kernel<61>);
  if (other == 67) return go(issue_probe_kernel<67>);
  if (other == 0) return go(issue_probe_kernel<0>);
  return FGATTN_E_FLAGS;
}

}  // namespace fg
