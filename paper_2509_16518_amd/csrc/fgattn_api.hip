// C-ABI entry points of libfgattn.so (see include/fgattn.h), the ordering pre-pass and the
// mask validator.  Host code here only validates arguments and enqueues kernels.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <mutex>

#include "fgattn.h"
#include "fgattn_launch.hpp"

namespace fg {

// ------------------------------------------------------------------------------------------
// Ordering pre-pass (paper Sec. 4.2 "Load balancing", Appendix B): the cost of a work item is
// the length of its key/value list; items are handed out longest first.  Here the order is
// built per head -- all workgroups drain one head before the next, so concurrently running
// items share that head's K/V in cache -- and longest-first inside a head.
// blockIdx.x = (batch, head) slice; blockIdx.y splits the slice's query blocks when they are ranked exactly.
// workspace layout: int32 ctrl[64] (ctrl[1] finished-workgroup count, ctrl[8 + q] head of the
// queue of XCD q, which covers the q-th eighth of the slices), then int32 order[n_items].
// ------------------------------------------------------------------------------------------
constexpr int kPlanThreads = 256;
constexpr int kRankMax = 4096;     // slices with at most this many query blocks are ranked exactly
constexpr int kBuckets = 2048;     // larger slices: bucket sort on the (scaled) cost

__global__ void __launch_bounds__(kPlanThreads) plan_kernel(const int64_t* indptr, int32_t* ctrl, int32_t* order, int QB,
                                                             int sorted) {
  __shared__ int s_cost[kRankMax];
  __shared__ int s_hist[kBuckets];
  __shared__ int s_max;
  const int tid = threadIdx.x;
  const int64_t base = (int64_t)blockIdx.x * QB;
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid < 16) ctrl[tid] = 0;
  if (!sorted || indptr == nullptr) {
    if (blockIdx.y == 0)
      for (int j = tid; j < QB; j += kPlanThreads) order[base + j] = (int32_t)(base + j);
    return;
  }
  auto cost_of = [&](int j) -> int {
    int64_t c = indptr[base + j + 1] - indptr[base + j];
    return c > 0x7fffffff ? 0x7fffffff : (c < 0 ? 0 : (int)c);
  };
  if (QB <= kRankMax) {
    // exact rank by counting; blockIdx.y splits the query blocks of the slice, four lanes share one block's count
    for (int j = tid; j < QB; j += kPlanThreads) s_cost[j] = cost_of(j);
    __syncthreads();
    const int part = tid & 3;
    for (int j0 = blockIdx.y * (kPlanThreads / 4); j0 < QB; j0 += gridDim.y * (kPlanThreads / 4)) {
      const int j = j0 + (tid >> 2);
      const int c = j < QB ? s_cost[j] : 0;
      int rank = 0;
      for (int i = part; i < QB; i += 4) {
        const int ci = s_cost[i];
        rank += (ci > c) || (ci == c && i < j);
      }
      rank += __shfl_xor(rank, 1);
      rank += __shfl_xor(rank, 2);
      if (part == 0 && j < QB) order[base + rank] = (int32_t)(base + j);
    }
    return;
  }
  if (blockIdx.y != 0) return;
  // bucket path: descending buckets over [0, max cost]
  if (tid == 0) s_max = 1;
  for (int i = tid; i < kBuckets; i += kPlanThreads) s_hist[i] = 0;
  __syncthreads();
  int mx = 1;
  for (int j = tid; j < QB; j += kPlanThreads) mx = max(mx, cost_of(j));
  atomicMax(&s_max, mx);
  __syncthreads();
  const int64_t cmax = s_max;
  auto bucket_of = [&](int c) -> int { return (kBuckets - 1) - (int)(((int64_t)c * (kBuckets - 1)) / cmax); };
  for (int j = tid; j < QB; j += kPlanThreads) atomicAdd(&s_hist[bucket_of(cost_of(j))], 1);
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < kBuckets; i++) {
      int n = s_hist[i];
      s_hist[i] = run;
      run += n;
    }
  }
  __syncthreads();
  for (int j = tid; j < QB; j += kPlanThreads) {
    const int pos = atomicAdd(&s_hist[bucket_of(cost_of(j))], 1);
    order[base + pos] = (int32_t)(base + j);
  }
}

// ------------------------------------------------------------------------------------------
// Mask validator (test helper): one workgroup per work item.
// ------------------------------------------------------------------------------------------
constexpr int kValBits = 1 << 18;   // key groups checked per pass (bitmap in LDS)

__global__ void __launch_bounds__(256) validate_kernel(const int64_t* indptr, const int32_t* indices, int G, int* bad) {
  __shared__ unsigned s_bits[kValBits / 32];
  const int64_t w = blockIdx.x;
  const int tid = threadIdx.x;
  const int64_t beg = indptr[w], end = indptr[w + 1];
  if (w == 0 && tid == 0 && beg != 0) atomicOr(bad, 1);
  if (end < beg) {
    if (tid == 0) atomicOr(bad, 2);
    return;
  }
  for (int lo = 0; lo < G; lo += kValBits) {
    for (int i = tid; i < kValBits / 32; i += 256) s_bits[i] = 0;
    __syncthreads();
    for (int64_t e = beg + tid; e < end; e += 256) {
      const int gid = indices[e];
      if (gid < 0 || gid >= G) {
        atomicOr(bad, 4);
      } else if (gid >= lo && gid < lo + kValBits) {
        const unsigned bit = 1u << ((gid - lo) & 31);
        const unsigned old = atomicOr(&s_bits[(gid - lo) >> 5], bit);
        if (old & bit) atomicOr(bad, 8);
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct DeviceInfo {
  bool known = false;
  bool gfx950 = false;
  int cus = 0;
};
static DeviceInfo g_dev[64];
static std::mutex g_dev_mutex;   // first calls from several host threads fill the table one at a time

static int device_info(DeviceInfo* out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FGATTN_E_DEVICE;
  std::lock_guard<std::mutex> lock(g_dev_mutex);
  DeviceInfo& d = g_dev[dev];
  if (!d.known) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return FGATTN_E_DEVICE;
    d.gfx950 = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    d.cus = prop.multiProcessorCount;
    d.known = true;
  }
  *out = d;
  return d.gfx950 ? FGATTN_OK : FGATTN_E_DEVICE;
}

static int64_t n_items_of(const fgattn_params* p) {
  return (int64_t)p->B * p->H * (((int64_t)p->L + p->M - 1) / p->M);
}

static int check_shape(const fgattn_params* p) {
  if (p == nullptr) return FGATTN_E_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1 || p->N < 1) return FGATTN_E_SHAPE;
  if (p->d != 64 && p->d != 128) return FGATTN_E_SHAPE;
  if (p->M != 16 && p->M != 32 && p->M != 64 && p->M != 128) return FGATTN_E_SHAPE;
  if ((int64_t)p->L + p->N > 0x7fffffffLL) return FGATTN_E_SHAPE;
  if (p->L > (1 << 24)) return FGATTN_E_SHAPE;   // key row * row bytes uses 24-bit multiplies
  if (n_items_of(p) > 0x7fffffffLL) return FGATTN_E_SHAPE;
  if (p->flags & ~(FGATTN_FLAG_STATIC_ASSIGN | FGATTN_FLAG_FIFO_QUEUE | FGATTN_FLAG_REUSE_PLAN | FGATTN_FLAG_MASK_ROWS_IN_HBM |
                   FGATTN_FLAG_MASK_ONE_TILE_CHUNKS))
    return FGATTN_E_FLAGS;
  return FGATTN_OK;
}

static int check_tensors(const void* q, const void* k, const void* v, const void* out, const float* lse,
                         const fgattn_params* p) {
  if (!q || !k || !v || !out || !lse) return FGATTN_E_NULL;
  const int64_t rows[4] = {p->q_stride_l, p->k_stride_l, p->v_stride_l, p->o_stride_l};
  for (int i = 0; i < 4; i++)
    if (rows[i] < p->d || (rows[i] % 8) != 0 || rows[i] * 2 >= (1 << 24)) return FGATTN_E_STRIDE;
  const int64_t outer[8] = {p->q_stride_b, p->q_stride_h, p->k_stride_b, p->k_stride_h,
                            p->v_stride_b, p->v_stride_h, p->o_stride_b, p->o_stride_h};
  for (int i = 0; i < 8; i++)
    if (outer[i] < 0 || (outer[i] % 8) != 0) return FGATTN_E_STRIDE;
  const void* ptrs[4] = {q, k, v, out};
  for (int i = 0; i < 4; i++)
    if ((reinterpret_cast<uintptr_t>(ptrs[i]) & 15) != 0) return FGATTN_E_ALIGN;
  if ((reinterpret_cast<uintptr_t>(lse) & 3) != 0) return FGATTN_E_ALIGN;
  // the gather addresses K/V rows with 32-bit byte offsets from the (batch, head) slice base; every lane offset
  // also carries a +4096 bias (the base pointer is moved down by as much, see gather16_next), which must not wrap
  const int64_t last = (int64_t)p->L - 1;
  if (last * p->k_stride_l * 2 + 2 * p->d + 4096 > 0xffffffffLL || last * p->v_stride_l * 2 + 2 * p->d + 4096 > 0xffffffffLL)
    return FGATTN_E_STRIDE;
  if (!isfinite(p->scale)) return FGATTN_E_SCALE;
  return FGATTN_OK;
}

static int check_workspace(const fgattn_params* p, const void* workspace, size_t bytes) {
  if (!workspace) return FGATTN_E_NULL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return FGATTN_E_ALIGN;
  if (bytes < fgattn_workspace_bytes(p)) return FGATTN_E_WORKSPACE;
  return FGATTN_OK;
}

static int run_plan(const int64_t* indptr, const fgattn_params* p, void* workspace, hipStream_t stream, int QB = 0) {
  int32_t* ctrl = static_cast<int32_t*>(workspace);
  int32_t* order = ctrl + 64;
  if (QB == 0) QB = (p->L + p->M - 1) / p->M;
  const int sorted = (p->flags & (FGATTN_FLAG_STATIC_ASSIGN | FGATTN_FLAG_FIFO_QUEUE)) ? 0 : 1;
  const int splits = QB <= kRankMax ? (QB + kPlanThreads / 4 - 1) / (kPlanThreads / 4) : 1;   // 64 query blocks per workgroup
  hipLaunchKernelGGL(plan_kernel, dim3(p->B * p->H, splits < 64 ? splits : 64), dim3(kPlanThreads), 0, stream, indptr, ctrl,
                     order, QB, sorted);
  return hipGetLastError() == hipSuccess ? FGATTN_OK : FGATTN_E_DEVICE;
}

static int run_forward(const void* q, const void* k, const void* v, const int64_t* indptr, const int32_t* indices,
                       const fgattn_params* p, void* out, float* lse, void* workspace, size_t workspace_bytes,
                       void* stream_v, int part = 0, const int32_t* group_tiles = nullptr,
                       const uint8_t* group_memb = nullptr) {
  int rc = check_shape(p);
  if (rc) return rc;
  rc = check_tensors(q, k, v, out, lse, p);
  if (rc) return rc;
  rc = check_workspace(p, workspace, workspace_bytes);
  if (rc) return rc;
  DeviceInfo dev;
  rc = device_info(&dev);
  if (rc) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  const bool grouped = group_tiles != nullptr;
  const int R = grouped ? 128 / p->M : 1;                                   // member tiles per group
  const int QB_tiles = (p->L + p->M - 1) / p->M;
  const int QB_items = grouped ? (QB_tiles + R - 1) / R : QB_tiles;         // work items per (batch, head) slice
  if (!(p->flags & FGATTN_FLAG_REUSE_PLAN)) {
    rc = run_plan(indptr, p, workspace, stream, QB_items);
    if (rc) return rc;
  }
  FwdArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.indptr = indptr;
  a.indices = indices;
  a.counter = static_cast<int32_t*>(workspace);
  a.order = a.counter + 64;
  a.q_sb = p->q_stride_b; a.q_sh = p->q_stride_h; a.q_sl = p->q_stride_l;
  a.k_sb = p->k_stride_b; a.k_sh = p->k_stride_h; a.k_sl = p->k_stride_l;
  a.v_sb = p->v_stride_b; a.v_sh = p->v_stride_h; a.v_sl = p->v_stride_l;
  a.o_sb = p->o_stride_b; a.o_sh = p->o_stride_h; a.o_sl = p->o_stride_l;
  a.H = p->H;
  a.L = p->L;
  a.M = grouped ? 128 : p->M;
  a.N = indptr ? p->N : 1;
  a.group_tiles = group_tiles;
  a.memb = group_memb;
  a.tile_rows = p->M;
  a.R = R;
  const int NT = a.M <= 32 ? 32 : a.M == 64 ? 64 : 32;   // keys per LDS tile of the variant launched for M
  a.nt_div_n = NT / a.N;
  a.nt_mod_n = NT % a.N;
  a.n_recip16 = (65536u + (uint32_t)a.N - 1) / (uint32_t)a.N;
  a.QB = QB_items;
  a.n_items = (int32_t)((int64_t)p->B * p->H * QB_items);
  a.static_assign = (p->flags & FGATTN_FLAG_STATIC_ASSIGN) ? 1 : 0;
  const float sabs = fabsf(p->scale);
  // scale = 0 is run with a tiny positive exponent factor: valid keys still get p = exp2(tiny * s) = 1 exactly,
  // while masked keys (score -inf) get exactly 0 instead of exp2(-inf * 0) = NaN
  a.c_log2 = sabs * 1.44269504088896340736f;
  if (!(a.c_log2 > 1e-30f)) a.c_log2 = 1e-30f;
  a.scale_abs = sabs;
  a.q_sign = p->scale < 0.0f ? 0x80008000u : 0u;
  if (part != 0) return launch_part(a, part, dev.cus, stream);
  if (grouped) return launch_grouped(a, p->d, dev.cus, stream);
  return launch_forward(a, p->d, dev.cus, stream, nullptr);
}

// ------------------------------------------------------------------------------------------
// Fixed scratch for fgattn_forward_static: the same layout as the caller-provided workspace
// (int32 ctrl[64], then int32 order[n_items]) in the library's device image.  `scratch` is a
// host-side stand-in for the symbol, not a device address: host code uses the per-device
// address that hipGetSymbolAddress returns (each GPU holds its own copy at its own address).
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[64 + FGATTN_STATIC_MAX_ITEMS];
static void* g_scratch_ptr[64];   // per device, filled on the first call with that device current
static std::mutex g_scratch_mutex;

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return FGATTN_E_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return FGATTN_E_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FGATTN_OK;
}

}  // namespace fg

extern "C" {

size_t fgattn_workspace_bytes(const fgattn_params* p) {
  if (fg::check_shape(p) != FGATTN_OK) return 0;
  size_t bytes = 256 + sizeof(int32_t) * (size_t)fg::n_items_of(p);
  return (bytes + 255) & ~(size_t)255;
}

int fgattn_forward(const void* q, const void* k, const void* v, const int64_t* mask_indptr, const int32_t* mask_indices,
                   const fgattn_params* p, void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (!mask_indptr || !mask_indices) return FGATTN_E_NULL;
  return fg::run_forward(q, k, v, mask_indptr, mask_indices, p, out, lse, workspace, workspace_bytes, stream);
}

int fgattn_forward_static(const void* q, const void* k, const void* v, const int64_t* mask_indptr,
                          const int32_t* mask_indices, const fgattn_params* p, void* out, float* lse, void* stream) {
  if (!mask_indptr || !mask_indices) return FGATTN_E_NULL;
  int rc = fg::check_shape(p);
  if (rc) return rc;
  if (fg::n_items_of(p) > FGATTN_STATIC_MAX_ITEMS) return FGATTN_E_STATIC_LIMIT;
  rc = fg::check_tensors(q, k, v, out, lse, p);
  if (rc) return rc;
  void* ws = nullptr;
  rc = fg::static_scratch(&ws);
  if (rc) return rc;
  // the ordering pre-pass clears the queue counters itself (a kernel, no memset), so nothing else needs zeroing
  return fg::run_forward(q, k, v, mask_indptr, mask_indices, p, out, lse, ws,
                         sizeof(int32_t) * (64 + (size_t)FGATTN_STATIC_MAX_ITEMS), stream);
}

int fgattn_dense_forward(const void* q, const void* k, const void* v, const fgattn_params* p, void* out, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (p == nullptr) return FGATTN_E_NULL;
  fgattn_params pd = *p;
  pd.N = 1;   // there is no mask, hence no key groups: whatever the caller left in N is ignored
  return fg::run_forward(q, k, v, nullptr, nullptr, &pd, out, lse, workspace, workspace_bytes, stream);
}

int fgattn_forward_part(const void* q, const void* k, const void* v, const int64_t* mask_indptr,
                        const int32_t* mask_indices, const fgattn_params* p, void* out, float* lse, void* workspace,
                        size_t workspace_bytes, int part, void* stream) {
  if (!mask_indptr || !mask_indices) return FGATTN_E_NULL;
  if (part < FGATTN_PART_GATHER || part > FGATTN_PART_GATHER_ONE_WG) return FGATTN_E_FLAGS;
  if (p && ((p->M != 64 && p->M != 128) || p->d != 128 || p->N != 1)) return FGATTN_E_SHAPE;
  if (p && p->M != 64 && part > FGATTN_PART_COMPUTE) return FGATTN_E_SHAPE;
  return fg::run_forward(q, k, v, mask_indptr, mask_indices, p, out, lse, workspace, workspace_bytes, stream, part);
}

int fgattn_issue_probe(int other_valu_per_16_mfma, int iters, void* scratch, size_t scratch_bytes, double* flop, void* stream) {
  if (!scratch || !flop) return FGATTN_E_NULL;
  if (iters < 1 || iters > (1 << 20)) return FGATTN_E_SHAPE;
  fg::DeviceInfo dev;
  int rc = fg::device_info(&dev);
  if (rc) return rc;
  if (scratch_bytes < (size_t)2 * dev.cus * 256 * sizeof(float)) return FGATTN_E_WORKSPACE;
  *flop = 2.0 * dev.cus * 4 * (double)iters * 16 * 32768.0;
  return fg::launch_issue_probe(other_valu_per_16_mfma, iters, static_cast<float*>(scratch), dev.cus, static_cast<hipStream_t>(stream));
}

int fgattn_forward_grouped(const void* q, const void* k, const void* v, const int32_t* group_tiles,
                           const int64_t* union_indptr, const int32_t* union_indices, const uint8_t* union_members,
                           const fgattn_params* p, void* out, float* lse, void* workspace, size_t workspace_bytes,
                           void* stream) {
  if (!group_tiles || !union_indptr || !union_indices || !union_members) return FGATTN_E_NULL;
  return fg::run_forward(q, k, v, union_indptr, union_indices, p, out, lse, workspace, workspace_bytes, stream, 0,
                         group_tiles, union_members);
}

int fgattn_plan(const int64_t* mask_indptr, const fgattn_params* p, void* workspace, size_t workspace_bytes,
                void* stream) {
  if (!mask_indptr) return FGATTN_E_NULL;
  int rc = fg::check_shape(p);
  if (rc) return rc;
  rc = fg::check_workspace(p, workspace, workspace_bytes);
  if (rc) return rc;
  fg::DeviceInfo dev;
  rc = fg::device_info(&dev);
  if (rc) return rc;
  return fg::run_plan(mask_indptr, p, workspace, static_cast<hipStream_t>(stream));
}

int fgattn_validate_mask(const int64_t* mask_indptr, const int32_t* mask_indices, const fgattn_params* p,
                         void* workspace, size_t workspace_bytes, void* stream_v) {
  if (!mask_indptr || !mask_indices) return FGATTN_E_NULL;
  int rc = fg::check_shape(p);
  if (rc) return rc;
  rc = fg::check_workspace(p, workspace, workspace_bytes);
  if (rc) return rc;
  fg::DeviceInfo dev;
  rc = fg::device_info(&dev);
  if (rc) return rc;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  int* bad = static_cast<int*>(workspace);
  int zero = 0, host_bad = 0;
  if (hipMemcpyAsync(bad, &zero, sizeof(int), hipMemcpyHostToDevice, stream) != hipSuccess) return FGATTN_E_DEVICE;
  const int G = (p->L + p->N - 1) / p->N;
  hipLaunchKernelGGL(fg::validate_kernel, dim3((unsigned)fg::n_items_of(p)), dim3(256), 0, stream, mask_indptr,
                     mask_indices, G, bad);
  if (hipGetLastError() != hipSuccess) return FGATTN_E_DEVICE;
  if (hipMemcpyAsync(&host_bad, bad, sizeof(int), hipMemcpyDeviceToHost, stream) != hipSuccess) return FGATTN_E_DEVICE;
  if (hipStreamSynchronize(stream) != hipSuccess) return FGATTN_E_DEVICE;
  return host_bad ? FGATTN_E_MASK : FGATTN_OK;
}

int fgattn_grid_size(const fgattn_params* p) {
  if (fg::check_shape(p) != FGATTN_OK) return 0;
  fg::DeviceInfo dev;
  if (fg::device_info(&dev) != FGATTN_OK) return 0;
  fg::FwdArgs a;
  memset(&a, 0, sizeof(a));
  a.M = p->M;
  a.N = p->N;
  a.L = p->L;
  a.n_items = (int32_t)fg::n_items_of(p);
  a.indptr = reinterpret_cast<const int64_t*>(&a);   // any non-null value: report the sparse variant's grid
  int grid = 0;
  if (fg::launch_forward(a, p->d, dev.cus, nullptr, &grid) != FGATTN_OK) return 0;
  return grid;
}

const char* fgattn_strerror(int code) {
  switch (code) {
    case FGATTN_OK: return "ok";
    case FGATTN_E_NULL: return "a required pointer is NULL";
    case FGATTN_E_SHAPE: return "unsupported shape (need B,H,L >= 1, d in {64,128}, M in {16,32,64,128}, N >= 1)";
    case FGATTN_E_STRIDE: return "strides must be multiples of 8 elements and row strides >= d";
    case FGATTN_E_ALIGN: return "q/k/v/out must be 16-byte aligned and the workspace 256-byte aligned";
    case FGATTN_E_WORKSPACE: return "workspace too small (see fgattn_workspace_bytes)";
    case FGATTN_E_SCALE: return "scale must be finite";
    case FGATTN_E_DEVICE: return "no gfx950 device current, or a HIP runtime call failed";
    case FGATTN_E_MASK: return "mask failed validation";
    case FGATTN_E_FLAGS: return "unknown flag bits";
    case FGATTN_E_STATIC_LIMIT: return "fgattn_forward_static: more work items than FGATTN_STATIC_MAX_ITEMS";
    default: return "unknown fgattn error code";
  }
}

}  // extern "C"

namespace fg {
int launch_forward(const FwdArgs& a, int d, int cus, hipStream_t stream, int* grid_only) {
  if (a.M <= 32) return launch_mt32(a, d, cus, stream, grid_only);
  if (a.M == 64) return launch_mt64(a, d, cus, stream, grid_only);
  return launch_mt128(a, d, cus, stream, grid_only);
}
}  // namespace fg
