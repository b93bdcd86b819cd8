/*
 * fgattn.h -- C ABI of the MI355X (gfx950) forward kernel for fine-grained sparse attention.
 *
 * What it computes (paper Sec. 2 "Efficient dense attention" / "Efficient block sparse
 * attention", Sec. 4.1 and Fig. 1b): per batch b, head h and query block i (rows
 * [i*M, min((i+1)*M, L))), softmax(scale * Q K^T) restricted to the keys of the active
 * key groups listed for that block, times V.  A key group g covers keys
 * [g*N, min((g+1)*N, L)).  A skipped key takes no part in the softmax.
 *
 * All tensor and mask pointers are DEVICE pointers owned by the caller.  The library
 * allocates no device memory; scratch space (work order + queue counter) is the
 * caller-provided `workspace` of at least fgattn_workspace_bytes() bytes, 256-byte aligned.
 * Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = default stream)
 * and never synchronise the host, except fgattn_validate_mask.  Two calls that share a
 * workspace must be ordered on one stream.
 *
 * Return value: 0 (FGATTN_OK) or a negative FGATTN_E* code; fgattn_strerror() names it.
 * No C++ exceptions cross this boundary.
 */
#ifndef FGATTN_H_
#define FGATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FGATTN_OK = 0,
  FGATTN_E_NULL = -1,        /* a required pointer is NULL */
  FGATTN_E_SHAPE = -2,       /* B,H,L < 1; L > 2^24; d not in {64,128}; M not in {16,32,64,128}; N < 1;
                                L+N overflows int32 */
  FGATTN_E_STRIDE = -3,      /* a stride is not a multiple of 8 elements, a row stride is smaller than d, or a K/V
                                (batch, head) slice spans 4 GiB or more, or a row stride is 16 MiB or more */
  FGATTN_E_ALIGN = -4,       /* q/k/v/out not 16-byte aligned, or workspace not 256-byte aligned */
  FGATTN_E_WORKSPACE = -5,   /* workspace_bytes too small */
  FGATTN_E_SCALE = -6,       /* scale is not finite */
  FGATTN_E_DEVICE = -7,      /* not a gfx950 device, or a HIP runtime call failed */
  FGATTN_E_MASK = -8,        /* fgattn_validate_mask found a bad mask */
  FGATTN_E_FLAGS = -9,       /* unknown flag bits */
  FGATTN_E_STATIC_LIMIT = -10 /* fgattn_forward_static: more work items than FGATTN_STATIC_MAX_ITEMS */
};

enum {
  /* Scheduling of work items (one item = one query block of one head) onto the persistent
   * workgroups; paper Sec. 4.2 "Load balancing" and Appendix B.  Default (0): per head, items
   * ordered by decreasing active-list length and fetched from device-side queues (one per XCD over a
   * contiguous share of the heads; a workgroup whose queue is empty takes from the others). */
  FGATTN_FLAG_STATIC_ASSIGN = 1,  /* ablation "no scheduler": item j goes to workgroup j mod grid, natural order */
  FGATTN_FLAG_FIFO_QUEUE = 2,     /* device-side queue, but natural order (no longest-first ordering) */
  FGATTN_FLAG_REUSE_PLAN = 4,     /* skip the ordering pre-pass: `workspace` already holds the order built by an
                                     earlier fgattn_forward/fgattn_plan call for the same mask and params */
  /* Read by the fgattn_mask_* calls only (the others ignore it): use the general selection kernel, which reads a
   * row of scores from device memory in every pass, also for rows of at most 32768 key blocks (which otherwise
   * take the kernel that reads the row once).  Same results; pass the same flags to all three mask calls. */
  FGATTN_FLAG_MASK_ROWS_IN_HBM = 8,
  /* Read by the fgattn_mask_* calls only: a score buffer of the smallest size (one tile of 128 query blocks)
   * instead of up to 1 GiB, so that small inputs also take several chunks.  Same results; it changes the
   * workspace size, so pass the same flags to all three mask calls. */
  FGATTN_FLAG_MASK_ONE_TILE_CHUNKS = 16
};

typedef struct fgattn_params {
  int32_t B, H, L, d;            /* batch, heads, tokens, head dim (64 or 128) */
  int32_t M, N;                  /* query-block rows (16, 32, 64 or 128); keys per key group (>= 1) */
  /* strides in ELEMENTS (bf16); the last dimension (d) is contiguous; row strides must be multiples of 8 */
  int64_t q_stride_b, q_stride_h, q_stride_l;
  int64_t k_stride_b, k_stride_h, k_stride_l;
  int64_t v_stride_b, v_stride_h, v_stride_l;
  int64_t o_stride_b, o_stride_h, o_stride_l;
  float scale;                   /* multiplies Q K^T; the paper uses 1/sqrt(d) (Sec. 2) */
  int32_t flags;                 /* FGATTN_FLAG_* */
} fgattn_params;

/* Bytes of device workspace fgattn_forward / fgattn_dense_forward / fgattn_plan need for `p`
 * (0 if p is NULL or its shape is invalid). */
size_t fgattn_workspace_bytes(const fgattn_params* p);

/*
 * Sparse forward pass (paper Sec. 4.1 gather-load + Sec. 4.2 / Appendix B scheduler).
 *   q, k, v      : bf16, logical shape [B, H, L, d], addressed through the strides in `p`.
 *   mask_indptr  : int64 [B*H*ceil(L/M) + 1], non-decreasing, mask_indptr[0] == 0.  Work item
 *                  w = (b*H + h)*ceil(L/M) + i owns mask_indices[mask_indptr[w] : mask_indptr[w+1]].
 *   mask_indices : int32 key-GROUP ids in [0, ceil(L/N)); any order; no duplicates within an item.
 *                  Contents are NOT checked here (out-of-range ids are undefined behaviour);
 *                  use fgattn_validate_mask in tests.
 *   out          : bf16, same logical shape as q (strides o_stride_*).  Rows >= L are not written.
 *   lse          : fp32 [B, H, L] contiguous: natural-log of sum_k exp(scale * q.k) over the active
 *                  keys; an item with an empty list gets out = 0 and lse = -inf.
 * Enqueues an ordering pre-pass (unless FGATTN_FLAG_REUSE_PLAN) and one persistent kernel.
 */
int fgattn_forward(const void* q, const void* k, const void* v, const int64_t* mask_indptr,
                   const int32_t* mask_indices, const fgattn_params* p, void* out, float* lse, void* workspace,
                   size_t workspace_bytes, void* stream);

/* Dense attention (0% sparsity: every key active), the comparison kernel of the same build
 * (paper Sec. 2 "Efficient dense attention").  Same arguments minus the mask; p->N is ignored
 * (fgattn_workspace_bytes still wants N >= 1). */
int fgattn_dense_forward(const void* q, const void* k, const void* v, const fgattn_params* p, void* out, float* lse,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sparse forward pass over GROUPED query tiles (paper Sec. 4.2 "Grouping Query Tiles Attending to Similar Sets of
 * Keys/Values"): R = 128 / M query tiles of M rows form one work item that gathers the UNION of their key lists
 * once; every tile still attends only to its own key blocks (the result equals fgattn_forward's on the
 * ungrouped mask).  With G_s = ceil(ceil(L/M) / R) groups per (batch, head) slice:
 *   group_tiles   : int32 [B*H*G_s * R]: the member tiles of each group as tile indices inside the slice
 *                   (tile t covers rows [t*M, (t+1)*M)); -1 = no member in this position; every tile of a slice
 *                   must appear exactly once.
 *   union_indptr  : int64 [B*H*G_s + 1], union_indices: int32 key-block ids of each group's union (any order, no
 *                   duplicates), union_members: uint8, one per entry of union_indices: bit r set iff member r of
 *                   the group selected that key block.
 * Everything else as in fgattn_forward (same workspace size; FGATTN_FLAG_REUSE_PLAN refers to a plan made by
 * this call).  Contents of the four arrays are not checked.
 */
int fgattn_forward_grouped(const void* q, const void* k, const void* v, const int32_t* group_tiles,
                           const int64_t* union_indptr, const int32_t* union_indices, const uint8_t* union_members,
                           const fgattn_params* p, void* out, float* lse, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * Grouping pre-pass for fgattn_forward_grouped (paper Sec. 4.2), on the device.
 *   mode FGATTN_GROUP_CONSECUTIVE: R = 128/M consecutive query tiles per group ("merge-consecutive", Sec. 5);
 *   mode FGATTN_GROUP_XOR: the section's greedy heuristic on the distance d(i,j) = number of key blocks selected
 *     by exactly one of the tiles i, j: the first ungrouped tile of a (batch, head) slice becomes a group's
 *     representative and takes the R-1 ungrouped tiles closest to it (equal distances: lower index first;
 *     members are listed representative first, then by (distance, index); the last group of a slice may be short).
 * fgattn_group_select: reads the ungrouped CSR mask (as given to fgattn_forward; ids are not checked), writes
 *   group_tiles (int32 [B*H*G_s*R], -1 padding) and union_indptr (int64 [B*H*G_s + 1]); `workspace` (device,
 *   256-byte aligned, >= fgattn_group_workspace_bytes(p, mode)) keeps the bit rows for the second call
 *   (one bit per (query tile, key block), plus 4 bytes per pair of query tiles of a slice in XOR mode).
 * fgattn_group_emit: after the caller has read nnz = union_indptr[last]: writes union_indices (ascending ids per
 *   group) and union_members; entries beyond `capacity` are dropped, never written out of bounds.
 * Limits: ceil(L/N) <= 491520 key blocks, ceil(L/M) <= 49152 query tiles per slice (else FGATTN_E_SHAPE); an unknown
 * mode gives FGATTN_E_FLAGS.  Asynchronous on `stream`, no allocation.
 */
#define FGATTN_GROUP_CONSECUTIVE 0
#define FGATTN_GROUP_XOR 1
size_t fgattn_group_workspace_bytes(const fgattn_params* p, int mode);
int fgattn_group_select(const int64_t* mask_indptr, const int32_t* mask_indices, const fgattn_params* p, int mode,
                        int32_t* group_tiles, int64_t* union_indptr, void* workspace, size_t workspace_bytes,
                        void* stream);
int fgattn_group_emit(const fgattn_params* p, int mode, const int32_t* group_tiles, const int64_t* union_indptr,
                      int32_t* union_indices, uint8_t* union_members, int64_t capacity, const void* workspace,
                      size_t workspace_bytes, void* stream);

/* Only the ordering pre-pass of fgattn_forward (Appendix B: cost of an item = length of its
 * key/value list; longest first): fills `workspace`.  A later fgattn_forward with
 * FGATTN_FLAG_REUSE_PLAN and the same mask/params skips it. */
int fgattn_plan(const int64_t* mask_indptr, const fgattn_params* p, void* workspace, size_t workspace_bytes,
                void* stream);

/* Slow, SYNCHRONOUS check of a device-resident mask: indptr starts at 0 and is non-decreasing,
 * every id is in [0, ceil(L/N)), no id repeats within an item.  Uses the first 256 bytes of
 * `workspace`.  Returns FGATTN_OK or FGATTN_E_MASK. */
int fgattn_validate_mask(const int64_t* mask_indptr, const int32_t* mask_indices, const fgattn_params* p,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Mean-query/key top-p mask (paper Sec. 4.3): builds, on the device, the CSR mask fgattn_forward reads.
 *   q_avg(i) = mean of the rows of query block i (M rows), k_avg(j) = mean of the rows of key block j (N rows),
 *   A_hat(i,:) = softmax_j(scale * <q_avg(i), k_avg(j)>); per query block the key blocks are ranked by A_hat
 *   (equal values: lower id first) and the smallest prefix whose mass is at least top_p is kept.
 * Reading of what the paper leaves open: the block means are bf16 tensors (fp32 sum in row order, fp32 divide,
 * one rounding to nearest even); scores and masses are fp32 / 2^-40 fixed point.
 *
 * fgattn_mask_select: q, k as in fgattn_forward (strides from `p`; v/out strides ignored).  Writes
 *   mask_indptr (device, int64 [B*H*ceil(L/M) + 1]) and keeps the per-block cut in `workspace`
 *   (device, 256-byte aligned, at least fgattn_mask_workspace_bytes(p)).  top_p must be in (0, 1]
 *   (FGATTN_E_SCALE otherwise).
 *   Workspace size: the block means (2*d bytes per query block, and per key block unless B == 1 and N == 1),
 *   20 bytes per query block, one bit per (query block, key block), and a buffer for fp32 scores that is
 *   bounded: the scores are produced and consumed in chunks of whole tiles of 128 query blocks, and the buffer
 *   holds min(all tiles, max(1, floor(1 GiB / tile))) tiles, a tile being 128 * 4 * ceil32(ceil(L/N)) bytes.
 *   So it never exceeds max(1 GiB, one tile); a tile is below 1 GiB up to 2 097 152 key blocks.
 * fgattn_mask_emit: after the caller has read nnz = mask_indptr[last] and provided mask_indices (device, int32,
 *   capacity >= nnz entries): writes the kept key-block ids of every query block in ascending order.  Entries
 *   that would fall beyond `indices_capacity` are dropped, never written out of bounds.  `workspace` must be the
 *   one fgattn_mask_select filled for the same `p`.
 * Both are asynchronous on `stream`, allocate nothing, and return FGATTN_* codes like the other calls.
 */
size_t fgattn_mask_workspace_bytes(const fgattn_params* p);
int fgattn_mask_select(const void* q, const void* k, const fgattn_params* p, float top_p, int64_t* mask_indptr,
                       void* workspace, size_t workspace_bytes, void* stream);
int fgattn_mask_emit(const fgattn_params* p, const int64_t* mask_indptr, int32_t* mask_indices, int64_t indices_capacity,
                     const void* workspace, size_t workspace_bytes, void* stream);

/* Number of persistent workgroups fgattn_forward would launch for `p` on the current device
 * (0 on error).  Informational: used by benchmarks to report the launch shape. */
int fgattn_grid_size(const fgattn_params* p);

const char* fgattn_strerror(int code);

/*
 * Entry point for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc).  Same computation, arguments, flags and error behaviour as
 * fgattn_forward, minus the workspace: the work order and the queue counters live in a fixed array inside the
 * library's device image (4 bytes per work item + 256 bytes; every GPU the library runs on holds its own copy
 * until the process ends).  It calls no hipMalloc / hipFree and no allocating library routine.
 *   limit : B * H * ceil(L/M) <= FGATTN_STATIC_MAX_ITEMS, else FGATTN_E_STATIC_LIMIT and nothing is enqueued;
 *   all calls on one GPU share that GPU's array: calls that may overlap there (different streams, different host
 *   threads) race -- order them on one stream; the array keeps the last call's contents, each call rebuilds what it
 *   reads (FGATTN_FLAG_REUSE_PLAN reuses the order left by the previous call of THIS entry point on the same GPU).
 */
#define FGATTN_STATIC_MAX_ITEMS 65536
int fgattn_forward_static(const void* q, const void* k, const void* v, const int64_t* mask_indptr,
                          const int32_t* mask_indices, const fgattn_params* p, void* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------------------------------------------
 * Measurement aids -- not part of the method, not needed by any caller of the path; benchmarks use them.
 * --------------------------------------------------------------------------------------------------------------- */

/* Runs one half of fgattn_forward's kernel on the same launch shape,
 * FGATTN_PART_GATHER = index translation and K/V row gathers only (the data movement of Sec. 4.1),
 * FGATTN_PART_COMPUTE = everything except the row gathers (MFMA, softmax, LDS reads on whatever the tiles hold),
 * FGATTN_PART_GATHER_RING3 = the gathers with a K ring of three tiles instead of two (more rows in flight),
 * FGATTN_PART_GATHER_ONE_WG = the gathers with one workgroup per compute unit instead of two (half the issuing waves).
 * Same arguments and error behaviour as fgattn_forward; only M = 64 or 128 with d = 128, N = 1 is built, the last
 * two parts only M = 64 (else FGATTN_E_SHAPE; an unknown `part` gives FGATTN_E_FLAGS).  `out` and `lse` are
 * overwritten with meaningless values. */
#define FGATTN_PART_GATHER 1
#define FGATTN_PART_COMPUTE 2
#define FGATTN_PART_GATHER_RING3 3
#define FGATTN_PART_GATHER_ONE_WG 4
int fgattn_forward_part(const void* q, const void* k, const void* v, const int64_t* mask_indptr,
                        const int32_t* mask_indices, const fgattn_params* p, void* out, float* lse, void* workspace,
                        size_t workspace_bytes, int part, void* stream);

/* Measurement aid, like fgattn_forward_part: the instruction-issue ceiling of the forward kernel's arithmetic.  Runs, with
 * the forward kernel's occupancy (two four-wave workgroups per compute unit), a loop of 16 MFMAs (32x32x16 bf16), 16
 * exponentials and `other_valu_per_16_mfma` ordinary vector instructions per trip, `iters` trips, no memory traffic:
 * what a SIMD sustains on the mix of one wave-tile of the key loop (Sec. 2's softmax between the two matrix products).
 * Built for other_valu_per_16_mfma = 67 (64-row sparse tile), 61 (128-row sparse tile), 59 (128-row dense tile), and 0 =
 * the MFMAs alone, without the exponentials; anything else gives FGATTN_E_FLAGS.  `scratch`: device memory, at least 2048 B per compute unit (results nobody
 * reads); *flop (host) receives the MFMA FLOP count of the launch, so that FLOP / measured time is the ceiling.
 * Asynchronous on `stream`. */
int fgattn_issue_probe(int other_valu_per_16_mfma, int iters, void* scratch, size_t scratch_bytes, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FGATTN_H_ */
