/*
 * libmaxk -- MaxK-GNN aggregation hot path for AMD MI355X (gfx950), C ABI.
 *
 *   H --maxk_topk_cbsr--> CBSR (sp_data, sp_index) --maxk_spgemm_fwd--> Y
 *   dY + sp_index --maxk_sspmm_bwd--> dXs            (plus a dense SpMM baseline)
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; the library
 *     borrows them for the call and never frees or retains them, except that a
 *     maxk_graph keeps (aliases) the three CSR arrays it was created from: they
 *     must stay alive and unchanged until maxk_graph_destroy.
 *   - Dense matrices are row-major fp32 with leading dimension = dim.
 *     sp_data / sp_index / dXs are row-major with leading dimension = k.
 *   - sp_index element width is index_bytes in {1,2,4} (uint8 / uint16 / int32),
 *     and dim must fit: dim <= 256, <= 65536, or any.  The paper uses uint8 when
 *     the hidden width is small and 4-byte integers otherwise (Sec. 4.3).
 *   - Outputs are OVERWRITTEN; the caller need not clear them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they do not synchronise the device.
 *     After maxk_graph_reserve* the compute calls allocate nothing (see there).
 *   - Return value: MAXK_OK (0) or a negative maxk_status.  Nothing throws,
 *     aborts or prints.  N == 0 is a valid no-op.  Array CONTENTS are not
 *     validated by the compute calls (NaN in H, column ids outside [0,N) and
 *     sp_index outside [0,dim) are contract violations).
 *   - Calls on one maxk_graph must not overlap in time (they share its workspace).
 *   - Tuning knobs, read from the environment once per handle by maxk_graph_create (results never depend on
 *     them): MAXK_CHUNK (entries per work item, default 2048), MAXK_SLAB_KB (KiB of dY per slab of the slab-pull
 *     backward kernel, default 3584), MAXK_FWD_PACK_MAX (largest CBSR row in bytes that the forward pass
 *     repacks into one record per node, default 96).
 */
#ifndef MAXK_H
#define MAXK_H

#include <stdint.h>

#if defined(__GNUC__)
#define MAXK_API __attribute__((visibility("default")))
#else
#define MAXK_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t maxk_status;
enum {
    MAXK_OK = 0,
    MAXK_INVALID_ARGUMENT = -1, /* null pointer, negative size, k outside [1,dim], bad index_bytes, misaligned pointer */
    MAXK_UNSUPPORTED = -2,      /* dim above MAXK_MAX_DIM */
    MAXK_HIP_ERROR = -3,        /* a HIP call failed; see maxk_last_hip_error() */
    MAXK_OUT_OF_MEMORY = -4,
    MAXK_SCRATCH_TOO_SMALL = -5 /* maxk_spgemm_fwd_noalloc: the graph's split rows need more than the fixed array */
};

/* Largest hidden width the kernels are compiled for. */
#define MAXK_MAX_DIM 1024

/* Which kernel maxk_sspmm_bwd runs (see maxk_graph_set_bwd_mode). */
enum {
    MAXK_BWD_AUTO = 0,    /* library's choice (the faster one on MI355X) */
    MAXK_BWD_PULL_CSC = 1,/* owner-computes over A^T stored as CSC: deterministic, no atomics */
    MAXK_BWD_PUSH_CSR = 2,/* Alg. 2's dataflow: stage dY[i,:] on chip, push along row i of A with fp32 atomics */
    MAXK_BWD_EXPAND_REDUCE = 3,/* Alg. 2's staging without atomics: write each entry's k products to a per-graph
                                  buffer (nnz*k floats, sequential), then sum them per destination node */
    MAXK_BWD_SLAB_PULL = 4,   /* owner-computes pull, tiled so the dY rows being gathered stay in L2: source rows are
                                  swept slab by slab, one launch per slab; deterministic, no atomics */
    MAXK_BWD_TILED = 5        /* Alg. 2's on-chip staging of dY rows, turned round: a workgroup keeps the dXs rows of a
                                  set of destination nodes in LDS and streams tiles of dY rows through LDS, so a dY row
                                  is fetched once per destination set instead of once per entry.  fp32 dY, k % 4 == 0,
                                  dim % 4 == 0, dim <= 512, 16-byte aligned dY; other calls run MAXK_BWD_SLAB_PULL */
};

/* Storage format of the CBSR values for the *_narrow entry points: fp32, or a 16-bit pattern in a uint16_t. */
enum {
    MAXK_VALUE_F32 = 0,
    MAXK_VALUE_BF16 = 1, /* bfloat16: the upper half of the fp32 pattern, 8 significant bits */
    MAXK_VALUE_F16 = 2   /* IEEE binary16, 11 significant bits, subnormals kept, |x| >= 65520 becomes infinity */
};

typedef struct maxk_graph maxk_graph;

/*
 * Load-time preprocessing of the adjacency (the paper's O(n) partition of rows
 * into edge groups, Sec. 4.1 "Warp Level Partition", done "during graph loading",
 * Sec. 4.2).  Takes A in CSR on the device: d_rowptr int32[N+1], d_colidx
 * int32[nnz], d_val fp32[nnz]; rows may be empty, columns need not be sorted,
 * duplicates add.  Builds and owns: the degree-ordered work-item lists with hub
 * rows split into bounded chunks, and A^T as CSC (value-carrying) for the
 * backward pull kernel.  Synchronises `stream` (it copies rowptr to the host).
 * Not part of the timed path.
 */
MAXK_API maxk_status maxk_graph_create(maxk_graph** out, int64_t N, int64_t nnz, const int32_t* d_rowptr,
                              const int32_t* d_colidx, const float* d_val, void* stream);

/* Frees everything the handle owns (not the caller's CSR).  NULL is a no-op. */
MAXK_API maxk_status maxk_graph_destroy(maxk_graph* g);

/*
 * Builds everything the handle's compute calls need for hidden width `dim`, MaxK `k` and (for the backward pass)
 * dY stored as `dy_value_type`: the partial-sum workspace of split rows, the forward pass's repack buffer, and
 * what the backward kernel that would run needs (the nnz*k float buffer of expand/reduce, the slab regrouping
 * of A^T for the slab height of (dim, dy_value_type), the visit lists of the LDS-tiled kernel for (dim, k)).
 * After it, compute calls with the same dim and k (forward, SpMM: any dim' <= dim, k' <= k) allocate nothing,
 * do not synchronise and read no environment variable.  Tables are cached per shape for the life of the handle,
 * so alternating several (dim, k) or dY formats never rebuilds one.  Without a reserve, the first compute call that
 * needs a table or a larger workspace builds it (synchronous allocations; the tables also sort A^T), later ones
 * reuse it; the same holds for a backward call whose pointers turn out too misaligned for the reserved kernel.
 * Synchronises the device.  maxk_graph_reserve is the fp32-dY form.
 */
MAXK_API maxk_status maxk_graph_reserve(maxk_graph* g, int32_t dim, int32_t k);
MAXK_API maxk_status maxk_graph_reserve_narrow(maxk_graph* g, int32_t dim, int32_t k, int32_t dy_value_type);

/* Selects the backward kernel (MAXK_BWD_*). */
MAXK_API maxk_status maxk_graph_set_bwd_mode(maxk_graph* g, int32_t mode);

/* The MAXK_BWD_* kernel maxk_sspmm_bwd would run for (dim, k) with the handle's current mode
 * (resolves MAXK_BWD_AUTO); negative maxk_status on bad arguments. */
MAXK_API int32_t maxk_graph_bwd_choice(const maxk_graph* g, int32_t dim, int32_t k);

/* Reads back sizes: any out pointer may be NULL. */
MAXK_API maxk_status maxk_graph_info(const maxk_graph* g, int64_t* N, int64_t* nnz, int64_t* n_fwd_items,
                            int64_t* n_split_rows, int64_t* max_degree, int64_t* workspace_bytes);

/*
 * MaxK nonlinearity + CBSR packing (Sec. 3.1 definition, Eq. 1; CBSR: Sec. 3.2
 * "Forward Computation").  For every row i of d_H[N x dim] keeps the k largest
 * entries by signed value; ties at the k-th value go to the lower column, so
 * exactly k survive.  d_sp_index[i,0..k) = kept columns in ascending order,
 * d_sp_data[i,t] = H[i, sp_index[i,t]] (identical bits).  -0.0 and +0.0 compare
 * equal; NaN is outside the contract.
 */
MAXK_API maxk_status maxk_topk_cbsr(const float* d_H, int64_t N, int32_t dim, int32_t k, float* d_sp_data, void* d_sp_index,
                           int32_t index_bytes, void* stream);

/*
 * Forward aggregation, row-wise-product SpGEMM with dense output (Eq. 2 left;
 * Sec. 3.2; Alg. 1):  Y[i,:] = sum_{p in row i} val[p] * X[col[p],:], where X
 * is the N x dim matrix the CBSR describes.  d_Y is fp32 [N x dim].  Entries of
 * a CBSR row may come in any order; fp32 accumulation order is unspecified.
 */
MAXK_API maxk_status maxk_spgemm_fwd(maxk_graph* g, const float* d_sp_data, const void* d_sp_index, int32_t index_bytes,
                            int32_t dim, int32_t k, float* d_Y, void* stream);

/*
 * maxk_spgemm_fwd for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same result.  The forward kernels' scratch memory -- the partial rows
 * of rows that were split over several work items (slots x dim floats), and the per-call repack of a small-k
 * CBSR -- lives in a fixed array of MAXK_NOALLOC_SCRATCH_BYTES inside the library's device image instead of the
 * handle's workspaces, so this call never calls hipMalloc, hipFree or any allocating routine, whatever was or was
 * not reserved.  Every GPU holds its own copy of the array from the moment the library is loaded there until the
 * process ends.  MAXK_SCRATCH_TOO_SMALL when the split rows alone need more than the array (nothing is launched);
 * when only the repacked CBSR does not fit, the kernel reads sp_data / sp_index directly (same result, slower at
 * small k).  Must be called with the device current on which the handle was created.  All calls on one GPU share
 * the array, on any handle and any stream: calls that overlap in time on one GPU race; order them on one stream
 * or with events.  Nothing in the array needs clearing between calls.
 */
#define MAXK_NOALLOC_SCRATCH_BYTES (32u << 20)
MAXK_API maxk_status maxk_spgemm_fwd_noalloc(maxk_graph* g, const float* d_sp_data, const void* d_sp_index,
                                             int32_t index_bytes, int32_t dim, int32_t k, float* d_Y, void* stream);

/*
 * The same two steps with the CBSR values stored in 2 bytes (value_type MAXK_VALUE_BF16 or _F16;
 * MAXK_VALUE_F32 makes them the plain calls).  The forward pass reads (4+ib) bytes per stored entry and
 * kept position (Sec. 4.3, traffic model of the SpGEMM); 16-bit values make that (2+ib).  Selection is done
 * on the fp32 input, so d_sp_index is identical to maxk_topk_cbsr's; d_sp_data[i,t] is the fp32 value
 * rounded to nearest (halfway cases to even), laid out [N x k] in uint16_t.  The forward kernel widens the
 * stored values exactly and multiplies and accumulates in fp32, so Y differs from the fp32 path only
 * through the rounding of the values: by at most 2^-8 (bf16) or 2^-11 (fp16, |x| in [6.2e-5, 65504])
 * of the sum of |terms| per element.  The backward pass does not read the values and is unchanged.
 */
MAXK_API maxk_status maxk_topk_cbsr_narrow(const float* d_H, int64_t N, int32_t dim, int32_t k, void* d_sp_data,
                                           int32_t value_type, void* d_sp_index, int32_t index_bytes, void* stream);
MAXK_API maxk_status maxk_spgemm_fwd_narrow(maxk_graph* g, const void* d_sp_data, int32_t value_type,
                                            const void* d_sp_index, int32_t index_bytes, int32_t dim, int32_t k,
                                            float* d_Y, void* stream);

/*
 * Backward aggregation, sampled SSpMM (Eq. 2 right; Eq. 3; Alg. 2 with the
 * destination read as the neighbour row):  for every stored entry (i,j) of A,
 * dXs[j,t] += val * dY[i, sp_index[j,t]], i.e. dXs = (A^T dY) at each row's CBSR
 * columns.  d_dY is fp32 [N x dim]; d_dXs is fp32 [N x k], laid out like sp_data.
 */
MAXK_API maxk_status maxk_sspmm_bwd(maxk_graph* g, const float* d_dY, const void* d_sp_index, int32_t index_bytes,
                           int32_t dim, int32_t k, float* d_dXs, void* stream);

/*
 * The backward pass reading dY stored in 2 bytes (value_type MAXK_VALUE_BF16 or _F16, patterns in uint16_t
 * [N x dim]; MAXK_VALUE_F32 makes it the plain call).  The sampled gather of Alg. 2 / Eq. 3 moves whole cache
 * lines of dY rows, so the row length in bytes is what the kernel's time follows.  Values are widened exactly;
 * products and sums are fp32 and d_dXs is fp32, so the result meets the bound of maxk_sspmm_bwd against the
 * definition evaluated on the 16-bit values.  Rounding fp32 gradients to 16 bits is the caller's decision.
 * The slab-pull kernel regroups A^T per slab height, and 16-bit rows use a height of their own
 * (maxk_graph_reserve_narrow builds it ahead of time).
 */
MAXK_API maxk_status maxk_sspmm_bwd_narrow(maxk_graph* g, const void* d_dY, int32_t value_type, const void* d_sp_index,
                                           int32_t index_bytes, int32_t dim, int32_t k, float* d_dXs, void* stream);

/*
 * MaxK backward (Sec. 3.1 definition, part (ii): the gradient keeps the sparsity pattern of the
 * forward pass): d_dense[i, sp_index[i,t]] = d_values[i,t], every other entry of d_dense[N x dim] = 0.
 * d_values is fp32 [N x k] (the dXs of maxk_sspmm_bwd).  Columns of a row must be distinct.
 */
MAXK_API maxk_status maxk_cbsr_scatter(const float* d_values, const void* d_sp_index, int32_t index_bytes, int64_t N,
                                       int32_t dim, int32_t k, float* d_dense, void* stream);

/*
 * Dense-feature SpMM Y = A * H on the same graph handle: the operator the paper
 * measures its speedups against (Sec. 5.2), here as a same-GPU baseline.
 */
MAXK_API maxk_status spmm_baseline(maxk_graph* g, const float* d_H, int32_t dim, float* d_Y, void* stream);

/* Text for a status code (static storage). */
MAXK_API const char* maxk_status_string(maxk_status s);

/* hipError_t (as int) of the last HIP failure seen by this thread, 0 if none. */
MAXK_API int32_t maxk_last_hip_error(void);

/* Library version, MAJOR*10000 + MINOR*100 + PATCH. */
MAXK_API int32_t maxk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MAXK_H */
