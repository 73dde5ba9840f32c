// Internal declarations shared by the translation units of libmaxk (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/maxk.h"

namespace maxk {

constexpr int kWave = 64;  // CDNA wavefront width

// One unit of scheduled work: a contiguous run of stored entries of one row
// (forward / push backward / dense SpMM) or of one column of A^T (pull backward).
// The paper's "edge group" (Sec. 4.1), sized for a 64-wide wavefront.
struct WorkItem {
    int32_t row;    // output row (or destination node for the CSC lists)
    int32_t begin;  // first stored entry
    int32_t end;    // one past the last
    int32_t slot;   // -1: this item owns the whole row and writes the result; else partial-sum slot
};

// A row whose entries were split over several items; its partial sums live in
// slots [slot_begin, slot_begin + slot_count) and are added up by a second kernel.
struct SplitRow {
    int32_t row;
    int32_t slot_begin;
    int32_t slot_count;
};

struct ItemList {
    WorkItem* d_items = nullptr;
    SplitRow* d_split = nullptr;
    int64_t n_items = 0;
    int64_t n_split = 0;
    int64_t n_slots = 0;
};

// A^T regrouped for the L2-tiled pull kernel: source rows are cut into slabs of `slab_rows`
// rows (a slab of dY fits one XCD's L2); in-entries are ordered by (slab of source, destination,
// source) and every non-empty (slab, destination) pair is one "visit".
struct SlabSet {
    int32_t slab_rows = 0;
    int32_t n_slabs = 0;
    int64_t n_visits = 0;
    int32_t* d_src = nullptr;          // [nnz] source row of each regrouped in-entry
    float* d_val = nullptr;            // [nnz]
    int32_t* d_visit_node = nullptr;   // [n_visits] destination node
    int32_t* d_visit_begin = nullptr;  // [n_visits + 1] first regrouped entry of the visit
    int64_t* h_slab_visit = nullptr;   // host [n_slabs + 1] first visit of each slab
    // visits with more than kSlabLongVisit entries (hub destinations) are worked on by a whole wavefront
    int64_t n_long = 0;
    int32_t* d_long_visit = nullptr;   // [n_long] visit numbers, grouped by slab
    int64_t* h_slab_long = nullptr;    // host [n_slabs + 1] first long visit of each slab
};

constexpr int kSlabLongVisit = 32;

// A^T regrouped for the LDS-tiled backward kernel: destinations are cut into sets of D nodes (a workgroup keeps one
// set's accumulators in LDS), sources into tiles of TR rows; every non-empty (tile, destination) pair is a visit,
// listed per (destination set, tile) and padded to whole wave instructions of E visits.
struct TiledSet {
    int32_t D = 0, TR = 0, E = 0, LPV = 0;  // destinations per set; rows per tile; visits per wave instruction; lanes per visit
    int32_t n_dsets = 0, n_tiles = 0;
    int32_t G = 0, R = 0, tiles_per_range = 0;  // destination sets per XCD; source ranges; tiles per range
    int32_t ovf_by_bucket = 0;                  // overflow entries: added bucket by bucket (1) or with LDS atomics (0)
    int64_t total_sets = 0, n_visits = 0, n_chain = 0;
    uint32_t* d_dir_sets = nullptr;  // [n_dsets * n_tiles + 1 (+ spare)] first wave instruction of each list
    uint2* d_rec = nullptr;          // [total_sets * E] visit records (first entry inline)
    uint4* d_extra = nullptr;        // [total_sets * E] second and third entry of a visit
    uint4* d_ovf = nullptr;          // [n_chain + 1] fourth and later entries of a visit (added at the end of the kernel)
    uint32_t* d_ovf_dir = nullptr;   // [n_dsets * R * lane groups + 1] overflow entries before every (workgroup, lane group)
    uint32_t* d_progress = nullptr;  // [8 * ceil(n_dsets / 8) * 32] progress marks of the running workgroups (pacing)
};

extern thread_local int32_t g_last_hip_error;

inline maxk_status hip_fail(hipError_t e)
{
    g_last_hip_error = (int32_t)e;
    (void)hipGetLastError();  // clear the sticky launch error, the code is kept above
    return e == hipErrorOutOfMemory ? MAXK_OUT_OF_MEMORY : MAXK_HIP_ERROR;
}

#define MAXK_HIP_TRY(expr)                                   \
    do {                                                     \
        hipError_t _e = (expr);                              \
        if (_e != hipSuccess) return ::maxk::hip_fail(_e);   \
    } while (0)

#define MAXK_LAUNCH_CHECK()                                  \
    do {                                                     \
        hipError_t _e = hipGetLastError();                   \
        if (_e != hipSuccess) return ::maxk::hip_fail(_e);   \
    } while (0)

// ---- storage formats of CBSR values: MAXK_VALUE_F32 / _BF16 / _F16 (the 16-bit ones are bit patterns in uint16_t) ----

template <int VT>
struct value_store { using type = uint16_t; };
template <>
struct value_store<MAXK_VALUE_F32> { using type = float; };
template <int VT>
using value_store_t = typename value_store<VT>::type;

inline int value_bytes(int value_type) { return value_type == MAXK_VALUE_F32 ? 4 : 2; }

// the fp32 value a stored pattern stands for (exact)
template <int VT>
__device__ __forceinline__ float widen_value(value_store_t<VT> x)
{
    if constexpr (VT == MAXK_VALUE_F32) return x;
    else if constexpr (VT == MAXK_VALUE_BF16) return __uint_as_float((uint32_t)x << 16);
    else return (float)__builtin_bit_cast(_Float16, x);
}

// round to nearest, halfway cases to even; beyond the largest finite value -> infinity (NaN is outside the contract)
template <int VT>
__device__ __forceinline__ value_store_t<VT> narrow_value(float x)
{
    if constexpr (VT == MAXK_VALUE_F32) return x;
    else if constexpr (VT == MAXK_VALUE_BF16) {
        const uint32_t b = __float_as_uint(x);
        // adding 0x7FFF (+1 when the kept part is odd) carries into the kept part exactly when the cut-off
        // part is above one half, or equals one half next to an odd neighbour
        return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
    } else {
        return __builtin_bit_cast(uint16_t, (_Float16)x);  // v_cvt_f16_f32, round-to-nearest-even mode, subnormals kept
    }
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---- launchers implemented in the kernel files (device pointers throughout) ----

maxk_status launch_topk(const float* H, int64_t N, int dim, int k, void* sp_data, int value_type, void* sp_index,
                        int index_bytes, hipStream_t s);

maxk_status launch_cbsr_scatter(const float* values, const void* sp_index, int index_bytes, int64_t N, int dim, int k,
                                float* dense, hipStream_t s);

// `packed`: workspace of N * fwd_packed_record_bytes(k, index_bytes, value bytes) bytes to use the packed-record
// path, or null
maxk_status launch_spgemm_fwd(const ItemList& items, const int32_t* col, const float* val, const void* sp_data,
                              int value_type, const void* sp_index, int index_bytes, int64_t N, char* packed, int dim,
                              int k, float* Y, float* partials, hipStream_t s);
int fwd_packed_index_offset(int k, int index_bytes, int val_bytes);  // where a record's indices start
int fwd_packed_record_bytes(int k, int index_bytes, int val_bytes);
int fwd_private_copies(int k);  // output-row copies the forward kernel keeps for MaxK k

maxk_status launch_spmm(const ItemList& items, const int32_t* col, const float* val, const float* H, int dim,
                        float* Y, float* partials, hipStream_t s);

// backward launchers: `dY` holds value_store_t<value_type> elements (fp32, or bf16 / fp16 patterns)
maxk_status launch_bwd_pull(const ItemList& csc_items, const int32_t* csc_src, const float* csc_val, const void* dY,
                            int value_type, const void* sp_index, int index_bytes, int dim, int k, float* dXs,
                            float* partials, hipStream_t s);

maxk_status launch_bwd_push(const ItemList& items, const int32_t* col, const float* val, const void* dY,
                            int value_type, const void* sp_index, int index_bytes, int64_t N, int dim, int k,
                            float* dXs, hipStream_t s);

maxk_status launch_bwd_expand_reduce(const ItemList& csr_items, const int32_t* col, const float* val,
                                     const ItemList& csc_items, const uint32_t* csc_entry, const void* dY,
                                     int value_type, const void* sp_index, int index_bytes, int dim, int k,
                                     float* expand, float* dXs, float* partials, hipStream_t s);

maxk_status launch_bwd_slab_pull(const SlabSet& S, const void* dY, int value_type, const void* sp_index,
                                 int index_bytes, int64_t N, int dim, int k, float* dXs, hipStream_t s);

// LDS-tiled backward kernel (fp32 dY, k % 4 == 0, dim % 4 == 0, dim <= 512)
struct TiledShape { int D = 0, TR = 0, n_dsets = 0; };
bool tiled_shape(int64_t N, int dim, int k, TiledShape& sh);  // false: (N, dim, k) not supported
int tiled_positions_per_lane(int k);
bool tiled_supports(const void* dY, int value_type, const void* sp_index, int index_bytes, int dim, int k);
maxk_status build_tiled(TiledSet& T, int64_t N, int64_t nnz, const int32_t* d_csc_ptr, const int32_t* d_csc_src,
                        const float* d_csc_val, int D, int TR, int k);
void free_tiled(TiledSet& T);
maxk_status launch_bwd_tiled(const TiledSet& T, const void* dY, int value_type, const void* sp_index, int index_bytes,
                             int64_t N, int dim, int k, float* dXs, hipStream_t s);

// shared by the push and slab kernels: p[0..n) = 0
maxk_status launch_fill_zero(float* p, int64_t n, hipStream_t s);

// out[row,:] = sum of the row's partial slots, for every split row (width = row length in floats)
maxk_status launch_combine(const ItemList& items, const float* partials, int width, float* out, hipStream_t s);

}  // namespace maxk
