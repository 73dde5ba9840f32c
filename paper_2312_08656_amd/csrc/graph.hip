// Graph handle: load-time preprocessing of the adjacency (the paper's O(n)
// partition of rows into edge groups "during graph loading", Sec. 4.1 / 4.2),
// and the extern "C" entry points of the library.
//
// Preprocessing builds, once per graph:
//   - the forward work-item list: rows cut into runs of at most `chunk` stored
//     entries, ordered longest first so the heavy tail of a power-law degree
//     distribution starts early and the short rows fill in behind it;
//   - A^T as value-carrying CSC (stable radix sort of the entries by column, so
//     in-entries of a node stay ordered by source row: deterministic sums) and
//     its work-item list, for the pull backward kernel;
//   - one partial-sum workspace shared by all kernels of the handle.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

#include "common.hpp"

struct maxk_graph {
    int64_t N = 0, nnz = 0;
    const int32_t* d_rowptr = nullptr;  // caller's CSR, aliased
    const int32_t* d_col = nullptr;
    const float* d_val = nullptr;
    maxk::ItemList csr_items;  // over rows of A
    maxk::ItemList csc_items;  // over columns of A (rows of A^T)
    int32_t* d_csc_ptr = nullptr;
    int32_t* d_csc_src = nullptr;
    float* d_csc_val = nullptr;
    uint32_t* d_csc_entry = nullptr;  // CSR entry id of every CSC position (the transposing permutation)
    float* d_partials = nullptr;
    int64_t partial_floats = 0;
    float* d_expand = nullptr;  // per-entry contributions of the expand/reduce backward kernel (nnz * k floats)
    int64_t expand_floats = 0;
    std::vector<maxk::SlabSet*> slab_cache;    // A^T regrouped per slab height (one per height ever asked for)
    std::vector<maxk::TiledSet*> tiled_cache;  // visit lists of the LDS-tiled kernel, one per (set size, k / 4)
    char* d_packed = nullptr;   // forward kernel's per-call repack of a small-k CBSR (one record per node)
    int64_t packed_bytes = 0;
    int64_t max_degree = 0;
    int32_t bwd_mode = MAXK_BWD_AUTO;
    int32_t chunk = 0;         // tuning knobs, read from the environment once, by maxk_graph_create
    int32_t slab_kb = 0;
    int32_t fwd_pack_max = 0;
    unsigned char* d_noalloc_scratch = nullptr;  // this device's copy of the library's fixed scratch array
    int device = 0;
};

// Scratch memory of maxk_spgemm_fwd_noalloc: a fixed array in the library's device image, one copy per GPU, alive
// until the process ends.  In host code this name is a handle for hipGetSymbolAddress only, never a pointer.
static __device__ __align__(256) unsigned char maxk_noalloc_scratch[MAXK_NOALLOC_SCRATCH_BYTES];

namespace maxk {

thread_local int32_t g_last_hip_error = 0;

namespace {

// Device address of the scratch array on the current device (asked for once per handle, by maxk_graph_create).
maxk_status noalloc_scratch_address(unsigned char** out)
{
    void* p = nullptr;
    MAXK_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(maxk_noalloc_scratch)));
    *out = static_cast<unsigned char*>(p);
    return p ? MAXK_OK : MAXK_HIP_ERROR;
}

int env_int(const char* name, int dflt, int lo, int hi)
{
    const char* v = std::getenv(name);
    if (!v || !*v) return dflt;
    long x = std::strtol(v, nullptr, 10);
    if (x < lo || x > hi) return dflt;
    return (int)x;
}

// Host side of the partition: ptr[n+1] -> items (longest first) + split rows.
void build_items(const std::vector<int32_t>& ptr, int64_t n, int chunk, std::vector<WorkItem>& items,
                 std::vector<SplitRow>& split, int64_t& n_slots, int64_t& max_len)
{
    items.clear();
    split.clear();
    n_slots = 0;
    max_len = 0;
    items.reserve((size_t)n + 1024);
    for (int64_t i = 0; i < n; ++i) {
        const int32_t b = ptr[i], e = ptr[i + 1];
        const int64_t len = (int64_t)e - b;
        max_len = std::max(max_len, len);
        if (len <= chunk) {
            items.push_back(WorkItem{(int32_t)i, b, e, -1});
        } else {
            // equal-sized pieces, each at most `chunk`
            const int64_t pieces = (len + chunk - 1) / chunk;
            split.push_back(SplitRow{(int32_t)i, (int32_t)n_slots, (int32_t)pieces});
            for (int64_t s = 0; s < pieces; ++s) {
                const int32_t pb = (int32_t)(b + len * s / pieces), pe = (int32_t)(b + len * (s + 1) / pieces);
                items.push_back(WorkItem{(int32_t)i, pb, pe, (int32_t)(n_slots + s)});
            }
            n_slots += pieces;
        }
    }
    std::stable_sort(items.begin(), items.end(), [](const WorkItem& a, const WorkItem& b) {
        return (a.end - a.begin) > (b.end - b.begin);
    });
}

maxk_status upload_items(const std::vector<WorkItem>& items, const std::vector<SplitRow>& split, int64_t n_slots,
                         ItemList& L, hipStream_t s)
{
    L.n_items = (int64_t)items.size();
    L.n_split = (int64_t)split.size();
    L.n_slots = n_slots;
    if (L.n_items) {
        MAXK_HIP_TRY(hipMalloc((void**)&L.d_items, sizeof(WorkItem) * items.size()));
        MAXK_HIP_TRY(hipMemcpyAsync(L.d_items, items.data(), sizeof(WorkItem) * items.size(), hipMemcpyHostToDevice, s));
    }
    if (L.n_split) {
        MAXK_HIP_TRY(hipMalloc((void**)&L.d_split, sizeof(SplitRow) * split.size()));
        MAXK_HIP_TRY(hipMemcpyAsync(L.d_split, split.data(), sizeof(SplitRow) * split.size(), hipMemcpyHostToDevice, s));
    }
    MAXK_HIP_TRY(hipStreamSynchronize(s));  // the host vectors go out of scope after this
    return MAXK_OK;
}

// row_of[p] = the row that stored entry p belongs to (binary search in rowptr)
__global__ __launch_bounds__(256) void entry_rows_kernel(const int32_t* __restrict__ rowptr, int64_t N, int64_t nnz,
                                                         int32_t* __restrict__ row_of, uint32_t* __restrict__ iota)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
        int64_t lo = 0, hi = N;  // largest i with rowptr[i] <= p
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)rowptr[mid] <= p) lo = mid; else hi = mid;
        }
        row_of[p] = (int32_t)lo;
        iota[p] = (uint32_t)p;
    }
}

// count[j] = stored entries in column j; ids outside [0,N) are tallied in count[N]
__global__ __launch_bounds__(256) void column_histogram_kernel(const int32_t* __restrict__ col, int64_t N,
                                                               int64_t nnz, int32_t* __restrict__ count)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
        const int32_t c = col[p];
        atomicAdd(&count[(c >= 0 && (int64_t)c < N) ? c : N], 1);
    }
}

__global__ __launch_bounds__(256) void gather_transposed_kernel(const uint32_t* __restrict__ perm,
                                                                const int32_t* __restrict__ row_of,
                                                                const float* __restrict__ val, int64_t nnz,
                                                                int32_t* __restrict__ csc_src,
                                                                float* __restrict__ csc_val)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += stride) {
        const uint32_t p = perm[q];
        csc_src[q] = row_of[p];
        csc_val[q] = val[p];
    }
}

// A^T in CSC: csc_ptr[N+1] (host copy returned), csc_src / csc_val on the device.
maxk_status build_csc(maxk_graph* g, std::vector<int32_t>& h_csc_ptr, hipStream_t s)
{
    const int64_t N = g->N, nnz = g->nnz;
    h_csc_ptr.assign((size_t)N + 1, 0);
    MAXK_HIP_TRY(hipMalloc((void**)&g->d_csc_ptr, sizeof(int32_t) * (size_t)(N + 1)));
    if (nnz == 0) {
        MAXK_HIP_TRY(hipMemsetAsync(g->d_csc_ptr, 0, sizeof(int32_t) * (size_t)(N + 1), s));
        MAXK_HIP_TRY(hipStreamSynchronize(s));
        return MAXK_OK;
    }
    MAXK_HIP_TRY(hipMalloc((void**)&g->d_csc_src, sizeof(int32_t) * (size_t)nnz));
    MAXK_HIP_TRY(hipMalloc((void**)&g->d_csc_val, sizeof(float) * (size_t)nnz));

    int32_t *d_row_of = nullptr, *d_count = nullptr;
    uint32_t *d_iota = nullptr, *d_keys_out = nullptr;
    MAXK_HIP_TRY(hipMalloc((void**)&g->d_csc_entry, sizeof(uint32_t) * (size_t)nnz));
    uint32_t* d_perm = g->d_csc_entry;  // kept: the reduce phase of the backward pass gathers through it
    void* d_tmp = nullptr;
    maxk_status st = MAXK_OK;
    auto cleanup = [&]() {
        (void)hipFree(d_row_of); (void)hipFree(d_count); (void)hipFree(d_iota);
        (void)hipFree(d_keys_out); (void)hipFree(d_tmp);
    };
#define MAXK_TRY_CLEAN(expr)                        \
    do {                                            \
        hipError_t _e = (expr);                     \
        if (_e != hipSuccess) { cleanup(); return hip_fail(_e); } \
    } while (0)
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_row_of, sizeof(int32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_iota, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_keys_out, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_count, sizeof(int32_t) * (size_t)(N + 1)));
    MAXK_TRY_CLEAN(hipMemsetAsync(d_count, 0, sizeof(int32_t) * (size_t)(N + 1), s));

    const unsigned blocks = (unsigned)std::min<int64_t>((nnz + 255) / 256, 65536);
    hipLaunchKernelGGL(entry_rows_kernel, dim3(blocks), dim3(256), 0, s, g->d_rowptr, N, nnz, d_row_of, d_iota);
    hipLaunchKernelGGL(column_histogram_kernel, dim3(blocks), dim3(256), 0, s, g->d_col, N, nnz, d_count);
    MAXK_TRY_CLEAN(hipGetLastError());

    // stable sort of entry ids by column: in-entries of a node keep ascending source row
    int end_bit = 1;
    while (end_bit < 32 && ((int64_t)1 << end_bit) < N) ++end_bit;
    size_t tmp_bytes = 0;
    const uint32_t* keys_in = reinterpret_cast<const uint32_t*>(g->d_col);
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys_in, d_keys_out, d_iota, d_perm, (size_t)nnz, 0,
                                             (unsigned)end_bit, s));
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(d_tmp, tmp_bytes, keys_in, d_keys_out, d_iota, d_perm, (size_t)nnz, 0,
                                             (unsigned)end_bit, s));
    hipLaunchKernelGGL(gather_transposed_kernel, dim3(blocks), dim3(256), 0, s, d_perm, d_row_of, g->d_val, nnz,
                       g->d_csc_src, g->d_csc_val);
    MAXK_TRY_CLEAN(hipGetLastError());

    // column counts -> pointers (host scan over N values)
    std::vector<int32_t> h_count((size_t)N + 1);
    MAXK_TRY_CLEAN(hipMemcpyAsync(h_count.data(), d_count, sizeof(int32_t) * (size_t)(N + 1), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    int64_t run = 0;
    for (int64_t j = 0; j < N; ++j) {
        h_csc_ptr[(size_t)j] = (int32_t)run;
        run += h_count[(size_t)j];
    }
    h_csc_ptr[(size_t)N] = (int32_t)run;
    if (run != nnz) st = MAXK_INVALID_ARGUMENT;  // a column id fell outside [0,N)
    MAXK_TRY_CLEAN(hipMemcpyAsync(g->d_csc_ptr, h_csc_ptr.data(), sizeof(int32_t) * (size_t)(N + 1), hipMemcpyHostToDevice, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
#undef MAXK_TRY_CLEAN
    cleanup();
    return st;
}

maxk_status ensure_workspace(maxk_graph* g, int dim, int k)
{
    const int64_t need = std::max<int64_t>(g->csr_items.n_slots * (int64_t)dim, g->csc_items.n_slots * (int64_t)k);
    if (need <= g->partial_floats) return MAXK_OK;
    float* fresh = nullptr;
    MAXK_HIP_TRY(hipMalloc((void**)&fresh, sizeof(float) * (size_t)need));
    if (g->d_partials) {
        MAXK_HIP_TRY(hipDeviceSynchronize());  // nothing may still be using the old buffer
        (void)hipFree(g->d_partials);
    }
    g->d_partials = fresh;
    g->partial_floats = need;
    return MAXK_OK;
}

void free_slabs(SlabSet& S)
{
    (void)hipFree(S.d_src);
    (void)hipFree(S.d_val);
    (void)hipFree(S.d_visit_node);
    (void)hipFree(S.d_visit_begin);
    (void)hipFree(S.d_long_visit);
    std::free(S.h_slab_visit);
    std::free(S.h_slab_long);
    S = SlabSet();
}

// key[q] = slab(source of CSC position q) * N + destination of q;  iota[q] = q
__global__ __launch_bounds__(256) void slab_keys_kernel(const int32_t* __restrict__ csc_ptr,
                                                        const int32_t* __restrict__ csc_src, int64_t N, int64_t nnz,
                                                        int32_t slab_rows, uint64_t* __restrict__ key,
                                                        uint32_t* __restrict__ iota)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += stride) {
        int64_t lo = 0, hi = N;  // largest j with csc_ptr[j] <= q
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)csc_ptr[mid] <= q) lo = mid; else hi = mid;
        }
        key[q] = (uint64_t)(csc_src[q] / slab_rows) * (uint64_t)N + (uint64_t)lo;
        iota[q] = (uint32_t)q;
    }
}

__global__ __launch_bounds__(256) void slab_gather_kernel(const uint32_t* __restrict__ perm,
                                                          const uint64_t* __restrict__ key_sorted,
                                                          const int32_t* __restrict__ csc_src,
                                                          const float* __restrict__ csc_val, int64_t nnz,
                                                          int32_t* __restrict__ out_src, float* __restrict__ out_val,
                                                          uint32_t* __restrict__ head)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < nnz; r += stride) {
        const uint32_t q = perm[r];
        out_src[r] = csc_src[q];
        out_val[r] = csc_val[q];
        head[r] = (r == 0 || key_sorted[r] != key_sorted[r - 1]) ? 1u : 0u;
    }
}

// at every head position r (visit number v = rank[r] - 1): record the visit
__global__ __launch_bounds__(256) void slab_visits_kernel(const uint32_t* __restrict__ head,
                                                          const uint32_t* __restrict__ rank,
                                                          const uint64_t* __restrict__ key_sorted, int64_t N,
                                                          int64_t nnz, int32_t* __restrict__ visit_node,
                                                          int32_t* __restrict__ visit_begin,
                                                          int32_t* __restrict__ visit_slab)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < nnz; r += stride) {
        if (!head[r]) continue;
        const uint32_t v = rank[r] - 1u;
        const uint64_t key = key_sorted[r];
        visit_node[v] = (int32_t)(key % (uint64_t)N);
        visit_slab[v] = (int32_t)(key / (uint64_t)N);
        visit_begin[v] = (int32_t)r;
    }
}

// slab_first[s] = first visit whose slab is >= s (slab_first pre-filled with n_visits)
__global__ __launch_bounds__(256) void slab_first_kernel(const int32_t* __restrict__ visit_slab, int64_t n_visits,
                                                         int64_t* __restrict__ slab_first)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_visits; v += stride) {
        const int32_t sl = visit_slab[v];
        const int32_t prev = v ? visit_slab[v - 1] : -1;
        for (int32_t s = prev + 1; s <= sl; ++s) slab_first[s] = v;
    }
}

__global__ __launch_bounds__(256) void fill_i64_kernel(int64_t* __restrict__ p, int64_t n, int64_t value)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// Regroups A^T by slabs of `slab_rows` source rows (see SlabSet) into the empty set S.  Synchronises the device.
maxk_status build_slabs(maxk_graph* g, SlabSet& S, int32_t slab_rows)
{
    MAXK_HIP_TRY(hipDeviceSynchronize());
    const int64_t N = g->N, nnz = g->nnz;
    const int32_t n_slabs = (int32_t)((N + slab_rows - 1) / slab_rows);
    S.h_slab_visit = (int64_t*)std::calloc((size_t)n_slabs + 1, sizeof(int64_t));
    if (!S.h_slab_visit) return MAXK_OUT_OF_MEMORY;
    S.n_slabs = n_slabs;
    if (nnz == 0) {
        S.slab_rows = slab_rows;
        return MAXK_OK;
    }
    hipStream_t s = nullptr;
    uint64_t *d_key = nullptr, *d_key_sorted = nullptr;
    uint32_t *d_iota = nullptr, *d_perm = nullptr, *d_head = nullptr, *d_rank = nullptr;
    int32_t* d_visit_slab = nullptr;
    int64_t* d_slab_first = nullptr;
    void* d_tmp = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(d_key); (void)hipFree(d_key_sorted); (void)hipFree(d_iota); (void)hipFree(d_perm);
        (void)hipFree(d_head); (void)hipFree(d_rank); (void)hipFree(d_visit_slab); (void)hipFree(d_slab_first);
        (void)hipFree(d_tmp);
    };
#define MAXK_TRY_CLEAN(expr)                                                           \
    do {                                                                               \
        hipError_t _e = (expr);                                                        \
        if (_e != hipSuccess) { cleanup(); free_slabs(S); return hip_fail(_e); }       \
    } while (0)
    // 8 spare entries at the end: the row-accumulating kernel fetches entries eight at a time with scalar loads
    MAXK_TRY_CLEAN(hipMalloc((void**)&S.d_src, sizeof(int32_t) * (size_t)(nnz + 8)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&S.d_val, sizeof(float) * (size_t)(nnz + 8)));
    MAXK_TRY_CLEAN(hipMemsetAsync(S.d_src + nnz, 0, sizeof(int32_t) * 8, s));
    MAXK_TRY_CLEAN(hipMemsetAsync(S.d_val + nnz, 0, sizeof(float) * 8, s));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_key, sizeof(uint64_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_key_sorted, sizeof(uint64_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_iota, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_perm, sizeof(uint32_t) * (size_t)nnz));
    const unsigned blocks = (unsigned)std::min<int64_t>((nnz + 255) / 256, 65536);
    hipLaunchKernelGGL(slab_keys_kernel, dim3(blocks), dim3(256), 0, s, g->d_csc_ptr, g->d_csc_src, N, nnz, slab_rows,
                       d_key, d_iota);
    MAXK_TRY_CLEAN(hipGetLastError());
    int end_bit = 1;
    while (end_bit < 64 && ((uint64_t)1 << end_bit) < (uint64_t)n_slabs * (uint64_t)N) ++end_bit;
    size_t tmp_bytes = 0;
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(nullptr, tmp_bytes, d_key, d_key_sorted, d_iota, d_perm, (size_t)nnz, 0,
                                             (unsigned)end_bit, s));
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(d_tmp, tmp_bytes, d_key, d_key_sorted, d_iota, d_perm, (size_t)nnz, 0,
                                             (unsigned)end_bit, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    (void)hipFree(d_tmp); d_tmp = nullptr;
    (void)hipFree(d_key); d_key = nullptr;
    (void)hipFree(d_iota); d_iota = nullptr;
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_head, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_rank, sizeof(uint32_t) * (size_t)nnz));
    hipLaunchKernelGGL(slab_gather_kernel, dim3(blocks), dim3(256), 0, s, d_perm, d_key_sorted, g->d_csc_src,
                       g->d_csc_val, nnz, S.d_src, S.d_val, d_head);
    MAXK_TRY_CLEAN(hipGetLastError());
    tmp_bytes = 0;
    MAXK_TRY_CLEAN(rocprim::inclusive_scan(nullptr, tmp_bytes, d_head, d_rank, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::inclusive_scan(d_tmp, tmp_bytes, d_head, d_rank, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    uint32_t n_visits32 = 0;
    MAXK_TRY_CLEAN(hipMemcpyAsync(&n_visits32, d_rank + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    const int64_t n_visits = n_visits32;
    MAXK_TRY_CLEAN(hipMalloc((void**)&S.d_visit_node, sizeof(int32_t) * (size_t)n_visits));
    MAXK_TRY_CLEAN(hipMalloc((void**)&S.d_visit_begin, sizeof(int32_t) * (size_t)(n_visits + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_visit_slab, sizeof(int32_t) * (size_t)n_visits));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_slab_first, sizeof(int64_t) * (size_t)(n_slabs + 1)));
    hipLaunchKernelGGL(slab_visits_kernel, dim3(blocks), dim3(256), 0, s, d_head, d_rank, d_key_sorted, N, nnz,
                       S.d_visit_node, S.d_visit_begin, d_visit_slab);
    const int32_t nnz32 = (int32_t)nnz;
    MAXK_TRY_CLEAN(hipMemcpyAsync(S.d_visit_begin + n_visits, &nnz32, sizeof(int32_t), hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(fill_i64_kernel, dim3((unsigned)((n_slabs + 1 + 255) / 256)), dim3(256), 0, s, d_slab_first,
                       (int64_t)n_slabs + 1, n_visits);
    hipLaunchKernelGGL(slab_first_kernel, dim3((unsigned)std::min<int64_t>((n_visits + 255) / 256, 65536)), dim3(256), 0,
                       s, d_visit_slab, n_visits, d_slab_first);
    MAXK_TRY_CLEAN(hipGetLastError());
    MAXK_TRY_CLEAN(hipMemcpyAsync(S.h_slab_visit, d_slab_first, sizeof(int64_t) * (size_t)(n_slabs + 1),
                                  hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    // long visits (hub destinations inside one slab): listed per slab on the host
    {
        std::vector<int32_t> h_begin((size_t)n_visits + 1), h_long;
        MAXK_TRY_CLEAN(hipMemcpy(h_begin.data(), S.d_visit_begin, sizeof(int32_t) * (size_t)(n_visits + 1),
                                 hipMemcpyDeviceToHost));
        S.h_slab_long = (int64_t*)std::calloc((size_t)n_slabs + 1, sizeof(int64_t));
        if (!S.h_slab_long) { cleanup(); free_slabs(S); return MAXK_OUT_OF_MEMORY; }
        for (int32_t sl = 0; sl < n_slabs; ++sl) {
            S.h_slab_long[sl] = (int64_t)h_long.size();
            for (int64_t v = S.h_slab_visit[sl]; v < S.h_slab_visit[sl + 1]; ++v)
                if (h_begin[(size_t)v + 1] - h_begin[(size_t)v] > kSlabLongVisit) h_long.push_back((int32_t)v);
        }
        S.h_slab_long[n_slabs] = (int64_t)h_long.size();
        S.n_long = (int64_t)h_long.size();
        if (S.n_long) {
            MAXK_TRY_CLEAN(hipMalloc((void**)&S.d_long_visit, sizeof(int32_t) * h_long.size()));
            MAXK_TRY_CLEAN(hipMemcpy(S.d_long_visit, h_long.data(), sizeof(int32_t) * h_long.size(), hipMemcpyHostToDevice));
        }

    }
#undef MAXK_TRY_CLEAN
    cleanup();
    S.n_visits = n_visits;
    S.slab_rows = slab_rows;
    return MAXK_OK;
}

// Slab height for hidden width `dim`: a slab of dY should sit comfortably inside one XCD's 4 MB L2.
int32_t slab_rows_for(const maxk_graph* g, int dim, int val_bytes = 4)
{
    const int64_t rows = (int64_t)g->slab_kb * 1024 / ((int64_t)dim * val_bytes);
    return (int32_t)std::max<int64_t>(rows, 64);
}

// The regrouping of A^T for one slab height: built on first use (or by maxk_graph_reserve*), then kept until the
// handle is destroyed, so alternating hidden widths or dY formats on one handle never rebuilds anything.
maxk_status slabs_for(maxk_graph* g, int32_t slab_rows, SlabSet** out)
{
    for (SlabSet* S : g->slab_cache)
        if (S->slab_rows == slab_rows) { *out = S; return MAXK_OK; }
    SlabSet* S = new (std::nothrow) SlabSet();
    if (!S) return MAXK_OUT_OF_MEMORY;
    const maxk_status st = build_slabs(g, *S, slab_rows);
    if (st != MAXK_OK) { delete S; return st; }
    try { g->slab_cache.push_back(S); } catch (const std::bad_alloc&) { free_slabs(*S); delete S; return MAXK_OUT_OF_MEMORY; }
    *out = S;
    return MAXK_OK;
}

maxk_status tiled_for(maxk_graph* g, int dim, int k, TiledSet** out)
{
    TiledShape sh;
    if (!tiled_shape(g->N, dim, k, sh)) return MAXK_UNSUPPORTED;
    for (TiledSet* T : g->tiled_cache)
        if (T->D == sh.D && T->TR == sh.TR && T->LPV == k / tiled_positions_per_lane(k)) { *out = T; return MAXK_OK; }
    TiledSet* T = new (std::nothrow) TiledSet();
    if (!T) return MAXK_OUT_OF_MEMORY;
    const maxk_status st = build_tiled(*T, g->N, g->nnz, g->d_csc_ptr, g->d_csc_src, g->d_csc_val, sh.D, sh.TR, k);
    if (st != MAXK_OK) { delete T; return st; }
    try { g->tiled_cache.push_back(T); } catch (const std::bad_alloc&) { free_tiled(*T); delete T; return MAXK_OUT_OF_MEMORY; }
    *out = T;
    return MAXK_OK;
}

// The forward kernel repacks the CBSR when a row of it is well below a cache line.
bool fwd_uses_packed(const maxk_graph* g, int k, int index_bytes, int val_bytes)
{
    return k * (val_bytes + index_bytes) <= g->fwd_pack_max;
}

maxk_status ensure_packed(maxk_graph* g, int k, int index_bytes, int val_bytes)
{
    const int64_t need = g->N * (int64_t)fwd_packed_record_bytes(k, index_bytes, val_bytes);
    if (need <= g->packed_bytes) return MAXK_OK;
    char* fresh = nullptr;
    MAXK_HIP_TRY(hipMalloc((void**)&fresh, (size_t)need));
    if (g->d_packed) {
        MAXK_HIP_TRY(hipDeviceSynchronize());
        (void)hipFree(g->d_packed);
    }
    g->d_packed = fresh;
    g->packed_bytes = need;
    return MAXK_OK;
}

maxk_status ensure_expand(maxk_graph* g, int k)
{
    const int64_t need = g->nnz * (int64_t)k;
    if (need <= g->expand_floats) return MAXK_OK;
    float* fresh = nullptr;
    MAXK_HIP_TRY(hipMalloc((void**)&fresh, sizeof(float) * (size_t)need));
    if (g->d_expand) {
        MAXK_HIP_TRY(hipDeviceSynchronize());
        (void)hipFree(g->d_expand);
    }
    g->d_expand = fresh;
    g->expand_floats = need;
    return MAXK_OK;
}

// Backward kernel choice when the caller leaves it to the library (rates measured on MI355X).
// Slab pull gathers dY from L2 but re-reads and re-writes a destination's dXs row once per
// (slab, destination) visit, so it needs several in-entries per visit: dense neighbourhoods.
// Otherwise: expand/reduce moves 8k bytes per stored entry through HBM, plain pull touches about
// min(k, dim/32) cache lines of a dY row per entry whatever k is, so pull wins once k is large.
int auto_bwd_mode(const maxk_graph* g, int dim, int k, int val_bytes = 4, bool tiled_ok = true)
{
    const double n_slabs = std::ceil((double)g->N / slab_rows_for(g, dim, val_bytes));
    const double entries_per_visit = (double)g->nnz / std::max(1.0, (double)g->N * n_slabs);
    const double per_line = 128.0 / val_bytes;  // dY elements per cache line
    const double lines = dim <= per_line ? 1.0 : (dim / per_line) * (1.0 - std::pow(1.0 - per_line / dim, (double)k));
    if (entries_per_visit >= 2.0 && n_slabs * (double)g->N < 1.8e19) {
        // Dense neighbourhoods: slab pull or the LDS-tiled kernel, by cost models fitted on the dense and the
        // ogbn-proteins-like workload (256 CUs): slab pull moves the cache lines that an entry's k columns touch (plus
        // ~0.35 lines of streamed arrays) at ~5.2 ps per line, and pays ~10 us per slab launch; the tiled kernel pays
        // ~150 ns per (destination set, tile) step on each CU and ~(3.0 + 0.73 k) ps per entry.  Both models are
        // within 10 % of the measurements from k = 16 up (they run high at k = 8, where the choice is clear).
        TiledShape sh;
        if (tiled_ok && val_bytes == 4 && tiled_shape(g->N, dim, k, sh)) {
            const double n_tiles = std::ceil((double)g->N / sh.TR);
            const double t_slab = (double)g->nnz * (lines + 0.35) * 5.2e-12 + n_slabs * 10e-6;
            const double t_tiled = 150e-9 * sh.n_dsets * n_tiles / 256.0 + (double)g->nnz * (3.0e-12 + 0.73e-12 * k);
            // (graphs of a few thousand nodes: both models miss the fixed costs, and the tiled kernel, one launch,
            // measured faster at every k)
            const double margin = (double)sh.n_dsets * n_tiles < 256.0 * 256.0 ? 0.9 : 1.05;
            if (margin * t_tiled < t_slab && (double)sh.n_dsets * n_tiles < 2.6e8) return MAXK_BWD_TILED;
        }
        return MAXK_BWD_SLAB_PULL;
    }
    // `lines`: expected cache lines of a dY row touched by k sorted columns; measured crossover on four graphs:
    // expand/reduce (8k bytes per entry) beats pull (lines * 128 bytes per entry) while 8k < 44 * lines
    const double pull_cost = lines * 128.0 / 2.9;
    const double expand_cost = 8.0 * k;
    const bool fits = (double)g->nnz * k * 4.0 <= 96e9;
    return (fits && expand_cost < pull_cost) ? MAXK_BWD_EXPAND_REDUCE : MAXK_BWD_PULL_CSC;
}

bool bad_index_bytes(int index_bytes, int dim)
{
    if (index_bytes == 1) return dim > 256;
    if (index_bytes == 2) return dim > 65536;
    return index_bytes != 4;
}

}  // namespace
}  // namespace maxk

using namespace maxk;

extern "C" {

MAXK_API maxk_status maxk_graph_create(maxk_graph** out, int64_t N, int64_t nnz, const int32_t* d_rowptr,
                              const int32_t* d_colidx, const float* d_val, void* stream)
{
    if (!out) return MAXK_INVALID_ARGUMENT;
    *out = nullptr;
    if (N < 0 || nnz < 0 || N > 0x7FFFFFF0ll || nnz > 0x7FFFFFF0ll) return MAXK_INVALID_ARGUMENT;
    if (!d_rowptr || (nnz > 0 && (!d_colidx || !d_val))) return MAXK_INVALID_ARGUMENT;
    if (!aligned(d_rowptr, 4) || !aligned(d_colidx, 4) || !aligned(d_val, 4)) return MAXK_INVALID_ARGUMENT;
    hipStream_t s = (hipStream_t)stream;

    maxk_graph* g = new (std::nothrow) maxk_graph();
    if (!g) return MAXK_OUT_OF_MEMORY;
    g->N = N;
    g->nnz = nnz;
    g->d_rowptr = d_rowptr;
    g->d_col = d_colidx;
    g->d_val = d_val;
    g->chunk = env_int("MAXK_CHUNK", 2048, 64, 1 << 20);  // measured plateau: 2048 and up
    g->slab_kb = env_int("MAXK_SLAB_KB", 3584, 64, 1 << 20);
    g->fwd_pack_max = env_int("MAXK_FWD_PACK_MAX", 96, 0, 1 << 20);
    (void)hipGetDevice(&g->device);
    {
        const maxk_status sst = noalloc_scratch_address(&g->d_noalloc_scratch);
        if (sst != MAXK_OK) { delete g; return sst; }
    }

    maxk_status st = MAXK_OK;
    try {
        std::vector<int32_t> h_rowptr((size_t)N + 1);
        hipError_t e = hipMemcpyAsync(h_rowptr.data(), d_rowptr, sizeof(int32_t) * (size_t)(N + 1), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) { st = hip_fail(e); goto fail; }
        if (h_rowptr[0] != 0 || (int64_t)h_rowptr[(size_t)N] != nnz) { st = MAXK_INVALID_ARGUMENT; goto fail; }
        for (int64_t i = 0; i < N; ++i)
            if (h_rowptr[(size_t)i + 1] < h_rowptr[(size_t)i]) { st = MAXK_INVALID_ARGUMENT; goto fail; }

        std::vector<WorkItem> items;
        std::vector<SplitRow> split;
        int64_t n_slots = 0, max_len = 0;
        build_items(h_rowptr, N, g->chunk, items, split, n_slots, max_len);
        g->max_degree = max_len;
        st = upload_items(items, split, n_slots, g->csr_items, s);
        if (st != MAXK_OK) goto fail;

        std::vector<int32_t> h_csc_ptr;
        st = build_csc(g, h_csc_ptr, s);
        if (st != MAXK_OK) goto fail;
        build_items(h_csc_ptr, N, g->chunk, items, split, n_slots, max_len);
        st = upload_items(items, split, n_slots, g->csc_items, s);
        if (st != MAXK_OK) goto fail;
    } catch (const std::bad_alloc&) {
        st = MAXK_OUT_OF_MEMORY;
        goto fail;
    }
    *out = g;
    return MAXK_OK;
fail:
    maxk_graph_destroy(g);
    return st;
}

MAXK_API maxk_status maxk_graph_destroy(maxk_graph* g)
{
    if (!g) return MAXK_OK;
    (void)hipFree(g->csr_items.d_items);
    (void)hipFree(g->csr_items.d_split);
    (void)hipFree(g->csc_items.d_items);
    (void)hipFree(g->csc_items.d_split);
    (void)hipFree(g->d_csc_ptr);
    (void)hipFree(g->d_csc_src);
    (void)hipFree(g->d_csc_val);
    (void)hipFree(g->d_csc_entry);
    (void)hipFree(g->d_expand);
    (void)hipFree(g->d_packed);
    for (SlabSet* S : g->slab_cache) { free_slabs(*S); delete S; }
    for (TiledSet* T : g->tiled_cache) { free_tiled(*T); delete T; }
    (void)hipFree(g->d_partials);
    delete g;
    return MAXK_OK;
}

MAXK_API maxk_status maxk_graph_reserve_narrow(maxk_graph* g, int32_t dim, int32_t k, int32_t dy_value_type)
{
    if (!g || dim < 1 || k < 1 || k > dim) return MAXK_INVALID_ARGUMENT;
    if (dy_value_type < MAXK_VALUE_F32 || dy_value_type > MAXK_VALUE_F16) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (g->N == 0) return MAXK_OK;
    maxk_status st = ensure_workspace(g, dim, k);
    if (st != MAXK_OK) return st;
    for (int vb = 2; vb <= 4; vb += 2) {
        for (int ib = 1; ib <= 4; ib *= 2) {
            for (int kk = 1; kk <= k; ++kk) {  // the largest repacked record among k' <= k
                if (!fwd_uses_packed(g, kk, ib, vb)) break;
                if (kk == k || !fwd_uses_packed(g, kk + 1, ib, vb)) {
                    st = ensure_packed(g, kk, ib, vb);
                    if (st != MAXK_OK) return st;
                }
            }
        }
    }
    const int vb = value_bytes(dy_value_type);
    const int mode = g->bwd_mode == MAXK_BWD_AUTO ? auto_bwd_mode(g, dim, k, vb) : g->bwd_mode;
    if (mode == MAXK_BWD_TILED) {
        TiledSet* T = nullptr;
        st = tiled_for(g, dim, k, &T);
        if (st != MAXK_UNSUPPORTED) return st;
        // the compute call falls back to the slab kernel for shapes the tiled one does not take
    }
    if (mode == MAXK_BWD_SLAB_PULL || mode == MAXK_BWD_TILED) {
        SlabSet* S = nullptr;
        return g->nnz ? slabs_for(g, slab_rows_for(g, dim, vb), &S) : MAXK_OK;
    }
    return mode == MAXK_BWD_EXPAND_REDUCE ? ensure_expand(g, k) : MAXK_OK;
}

MAXK_API maxk_status maxk_graph_reserve(maxk_graph* g, int32_t dim, int32_t k)
{
    return maxk_graph_reserve_narrow(g, dim, k, MAXK_VALUE_F32);
}

MAXK_API maxk_status maxk_graph_set_bwd_mode(maxk_graph* g, int32_t mode)
{
    if (!g || mode < MAXK_BWD_AUTO || mode > MAXK_BWD_TILED) return MAXK_INVALID_ARGUMENT;
    g->bwd_mode = mode;
    return MAXK_OK;
}

MAXK_API int32_t maxk_graph_bwd_choice(const maxk_graph* g, int32_t dim, int32_t k)
{
    if (!g || dim < 1 || k < 1 || k > dim) return MAXK_INVALID_ARGUMENT;
    return g->bwd_mode == MAXK_BWD_AUTO ? auto_bwd_mode(g, dim, k) : g->bwd_mode;
}

MAXK_API maxk_status maxk_graph_info(const maxk_graph* g, int64_t* N, int64_t* nnz, int64_t* n_fwd_items, int64_t* n_split_rows,
                            int64_t* max_degree, int64_t* workspace_bytes)
{
    if (!g) return MAXK_INVALID_ARGUMENT;
    if (N) *N = g->N;
    if (nnz) *nnz = g->nnz;
    if (n_fwd_items) *n_fwd_items = g->csr_items.n_items;
    if (n_split_rows) *n_split_rows = g->csr_items.n_split;
    if (max_degree) *max_degree = g->max_degree;
    if (workspace_bytes)
        *workspace_bytes = (g->partial_floats + g->expand_floats) * (int64_t)sizeof(float) + g->packed_bytes;
    return MAXK_OK;
}

MAXK_API maxk_status maxk_topk_cbsr_narrow(const float* d_H, int64_t N, int32_t dim, int32_t k, void* d_sp_data,
                                           int32_t value_type, void* d_sp_index, int32_t index_bytes, void* stream)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim || bad_index_bytes(index_bytes, dim)) return MAXK_INVALID_ARGUMENT;
    if (value_type < MAXK_VALUE_F32 || value_type > MAXK_VALUE_F16) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (N > 0x7FFFFFF0ll) return MAXK_INVALID_ARGUMENT;
    if (N == 0) return MAXK_OK;
    if (!d_H || !d_sp_data || !d_sp_index) return MAXK_INVALID_ARGUMENT;
    if (!aligned(d_H, 4) || !aligned(d_sp_data, (size_t)value_bytes(value_type)) ||
        !aligned(d_sp_index, (size_t)index_bytes))
        return MAXK_INVALID_ARGUMENT;
    return launch_topk(d_H, N, dim, k, d_sp_data, value_type, d_sp_index, index_bytes, (hipStream_t)stream);
}

MAXK_API maxk_status maxk_topk_cbsr(const float* d_H, int64_t N, int32_t dim, int32_t k, float* d_sp_data, void* d_sp_index,
                           int32_t index_bytes, void* stream)
{
    return maxk_topk_cbsr_narrow(d_H, N, dim, k, d_sp_data, MAXK_VALUE_F32, d_sp_index, index_bytes, stream);
}

MAXK_API maxk_status maxk_spgemm_fwd_narrow(maxk_graph* g, const void* d_sp_data, int32_t value_type,
                                            const void* d_sp_index, int32_t index_bytes, int32_t dim, int32_t k,
                                            float* d_Y, void* stream)
{
    if (!g || dim < 1 || k < 1 || k > dim || bad_index_bytes(index_bytes, dim)) return MAXK_INVALID_ARGUMENT;
    if (value_type < MAXK_VALUE_F32 || value_type > MAXK_VALUE_F16) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (g->N == 0) return MAXK_OK;
    if (!d_sp_data || !d_sp_index || !d_Y) return MAXK_INVALID_ARGUMENT;
    const int vb = value_bytes(value_type);
    if (!aligned(d_sp_data, (size_t)vb) || !aligned(d_Y, 4) || !aligned(d_sp_index, (size_t)index_bytes))
        return MAXK_INVALID_ARGUMENT;
    maxk_status st = ensure_workspace(g, dim, k);
    if (st != MAXK_OK) return st;
    char* packed = nullptr;
    if (fwd_uses_packed(g, k, index_bytes, vb)) {
        st = ensure_packed(g, k, index_bytes, vb);
        if (st != MAXK_OK) return st;
        packed = g->d_packed;
    }
    return launch_spgemm_fwd(g->csr_items, g->d_col, g->d_val, d_sp_data, value_type, d_sp_index, index_bytes, g->N, packed,
                             dim, k, d_Y, g->d_partials, (hipStream_t)stream);
}

MAXK_API maxk_status maxk_spgemm_fwd(maxk_graph* g, const float* d_sp_data, const void* d_sp_index, int32_t index_bytes,
                            int32_t dim, int32_t k, float* d_Y, void* stream)
{
    return maxk_spgemm_fwd_narrow(g, d_sp_data, MAXK_VALUE_F32, d_sp_index, index_bytes, dim, k, d_Y, stream);
}

MAXK_API maxk_status maxk_spgemm_fwd_noalloc(maxk_graph* g, const float* d_sp_data, const void* d_sp_index,
                                             int32_t index_bytes, int32_t dim, int32_t k, float* d_Y, void* stream)
{
    if (!g || dim < 1 || k < 1 || k > dim || bad_index_bytes(index_bytes, dim)) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (g->N == 0) return MAXK_OK;
    if (!d_sp_data || !d_sp_index || !d_Y) return MAXK_INVALID_ARGUMENT;
    if (!aligned(d_sp_data, 4) || !aligned(d_Y, 4) || !aligned(d_sp_index, (size_t)index_bytes)) return MAXK_INVALID_ARGUMENT;
    int device = -1;
    MAXK_HIP_TRY(hipGetDevice(&device));
    if (device != g->device || !g->d_noalloc_scratch) return MAXK_INVALID_ARGUMENT;  // the array is per GPU
    // layout of the scratch array: [partial rows of split rows | repacked CBSR, if it fits]
    const int64_t partial_bytes = (g->csr_items.n_slots * (int64_t)dim * 4 + 255) & ~(int64_t)255;
    if (partial_bytes > (int64_t)MAXK_NOALLOC_SCRATCH_BYTES) return MAXK_SCRATCH_TOO_SMALL;
    float* partials = reinterpret_cast<float*>(g->d_noalloc_scratch);
    char* packed = nullptr;
    if (fwd_uses_packed(g, k, index_bytes, 4) &&
        partial_bytes + g->N * (int64_t)fwd_packed_record_bytes(k, index_bytes, 4) <= (int64_t)MAXK_NOALLOC_SCRATCH_BYTES)
        packed = reinterpret_cast<char*>(g->d_noalloc_scratch) + partial_bytes;
    // nothing in the array has to start at zero: the kernels write every partial row and every record they read
    return launch_spgemm_fwd(g->csr_items, g->d_col, g->d_val, d_sp_data, MAXK_VALUE_F32, d_sp_index, index_bytes, g->N,
                             packed, dim, k, d_Y, partials, (hipStream_t)stream);
}

MAXK_API maxk_status maxk_sspmm_bwd_narrow(maxk_graph* g, const void* d_dY, int32_t value_type, const void* d_sp_index,
                                           int32_t index_bytes, int32_t dim, int32_t k, float* d_dXs, void* stream)
{
    if (!g || dim < 1 || k < 1 || k > dim || bad_index_bytes(index_bytes, dim)) return MAXK_INVALID_ARGUMENT;
    if (value_type < MAXK_VALUE_F32 || value_type > MAXK_VALUE_F16) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (g->N == 0) return MAXK_OK;
    if (!d_dY || !d_sp_index || !d_dXs) return MAXK_INVALID_ARGUMENT;
    const int vb = value_bytes(value_type);
    if (!aligned(d_dY, (size_t)vb) || !aligned(d_dXs, 4) || !aligned(d_sp_index, (size_t)index_bytes))
        return MAXK_INVALID_ARGUMENT;
    maxk_status st = ensure_workspace(g, dim, k);
    if (st != MAXK_OK) return st;
    int mode = g->bwd_mode;
    const bool tiled_ok = tiled_supports(d_dY, value_type, d_sp_index, index_bytes, dim, k);
    if (mode == MAXK_BWD_AUTO) mode = auto_bwd_mode(g, dim, k, vb, tiled_ok);
    if (g->nnz == 0) return launch_fill_zero(d_dXs, g->N * (int64_t)k, (hipStream_t)stream);
    if (mode == MAXK_BWD_TILED) {
        TiledSet* T = nullptr;
        st = tiled_ok ? tiled_for(g, dim, k, &T) : MAXK_UNSUPPORTED;
        if (st == MAXK_OK)
            return launch_bwd_tiled(*T, d_dY, value_type, d_sp_index, index_bytes, g->N, dim, k, d_dXs, (hipStream_t)stream);
        if (st != MAXK_UNSUPPORTED) return st;
        mode = MAXK_BWD_SLAB_PULL;  // shapes, formats and alignments the tiled kernel does not take
    }
    if (mode == MAXK_BWD_SLAB_PULL) {
        SlabSet* S = nullptr;
        st = slabs_for(g, slab_rows_for(g, dim, vb), &S);
        if (st != MAXK_OK) return st;
        return launch_bwd_slab_pull(*S, d_dY, value_type, d_sp_index, index_bytes, g->N, dim, k, d_dXs, (hipStream_t)stream);
    }
    if (mode == MAXK_BWD_EXPAND_REDUCE) {
        st = ensure_expand(g, k);
        if (st != MAXK_OK) return st;
        return launch_bwd_expand_reduce(g->csr_items, g->d_col, g->d_val, g->csc_items, g->d_csc_entry, d_dY, value_type,
                                        d_sp_index, index_bytes, dim, k, g->d_expand, d_dXs, g->d_partials,
                                        (hipStream_t)stream);
    }
    if (mode == MAXK_BWD_PULL_CSC)
        return launch_bwd_pull(g->csc_items, g->d_csc_src, g->d_csc_val, d_dY, value_type, d_sp_index, index_bytes, dim, k,
                               d_dXs, g->d_partials, (hipStream_t)stream);
    return launch_bwd_push(g->csr_items, g->d_col, g->d_val, d_dY, value_type, d_sp_index, index_bytes, g->N, dim, k, d_dXs,
                           (hipStream_t)stream);
}

MAXK_API maxk_status maxk_sspmm_bwd(maxk_graph* g, const float* d_dY, const void* d_sp_index, int32_t index_bytes, int32_t dim,
                           int32_t k, float* d_dXs, void* stream)
{
    return maxk_sspmm_bwd_narrow(g, d_dY, MAXK_VALUE_F32, d_sp_index, index_bytes, dim, k, d_dXs, stream);
}

MAXK_API maxk_status maxk_cbsr_scatter(const float* d_values, const void* d_sp_index, int32_t index_bytes, int64_t N,
                                       int32_t dim, int32_t k, float* d_dense, void* stream)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim || bad_index_bytes(index_bytes, dim)) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (N > 0x7FFFFFF0ll) return MAXK_INVALID_ARGUMENT;
    if (N == 0) return MAXK_OK;
    if (!d_values || !d_sp_index || !d_dense) return MAXK_INVALID_ARGUMENT;
    if (!aligned(d_values, 4) || !aligned(d_dense, 4) || !aligned(d_sp_index, (size_t)index_bytes))
        return MAXK_INVALID_ARGUMENT;
    return launch_cbsr_scatter(d_values, d_sp_index, index_bytes, N, dim, k, d_dense, (hipStream_t)stream);
}

MAXK_API maxk_status spmm_baseline(maxk_graph* g, const float* d_H, int32_t dim, float* d_Y, void* stream)
{
    if (!g || dim < 1) return MAXK_INVALID_ARGUMENT;
    if (dim > MAXK_MAX_DIM) return MAXK_UNSUPPORTED;
    if (g->N == 0) return MAXK_OK;
    if (!d_H || !d_Y || !aligned(d_H, 4) || !aligned(d_Y, 4)) return MAXK_INVALID_ARGUMENT;
    maxk_status st = ensure_workspace(g, dim, 1);
    if (st != MAXK_OK) return st;
    return launch_spmm(g->csr_items, g->d_col, g->d_val, d_H, dim, d_Y, g->d_partials, (hipStream_t)stream);
}

MAXK_API const char* maxk_status_string(maxk_status s)
{
    switch (s) {
        case MAXK_OK: return "ok";
        case MAXK_INVALID_ARGUMENT: return "invalid argument";
        case MAXK_UNSUPPORTED: return "unsupported size";
        case MAXK_HIP_ERROR: return "HIP runtime error";
        case MAXK_OUT_OF_MEMORY: return "out of device or host memory";
        case MAXK_SCRATCH_TOO_SMALL: return "the input needs more scratch memory than the library's fixed array holds";
        default: return "unknown status";
    }
}

MAXK_API int32_t maxk_fwd_private_copies(int32_t k) { return k < 1 ? MAXK_INVALID_ARGUMENT : fwd_private_copies(k); }

MAXK_API maxk_status maxk_graph_cached_tables(const maxk_graph* g, int32_t* n_slab_tables, int32_t* n_tiled_tables)
{
    if (!g) return MAXK_INVALID_ARGUMENT;
    if (n_slab_tables) *n_slab_tables = (int32_t)g->slab_cache.size();
    if (n_tiled_tables) *n_tiled_tables = (int32_t)g->tiled_cache.size();
    return MAXK_OK;
}

int32_t maxk_last_hip_error(void) { return g_last_hip_error; }

MAXK_API int32_t maxk_version(void) { return 100; }

}  // extern "C"
