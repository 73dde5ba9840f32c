// Forward aggregation: row-wise-product SpGEMM with dense output
// (Eq. 2 left; Sec. 3.2 "Forward Computation"; prior art: Alg. 1).
//
// One 64-lane wavefront (= one workgroup, so no cross-wave barrier exists)
// owns one work item: a run of at most `chunk` stored entries of one row of A.
// It keeps the dense output row (dim floats) in LDS, streams the item's
// (col, val) pairs 64 at a time into registers with one coalesced load each,
// and walks a FLAT list of units (entry, quad) -- unit u belongs to entry
// u / (k/4) and covers CBSR positions 4*(u % (k/4)) .. +3 -- so all 64 lanes
// stay busy for every k that is a multiple of 4: each lane fetches one float4
// of sp_data and its 4 indices with one load each, U rounds in flight before
// the first LDS update.  The scatter-add into the row buffer is ds_add_f32.
// Rows longer than `chunk` write partial rows that a second kernel adds up
// (deterministic order, and it bounds the length of any fp32 running sum);
// every other row is written once, straight from LDS, fully coalesced.
#include "common.hpp"

namespace maxk {
namespace {

template <typename IdxT, int VEC>
struct IdxVec;
template <>
struct IdxVec<uint8_t, 4> {
    uint32_t w;
    __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint32_t*>(p); }
    __device__ __forceinline__ int get(int i) const { return (w >> (8 * i)) & 0xFFu; }
};
template <>
struct IdxVec<uint16_t, 4> {
    uint2 w;
    __device__ __forceinline__ void load(const uint16_t* p) { w = *reinterpret_cast<const uint2*>(p); }
    __device__ __forceinline__ int get(int i) const { return ((i < 2 ? w.x : w.y) >> (16 * (i & 1))) & 0xFFFFu; }
};
template <>
struct IdxVec<int32_t, 4> {
    int4 w;
    __device__ __forceinline__ void load(const int32_t* p) { w = *reinterpret_cast<const int4*>(p); }
    __device__ __forceinline__ int get(int i) const { return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w; }
};
template <typename IdxT>
struct IdxVec<IdxT, 1> {
    int w;
    __device__ __forceinline__ void load(const IdxT* p) { w = (int)*p; }
    __device__ __forceinline__ int get(int) const { return w; }
};

template <int VEC>
struct ValVec;
template <>
struct ValVec<4> {
    float4 w;
    __device__ __forceinline__ void load(const float* p) { w = *reinterpret_cast<const float4*>(p); }
    __device__ __forceinline__ float get(int i) const { return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w; }
};
template <>
struct ValVec<1> {
    float w;
    __device__ __forceinline__ void load(const float* p) { w = *p; }
    __device__ __forceinline__ float get(int) const { return w; }
};

constexpr int kRounds = 4;  // unit rounds in flight per wavefront

// VEC: CBSR entries per unit (4 when k % 4 == 0 and pointers are 16-byte aligned, else 1)
// KU : units per stored entry (k / VEC) when known at compile time, 0 = runtime
template <int VEC, int KU, typename IdxT>
__global__ __launch_bounds__(kWave) void spgemm_fwd_kernel(const WorkItem* __restrict__ items,
                                                           const int32_t* __restrict__ col,
                                                           const float* __restrict__ val,
                                                           const float* __restrict__ sp_data,
                                                           const IdxT* __restrict__ sp_index, int dim, int k, int ku_rt,
                                                           float* __restrict__ Y, float* __restrict__ partials)
{
    extern __shared__ float row_buf[];
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    for (int c = lane; c < dim; c += kWave) row_buf[c] = 0.f;
    __syncthreads();

    const int ku = KU ? KU : ku_rt;
    for (int base = it.begin; base < it.end; base += kWave) {
        const int n = min(kWave, it.end - base);
        int my_col = 0;
        float my_val = 0.f;
        if (lane < n) {
            my_col = col[base + lane];
            my_val = val[base + lane];
        }
        const int units = n * ku;
        for (int u0 = 0; u0 < units; u0 += kWave * kRounds) {
            ValVec<VEC> d[kRounds];
            IdxVec<IdxT, VEC> ix[kRounds];
            float a[kRounds];
            bool ok[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int u = u0 + r * kWave + lane;
                ok[r] = u < units;
                const int uc = ok[r] ? u : 0;
                const int e = uc / ku;
                const int q = uc - e * ku;
                const int c = __shfl(my_col, e);
                a[r] = __shfl(my_val, e);
                const int64_t off = (int64_t)c * k + q * VEC;
                d[r].load(sp_data + off);
                ix[r].load(sp_index + off);
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                if (ok[r]) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) atomicAdd(&row_buf[ix[r].get(j)], a[r] * d[r].get(j));
                }
            }
        }
    }
    __syncthreads();

    float* __restrict__ out = (it.slot < 0) ? Y + (int64_t)it.row * dim : partials + (int64_t)it.slot * dim;
    if ((dim & 3) == 0) {
        for (int c = lane * 4; c < dim; c += kWave * 4)
            *reinterpret_cast<float4*>(out + c) = *reinterpret_cast<const float4*>(row_buf + c);
    } else {
        for (int c = lane; c < dim; c += kWave) out[c] = row_buf[c];
    }
}

// out[row, c] = sum over the row's partial slots
__global__ __launch_bounds__(256) void combine_kernel(const SplitRow* __restrict__ split, int64_t n_split,
                                                      const float* __restrict__ partials, int width,
                                                      float* __restrict__ out)
{
    const int64_t r = blockIdx.x;
    if (r >= n_split) return;
    const SplitRow sr = split[r];
    for (int c = threadIdx.x; c < width; c += blockDim.x) {
        float acc = 0.f;
        const float* p = partials + (int64_t)sr.slot_begin * width + c;
        for (int s = 0; s < sr.slot_count; ++s) acc += p[(int64_t)s * width];
        out[(int64_t)sr.row * width + c] = acc;
    }
}

template <int VEC, typename IdxT>
maxk_status launch_ku(const ItemList& L, const int32_t* col, const float* val, const float* sp_data,
                      const IdxT* sp_index, int dim, int k, float* Y, float* partials, hipStream_t s)
{
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)L.n_items), block(kWave);
    const size_t lds = sizeof(float) * (size_t)dim;
    const int ku = k / VEC;
#define MAXK_FWD_CASE(KU)                                                                                          \
    hipLaunchKernelGGL((spgemm_fwd_kernel<VEC, KU, IdxT>), grid, block, lds, s, L.d_items, col, val, sp_data,      \
                       sp_index, dim, k, ku, Y, partials)
    if (VEC == 4) {
        switch (ku) {
            case 2: MAXK_FWD_CASE(2); break;
            case 4: MAXK_FWD_CASE(4); break;
            case 8: MAXK_FWD_CASE(8); break;
            case 16: MAXK_FWD_CASE(16); break;
            case 24: MAXK_FWD_CASE(24); break;
            case 32: MAXK_FWD_CASE(32); break;
            case 48: MAXK_FWD_CASE(48); break;
            default: MAXK_FWD_CASE(0); break;
        }
    } else {
        MAXK_FWD_CASE(0);
    }
#undef MAXK_FWD_CASE
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

}  // namespace

maxk_status launch_combine(const ItemList& L, const float* partials, int width, float* out, hipStream_t s)
{
    if (L.n_split == 0) return MAXK_OK;
    if (L.n_split > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)L.n_split), dim3(256), 0, s, L.d_split, L.n_split, partials,
                       width, out);
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

maxk_status launch_spgemm_fwd(const ItemList& L, const int32_t* col, const float* val, const float* sp_data,
                              const void* sp_index, int index_bytes, int dim, int k, float* Y, float* partials,
                              hipStream_t s)
{
    if (L.n_items == 0) return MAXK_OK;
    const bool vec = (k % 4 == 0) && aligned(sp_data, 16) && aligned(sp_index, (size_t)(4 * index_bytes));
    maxk_status st;
    if (vec) {
        if (index_bytes == 1) st = launch_ku<4>(L, col, val, sp_data, (const uint8_t*)sp_index, dim, k, Y, partials, s);
        else if (index_bytes == 2) st = launch_ku<4>(L, col, val, sp_data, (const uint16_t*)sp_index, dim, k, Y, partials, s);
        else st = launch_ku<4>(L, col, val, sp_data, (const int32_t*)sp_index, dim, k, Y, partials, s);
    } else {
        if (index_bytes == 1) st = launch_ku<1>(L, col, val, sp_data, (const uint8_t*)sp_index, dim, k, Y, partials, s);
        else if (index_bytes == 2) st = launch_ku<1>(L, col, val, sp_data, (const uint16_t*)sp_index, dim, k, Y, partials, s);
        else st = launch_ku<1>(L, col, val, sp_data, (const int32_t*)sp_index, dim, k, Y, partials, s);
    }
    if (st != MAXK_OK) return st;
    return launch_combine(L, partials, dim, Y, s);
}

}  // namespace maxk
