// Backward aggregation (Eq. 2 right; Eq. 3): dispatch over the storage format of dY, plus the pieces that
// do not read dY (clearing dXs, phase 2 of expand/reduce).  The kernels that read dY are in sspmm_bwd_impl.hpp.
#include "sspmm_bwd_impl.hpp"

namespace maxk {
namespace {

constexpr int kReduceUnroll = 4;

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

// Phase 2: dXs[j, :] = sum of the product rows of j's in-entries.  VEC = floats per lane (4 or 1);
// LPE = lanes per entry (power of two >= k / VEC, at most 64); 64 / LPE entries per wave instruction.
template <int VEC, int LPE>
__global__ __launch_bounds__(kWave) void bwd_reduce_kernel(const WorkItem* __restrict__ items,
                                                           const uint32_t* __restrict__ csc_entry,
                                                           const float* __restrict__ expand, int k,
                                                           float* __restrict__ dXs, float* __restrict__ partials)
{
    constexpr int G = kWave / LPE;
    const int lane = threadIdx.x;
    const int q = lane % LPE, g = lane / LPE;
    const int kq = k / VEC;  // lanes' worth of work per entry
    const WorkItem it = items[blockIdx.x];
    float* __restrict__ out = (it.slot < 0) ? dXs + (int64_t)it.row * k : partials + (int64_t)it.slot * k;
    for (int qq = q; qq < ((kq + LPE - 1) / LPE) * LPE; qq += LPE) {  // one pass unless k / VEC > 64
        const bool active = qq < kq;
        float acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
        for (int p0 = it.begin; p0 < it.end; p0 += G * kReduceUnroll) {
            float v[kReduceUnroll][VEC];
#pragma unroll
            for (int u = 0; u < kReduceUnroll; ++u) {
                const int p = p0 + u * G + g;
                const bool ok = active && p < it.end;
                const float* __restrict__ src = expand + (int64_t)csc_entry[ok ? p : it.begin] * k + (ok ? qq : 0) * VEC;
                if constexpr (VEC == 4) {
                    const float4 x = ok ? *reinterpret_cast<const float4*>(src) : make_float4(0.f, 0.f, 0.f, 0.f);
                    v[u][0] = x.x; v[u][1] = x.y; v[u][2] = x.z; v[u][3] = x.w;
                } else {
                    v[u][0] = ok ? *src : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < kReduceUnroll; ++u)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] += v[u][j];
        }
#pragma unroll
        for (int off = LPE; off < kWave; off <<= 1)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] += __shfl_xor(acc[j], off);
        if (g == 0 && active) {
            if constexpr (VEC == 4) *reinterpret_cast<float4*>(out + qq * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            else out[qq] = acc[0];
        }
    }
}

template <int VEC>
maxk_status launch_reduce_v(const ItemList& L, const uint32_t* csc_entry, const float* expand, int k, float* dXs,
                            float* partials, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
    const int kq = k / VEC;
#define MAXK_REDUCE(LPE) \
    hipLaunchKernelGGL((bwd_reduce_kernel<VEC, LPE>), grid, block, 0, s, L.d_items, csc_entry, expand, k, dXs, partials)
    if (kq <= 1) MAXK_REDUCE(1);
    else if (kq <= 2) MAXK_REDUCE(2);
    else if (kq <= 4) MAXK_REDUCE(4);
    else if (kq <= 8) MAXK_REDUCE(8);
    else if (kq <= 16) MAXK_REDUCE(16);
    else if (kq <= 32) MAXK_REDUCE(32);
    else MAXK_REDUCE(64);
#undef MAXK_REDUCE
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

#define MAXK_BY_FORMAT(FN, ...)                                                        \
    (value_type == MAXK_VALUE_BF16 ? FN<MAXK_VALUE_BF16>(__VA_ARGS__)                  \
     : value_type == MAXK_VALUE_F16 ? FN<MAXK_VALUE_F16>(__VA_ARGS__) : FN<MAXK_VALUE_F32>(__VA_ARGS__))

}  // namespace

maxk_status launch_bwd_pull(const ItemList& L, const int32_t* csc_src, const float* csc_val, const void* dY,
                            int value_type, const void* sp_index, int index_bytes, int dim, int k, float* dXs,
                            float* partials, hipStream_t s)
{
    if (L.n_items == 0) return MAXK_OK;
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    const maxk_status st = MAXK_BY_FORMAT(bwd_pull_format, L, csc_src, csc_val, dY, sp_index, index_bytes, dim, k, dXs, partials, s);
    if (st != MAXK_OK) return st;
    return launch_combine(L, partials, k, dXs, s);
}

maxk_status launch_bwd_push(const ItemList& L, const int32_t* col, const float* val, const void* dY, int value_type,
                            const void* sp_index, int index_bytes, int64_t N, int dim, int k, float* dXs,
                            hipStream_t s)
{
    const maxk_status st = launch_fill_zero(dXs, N * (int64_t)k, s);
    if (st != MAXK_OK || N * (int64_t)k == 0 || L.n_items == 0) return st;
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    return MAXK_BY_FORMAT(bwd_push_format, L, col, val, dY, sp_index, index_bytes, dim, k, dXs, s);
}

maxk_status launch_bwd_expand_reduce(const ItemList& csr_items, const int32_t* col, const float* val,
                                     const ItemList& csc_items, const uint32_t* csc_entry, const void* dY,
                                     int value_type, const void* sp_index, int index_bytes, int dim, int k,
                                     float* expand, float* dXs, float* partials, hipStream_t s)
{
    if (csc_items.n_items == 0) return MAXK_OK;
    if (csr_items.n_items > 0x7FFFFFFF || csc_items.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    maxk_status st = MAXK_OK;
    if (csr_items.n_items) {
        st = MAXK_BY_FORMAT(bwd_expand_format, csr_items, col, val, dY, sp_index, index_bytes, dim, k, expand, s);
        if (st != MAXK_OK) return st;
    }
    if (k % 4 == 0 && aligned(dXs, 16) && aligned(expand, 16)) st = launch_reduce_v<4>(csc_items, csc_entry, expand, k, dXs, partials, s);
    else st = launch_reduce_v<1>(csc_items, csc_entry, expand, k, dXs, partials, s);
    if (st != MAXK_OK) return st;
    return launch_combine(csc_items, partials, k, dXs, s);
}

maxk_status launch_fill_zero(float* p, int64_t n, hipStream_t s)
{
    if (n <= 0) return MAXK_OK;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

maxk_status launch_bwd_slab_pull(const SlabSet& S, const void* dY, int value_type, const void* sp_index,
                                 int index_bytes, int64_t N, int dim, int k, float* dXs, hipStream_t s)
{
    const maxk_status st = launch_fill_zero(dXs, N * (int64_t)k, s);
    if (st != MAXK_OK || S.n_visits == 0) return st;
    return MAXK_BY_FORMAT(bwd_slab_format, S, dY, sp_index, index_bytes, N, dim, k, dXs, s);
}

}  // namespace maxk
