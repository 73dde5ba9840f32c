// Dense-feature SpMM Y = A * H: the operator the paper measures its speedups
// against (Sec. 5.2), as a same-GPU baseline on the same work-item lists.
//
// One wavefront per work item; each lane keeps its slice of the output row in
// registers (float4 per 256 columns), every stored entry costs one coalesced
// read of a full H row, UNR entries in flight.  No LDS, no atomics; rows longer
// than the chunk go through the same partial-row combine as the forward kernel.
#include "common.hpp"

namespace maxk {
namespace {

constexpr int kUnroll = 8;

// R float4 accumulators per lane: dim <= 256 * R, dim % 4 == 0
template <int R>
__global__ __launch_bounds__(kWave) void spmm_vec_kernel(const WorkItem* __restrict__ items,
                                                         const int32_t* __restrict__ col,
                                                         const float* __restrict__ val, const float* __restrict__ H,
                                                         int dim, float* __restrict__ Y, float* __restrict__ partials)
{
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    float4 acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int p = it.begin; p < it.end; p += kUnroll) {
        float4 h[kUnroll][R];
        float a[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool ok = p + u < it.end;
            const int q = ok ? p + u : it.begin;
            a[u] = ok ? val[q] : 0.f;
            const float* __restrict__ hr = H + (int64_t)col[q] * dim;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int c = r * 256 + lane * 4;
                h[u][r] = (ok && c < dim) ? *reinterpret_cast<const float4*>(hr + c) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc[r].x += a[u] * h[u][r].x;
                acc[r].y += a[u] * h[u][r].y;
                acc[r].z += a[u] * h[u][r].z;
                acc[r].w += a[u] * h[u][r].w;
            }
        }
    }
    float* __restrict__ out = (it.slot < 0) ? Y + (int64_t)it.row * dim : partials + (int64_t)it.slot * dim;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * 256 + lane * 4;
        if (c < dim) *reinterpret_cast<float4*>(out + c) = acc[r];
    }
}

// any dim <= 64 * R, scalar loads
template <int R>
__global__ __launch_bounds__(kWave) void spmm_scalar_kernel(const WorkItem* __restrict__ items,
                                                            const int32_t* __restrict__ col,
                                                            const float* __restrict__ val,
                                                            const float* __restrict__ H, int dim,
                                                            float* __restrict__ Y, float* __restrict__ partials)
{
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    for (int p = it.begin; p < it.end; ++p) {
        const float a = val[p];
        const float* __restrict__ hr = H + (int64_t)col[p] * dim;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kWave + lane;
            if (c < dim) acc[r] += a * hr[c];
        }
    }
    float* __restrict__ out = (it.slot < 0) ? Y + (int64_t)it.row * dim : partials + (int64_t)it.slot * dim;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kWave + lane;
        if (c < dim) out[c] = acc[r];
    }
}

}  // namespace

maxk_status launch_spmm(const ItemList& L, const int32_t* col, const float* val, const float* H, int dim, float* Y,
                        float* partials, hipStream_t s)
{
    if (L.n_items == 0) return MAXK_OK;
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)L.n_items), block(kWave);
#define MAXK_SPMM(KERNEL) hipLaunchKernelGGL((KERNEL), grid, block, 0, s, L.d_items, col, val, H, dim, Y, partials)
    if (dim % 4 == 0 && aligned(H, 16) && aligned(Y, 16)) {
        if (dim <= 256) MAXK_SPMM(spmm_vec_kernel<1>);
        else if (dim <= 512) MAXK_SPMM(spmm_vec_kernel<2>);
        else MAXK_SPMM(spmm_vec_kernel<4>);
    } else {
        if (dim <= 256) MAXK_SPMM(spmm_scalar_kernel<4>);
        else if (dim <= 512) MAXK_SPMM(spmm_scalar_kernel<8>);
        else MAXK_SPMM(spmm_scalar_kernel<16>);
    }
#undef MAXK_SPMM
    MAXK_LAUNCH_CHECK();
    return launch_combine(L, partials, dim, Y, s);
}

}  // namespace maxk
