// Backward aggregation: sampled SSpMM  dXs = (A^T dY) at each row's CBSR columns
// (Eq. 2 right; Eq. 3; prior art: Alg. 2).  Two kernels with the same result:
//
//  pull (owner computes, A^T stored as CSC): one wavefront owns a run of the
//    in-entries of destination node j; lane t keeps sp_index[j,t] and a running
//    sum in registers and gathers dY[i, sp_index[j,t]] for each in-entry (i -> j).
//    No atomics, deterministic, but every entry touches up to min(k, dim/32)
//    cache lines of a dY row for only 4k useful bytes.
//
//  push (the dataflow of Alg. 2): one wavefront stages dY[i,:] in LDS with one
//    coalesced read, then walks row i of A; for entry (i -> j) it reads
//    sp_index[j,:] (contiguous), gathers from LDS and adds val * dY[i, idx] into
//    dXs[j,:] with hardware fp32 atomics (contiguous 4k bytes per entry).
//    Needs no transposed copy of A; dXs is cleared first by a fill kernel.
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include "common.hpp"

namespace maxk {
namespace {

constexpr int kPullUnroll = 4;

// ---------------------------------------------------------------- pull ----

// k <= 64: KP = power of two >= k lanes per in-entry, 64/KP entries per step
template <int KP, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_pull_small_kernel(const WorkItem* __restrict__ items,
                                                               const int32_t* __restrict__ csc_src,
                                                               const float* __restrict__ csc_val,
                                                               const float* __restrict__ dY,
                                                               const IdxT* __restrict__ sp_index, int dim, int k,
                                                               float* __restrict__ dXs, float* __restrict__ partials)
{
    constexpr int G = kWave / KP;
    const int lane = threadIdx.x;
    const int t = lane % KP, g = lane / KP;
    const WorkItem it = items[blockIdx.x];
    const bool active = t < k;
    const int my_idx = active ? (int)sp_index[(int64_t)it.row * k + t] : 0;
    float acc = 0.f;
    for (int p0 = it.begin; p0 < it.end; p0 += G * kPullUnroll) {
        float gv[kPullUnroll], a[kPullUnroll];
#pragma unroll
        for (int u = 0; u < kPullUnroll; ++u) {
            const int p = p0 + u * G + g;
            const bool ok = p < it.end;
            const int q = ok ? p : it.begin;
            a[u] = ok ? csc_val[q] : 0.f;
            const float x = dY[(int64_t)csc_src[q] * dim + my_idx];
            gv[u] = ok ? x : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPullUnroll; ++u) acc += a[u] * gv[u];
    }
#pragma unroll
    for (int off = KP; off < kWave; off <<= 1) acc += __shfl_xor(acc, off);
    if (g == 0 && active) {
        float* __restrict__ out = (it.slot < 0) ? dXs + (int64_t)it.row * k : partials + (int64_t)it.slot * k;
        out[t] = acc;
    }
}

// any k: lane handles positions t = lane, lane + 64, ...; one pass over the in-entries per 64 positions
template <typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_pull_wide_kernel(const WorkItem* __restrict__ items,
                                                              const int32_t* __restrict__ csc_src,
                                                              const float* __restrict__ csc_val,
                                                              const float* __restrict__ dY,
                                                              const IdxT* __restrict__ sp_index, int dim, int k,
                                                              float* __restrict__ dXs, float* __restrict__ partials)
{
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    float* __restrict__ out = (it.slot < 0) ? dXs + (int64_t)it.row * k : partials + (int64_t)it.slot * k;
    for (int t = lane; t < k; t += kWave) {
        const int my_idx = (int)sp_index[(int64_t)it.row * k + t];
        float acc = 0.f;
        for (int p0 = it.begin; p0 < it.end; p0 += kPullUnroll) {
            float gv[kPullUnroll], a[kPullUnroll];
#pragma unroll
            for (int u = 0; u < kPullUnroll; ++u) {
                const bool ok = p0 + u < it.end;
                const int q = ok ? p0 + u : it.begin;
                a[u] = ok ? csc_val[q] : 0.f;
                const float x = dY[(int64_t)csc_src[q] * dim + my_idx];
                gv[u] = ok ? x : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kPullUnroll; ++u) acc += a[u] * gv[u];
        }
        out[t] = acc;
    }
}

// ---------------------------------------------------------------- push ----

constexpr int kPushRounds = 4;

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

// K > 0: k known at compile time
template <int K, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_push_kernel(const WorkItem* __restrict__ items,
                                                         const int32_t* __restrict__ col,
                                                         const float* __restrict__ val, const float* __restrict__ dY,
                                                         const IdxT* __restrict__ sp_index, int dim, int k_rt,
                                                         float* __restrict__ dXs)
{
    extern __shared__ float g_row[];
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    if (it.begin == it.end) return;
    const int k = K ? K : k_rt;
    const float* __restrict__ src = dY + (int64_t)it.row * dim;
    for (int c = lane; c < dim; c += kWave) g_row[c] = src[c];
    __syncthreads();

    for (int base = it.begin; base < it.end; base += kWave) {
        const int n = min(kWave, it.end - base);
        int my_col = 0;
        float my_val = 0.f;
        if (lane < n) {
            my_col = col[base + lane];
            my_val = val[base + lane];
        }
        const int units = n * k;
        for (int u0 = 0; u0 < units; u0 += kWave * kPushRounds) {
            int ix[kPushRounds];
            int64_t off[kPushRounds];
            float a[kPushRounds];
            bool ok[kPushRounds];
#pragma unroll
            for (int r = 0; r < kPushRounds; ++r) {
                const int u = u0 + r * kWave + lane;
                ok[r] = u < units;
                const int uc = ok[r] ? u : 0;
                const int e = uc / k;
                const int t = uc - e * k;
                const int j = __shfl(my_col, e);
                a[r] = __shfl(my_val, e);
                off[r] = (int64_t)j * k + t;
                ix[r] = (int)sp_index[off[r]];
            }
#pragma unroll
            for (int r = 0; r < kPushRounds; ++r)
                if (ok[r]) unsafeAtomicAdd(dXs + off[r], a[r] * g_row[ix[r]]);
        }
    }
}

template <typename IdxT>
maxk_status launch_pull_t(const ItemList& L, const int32_t* csc_src, const float* csc_val, const float* dY,
                          const IdxT* sp_index, int dim, int k, float* dXs, float* partials, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
#define MAXK_PULL(KERNEL) \
    hipLaunchKernelGGL((KERNEL), grid, block, 0, s, L.d_items, csc_src, csc_val, dY, sp_index, dim, k, dXs, partials)
    if (k <= 1) MAXK_PULL((bwd_pull_small_kernel<1, IdxT>));
    else if (k <= 2) MAXK_PULL((bwd_pull_small_kernel<2, IdxT>));
    else if (k <= 4) MAXK_PULL((bwd_pull_small_kernel<4, IdxT>));
    else if (k <= 8) MAXK_PULL((bwd_pull_small_kernel<8, IdxT>));
    else if (k <= 16) MAXK_PULL((bwd_pull_small_kernel<16, IdxT>));
    else if (k <= 32) MAXK_PULL((bwd_pull_small_kernel<32, IdxT>));
    else if (k <= 64) MAXK_PULL((bwd_pull_small_kernel<64, IdxT>));
    else MAXK_PULL((bwd_pull_wide_kernel<IdxT>));
#undef MAXK_PULL
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <typename IdxT>
maxk_status launch_push_t(const ItemList& L, const int32_t* col, const float* val, const float* dY,
                          const IdxT* sp_index, int dim, int k, float* dXs, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
    const size_t lds = sizeof(float) * (size_t)dim;
#define MAXK_PUSH(K) \
    hipLaunchKernelGGL((bwd_push_kernel<K, IdxT>), grid, block, lds, s, L.d_items, col, val, dY, sp_index, dim, k, dXs)
    switch (k) {
        case 8: MAXK_PUSH(8); break;
        case 16: MAXK_PUSH(16); break;
        case 32: MAXK_PUSH(32); break;
        case 64: MAXK_PUSH(64); break;
        case 96: MAXK_PUSH(96); break;
        case 128: MAXK_PUSH(128); break;
        case 192: MAXK_PUSH(192); break;
        default: MAXK_PUSH(0); break;
    }
#undef MAXK_PUSH
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

}  // namespace

maxk_status launch_bwd_pull(const ItemList& L, const int32_t* csc_src, const float* csc_val, const float* dY,
                            const void* sp_index, int index_bytes, int dim, int k, float* dXs, float* partials,
                            hipStream_t s)
{
    if (L.n_items == 0) return MAXK_OK;
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    maxk_status st;
    if (index_bytes == 1) st = launch_pull_t(L, csc_src, csc_val, dY, (const uint8_t*)sp_index, dim, k, dXs, partials, s);
    else if (index_bytes == 2) st = launch_pull_t(L, csc_src, csc_val, dY, (const uint16_t*)sp_index, dim, k, dXs, partials, s);
    else st = launch_pull_t(L, csc_src, csc_val, dY, (const int32_t*)sp_index, dim, k, dXs, partials, s);
    if (st != MAXK_OK) return st;
    return launch_combine(L, partials, k, dXs, s);
}

maxk_status launch_bwd_push(const ItemList& L, const int32_t* col, const float* val, const float* dY,
                            const void* sp_index, int index_bytes, int64_t N, int dim, int k, float* dXs,
                            hipStream_t s)
{
    const int64_t n = N * (int64_t)k;
    if (n == 0) return MAXK_OK;
    {
        int64_t blocks = (n + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        if (blocks < 1) blocks = 1;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, dXs, n);
        MAXK_LAUNCH_CHECK();
    }
    if (L.n_items == 0) return MAXK_OK;
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    if (index_bytes == 1) return launch_push_t(L, col, val, dY, (const uint8_t*)sp_index, dim, k, dXs, s);
    if (index_bytes == 2) return launch_push_t(L, col, val, dY, (const uint16_t*)sp_index, dim, k, dXs, s);
    return launch_push_t(L, col, val, dY, (const int32_t*)sp_index, dim, k, dXs, s);
}

}  // namespace maxk
