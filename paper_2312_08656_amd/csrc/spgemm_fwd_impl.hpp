// Forward aggregation: row-wise-product SpGEMM with dense output
// (Eq. 2 left; Sec. 3.2 "Forward Computation"; prior art: Alg. 1).
//
// One 64-lane wavefront (= one workgroup, so no cross-wave barrier exists)
// owns one work item: a run of at most `chunk` stored entries of one row of A.
// The item's (col, val) pairs are staged 64 at a time through LDS, and the
// wavefront walks a FLAT list of units (entry e, position t): unit u belongs to
// entry u / k and CBSR position u % k, so all 64 lanes stay busy for every k and
// the k lanes of one entry read k contiguous values and k contiguous indices.
//
// Accumulation.  LDS floating-point atomics (ds_add_f32) retire about one lane
// every three clocks on this chip (measured: ~190 clocks per wave instruction),
// which capped the first version of this kernel at ~200 G updates/s no matter
// the memory system.  A plain LDS read-add-write pair is ~14x faster, and it is
// safe here without atomics because (a) the k positions of one CBSR row are
// distinct columns, and (b) the entries that share one wave instruction (at most
// NB = ceil(64/k)+1 consecutive ones) accumulate into NB PRIVATE copies of the
// output row (copy e % NB), while LDS operations of one wavefront execute in
// program order.  The copies are added up when the row is written out.
// Rows longer than `chunk` write partial rows that a second kernel adds up
// (deterministic order, and it bounds the length of any fp32 running sum);
// every other row is written once, straight from LDS, fully coalesced.
// Shapes whose private copies would not fit comfortably in LDS (tiny k with a
// very wide row) fall back to the single-copy kernel with LDS atomics.
//
// This header holds the kernel templates; one translation unit per storage format of the CBSR values
// (fp32, bf16, fp16) instantiates them, so the three compile side by side.
#pragma once

#include <algorithm>

#include "common.hpp"

namespace maxk {

// Private output-row copies needed so that entries sharing a wave instruction never collide.
__host__ __device__ constexpr int private_copies(int k)
{
    return (k >= kWave) ? ((k % kWave == 0) ? 1 : 2) : ((kWave % k == 0) ? kWave / k : (kWave - 1) / k + 2);
}

constexpr size_t kMaxPrivateLds = 40 * 1024;  // above this the private copies cost too much occupancy

// Floats between the end of one private copy and the start of the next (a multiple of 4).  Padding shifts the copies
// against each other in the LDS banks; measured without effect (the columns of different entries are unrelated, so
// their bank conflicts are those of random addresses), hence 0.
#ifndef MAXK_FWD_COPY_PAD
#define MAXK_FWD_COPY_PAD 0
#endif
constexpr int kCopyPad = MAXK_FWD_COPY_PAD;

// implemented once per storage format (spgemm_fwd_f32.hip, _bf16.hip, _f16.hip)
template <int VT>
maxk_status launch_fwd_format(const ItemList& L, const int32_t* col, const float* val, const void* sp_data,
                              const void* sp_index, int index_bytes, int64_t N, char* packed, int dim, int k,
                              float* Y, float* partials, hipStream_t s);

namespace {


constexpr int kRounds = 4;  // unit rounds in flight per wavefront (fallback kernel)

// Fallback for shapes whose private copies would not fit in LDS: a single copy of the output row,
// updated with LDS floating-point atomics (slow on this chip, see the header comment).
template <int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void spgemm_fwd_atomic_kernel(const WorkItem* __restrict__ items,
                                                                  const int32_t* __restrict__ col,
                                                                  const float* __restrict__ val,
                                                                  const value_store_t<VT>* __restrict__ sp_data,
                                                                  const IdxT* __restrict__ sp_index, int dim, int k,
                                                                  float* __restrict__ Y, float* __restrict__ partials)
{
    extern __shared__ float row_buf[];
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    for (int c = lane; c < dim; c += kWave) row_buf[c] = 0.f;
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
        for (int u0 = 0; u0 < units; u0 += kWave * kRounds) {
            float d[kRounds], a[kRounds];
            int ix[kRounds];
            bool ok[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int u = u0 + r * kWave + lane;
                ok[r] = u < units;
                const int uc = ok[r] ? u : 0;
                const int e = uc / k;
                const int t = uc - e * k;
                const int c = __shfl(my_col, e);
                a[r] = __shfl(my_val, e);
                const int64_t off = (int64_t)c * k + t;
                d[r] = widen_value<VT>(sp_data[off]);
                ix[r] = (int)sp_index[off];
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r)
                if (ok[r]) atomicAdd(&row_buf[ix[r]], a[r] * d[r]);
        }
    }
    __syncthreads();

    float* __restrict__ out = (it.slot < 0) ? Y + (int64_t)it.row * dim : partials + (int64_t)it.slot * dim;
    for (int c = lane; c < dim; c += kWave) out[c] = row_buf[c];
}

// For small k a CBSR row is a fraction of a cache line in EACH of the two arrays, and the kernel is
// bound by the number of row requests (~137 G/s measured), not by bytes.  The packed path reads a
// per-call repack instead: one record per node, k values followed by k indices, so an entry costs
// one request.  The repack reads and writes N*k*(4+ib) bytes, against nnz*k*(4+ib) for the kernel
// (2+ib with 16-bit values; the indices start at the next multiple of their own width).
template <int VT, typename IdxT>
__global__ __launch_bounds__(256) void pack_cbsr_kernel(const value_store_t<VT>* __restrict__ sp_data,
                                                        const IdxT* __restrict__ sp_index, int64_t n_units, int k,
                                                        int rec_bytes, int idx_off, char* __restrict__ packed)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < n_units; u += stride) {
        const int64_t node = u / k;
        const int t = (int)(u - node * k);
        char* rec = packed + node * rec_bytes;
        reinterpret_cast<value_store_t<VT>*>(rec)[t] = sp_data[u];
        reinterpret_cast<IdxT*>(rec + idx_off)[t] = sp_index[u];
    }
}

// K: MaxK k when known at compile time (0 = runtime); ROUNDS: 64-unit rounds in flight;
// PACKED: read the per-node (values, indices) records of pack_cbsr_kernel instead of the two arrays
// VT: storage format of the CBSR values (widened exactly; products and sums are fp32 in every format)
template <int K, int ROUNDS, bool PACKED, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void spgemm_fwd_rmw_kernel(const WorkItem* __restrict__ items,
                                                               const int32_t* __restrict__ col,
                                                               const float* __restrict__ val,
                                                               const value_store_t<VT>* __restrict__ sp_data,
                                                               const IdxT* __restrict__ sp_index,
                                                               const char* __restrict__ packed, int rec_bytes,
                                                               int idx_off,
                                                               int dim, int k_rt, int nb_rt, int vec_out,
                                                               float* __restrict__ Y, float* __restrict__ partials)
{
    // vec_out: dim % 4 == 0 and Y / partials 16-byte aligned, so that a row is written with 16-byte stores
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int k = K ? K : k_rt;
    const int nb = K ? private_copies(K) : nb_rt;
    const int lane = threadIdx.x;
    float* __restrict__ row_buf = lds;                                         // nb copies of the output row
    const int cs = dim + kCopyPad;                                             // floats from one copy to the next
    int2* __restrict__ entry_buf = reinterpret_cast<int2*>(lds + ((nb * cs + 1) & ~1));  // 64 staged (col, val)
    const WorkItem it = items[blockIdx.x];
    if (((nb * cs) & 3) == 0) {
        for (int c = lane * 4; c < nb * cs; c += kWave * 4)
            *reinterpret_cast<float4*>(row_buf + c) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        for (int c = lane; c < nb * cs; c += kWave) row_buf[c] = 0.f;
    }

    for (int base = it.begin; base < it.end; base += kWave) {
        const int n = min(kWave, it.end - base);
        __syncthreads();  // previous batch fully consumed (and the zero fill done)
        if (lane < n) entry_buf[lane] = make_int2(col[base + lane], __float_as_int(val[base + lane]));
        __syncthreads();
        const int units = n * k;
        for (int u0 = 0; u0 < units; u0 += kWave * ROUNDS) {
            float d[ROUNDS], a[ROUNDS];
            int at[ROUNDS];
            bool ok[ROUNDS];
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
                const int u = u0 + r * kWave + lane;
                ok[r] = u < units;
                const int uc = ok[r] ? u : 0;
                const int e = uc / k;
                const int t = uc - e * k;
                const int2 ed = entry_buf[e];
                a[r] = __int_as_float(ed.y);
                if constexpr (PACKED) {
                    const char* rec = packed + (int64_t)ed.x * rec_bytes;
                    d[r] = widen_value<VT>(reinterpret_cast<const value_store_t<VT>*>(rec)[t]);
                    at[r] = (e % nb) * cs + (int)reinterpret_cast<const IdxT*>(rec + idx_off)[t];
                } else {
                    const int64_t off = (int64_t)ed.x * k + t;
                    d[r] = widen_value<VT>(sp_data[off]);
                    at[r] = (e % nb) * cs + (int)sp_index[off];
                }
            }
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
                if (ok[r]) {
                    const float old = row_buf[at[r]];
                    row_buf[at[r]] = old + a[r] * d[r];
                }
            }
        }
    }
    __syncthreads();

    float* __restrict__ out = (it.slot < 0) ? Y + (int64_t)it.row * dim : partials + (int64_t)it.slot * dim;
    if (vec_out) {
        for (int c = lane * 4; c < dim; c += kWave * 4) {
            float4 acc = *reinterpret_cast<const float4*>(row_buf + c);
            for (int b = 1; b < nb; ++b) {
                const float4 x = *reinterpret_cast<const float4*>(row_buf + b * cs + c);
                acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
            }
            *reinterpret_cast<float4*>(out + c) = acc;
        }
    } else {
        for (int c = lane; c < dim; c += kWave) {
            float acc = row_buf[c];
            for (int b = 1; b < nb; ++b) acc += row_buf[b * cs + c];
            out[c] = acc;
        }
    }
}


template <int VT, typename IdxT>
maxk_status launch_atomic(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* sp_data,
                          const IdxT* sp_index, int dim, int k, float* Y, float* partials, hipStream_t s)
{
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    hipLaunchKernelGGL((spgemm_fwd_atomic_kernel<VT, IdxT>), dim3((unsigned)L.n_items), dim3(kWave),
                       sizeof(float) * (size_t)dim, s, L.d_items, col, val, sp_data, sp_index, dim, k, Y, partials);
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <bool PACKED, int VT, typename IdxT>
maxk_status launch_rmw(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* sp_data,
                       const IdxT* sp_index, const char* packed, int rec_bytes, int idx_off, int dim, int k, float* Y,
                       float* partials, hipStream_t s)
{
    if (L.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)L.n_items), block(kWave);
    const int nb = private_copies(k);
    const size_t lds = sizeof(float) * (size_t)((nb * (dim + kCopyPad) + 1) & ~1) + sizeof(int2) * kWave;
    const int vec_out = dim % 4 == 0 && aligned(Y, 16) && aligned(partials, 16);
#define MAXK_FWD_RMW(K, R)                                                                                        \
    hipLaunchKernelGGL((spgemm_fwd_rmw_kernel<K, R, PACKED, VT, IdxT>), grid, block, lds, s, L.d_items, col, val, \
                       sp_data, sp_index, packed, rec_bytes, idx_off, dim, k, nb, vec_out, Y, partials)
    switch (k) {
        case 8: MAXK_FWD_RMW(8, 8); break;
        case 16: MAXK_FWD_RMW(16, 8); break;
        case 32: MAXK_FWD_RMW(32, 8); break;
        case 64: MAXK_FWD_RMW(64, 8); break;
        case 96: MAXK_FWD_RMW(96, 8); break;
        case 128: MAXK_FWD_RMW(128, 8); break;
        case 192: MAXK_FWD_RMW(192, 8); break;
        default: MAXK_FWD_RMW(0, 8); break;
    }
#undef MAXK_FWD_RMW
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <int VT, typename IdxT>
maxk_status launch_rmw_i(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* sp_data,
                         const IdxT* sp_index, int64_t N, char* packed, int dim, int k, float* Y, float* partials,
                         hipStream_t s)
{
    if (packed) {
        const int vb = (int)sizeof(value_store_t<VT>);
        const int rec_bytes = fwd_packed_record_bytes(k, (int)sizeof(IdxT), vb);
        const int idx_off = fwd_packed_index_offset(k, (int)sizeof(IdxT), vb);
        const int64_t n_units = N * (int64_t)k;
        const unsigned blocks = (unsigned)std::min<int64_t>((n_units + 255) / 256, 65536);
        hipLaunchKernelGGL((pack_cbsr_kernel<VT, IdxT>), dim3(blocks), dim3(256), 0, s, sp_data, sp_index, n_units, k,
                           rec_bytes, idx_off, packed);
        MAXK_LAUNCH_CHECK();
        return launch_rmw<true, VT>(L, col, val, sp_data, sp_index, packed, rec_bytes, idx_off, dim, k, Y, partials, s);
    }
    return launch_rmw<false, VT>(L, col, val, sp_data, sp_index, nullptr, 0, 0, dim, k, Y, partials, s);
}

// everything but the final sum of split rows, for one storage format of the values
template <int VT>
maxk_status launch_fwd_vt(const ItemList& L, const int32_t* col, const float* val, const void* sp_data_v,
                          const void* sp_index, int index_bytes, int64_t N, char* packed, int dim, int k, float* Y,
                          float* partials, hipStream_t s)
{
    const auto* sp_data = (const value_store_t<VT>*)sp_data_v;
    const size_t private_lds = sizeof(float) * (size_t)private_copies(k) * (size_t)dim;
    if (private_lds <= kMaxPrivateLds) {
        if (index_bytes == 1) return launch_rmw_i<VT>(L, col, val, sp_data, (const uint8_t*)sp_index, N, packed, dim, k, Y, partials, s);
        if (index_bytes == 2) return launch_rmw_i<VT>(L, col, val, sp_data, (const uint16_t*)sp_index, N, packed, dim, k, Y, partials, s);
        return launch_rmw_i<VT>(L, col, val, sp_data, (const int32_t*)sp_index, N, packed, dim, k, Y, partials, s);
    }
    if (index_bytes == 1) return launch_atomic<VT>(L, col, val, sp_data, (const uint8_t*)sp_index, dim, k, Y, partials, s);
    if (index_bytes == 2) return launch_atomic<VT>(L, col, val, sp_data, (const uint16_t*)sp_index, dim, k, Y, partials, s);
    return launch_atomic<VT>(L, col, val, sp_data, (const int32_t*)sp_index, dim, k, Y, partials, s);
}

}  // namespace
}  // namespace maxk
