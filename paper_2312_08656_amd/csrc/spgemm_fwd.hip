// Forward aggregation (Eq. 2 left; Sec. 3.2): dispatch over the storage format of the CBSR values, the
// packed-record geometry, and the kernel that adds up the partial rows of split rows.
// The kernels are in spgemm_fwd_impl.hpp.
#include "spgemm_fwd_impl.hpp"

namespace maxk {
namespace {

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

// Records are padded to a multiple of 64 bytes so that none straddles more 64-byte sectors than it
// must (measured on the dense workload: 1.34 -> 1.26 ms at k = 8, 2.10 -> 1.58 ms at k = 16).
int fwd_packed_index_offset(int k, int index_bytes, int val_bytes)
{
    return (k * val_bytes + index_bytes - 1) / index_bytes * index_bytes;
}

int fwd_packed_record_bytes(int k, int index_bytes, int val_bytes)
{
    return (fwd_packed_index_offset(k, index_bytes, val_bytes) + k * index_bytes + 63) & ~63;
}

int fwd_private_copies(int k) { return private_copies(k); }

maxk_status launch_spgemm_fwd(const ItemList& L, const int32_t* col, const float* val, const void* sp_data,
                              int value_type, const void* sp_index, int index_bytes, int64_t N, char* packed, int dim,
                              int k, float* Y, float* partials, hipStream_t s)
{
    if (L.n_items == 0) return MAXK_OK;
    maxk_status st;
    if (value_type == MAXK_VALUE_BF16)
        st = launch_fwd_format<MAXK_VALUE_BF16>(L, col, val, sp_data, sp_index, index_bytes, N, packed, dim, k, Y, partials, s);
    else if (value_type == MAXK_VALUE_F16)
        st = launch_fwd_format<MAXK_VALUE_F16>(L, col, val, sp_data, sp_index, index_bytes, N, packed, dim, k, Y, partials, s);
    else
        st = launch_fwd_format<MAXK_VALUE_F32>(L, col, val, sp_data, sp_index, index_bytes, N, packed, dim, k, Y, partials, s);
    if (st != MAXK_OK) return st;
    return launch_combine(L, partials, dim, Y, s);
}

}  // namespace maxk
