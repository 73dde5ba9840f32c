// Backward SSpMM kernels for dY stored as bf16 (see sspmm_bwd_impl.hpp).
#include "sspmm_bwd_impl.hpp"

namespace maxk {

template <>
maxk_status bwd_pull_format<MAXK_VALUE_BF16>(const ItemList& L, const int32_t* csc_src, const float* csc_val, const void* dY,
                                  const void* sp_index, int index_bytes, int dim, int k, float* dXs, float* partials,
                                  hipStream_t s)
{
    return pull_format<MAXK_VALUE_BF16>(L, csc_src, csc_val, dY, sp_index, index_bytes, dim, k, dXs, partials, s);
}

template <>
maxk_status bwd_push_format<MAXK_VALUE_BF16>(const ItemList& L, const int32_t* col, const float* val, const void* dY,
                                  const void* sp_index, int index_bytes, int dim, int k, float* dXs, hipStream_t s)
{
    return push_format<MAXK_VALUE_BF16>(L, col, val, dY, sp_index, index_bytes, dim, k, dXs, s);
}

template <>
maxk_status bwd_expand_format<MAXK_VALUE_BF16>(const ItemList& L, const int32_t* col, const float* val, const void* dY,
                                    const void* sp_index, int index_bytes, int dim, int k, float* expand, hipStream_t s)
{
    return expand_format<MAXK_VALUE_BF16>(L, col, val, dY, sp_index, index_bytes, dim, k, expand, s);
}

template <>
maxk_status bwd_slab_format<MAXK_VALUE_BF16>(const SlabSet& S, const void* dY, const void* sp_index, int index_bytes, int64_t N,
                                  int dim, int k, float* dXs, hipStream_t s)
{
    return slab_format<MAXK_VALUE_BF16>(S, dY, sp_index, index_bytes, N, dim, k, dXs, s);
}

}  // namespace maxk
