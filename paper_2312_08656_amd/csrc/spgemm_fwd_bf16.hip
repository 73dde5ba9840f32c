// Forward SpGEMM kernels for CBSR values stored as bf16 (see spgemm_fwd_impl.hpp).
#include "spgemm_fwd_impl.hpp"

namespace maxk {

template <>
maxk_status launch_fwd_format<MAXK_VALUE_BF16>(const ItemList& L, const int32_t* col, const float* val, const void* sp_data,
                                              const void* sp_index, int index_bytes, int64_t N, char* packed, int dim, int k,
                                              float* Y, float* partials, hipStream_t s)
{
    return launch_fwd_vt<MAXK_VALUE_BF16>(L, col, val, sp_data, sp_index, index_bytes, N, packed, dim, k, Y, partials, s);
}

}  // namespace maxk
