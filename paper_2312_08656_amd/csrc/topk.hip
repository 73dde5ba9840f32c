// MaxK selection + CBSR packing (Sec. 3.1 definition, Eq. 1; CBSR of Sec. 3.2).
//
// One 64-lane wavefront owns one row of H, held entirely in registers
// (E values per lane).  The paper's kernel bisects a floating-point pivot
// between min and max and stops after at most 10 rounds, which cannot separate
// equal values at rank k.  Here the k-th largest value is found EXACTLY by a
// most-significant-bit-first radix descent on order-preserving integer keys:
// each step is E compares + E wave ballots + scalar popcounts, no LDS and no
// barrier, and the descent stops early as soon as a prefix keeps exactly k
// entries (the usual case for continuous data, after ~10 bits).  Ties at the
// k-th value are resolved toward the lower column with ballot prefix counts,
// and the same prefix counts give every survivor its slot in the CBSR row, so
// indices come out ascending.
#include "common.hpp"

namespace maxk {
namespace {

__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if ((b << 1) == 0u) b = 0u;  // -0.0 and +0.0 compare equal
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Column of element e of lane l: chunks of 64*V columns, V consecutive per lane.
template <int V>
__device__ __forceinline__ int column_of(int lane, int e)
{
    return (e / V) * (kWave * V) + lane * V + (e % V);
}

// pos[e] = number of flagged elements that precede (lane, e) in column order
template <int E, int V>
__device__ __forceinline__ void column_order_prefix(const bool (&flag)[E], int (&pos)[E])
{
    int before_chunks = 0;
#pragma unroll
    for (int c = 0; c < E / V; ++c) {
        int in_chunk_before_lane = 0, chunk_total = 0;
        uint64_t m[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            m[v] = __builtin_amdgcn_ballot_w64(flag[c * V + v]);
            in_chunk_before_lane += lanes_below(m[v]);
            chunk_total += __builtin_popcountll(m[v]);
        }
        int own = 0;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            pos[c * V + v] = before_chunks + in_chunk_before_lane + own;
            own += flag[c * V + v] ? 1 : 0;
        }
        before_chunks += chunk_total;
    }
}

// VT: storage format of the values written (MAXK_VALUE_*); selection always works on the fp32 input
template <int E, int V, int VT, typename IdxT>
__global__ __launch_bounds__(256) void topk_cbsr_kernel(const float* __restrict__ H, int64_t N, int dim, int k,
                                                        value_store_t<VT>* __restrict__ sp_data,
                                                        IdxT* __restrict__ sp_index)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (row >= N) return;
    const float* __restrict__ h = H + row * (int64_t)dim;

    float v[E];
    uint32_t key[E];
#pragma unroll
    for (int c = 0; c < E / V; ++c) {
        const int base = c * (kWave * V) + lane * V;
        if constexpr (V == 4) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            const bool in = base < dim;  // dim % 4 == 0 on this path
            if (in) x = *reinterpret_cast<const float4*>(h + base);
            v[c * 4 + 0] = x.x; v[c * 4 + 1] = x.y; v[c * 4 + 2] = x.z; v[c * 4 + 3] = x.w;
#pragma unroll
            for (int j = 0; j < 4; ++j) key[c * 4 + j] = in ? order_key(v[c * 4 + j]) : 0u;
        } else if constexpr (V == 2) {
            float2 x = make_float2(0.f, 0.f);
            const bool in = base < dim;  // dim % 2 == 0 on this path
            if (in) x = *reinterpret_cast<const float2*>(h + base);
            v[c * 2 + 0] = x.x; v[c * 2 + 1] = x.y;
#pragma unroll
            for (int j = 0; j < 2; ++j) key[c * 2 + j] = in ? order_key(v[c * 2 + j]) : 0u;
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const bool in = base + j < dim;
                v[c * V + j] = in ? h[base + j] : 0.f;
                key[c * V + j] = in ? order_key(v[c * V + j]) : 0u;  // 0 ranks below every non-NaN key
            }
        }
    }

    // k-th largest key by MSB-first descent; `exact` = the prefix already keeps exactly k.
    // Everything but the compares is wave-uniform; readfirstlane tells the compiler so, which keeps
    // the prefix, the candidate and the counts in scalar registers (4 vector compares per step).
    uint32_t prefix = 0u;
    bool exact = false;
#pragma unroll
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = prefix | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= cand));
        cnt = __builtin_amdgcn_readfirstlane(cnt);
        if (cnt >= k) {
            prefix = cand;
            if (cnt == k) { exact = true; break; }
        }
    }

    bool sel[E];
    if (exact) {
#pragma unroll
        for (int e = 0; e < E; ++e) sel[e] = key[e] >= prefix;
    } else {
        // prefix is the k-th largest key and more than k entries are >= it: take all
        // strictly larger ones, then the leftmost (k - those) of the equal ones
        bool eq[E];
        int greater = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            eq[e] = key[e] == prefix;
            greater += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] > prefix));
        }
        const int need = k - greater;
        int rank[E];
        column_order_prefix<E, V>(eq, rank);
#pragma unroll
        for (int e = 0; e < E; ++e) sel[e] = key[e] > prefix || (eq[e] && rank[e] < need);
    }

    int pos[E];
    column_order_prefix<E, V>(sel, pos);
    value_store_t<VT>* __restrict__ od = sp_data + row * (int64_t)k;
    IdxT* __restrict__ oi = sp_index + row * (int64_t)k;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (sel[e]) {
            od[pos[e]] = narrow_value<VT>(v[e]);
            oi[pos[e]] = (IdxT)column_of<V>(lane, e);
        }
    }
}

// MaxK backward: dense[row, sp_index[row,t]] = values[row,t], zeros elsewhere.  One wavefront per row;
// the row is assembled in LDS so that it leaves the CU as one coalesced write.
template <typename IdxT>
__global__ __launch_bounds__(256) void cbsr_scatter_kernel(const float* __restrict__ values,
                                                           const IdxT* __restrict__ sp_index, int64_t N, int dim,
                                                           int k, float* __restrict__ dense)
{
    extern __shared__ float rows[];  // 4 rows of dim floats
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    const int64_t row = (int64_t)blockIdx.x * 4 + w;
    float* __restrict__ buf = rows + w * dim;
    for (int c = lane; c < dim; c += kWave) buf[c] = 0.f;
    __syncthreads();
    if (row < N)
        for (int t = lane; t < k; t += kWave) buf[(int)sp_index[row * (int64_t)k + t]] = values[row * (int64_t)k + t];
    __syncthreads();
    if (row < N) {
        float* __restrict__ out = dense + row * (int64_t)dim;
        for (int c = lane; c < dim; c += kWave) out[c] = buf[c];
    }
}

template <int E, int V, int VT>
maxk_status launch_v(const float* H, int64_t N, int dim, int k, void* sp_data, void* sp_index, int index_bytes,
                     hipStream_t s)
{
    const int rows_per_block = 4;
    const int64_t blocks = (N + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(rows_per_block * kWave);
    auto* od = (value_store_t<VT>*)sp_data;
    switch (index_bytes) {
        case 1: hipLaunchKernelGGL((topk_cbsr_kernel<E, V, VT, uint8_t>), grid, block, 0, s, H, N, dim, k, od, (uint8_t*)sp_index); break;
        case 2: hipLaunchKernelGGL((topk_cbsr_kernel<E, V, VT, uint16_t>), grid, block, 0, s, H, N, dim, k, od, (uint16_t*)sp_index); break;
        default: hipLaunchKernelGGL((topk_cbsr_kernel<E, V, VT, int32_t>), grid, block, 0, s, H, N, dim, k, od, (int32_t*)sp_index); break;
    }
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <int E, int V>
maxk_status launch_e(const float* H, int64_t N, int dim, int k, void* sp_data, int value_type, void* sp_index,
                     int index_bytes, hipStream_t s)
{
    if (value_type == MAXK_VALUE_BF16) return launch_v<E, V, MAXK_VALUE_BF16>(H, N, dim, k, sp_data, sp_index, index_bytes, s);
    if (value_type == MAXK_VALUE_F16) return launch_v<E, V, MAXK_VALUE_F16>(H, N, dim, k, sp_data, sp_index, index_bytes, s);
    return launch_v<E, V, MAXK_VALUE_F32>(H, N, dim, k, sp_data, sp_index, index_bytes, s);
}

}  // namespace

maxk_status launch_cbsr_scatter(const float* values, const void* sp_index, int index_bytes, int64_t N, int dim, int k,
                                float* dense, hipStream_t s)
{
    if (N == 0) return MAXK_OK;
    const int64_t blocks = (N + 3) / 4;
    if (blocks > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(4 * kWave);
    const size_t lds = sizeof(float) * 4 * (size_t)dim;
    if (index_bytes == 1) hipLaunchKernelGGL((cbsr_scatter_kernel<uint8_t>), grid, block, lds, s, values, (const uint8_t*)sp_index, N, dim, k, dense);
    else if (index_bytes == 2) hipLaunchKernelGGL((cbsr_scatter_kernel<uint16_t>), grid, block, lds, s, values, (const uint16_t*)sp_index, N, dim, k, dense);
    else hipLaunchKernelGGL((cbsr_scatter_kernel<int32_t>), grid, block, lds, s, values, (const int32_t*)sp_index, N, dim, k, dense);
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

maxk_status launch_topk(const float* H, int64_t N, int dim, int k, void* sp_data, int value_type, void* sp_index,
                        int index_bytes, hipStream_t s)
{
    if (N == 0) return MAXK_OK;
    // E values per lane in chunks of V consecutive columns (one 4*V-byte load each).  The scalar work of the
    // descent grows with E, so E is kept at ceil(dim / 64) where a vector width divides it.
    const bool vec4 = (dim % 4 == 0) && aligned(H, 16);
    const bool vec2 = (dim % 2 == 0) && aligned(H, 8);
    if (vec2 && dim > 64 && dim <= 128) return launch_e<2, 2>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    if (vec4 && dim <= 256) return launch_e<4, 4>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    if (vec2 && dim > 256 && dim <= 384) return launch_e<6, 2>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    if (vec4) {
        if (dim <= 512) return launch_e<8, 4>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
        if (dim <= 768) return launch_e<12, 4>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
        return launch_e<16, 4>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    }
    if (dim <= 64) return launch_e<1, 1>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    if (dim <= 256) return launch_e<4, 1>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    if (dim <= 512) return launch_e<8, 1>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
    return launch_e<16, 1>(H, N, dim, k, sp_data, value_type, sp_index, index_bytes, s);
}

}  // namespace maxk
