// MaxK selection + CBSR packing (Sec. 3.1 definition, Eq. 1; CBSR of Sec. 3.2).
//
// One 64-lane wavefront owns one row of H, held entirely in registers
// (E values per lane).  The paper's kernel bisects a floating-point pivot
// between min and max and stops after at most 10 rounds, which cannot separate
// equal values at rank k.  Here the selection is EXACT, in two stages.
// Stage 1 is the paper's idea made exact: move a pivot on the value axis, but
// stop only when the pivot keeps exactly k entries (any such pivot gives the
// one correct set); a step is E compares + E wave ballots + scalar popcounts,
// no LDS and no barrier.  A search that bisects [-max|x|, +max|x|] needs about
// 8 steps on continuous data whatever the exponent range (log2(range / gap at
// rank k)); one that starts at the pivot of the row before needs about 5.5 when
// neighbouring rows are alike, and up to 7 more than the bisection when they
// are not (the step doubles until the count changes sides).  The kernel is bound by scalar-unit issue (~12 scalar instructions per
// step, one scalar instruction per clock per CU), so fewer steps is what
// shortens it.
// Stage 2 runs only for rows stage 1 cannot settle (ties at rank k, infinities,
// k = dim): a most-significant-bit-first radix descent on order-preserving
// integer keys finds the k-th largest value itself, and ties at that value are
// resolved toward the lower column with ballot prefix counts.  The same prefix
// counts give every survivor its slot in the CBSR row, so indices come out
// ascending.
#include <algorithm>
#include <type_traits>

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

// Largest value of a non-negative quantity over the wavefront, as a wave-uniform bit pattern.  Data-parallel-primitive
// moves: a running maximum over the 16 lanes of each row (shifts by 1, 2, 4, 8; lanes shifted in from outside read 0),
// then lane 15 of each row into the next row and lane 31 into the upper half; lane 63 ends up with the result.
__device__ __forceinline__ uint32_t wave_max_nonneg(float x)
{
    // bit patterns of non-negative floats order like unsigned integers
    auto step = [](uint32_t v, auto ctrl, auto rows) {
        const uint32_t moved = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, decltype(ctrl)::value,
                                                                     decltype(rows)::value, 0xF, true);
        return v > moved ? v : moved;
    };
    using std::integral_constant;
    uint32_t b = __float_as_uint(x);
    b = step(b, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{});  // row_shr:1
    b = step(b, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{});  // row_shr:2
    b = step(b, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{});  // row_shr:4
    b = step(b, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{});  // row_shr:8
    b = step(b, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});  // row_bcast:15 into rows 1 and 3
    b = step(b, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});  // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)b, 63);
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

constexpr int kPivotSteps = 16;  // pivots tried before a row is handed to the radix descent (99 % need <= 14)

// What a wavefront carries from one row to its next: the pivot that selected the last row is the first one tried on
// the next.  Rows of one feature matrix mostly have their k-th largest value in about the same place, and a search
// that starts next to it needs about 5 pivots where one that starts from the row's range needs about 8.  All three
// fields are wave-uniform.
struct PivotHint {
    float pivot = 0.f;                // first pivot to try (clamped to the row's range)
    float step = 0.5f;                // first step, as a fraction of max|x|
    uint32_t bracketed = 0x80000000u;  // sign bit set: the target is known to lie within `step` (plain bisection)
};

// One row of H into registers: chunks of 64*V columns, V consecutive columns per lane.  Lanes past the row hold
// copies of its last chunk; select_row replaces them.  Nothing here touches the loaded values, so the loads of the
// rows ahead stay in flight until the row is used.
template <int E, int V>
__device__ __forceinline__ void load_row(const float* __restrict__ h, int dim, int lane, float (&v)[E])
{
#pragma unroll
    for (int c = 0; c < E / V; ++c) {
        const int base = c * (kWave * V) + lane * V;
        // every lane loads (lanes past the row re-read its last chunk and drop the result), so that no branch
        // surrounds the load and its place among the memory operations in flight is fixed
        const bool in = base < dim;  // dim % V == 0 on the vector paths
        const int at = in ? base : dim - V;
        if constexpr (V == 4) {
            const float4 x = *reinterpret_cast<const float4*>(h + at);
            v[c * 4 + 0] = x.x; v[c * 4 + 1] = x.y; v[c * 4 + 2] = x.z; v[c * 4 + 3] = x.w;
        } else if constexpr (V == 2) {
            const float2 x = *reinterpret_cast<const float2*>(h + at);
            v[c * 2 + 0] = x.x; v[c * 2 + 1] = x.y;
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) v[c * V + j] = h[base + j < dim ? base + j : dim - 1];
        }
    }
}

// CBSR packing of the selected entries of one row.  `stage` is this wavefront's own LDS area of 2*k + 64 words: the
// survivors are put there in CBSR order (value bits in [0, k), columns in [k, 2k)) and leave as whole-row stores, the
// t-th survivor by lane t.  Entries that are not selected are written to word 2k + lane, which nobody reads, so
// that no branch surrounds the LDS writes.  LDS operations of one wavefront execute in program order, so no barrier
// is needed inside the wavefront.
template <int E, int V, int VT, typename IdxT>
__device__ __forceinline__ void write_row(const bool (&sel)[E], const float (&v)[E], int k, int lane,
                                          uint32_t* __restrict__ stage, value_store_t<VT>* __restrict__ od,
                                          IdxT* __restrict__ oi)
{
    int pos[E];
    column_order_prefix<E, V>(sel, pos);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        stage[sel[e] ? pos[e] : 2 * k + lane] = __float_as_uint(v[e]);
        stage[sel[e] ? k + pos[e] : 2 * k + lane] = (uint32_t)column_of<V>(lane, e);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // The first 64 survivors: one store of each kind, issued by every lane (lanes past k repeat entry k-1), so that
    // the number of memory operations in flight never depends on a branch and the waits for the row loads are exact.
    const int t0 = lane < k ? lane : k - 1;
    od[t0] = narrow_value<VT>(__uint_as_float(stage[t0]));
    oi[t0] = (IdxT)stage[k + t0];
    for (int t = lane + kWave; t < k; t += kWave) {
        od[t] = narrow_value<VT>(__uint_as_float(stage[t]));
        oi[t] = (IdxT)stage[k + t];
    }
    __builtin_amdgcn_wave_barrier();  // the next row's survivors go to the same area
}

// Selection and CBSR packing of one row held in registers.  `stage` is this wavefront's own LDS area (see write_row).
// VT: storage format of the values written (MAXK_VALUE_*); selection always works on the fp32 input
// PAD: the row is shorter than the E*64 columns the lanes cover
template <int E, int V, bool PAD, int VT, typename IdxT>
__device__ __forceinline__ void select_row(const float (&raw)[E], int dim, int k, int lane, PivotHint& hint,
                                           uint32_t* __restrict__ stage, value_store_t<VT>* __restrict__ od,
                                           IdxT* __restrict__ oi)
{
    // columns past `dim` count as -inf: below every real entry in either stage, never selected
    float v[E];
    float amax = 0.f;  // largest magnitude of the row (the padding does not count)
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const bool in = !PAD || column_of<V>(lane, e) < dim;
        v[e] = in ? raw[e] : -__builtin_inff();
        amax = fmaxf(amax, in ? fabsf(raw[e]) : 0.f);
    }

    // Stage 1: search for a pivot on the value axis that keeps exactly k.  A wavefront's first row starts at pivot 0
    // and bisects [-max|x|, max|x|] (steps max|x| / 2, / 4, ...).  Later rows start at the pivot of the row before
    // (clamped to this row's range) with a step of max|x| / 32, which doubles while the count stays on the same
    // side of k and halves from the first change of side on.  The counts are scalar (ballot + scalar popcount).  The
    // pivot and the step are the same in every lane but are kept in vector registers (the empty asm hides that they
    // are uniform): the compares read them there, and a scalar copy would cost a move and wait states between
    // dependent vector and scalar instructions on every step.  The scalar unit's issue rate is what bounds this
    // kernel.
    const uint32_t amax_bits = wave_max_nonneg(amax);
    float pivot = 0.f;
    int kept = -1;  // entries the last pivot keeps
    if (amax_bits - 1u < 0x7F7FFFFFu && k < dim) {  // finite, not all zero (k = dim: every pivot above -max|x| keeps too few)
        constexpr uint32_t kSign = 0x80000000u;
        const float row_max = __uint_as_float(amax_bits);
        pivot = __builtin_amdgcn_fmed3f(hint.pivot, -row_max, row_max);
        uint32_t step_bits = __float_as_uint(hint.step * row_max);  // the step, signed: + moves the pivot up
        uint32_t bracketed = hint.bracketed;
        asm volatile("" : "+v"(pivot), "+v"(step_bits), "+v"(bracketed));
        const auto count = [&](float p) {
            int cnt = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v[e] >= p));
            return cnt;
        };
        kept = count(pivot);
        if (kept != k) {
            step_bits |= kept > k ? 0u : kSign;  // too few kept: move the pivot down
            for (int step = 1; step < kPivotSteps; ++step) {
                pivot += __uint_as_float(step_bits);
                kept = count(pivot);
                if (kept == k) break;
                const uint32_t down = kept > k ? 0u : kSign;
                bracketed |= down ^ step_bits;  // (sign bit) the count changed sides: the target is within the last step
                const float scale = (int32_t)bracketed < 0 ? 0.5f : 2.f;
                step_bits = __float_as_uint(__uint_as_float((step_bits & ~kSign) | down) * scale);
            }
        }
        if (kept == k) {
            hint.pivot = pivot;
            hint.step = 0.03125f;
            hint.bracketed = 0u;
        }
    }

    bool sel[E];
    if (kept == k) {
#pragma unroll
        for (int e = 0; e < E; ++e) sel[e] = v[e] >= pivot;
        write_row<E, V, VT, IdxT>(sel, v, k, lane, stage, od, oi);
        return;
    }
    {
        // Stage 2 (rows without such a pivot within kPivotSteps): k-th largest key by MSB-first descent;
        // `exact` = the prefix already keeps exactly k.  Padding columns get key 0, below every non-NaN key.
        uint32_t key[E];
#pragma unroll
        for (int e = 0; e < E; ++e) key[e] = (!PAD || column_of<V>(lane, e) < dim) ? order_key(v[e]) : 0u;
        uint32_t prefix = 0u;
        bool exact = false;
#pragma unroll 1
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
    }

    write_row<E, V, VT, IdxT>(sel, v, k, lane, stage, od, oi);
}

// One wavefront owns `rows_per_wave` consecutive rows and keeps the loads of the next two rows in flight while it
// selects from the current one: a row is only 4*dim bytes, and with one row per wavefront the kernel waited on
// memory latency (32 wavefronts per CU x 1 KB in flight).
template <int E, int V, bool PAD, int VT, typename IdxT>
__global__ __launch_bounds__(256) void topk_cbsr_kernel(const float* __restrict__ H, int64_t N, int dim, int k,
                                                        int rows_per_wave, value_store_t<VT>* __restrict__ sp_data,
                                                        IdxT* __restrict__ sp_index)
{
    extern __shared__ uint32_t topk_stage[];  // 2*k + 64 words per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform: rows and loop are scalar
    uint32_t* __restrict__ stage = topk_stage + w * (2 * k + kWave);
    const int64_t first = ((int64_t)blockIdx.x * (blockDim.x / kWave) + w) * rows_per_wave;
    if (first >= N) return;
    const int n = (int)(N - first < rows_per_wave ? N - first : rows_per_wave);  // rows of this wavefront
    const float* __restrict__ h0 = H + first * (int64_t)dim;
    value_store_t<VT>* __restrict__ od0 = sp_data + first * (int64_t)k;
    IdxT* __restrict__ oi0 = sp_index + first * (int64_t)k;

    // Three register buffers take turns (no copies: a copy would have to wait for the newest load).  Every turn
    // issues exactly one row load - past the wavefront's last row it re-reads that row - so that the number of
    // memory operations in flight is the same on every path and the waits can be exact.
    float a[E], b[E], c[E];
    PivotHint hint;
    // rows_per_wave * dim and rows_per_wave * k fit 32 bits (at most 8 rows of at most MAXK_MAX_DIM columns)
#define MAXK_TOPK_LOAD(buf, i) load_row<E, V>(h0 + ((i) < n ? (i) : n - 1) * dim, dim, lane, buf)
#define MAXK_TOPK_SELECT(buf, i) \
    select_row<E, V, PAD, VT, IdxT>(buf, dim, k, lane, hint, stage, od0 + (i) * k, oi0 + (i) * k)
    MAXK_TOPK_LOAD(a, 0);
    MAXK_TOPK_LOAD(b, 1);
    // Whole turns of three rows; the loop is left only at its end (an exit from the middle would reach the loop's
    // latch with a load still in flight on that path, and the waits of every turn would have to allow for it).
    int i = 0;
    for (; i + 2 < n; i += 3) {
        MAXK_TOPK_LOAD(c, i + 2);
        MAXK_TOPK_SELECT(a, i);
        MAXK_TOPK_LOAD(a, i + 3);
        MAXK_TOPK_SELECT(b, i + 1);
        MAXK_TOPK_LOAD(b, i + 4);
        MAXK_TOPK_SELECT(c, i + 2);
    }
    if (i < n) {  // one or two rows left: they are in a and b
        MAXK_TOPK_SELECT(a, i);
        if (i + 1 < n) MAXK_TOPK_SELECT(b, i + 1);
    }
#undef MAXK_TOPK_LOAD
#undef MAXK_TOPK_SELECT
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
    const int waves_per_block = 4;
    // rows per wavefront: up to 8, fewer when that would leave CUs without work (256 CUs x 32 wavefronts)
    int rows_per_wave = (int)std::min<int64_t>(8, std::max<int64_t>(1, N / (256 * 32)));
    const int64_t rows_per_block = (int64_t)waves_per_block * rows_per_wave;
    const int64_t blocks = (N + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(waves_per_block * kWave);
    const size_t lds = sizeof(uint32_t) * (2 * (size_t)k + kWave) * waves_per_block;  // k <= MAXK_MAX_DIM: at most 33 KiB
    auto* od = (value_store_t<VT>*)sp_data;
#define MAXK_TOPK_LAUNCH(PAD, IDX) \
    hipLaunchKernelGGL((topk_cbsr_kernel<E, V, PAD, VT, IDX>), grid, block, lds, s, H, N, dim, k, rows_per_wave, od, (IDX*)sp_index)
    const bool pad = dim != E * kWave;
    switch (index_bytes) {
        case 1: if (pad) MAXK_TOPK_LAUNCH(true, uint8_t); else MAXK_TOPK_LAUNCH(false, uint8_t); break;
        case 2: if (pad) MAXK_TOPK_LAUNCH(true, uint16_t); else MAXK_TOPK_LAUNCH(false, uint16_t); break;
        default: if (pad) MAXK_TOPK_LAUNCH(true, int32_t); else MAXK_TOPK_LAUNCH(false, int32_t); break;
    }
#undef MAXK_TOPK_LAUNCH
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
