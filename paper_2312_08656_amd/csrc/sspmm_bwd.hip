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
//    Bound by the rate at which L2 retires fp32 atomics (~330 G/s measured), not bytes.
//
//  expand/reduce (Alg. 2's staging, no atomics): phase 1 is the push kernel with
//    the atomic replaced by a plain store of each entry's k products into a
//    per-graph buffer in CSR entry order (one long sequential, fully coalesced
//    write); phase 2 walks A^T in CSC order and, for destination j, gathers the
//    4k-byte product rows of its in-entries (full cache lines, float4 per lane)
//    and sums them in registers.  Moves 8k bytes per entry instead of 4k, but at
//    memory bandwidth instead of atomic rate, and the result is deterministic.
//
//  slab pull (owner computes, tiled for L2): the pull kernel is bound by fetching
//    ~dim/32 cache lines of a dY row per entry from beyond L2 (~7 G rows/s at
//    dim 256); the same sampled gather runs at ~30 G rows/s when the rows sit in
//    the XCD's 4 MB L2.  So the source rows are swept in slabs of a few MB of dY,
//    ONE LAUNCH PER SLAB (every XCD gathers from the same slab, so each L2 holds
//    one copy; the launch boundary is what keeps all wavefronts on one slab --
//    letting them run ahead into the next slab was measured to lose the locality,
//    and it would also race on dXs): a launch walks the non-empty
//    (slab, destination) visits and adds the visit's in-entries to the
//    destination's dXs row (read-modify-write, the row is revisited once per
//    slab).  Pays off when a visit has several entries, i.e. dense neighbourhoods.
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <algorithm>

#include "common.hpp"

namespace maxk {
namespace {

// VEC consecutive sp_index entries fetched with one load
template <typename IdxT, int VEC>
struct IdxPack;
template <>
struct IdxPack<uint8_t, 4> {
    uint32_t w;
    __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint32_t*>(p); }
    __device__ __forceinline__ int get(int i) const { return (w >> (8 * i)) & 0xFFu; }
};
template <>
struct IdxPack<uint16_t, 4> {
    uint2 w;
    __device__ __forceinline__ void load(const uint16_t* p) { w = *reinterpret_cast<const uint2*>(p); }
    __device__ __forceinline__ int get(int i) const { return ((i < 2 ? w.x : w.y) >> (16 * (i & 1))) & 0xFFFFu; }
};
template <>
struct IdxPack<int32_t, 4> {
    int4 w;
    __device__ __forceinline__ void load(const int32_t* p) { w = *reinterpret_cast<const int4*>(p); }
    __device__ __forceinline__ int get(int i) const { return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w; }
};
template <typename IdxT>
struct IdxPack<IdxT, 1> {
    int w;
    __device__ __forceinline__ void load(const IdxT* p) { w = (int)*p; }
    __device__ __forceinline__ int get(int) const { return w; }
};

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

// -------------------------------------------------------- expand / reduce ----

constexpr int kExpandRounds = 8;
constexpr int kReduceUnroll = 4;

// Phase 1: expand[p*k + t] = val[p] * dY[row(p), sp_index[col[p]*k + t]] for every stored entry p.
// VEC = CBSR positions per lane (4: one packed index load + one float4 store per lane; else 1).
template <int K, int VEC, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_expand_kernel(const WorkItem* __restrict__ items,
                                                           const int32_t* __restrict__ col,
                                                           const float* __restrict__ val, const float* __restrict__ dY,
                                                           const IdxT* __restrict__ sp_index, int dim, int k_rt,
                                                           float* __restrict__ expand)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    if (it.begin == it.end) return;
    const int k = K ? K : k_rt;
    const int kq = k / VEC;  // units per stored entry
    float* __restrict__ g_row = lds;                                                  // dY[row,:]
    int2* __restrict__ entry_buf = reinterpret_cast<int2*>(lds + ((dim + 1) & ~1));   // 64 staged (col, val)
    const float* __restrict__ src = dY + (int64_t)it.row * dim;
    for (int c = lane; c < dim; c += kWave) g_row[c] = src[c];

    for (int base = it.begin; base < it.end; base += kWave) {
        const int n = min(kWave, it.end - base);
        __syncthreads();
        if (lane < n) entry_buf[lane] = make_int2(col[base + lane], __float_as_int(val[base + lane]));
        __syncthreads();
        const int units = n * kq;
        float* __restrict__ dst = expand + (int64_t)base * k;  // this batch's products are contiguous
        for (int u0 = 0; u0 < units; u0 += kWave * kExpandRounds) {
            IdxPack<IdxT, VEC> ix[kExpandRounds];
            float a[kExpandRounds];
            bool ok[kExpandRounds];
#pragma unroll
            for (int r = 0; r < kExpandRounds; ++r) {
                const int u = u0 + r * kWave + lane;
                ok[r] = u < units;
                const int uc = ok[r] ? u : 0;
                const int e = uc / kq;
                const int q = uc - e * kq;
                const int2 ed = entry_buf[e];
                a[r] = __int_as_float(ed.y);
                ix[r].load(sp_index + (int64_t)ed.x * k + q * VEC);
            }
#pragma unroll
            for (int r = 0; r < kExpandRounds; ++r) {
                if (ok[r]) {
                    const int u = u0 + r * kWave + lane;
                    if constexpr (VEC == 4) {
                        *reinterpret_cast<float4*>(dst + (int64_t)u * 4) =
                            make_float4(a[r] * g_row[ix[r].get(0)], a[r] * g_row[ix[r].get(1)],
                                        a[r] * g_row[ix[r].get(2)], a[r] * g_row[ix[r].get(3)]);
                    } else {
                        dst[u] = a[r] * g_row[ix[r].get(0)];
                    }
                }
            }
        }
    }
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

template <int VEC, typename IdxT>
maxk_status launch_expand_t(const ItemList& L, const int32_t* col, const float* val, const float* dY,
                            const IdxT* sp_index, int dim, int k, float* expand, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
    const size_t lds = sizeof(float) * (size_t)((dim + 1) & ~1) + sizeof(int2) * kWave;
#define MAXK_EXPAND(K) \
    hipLaunchKernelGGL((bwd_expand_kernel<K, VEC, IdxT>), grid, block, lds, s, L.d_items, col, val, dY, sp_index, dim, k, expand)
    switch (k) {
        case 8: MAXK_EXPAND(8); break;
        case 16: MAXK_EXPAND(16); break;
        case 32: MAXK_EXPAND(32); break;
        case 64: MAXK_EXPAND(64); break;
        case 96: MAXK_EXPAND(96); break;
        case 128: MAXK_EXPAND(128); break;
        case 192: MAXK_EXPAND(192); break;
        default: MAXK_EXPAND(0); break;
    }
#undef MAXK_EXPAND
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <typename IdxT>
maxk_status launch_expand_i(const ItemList& L, const int32_t* col, const float* val, const float* dY,
                            const IdxT* sp_index, int dim, int k, float* expand, hipStream_t s)
{
    const bool vec = (k % 4 == 0) && aligned(sp_index, 4 * sizeof(IdxT)) && aligned(expand, 16);
    return vec ? launch_expand_t<4>(L, col, val, dY, sp_index, dim, k, expand, s)
               : launch_expand_t<1>(L, col, val, dY, sp_index, dim, k, expand, s);
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

// ------------------------------------------------------------- slab pull ----

// dY[row * dim + col] with the element offset held in 32 bits when OFF32 (the launcher checks
// that the whole of dY spans less than 4 GiB): one SGPR base + 32-bit lane offsets instead of
// 64-bit lane addresses, which is what keeps the kernel at 8 waves per SIMD.
template <bool OFF32>
__device__ __forceinline__ float load_sampled(const float* __restrict__ dY, int32_t row, int dim, int32_t col)
{
    if constexpr (OFF32) {
        const uint32_t byte_off = ((uint32_t)row * (uint32_t)dim + (uint32_t)col) * 4u;
        return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(dY) + byte_off);
    } else {
        return dY[(int64_t)row * dim + col];
    }
}

// VEC CBSR positions per lane, STRIDED: lane q of a visit holds positions q, q + k/VEC, q + 2k/VEC, ...
// so that one gather instruction covers k/VEC CONSECUTIVE (ascending-column) positions of each visit
// and every cache line of a dY row is requested by one instruction only;
// LPD lanes per destination (power of two >= min(k / VEC, 64)); 64 / LPD visits per wave step.
// Visits longer than kSlabLongVisit entries are skipped by the lane groups and worked on by whole
// wavefronts instead (the first n_long_blocks workgroups): the 64 / LPD groups take every G-th entry
// and their sums are added across the wave, so a hub destination does not become the launch's tail.
// Within one launch every destination occurs in at most one visit, so the read-modify-write of its
// dXs row needs no atomics; launches of consecutive slabs are ordered by the stream.
template <int VEC, int LPD, bool OFF32, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_slab_kernel(const int32_t* __restrict__ visit_node,
                                                         const int32_t* __restrict__ visit_begin, int64_t v_begin,
                                                         int64_t v_end, const int32_t* __restrict__ long_visit,
                                                         int64_t l_begin, int64_t l_end, int n_long_blocks,
                                                         const int32_t* __restrict__ slab_src,
                                                         const float* __restrict__ slab_val,
                                                         const float* __restrict__ dY,
                                                         const IdxT* __restrict__ sp_index, int dim, int k,
                                                         float* __restrict__ dXs)
{
    constexpr int G = kWave / LPD;
    const int lane = threadIdx.x;
    const int q0 = lane % LPD, g = lane / LPD;
    const int kq = k / VEC;
    if ((int)blockIdx.x < n_long_blocks) {
        for (int64_t l = l_begin + blockIdx.x; l < l_end; l += n_long_blocks) {
            const int64_t v = long_visit[l];
            const int64_t j = visit_node[v];
            const int b = visit_begin[v], e = visit_begin[v + 1];
            for (int qb = 0; qb < kq; qb += LPD) {  // one pass unless k / VEC > 64
                const int q = qb + q0;
                const bool active = q < kq;
                const int64_t o = j * k + (active ? q : 0);  // lane's positions: o + c * kq
                int32_t my[VEC];
                float acc[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    my[c] = (int32_t)sp_index[o + c * kq];
                    acc[c] = 0.f;
                }
                for (int p0 = b; p0 < e; p0 += G * 4) {
                    float gv[4][VEC], a[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int p = p0 + u * G + g;
                        const bool ok = p < e;
                        const int pc = ok ? p : b;
                        const int32_t row = slab_src[pc];
                        a[u] = ok ? slab_val[pc] : 0.f;
#pragma unroll
                        for (int c = 0; c < VEC; ++c) {
                            const float x = load_sampled<OFF32>(dY, row, dim, my[c]);
                            gv[u][c] = ok ? x : 0.f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int c = 0; c < VEC; ++c) acc[c] += a[u] * gv[u][c];
                }
#pragma unroll
                for (int off = LPD; off < kWave; off <<= 1)
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[c] += __shfl_xor(acc[c], off);
                if (g == 0 && active) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) dXs[o + c * kq] += acc[c];
                }
            }
        }
        return;
    }
    // The kernel is bound by L1 tag look-ups (rocprof: ~1 per clock per CU), and a load whose lanes all read
    // one address still costs one look-up per 4 lanes.  So everything that is the same for the lanes of a
    // visit (header, sources, values) is fetched by as few lanes as possible -- lane u of the group fetches
    // entry u -- and handed round with lane shuffles, which do not go through the L1.
    const int64_t first = (int64_t)(blockIdx.x - n_long_blocks) * G;
    const int64_t stride = (int64_t)(gridDim.x - n_long_blocks) * G;
    const int gbase = g * LPD;  // first lane of this lane group
    for (int64_t v0 = v_begin + first; v0 < v_end; v0 += stride) {  // uniform; one step when the grid covers all visits
        const int64_t v = v0 + g;
        const bool have = v < v_end;
        int b, e;
        int64_t j;
        if constexpr (LPD >= 2) {
            int hdr = 0, nd = 0;
            if (have && q0 < 2) hdr = visit_begin[v + q0];
            if (have && q0 == 0) nd = visit_node[v];
            b = __shfl(hdr, gbase);
            e = __shfl(hdr, gbase + 1);
            j = __shfl(nd, gbase);
        } else {
            b = have ? visit_begin[v] : 0;
            e = have ? visit_begin[v + 1] : 0;
            j = have ? visit_node[v] : 0;
        }
        const int cnt = e - b;
        const bool work = have && cnt <= kSlabLongVisit;
        for (int qb = 0; qb < kq; qb += LPD) {  // one pass unless k / VEC > 64
            const int q = qb + q0;
            const bool active = work && q < kq;
            const int64_t o = j * k + (active ? q : 0);  // lane's positions: o + c * kq
            int32_t my[VEC];
            float acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                my[c] = active ? (int32_t)sp_index[o + c * kq] : 0;
                acc[c] = active ? dXs[o + c * kq] : 0.f;
            }
            for (int p0 = 0; p0 < kSlabLongVisit; p0 += LPD) {
                if (!__any(work && p0 < cnt)) break;
                const bool mine = work && p0 + q0 < cnt;
                const int32_t src_m = mine ? slab_src[b + p0 + q0] : 0;
                const float val_m = mine ? slab_val[b + p0 + q0] : 0.f;
                const int nb = work ? min(LPD, cnt - p0) : 0;  // entries of this batch for this group
                for (int u0 = 0; u0 < LPD; u0 += 4) {
                    if (!__any(u0 < nb)) break;
                    float gv[4][VEC], a[4];
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) {
                        const int u = u0 + uu;
                        const int from = gbase + (u < LPD ? u : 0);
                        const int32_t row = __shfl(src_m, from);
                        const float av = __shfl(val_m, from);
                        const bool ok = active && u < nb;
                        a[uu] = ok ? av : 0.f;
#pragma unroll
                        for (int c = 0; c < VEC; ++c) {
                            float x = 0.f;
                            if (ok) x = load_sampled<OFF32>(dY, row, dim, my[c]);
                            gv[uu][c] = x;
                        }
                    }
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu)
#pragma unroll
                        for (int c = 0; c < VEC; ++c) acc[c] += a[uu] * gv[uu][c];
                }
            }
            if (active) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) dXs[o + c * kq] = acc[c];
            }
        }
    }
}

// One wave step per workgroup measured best (6.8 -> 6.4 ms at k=32 against a grid capped at the number of
// resident wavefronts): the hardware dispatcher hides the two dependent loads that open a visit better
// than a software loop over visits does.
inline int64_t slab_grid_cap() { return 0x7FFF0000ll; }

template <int VEC, bool OFF32, typename IdxT>
maxk_status launch_slab_t(const SlabSet& S, const float* dY, const IdxT* sp_index, int dim, int k, float* dXs,
                          hipStream_t s)
{
    const int kq = k / VEC;
    for (int32_t sl = 0; sl < S.n_slabs; ++sl) {
        const int64_t vb = S.h_slab_visit[sl], ve = S.h_slab_visit[sl + 1];
        if (vb >= ve) continue;
        const int64_t lb = S.h_slab_long[sl], le = S.h_slab_long[sl + 1];
        const int nlb = (int)std::min<int64_t>(le - lb, 4096);
#define MAXK_SLAB(LPD)                                                                                             \
    do {                                                                                                           \
        const int64_t tasks = (ve - vb + (kWave / LPD) - 1) / (kWave / LPD);                                       \
        const unsigned grid = (unsigned)std::min<int64_t>(tasks, slab_grid_cap());                                 \
        hipLaunchKernelGGL((bwd_slab_kernel<VEC, LPD, OFF32, IdxT>), dim3(grid + (unsigned)nlb), dim3(kWave), 0, s,      \
                           S.d_visit_node, S.d_visit_begin, vb, ve, S.d_long_visit, lb, le, nlb, S.d_src, S.d_val, \
                           dY, sp_index, dim, k, dXs);                                                             \
    } while (0)
        if (kq <= 1) MAXK_SLAB(1);
        else if (kq <= 2) MAXK_SLAB(2);
        else if (kq <= 4) MAXK_SLAB(4);
        else if (kq <= 8) MAXK_SLAB(8);
        else if (kq <= 16) MAXK_SLAB(16);
        else if (kq <= 32) MAXK_SLAB(32);
        else MAXK_SLAB(64);
#undef MAXK_SLAB
    }
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <typename IdxT>
maxk_status launch_slab_i(const SlabSet& S, const float* dY, const IdxT* sp_index, int64_t N, int dim, int k,
                          float* dXs, hipStream_t s)
{
    const bool off32 = N * (int64_t)dim * 4 <= 0xFFFFFFFFll;
    // positions per lane, measured on the dense workload (ms at k = 8 / 16 / 32 / 64 / 128):
    //   1: 3.69 / 4.71 / 5.79 / 8.32 / 13.8     2: 3.83 / 4.83 / 5.57 / 6.75 / 14.5     4: 4.47 / 5.38 / 6.21 / 6.84 / 9.63
    if (k <= 16)
        return off32 ? launch_slab_t<1, true>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<1, false>(S, dY, sp_index, dim, k, dXs, s);
    if (k % 2 == 0 && k <= 64)
        return off32 ? launch_slab_t<2, true>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<2, false>(S, dY, sp_index, dim, k, dXs, s);
    if (k % 4 == 0)
        return off32 ? launch_slab_t<4, true>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<4, false>(S, dY, sp_index, dim, k, dXs, s);
    return off32 ? launch_slab_t<1, true>(S, dY, sp_index, dim, k, dXs, s)
                 : launch_slab_t<1, false>(S, dY, sp_index, dim, k, dXs, s);
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

maxk_status launch_bwd_expand_reduce(const ItemList& csr_items, const int32_t* col, const float* val,
                                     const ItemList& csc_items, const uint32_t* csc_entry, const float* dY,
                                     const void* sp_index, int index_bytes, int dim, int k, float* expand,
                                     float* dXs, float* partials, hipStream_t s)
{
    if (csc_items.n_items == 0) return MAXK_OK;
    if (csr_items.n_items > 0x7FFFFFFF || csc_items.n_items > 0x7FFFFFFF) return MAXK_UNSUPPORTED;
    maxk_status st = MAXK_OK;
    if (csr_items.n_items) {
        if (index_bytes == 1) st = launch_expand_i(csr_items, col, val, dY, (const uint8_t*)sp_index, dim, k, expand, s);
        else if (index_bytes == 2) st = launch_expand_i(csr_items, col, val, dY, (const uint16_t*)sp_index, dim, k, expand, s);
        else st = launch_expand_i(csr_items, col, val, dY, (const int32_t*)sp_index, dim, k, expand, s);
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

maxk_status launch_bwd_slab_pull(const SlabSet& S, const float* dY, const void* sp_index, int index_bytes, int64_t N,
                                 int dim, int k, float* dXs, hipStream_t s)
{
    maxk_status st = launch_fill_zero(dXs, N * (int64_t)k, s);
    if (st != MAXK_OK || S.n_visits == 0) return st;
    if (index_bytes == 1) return launch_slab_i(S, dY, (const uint8_t*)sp_index, N, dim, k, dXs, s);
    if (index_bytes == 2) return launch_slab_i(S, dY, (const uint16_t*)sp_index, N, dim, k, dXs, s);
    return launch_slab_i(S, dY, (const int32_t*)sp_index, N, dim, k, dXs, s);
}

}  // namespace maxk
