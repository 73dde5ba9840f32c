// Backward aggregation: sampled SSpMM  dXs = (A^T dY) at each row's CBSR columns
// (Eq. 2 right; Eq. 3; prior art: Alg. 2).  Four kernels with the same result:
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
//    Two forms: the sampled gather (small k), and from k >= dim/8 a form that adds
//    up whole dY rows in registers and samples the sum once per visit.
//
// This header holds the kernel templates that read dY; one translation unit per storage format of dY
// (fp32, bf16, fp16: the 16-bit formats are widened exactly, products and sums are fp32 throughout)
// instantiates them, so the three compile side by side.
#pragma once

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <algorithm>

#include "common.hpp"

namespace maxk {

// implemented once per storage format of dY (sspmm_bwd_f32.hip, _bf16.hip, _f16.hip)
template <int VT>
maxk_status bwd_pull_format(const ItemList& L, const int32_t* csc_src, const float* csc_val, const void* dY,
                            const void* sp_index, int index_bytes, int dim, int k, float* dXs, float* partials,
                            hipStream_t s);
template <int VT>
maxk_status bwd_push_format(const ItemList& L, const int32_t* col, const float* val, const void* dY,
                            const void* sp_index, int index_bytes, int dim, int k, float* dXs, hipStream_t s);
template <int VT>
maxk_status bwd_expand_format(const ItemList& L, const int32_t* col, const float* val, const void* dY,
                              const void* sp_index, int index_bytes, int dim, int k, float* expand, hipStream_t s);
template <int VT>
maxk_status bwd_slab_format(const SlabSet& S, const void* dY, const void* sp_index, int index_bytes, int64_t N,
                            int dim, int k, float* dXs, hipStream_t s);

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
template <int KP, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_pull_small_kernel(const WorkItem* __restrict__ items,
                                                               const int32_t* __restrict__ csc_src,
                                                               const float* __restrict__ csc_val,
                                                               const value_store_t<VT>* __restrict__ dY,
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
            const float x = widen_value<VT>(dY[(int64_t)csc_src[q] * dim + my_idx]);
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
template <int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_pull_wide_kernel(const WorkItem* __restrict__ items,
                                                              const int32_t* __restrict__ csc_src,
                                                              const float* __restrict__ csc_val,
                                                              const value_store_t<VT>* __restrict__ dY,
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
                const float x = widen_value<VT>(dY[(int64_t)csc_src[q] * dim + my_idx]);
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

// K > 0: k known at compile time
template <int K, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_push_kernel(const WorkItem* __restrict__ items,
                                                         const int32_t* __restrict__ col,
                                                         const float* __restrict__ val, const value_store_t<VT>* __restrict__ dY,
                                                         const IdxT* __restrict__ sp_index, int dim, int k_rt,
                                                         float* __restrict__ dXs)
{
    extern __shared__ float g_row[];
    const int lane = threadIdx.x;
    const WorkItem it = items[blockIdx.x];
    if (it.begin == it.end) return;
    const int k = K ? K : k_rt;
    const value_store_t<VT>* __restrict__ src = dY + (int64_t)it.row * dim;
    for (int c = lane; c < dim; c += kWave) g_row[c] = widen_value<VT>(src[c]);
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

// Phase 1: expand[p*k + t] = val[p] * dY[row(p), sp_index[col[p]*k + t]] for every stored entry p.
// VEC = CBSR positions per lane (4: one packed index load + one float4 store per lane; else 1).
template <int K, int VEC, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_expand_kernel(const WorkItem* __restrict__ items,
                                                           const int32_t* __restrict__ col,
                                                           const float* __restrict__ val, const value_store_t<VT>* __restrict__ dY,
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
    const value_store_t<VT>* __restrict__ src = dY + (int64_t)it.row * dim;
    for (int c = lane; c < dim; c += kWave) g_row[c] = widen_value<VT>(src[c]);

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

template <int VEC, int VT, typename IdxT>
maxk_status launch_expand_t(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* dY,
                            const IdxT* sp_index, int dim, int k, float* expand, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
    const size_t lds = sizeof(float) * (size_t)((dim + 1) & ~1) + sizeof(int2) * kWave;
#define MAXK_EXPAND(K) \
    hipLaunchKernelGGL((bwd_expand_kernel<K, VEC, VT, IdxT>), grid, block, lds, s, L.d_items, col, val, dY, sp_index, dim, k, expand)
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

template <int VT, typename IdxT>
maxk_status launch_expand_i(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* dY,
                            const IdxT* sp_index, int dim, int k, float* expand, hipStream_t s)
{
    const bool vec = (k % 4 == 0) && aligned(sp_index, 4 * sizeof(IdxT)) && aligned(expand, 16);
    return vec ? launch_expand_t<4, VT>(L, col, val, dY, sp_index, dim, k, expand, s)
               : launch_expand_t<1, VT>(L, col, val, dY, sp_index, dim, k, expand, s);
}

// ------------------------------------------------------------- slab pull ----

// dY[row * dim + col] with the byte offset held in 32 bits when OFF32 (the launcher checks
// that the whole of dY spans less than 4 GiB): one SGPR base + 32-bit lane offsets instead of
// 64-bit lane addresses, which is what keeps the kernel at 8 waves per SIMD.
template <bool OFF32, int VT>
__device__ __forceinline__ float load_sampled(const value_store_t<VT>* __restrict__ dY, int32_t row, int dim, int32_t col)
{
    using T = value_store_t<VT>;
    if constexpr (OFF32) {
        const uint32_t byte_off = ((uint32_t)row * (uint32_t)dim + (uint32_t)col) * (uint32_t)sizeof(T);
        if constexpr (sizeof(T) == 4) {
            return widen_value<VT>(*reinterpret_cast<const T*>(reinterpret_cast<const char*>(dY) + byte_off));
        } else {
            // 16-bit elements: fetch the aligned dword that holds the element and pick the half.  Two-byte
            // gathers were measured far slower than dword gathers here (15.8 against 9.6 ms at k = 128 for half
            // the cache lines).  The launcher takes this path only when dY is 4-byte aligned and holds an even
            // number of elements, so the dword never reaches past the array.
            const uint32_t w = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(dY) + (byte_off & ~3u));
            if constexpr (VT == MAXK_VALUE_BF16) return __uint_as_float((byte_off & 2u) ? (w & 0xFFFF0000u) : (w << 16));
            else return widen_value<VT>((uint16_t)((byte_off & 2u) ? (w >> 16) : (w & 0xFFFFu)));
        }
    } else {
        return widen_value<VT>(dY[(int64_t)row * dim + col]);
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
template <int VEC, int LPD, bool OFF32, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_slab_kernel(const int32_t* __restrict__ visit_node,
                                                         const int32_t* __restrict__ visit_begin, int64_t v_begin,
                                                         int64_t v_end, const int32_t* __restrict__ long_visit,
                                                         int64_t l_begin, int64_t l_end, int n_long_blocks,
                                                         int long_pad, int64_t tasks_per_xcd,
                                                         const int32_t* __restrict__ slab_src,
                                                         const float* __restrict__ slab_val,
                                                         const value_store_t<VT>* __restrict__ dY,
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
                            const float x = load_sampled<OFF32, VT>(dY, row, dim, my[c]);
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
    // Workgroup b runs on XCD b % 8 (measured).  The visits of the launch are cut into 8 contiguous ranges, one per
    // XCD, so that the streamed arrays (headers, entries, CBSR indices: several visits per cache line) are pulled
    // into one L2 only instead of into up to four.  Blocks [n_long_blocks, long_pad) idle so that the ranges line up.
    const int64_t wg = (int64_t)blockIdx.x - long_pad;
    if (wg < 0) return;
    const int64_t v0 = v_begin + ((wg & 7) * tasks_per_xcd + (wg >> 3)) * G;
    if ((wg >> 3) >= tasks_per_xcd || v0 >= v_end) return;
    const int gbase = g * LPD;  // first lane of this lane group
    {
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
                            if (ok) x = load_sampled<OFF32, VT>(dY, row, dim, my[c]);
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

// ---- slab pull, row-accumulating form (large k) ----
//
// From k = 32 up the sampled gather above spends about one L1 access per sampled element.  Here a visit
// instead adds up WHOLE dY rows -- one 16-byte load per lane covers a 1 KB row with 16 L1 accesses -- into
// the full row of (A^T dY)[j, :] held in registers (lane l keeps columns 4l..4l+3 of every 256-column chunk),
// and samples that row at the destination's k columns once per visit, through LDS.  The arithmetic grows from
// k to dim multiply-adds per entry, which the vector units absorb; cache lines per entry are those of the
// whole row, so this form is for k large enough that the sampled form touches all of them anyway.
// One wavefront walks VPW consecutive visits; the entries of the next visit are fetched while the rows of the
// current one are in flight.
// A lane's share of a dY row: 4 consecutive elements (16 bytes of fp32, 8 bytes of a 16-bit format; 16-byte pieces
// on half the lanes were measured slower for the 16-bit formats).
template <int VT>
struct row_piece { using type = float4; static constexpr int n = 4; };
template <>
struct row_piece<MAXK_VALUE_BF16> { using type = uint2; static constexpr int n = 4; };
template <>
struct row_piece<MAXK_VALUE_F16> { using type = uint2; static constexpr int n = 4; };

template <int VT>
__device__ __forceinline__ void fma_piece(float (&acc)[row_piece<VT>::n], float a, typename row_piece<VT>::type x)
{
    if constexpr (VT == MAXK_VALUE_F32) {
        acc[0] += a * x.x; acc[1] += a * x.y; acc[2] += a * x.z; acc[3] += a * x.w;
    } else {
        const uint32_t w[2] = {x.x, x.y};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            acc[2 * i] += a * widen_value<VT>((uint16_t)(w[i] & 0xFFFFu));
            acc[2 * i + 1] += a * widen_value<VT>((uint16_t)(w[i] >> 16));
        }
    }
}

constexpr int kRowAccInFlight = 8;  // dY rows a wavefront has in flight

// Eight consecutive regrouped entries (source row, weight).  Their addresses are wave-uniform, so they are fetched
// with scalar loads into scalar registers: no vector instruction and no L1 access is spent on them.
struct entry_batch {
    int32_t row[kRowAccInFlight];
    float w[kRowAccInFlight];
};

__device__ __forceinline__ entry_batch load_entry_batch(const int32_t* __restrict__ slab_src,
                                                        const float* __restrict__ slab_val, int pos)
{
    entry_batch en;  // may read up to 8 entries past the last one of the launch: the arrays are padded by 8
#pragma unroll
    for (int i = 0; i < kRowAccInFlight; ++i) {
        en.row[i] = slab_src[pos + i];
        en.w[i] = slab_val[pos + i];
    }
    return en;
}

// CNT rows loaded back to back, then added up.  The count is a template parameter so that a batch is straight-line
// code with exactly its own loads -- padding short batches with repeated rows cost 16 L1 accesses per padded row,
// and branches around single loads stopped the compiler from keeping a batch's rows in flight together.
// FULL: dim == RC * 256, every lane holds valid columns in every chunk.
template <int CNT, int RC, bool FULL, int VT>
__device__ __forceinline__ void rowacc_batch(float (&acc)[RC][row_piece<VT>::n], const entry_batch& en,
                                             const value_store_t<VT>* __restrict__ dY, int dim, int lane,
                                             const bool (&col_ok)[RC])
{
    using piece_t = typename row_piece<VT>::type;
    constexpr int EPL = row_piece<VT>::n;
    constexpr int CHUNK = kWave * EPL;
    piece_t x[CNT][RC];
#pragma unroll
    for (int uu = 0; uu < CNT; ++uu) {
        const value_store_t<VT>* __restrict__ r = dY + (int64_t)en.row[uu] * dim + lane * EPL;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
            if constexpr (FULL) {
                x[uu][c] = *reinterpret_cast<const piece_t*>(r + c * CHUNK);
            } else {
                piece_t z = {};
                if (col_ok[c]) z = *reinterpret_cast<const piece_t*>(r + c * CHUNK);
                x[uu][c] = z;
            }
        }
    }
#pragma unroll
    for (int uu = 0; uu < CNT; ++uu)
#pragma unroll
        for (int c = 0; c < RC; ++c) fma_piece<VT>(acc[c], en.w[uu], x[uu][c]);
}

// RC: chunks of 64 row pieces (256 columns) that cover a row
template <int RC, bool FULL, int VT, typename IdxT>
__global__ __launch_bounds__(kWave) void bwd_slab_rowacc_kernel(const int32_t* __restrict__ visit_node,
                                                                const int32_t* __restrict__ visit_begin,
                                                                int64_t v_begin, int64_t v_end, int visits_per_wave,
                                                                int64_t tasks_per_xcd,
                                                                const int32_t* __restrict__ slab_src,
                                                                const float* __restrict__ slab_val,
                                                                const value_store_t<VT>* __restrict__ dY,
                                                                const IdxT* __restrict__ sp_index, int dim, int k,
                                                                float* __restrict__ dXs)
{
    constexpr int EPL = row_piece<VT>::n;      // elements per lane and chunk
    constexpr int CHUNK = kWave * EPL;         // columns per chunk
    constexpr int U = kRowAccInFlight;
    __shared__ __attribute__((aligned(16))) float row_acc[RC * CHUNK];
    const int lane = threadIdx.x;
    const int64_t wg = blockIdx.x;  // workgroup b runs on XCD b % 8: each XCD takes a contiguous range of visits
    if ((wg >> 3) >= tasks_per_xcd) return;
    const int64_t v0 = v_begin + ((wg & 7) * tasks_per_xcd + (wg >> 3)) * visits_per_wave;
    if (v0 >= v_end) return;
    const int nv = (int)min((int64_t)visits_per_wave, v_end - v0);  // <= 32
    const int hdr_begin = (lane <= nv) ? visit_begin[v0 + lane] : 0;
    const int hdr_node = (lane < nv) ? visit_node[v0 + lane] : 0;
    bool col_ok[RC];
#pragma unroll
    for (int c = 0; c < RC; ++c) col_ok[c] = c * CHUNK + lane * EPL < dim;  // dim % 4 == 0 on this path

    // the entries of consecutive visits are consecutive in the regrouped arrays: one running position
    int pos = __builtin_amdgcn_readfirstlane(__shfl(hdr_begin, 0));
    entry_batch cur = load_entry_batch(slab_src, slab_val, pos);
    for (int n = 0; n < nv; ++n) {
        const int64_t j = __builtin_amdgcn_readfirstlane(__shfl(hdr_node, n));
        const int e = __builtin_amdgcn_readfirstlane(__shfl(hdr_begin, n + 1));
        // the destination's columns and its dXs values are asked for now and used after the rows (k <= 128: two
        // per lane are held in registers; beyond that the tail is fetched at the end)
        int col_t[2];
        float dx_t[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = lane + h * kWave;
            col_t[h] = (t < k) ? (int)sp_index[j * k + t] : 0;
            dx_t[h] = (t < k) ? dXs[j * k + t] : 0.f;
        }
        float acc[RC][EPL];
#pragma unroll
        for (int c = 0; c < RC; ++c)
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[c][i] = 0.f;
        while (pos < e) {
            const int cnt = min(e - pos, U);
            // the next batch (of this visit or the next one) is fetched under this batch's row loads
            const entry_batch nxt = load_entry_batch(slab_src, slab_val, pos + cnt);
            switch (cnt) {
                case 1: rowacc_batch<1, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 2: rowacc_batch<2, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 3: rowacc_batch<3, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 4: rowacc_batch<4, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 5: rowacc_batch<5, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 6: rowacc_batch<6, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                case 7: rowacc_batch<7, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
                default: rowacc_batch<8, RC, FULL, VT>(acc, cur, dY, dim, lane, col_ok); break;
            }
            cur = nxt;
            pos += cnt;
        }
        // the visit's share of (A^T dY)[j, :] -> LDS, then dXs[j, t] += row[sp_index[j, t]].  Lanes read what other
        // lanes wrote: a barrier after the writes, and one before the next visit overwrites the row (the workgroup
        // is one wavefront, so these cost a wait for the LDS queue and no more).
#pragma unroll
        for (int c = 0; c < RC; ++c)
#pragma unroll
            for (int i = 0; i < EPL; i += 4)
                *reinterpret_cast<float4*>(row_acc + c * CHUNK + lane * EPL + i) =
                    make_float4(acc[c][i], acc[c][i + 1], acc[c][i + 2], acc[c][i + 3]);
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = lane + h * kWave;
            if (t < k) dXs[j * k + t] = dx_t[h] + row_acc[col_t[h]];
        }
        for (int t = lane + 2 * kWave; t < k; t += kWave) {
            const int col = (int)sp_index[j * k + t];
            dXs[j * k + t] += row_acc[col];
        }
        __syncthreads();
    }
}

// One wave step per workgroup measured best (6.8 -> 6.4 ms at k=32 against a grid capped at the number of
// resident wavefronts): the hardware dispatcher hides the two dependent loads that open a visit better
// than a software loop over visits does.

template <int VEC, bool OFF32, int VT, typename IdxT>
maxk_status launch_slab_t(const SlabSet& S, const value_store_t<VT>* dY, const IdxT* sp_index, int dim, int k, float* dXs,
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
        const int64_t per_xcd = (tasks + 7) / 8;                                                                   \
        const int long_pad = (nlb + 7) & ~7;                                                                       \
        if (per_xcd * 8 + long_pad > 0x7FFFFFFFll) return MAXK_UNSUPPORTED;                                       \
        hipLaunchKernelGGL((bwd_slab_kernel<VEC, LPD, OFF32, VT, IdxT>), dim3((unsigned)(per_xcd * 8 + long_pad)), \
                           dim3(kWave), 0, s, S.d_visit_node, S.d_visit_begin, vb, ve, S.d_long_visit, lb, le, nlb, \
                           long_pad, per_xcd, S.d_src, S.d_val, dY, sp_index, dim, k, dXs);                         \
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

template <int RC, int VT, typename IdxT>
maxk_status launch_slab_rowacc(const SlabSet& S, const value_store_t<VT>* dY, const IdxT* sp_index, int dim, int k,
                               float* dXs, hipStream_t s)
{
    const int vpw = 4;  // consecutive visits per wavefront (4 and 8 measured alike)
    for (int32_t sl = 0; sl < S.n_slabs; ++sl) {
        const int64_t vb = S.h_slab_visit[sl], ve = S.h_slab_visit[sl + 1];
        if (vb >= ve) continue;
        const int64_t tasks = (ve - vb + vpw - 1) / vpw;
        const int64_t per_xcd = (tasks + 7) / 8;
        if (per_xcd * 8 > 0x7FFFFFFFll) return MAXK_UNSUPPORTED;
        if (dim == RC * 256)
            hipLaunchKernelGGL((bwd_slab_rowacc_kernel<RC, true, VT, IdxT>), dim3((unsigned)(per_xcd * 8)), dim3(kWave), 0,
                               s, S.d_visit_node, S.d_visit_begin, vb, ve, vpw, per_xcd, S.d_src, S.d_val, dY, sp_index,
                               dim, k, dXs);
        else
            hipLaunchKernelGGL((bwd_slab_rowacc_kernel<RC, false, VT, IdxT>), dim3((unsigned)(per_xcd * 8)), dim3(kWave),
                               0, s, S.d_visit_node, S.d_visit_begin, vb, ve, vpw, per_xcd, S.d_src, S.d_val, dY, sp_index,
                               dim, k, dXs);
    }
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <int VT, typename IdxT>
maxk_status launch_slab_i(const SlabSet& S, const value_store_t<VT>* dY, const IdxT* sp_index, int64_t N, int dim, int k,
                          float* dXs, hipStream_t s)
{
    // Row-accumulating form from the k where it was measured faster on the dense workload (dim 256; ms, sampled /
    // row-accumulating): fp32 k=24 5.26 / 5.39, k=32 5.42 / 5.41, k=64 6.64 / 5.76, k=128 9.62 / 6.70;
    // 16-bit dY k=8 3.1 / 4.3, k=16 4.1 / 4.2, k=32 5.8 / 4.3, k=128 11.5 / 4.8.  Other widths use the same ratios.
    const bool rowacc = sizeof(value_store_t<VT>) == 4 ? 8 * k >= dim : 16 * k > dim;
    if (rowacc && dim % 4 == 0 && aligned(dY, 16)) {
        if (dim <= 256) return launch_slab_rowacc<1, VT>(S, dY, sp_index, dim, k, dXs, s);
        if (dim <= 512) return launch_slab_rowacc<2, VT>(S, dY, sp_index, dim, k, dXs, s);
        if (dim <= 1024) return launch_slab_rowacc<4, VT>(S, dY, sp_index, dim, k, dXs, s);
    }
    const bool off32 = N * (int64_t)dim * (int64_t)sizeof(value_store_t<VT>) <= 0xFFFFFFFFll &&
                       (sizeof(value_store_t<VT>) == 4 || (aligned(dY, 4) && (N * (int64_t)dim) % 2 == 0));
    // positions per lane, measured on the dense workload (ms at k = 8 / 16 / 32 / 64 / 128):
    //   1: 3.69 / 4.71 / 5.79 / 8.32 / 13.8     2: 3.83 / 4.83 / 5.57 / 6.75 / 14.5     4: 4.47 / 5.38 / 6.21 / 6.84 / 9.63
    if (k <= 16)
        return off32 ? launch_slab_t<1, true, VT>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<1, false, VT>(S, dY, sp_index, dim, k, dXs, s);
    // 16-bit dY: two positions per lane stay best up to k = 128 (11.3 ms against 15.9 with four)
    if (k % 2 == 0 && (k <= 64 || sizeof(value_store_t<VT>) == 2))
        return off32 ? launch_slab_t<2, true, VT>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<2, false, VT>(S, dY, sp_index, dim, k, dXs, s);
    if (k % 4 == 0)
        return off32 ? launch_slab_t<4, true, VT>(S, dY, sp_index, dim, k, dXs, s)
                     : launch_slab_t<4, false, VT>(S, dY, sp_index, dim, k, dXs, s);
    return off32 ? launch_slab_t<1, true, VT>(S, dY, sp_index, dim, k, dXs, s)
                 : launch_slab_t<1, false, VT>(S, dY, sp_index, dim, k, dXs, s);
}

template <int VT, typename IdxT>
maxk_status launch_pull_t(const ItemList& L, const int32_t* csc_src, const float* csc_val, const value_store_t<VT>* dY,
                          const IdxT* sp_index, int dim, int k, float* dXs, float* partials, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
#define MAXK_PULL(KERNEL) \
    hipLaunchKernelGGL((KERNEL), grid, block, 0, s, L.d_items, csc_src, csc_val, dY, sp_index, dim, k, dXs, partials)
    if (k <= 1) MAXK_PULL((bwd_pull_small_kernel<1, VT, IdxT>));
    else if (k <= 2) MAXK_PULL((bwd_pull_small_kernel<2, VT, IdxT>));
    else if (k <= 4) MAXK_PULL((bwd_pull_small_kernel<4, VT, IdxT>));
    else if (k <= 8) MAXK_PULL((bwd_pull_small_kernel<8, VT, IdxT>));
    else if (k <= 16) MAXK_PULL((bwd_pull_small_kernel<16, VT, IdxT>));
    else if (k <= 32) MAXK_PULL((bwd_pull_small_kernel<32, VT, IdxT>));
    else if (k <= 64) MAXK_PULL((bwd_pull_small_kernel<64, VT, IdxT>));
    else MAXK_PULL((bwd_pull_wide_kernel<VT, IdxT>));
#undef MAXK_PULL
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

template <int VT, typename IdxT>
maxk_status launch_push_t(const ItemList& L, const int32_t* col, const float* val, const value_store_t<VT>* dY,
                          const IdxT* sp_index, int dim, int k, float* dXs, hipStream_t s)
{
    dim3 grid((unsigned)L.n_items), block(kWave);
    const size_t lds = sizeof(float) * (size_t)dim;
#define MAXK_PUSH(K) \
    hipLaunchKernelGGL((bwd_push_kernel<K, VT, IdxT>), grid, block, lds, s, L.d_items, col, val, dY, sp_index, dim, k, dXs)
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


// ---- one storage format of dY: everything above behind four functions ----

template <int VT>
maxk_status pull_format(const ItemList& L, const int32_t* csc_src, const float* csc_val, const void* dY_v,
                        const void* sp_index, int index_bytes, int dim, int k, float* dXs, float* partials,
                        hipStream_t s)
{
    const auto* dY = (const value_store_t<VT>*)dY_v;
    if (index_bytes == 1) return launch_pull_t<VT>(L, csc_src, csc_val, dY, (const uint8_t*)sp_index, dim, k, dXs, partials, s);
    if (index_bytes == 2) return launch_pull_t<VT>(L, csc_src, csc_val, dY, (const uint16_t*)sp_index, dim, k, dXs, partials, s);
    return launch_pull_t<VT>(L, csc_src, csc_val, dY, (const int32_t*)sp_index, dim, k, dXs, partials, s);
}

template <int VT>
maxk_status push_format(const ItemList& L, const int32_t* col, const float* val, const void* dY_v, const void* sp_index,
                        int index_bytes, int dim, int k, float* dXs, hipStream_t s)
{
    const auto* dY = (const value_store_t<VT>*)dY_v;
    if (index_bytes == 1) return launch_push_t<VT>(L, col, val, dY, (const uint8_t*)sp_index, dim, k, dXs, s);
    if (index_bytes == 2) return launch_push_t<VT>(L, col, val, dY, (const uint16_t*)sp_index, dim, k, dXs, s);
    return launch_push_t<VT>(L, col, val, dY, (const int32_t*)sp_index, dim, k, dXs, s);
}

template <int VT>
maxk_status expand_format(const ItemList& L, const int32_t* col, const float* val, const void* dY_v,
                          const void* sp_index, int index_bytes, int dim, int k, float* expand, hipStream_t s)
{
    const auto* dY = (const value_store_t<VT>*)dY_v;
    if (index_bytes == 1) return launch_expand_i<VT>(L, col, val, dY, (const uint8_t*)sp_index, dim, k, expand, s);
    if (index_bytes == 2) return launch_expand_i<VT>(L, col, val, dY, (const uint16_t*)sp_index, dim, k, expand, s);
    return launch_expand_i<VT>(L, col, val, dY, (const int32_t*)sp_index, dim, k, expand, s);
}

template <int VT>
maxk_status slab_format(const SlabSet& S, const void* dY_v, const void* sp_index, int index_bytes, int64_t N, int dim,
                        int k, float* dXs, hipStream_t s)
{
    const auto* dY = (const value_store_t<VT>*)dY_v;
    if (index_bytes == 1) return launch_slab_i<VT>(S, dY, (const uint8_t*)sp_index, N, dim, k, dXs, s);
    if (index_bytes == 2) return launch_slab_i<VT>(S, dY, (const uint16_t*)sp_index, N, dim, k, dXs, s);
    return launch_slab_i<VT>(S, dY, (const int32_t*)sp_index, N, dim, k, dXs, s);
}

}  // namespace
}  // namespace maxk
