// Backward aggregation, LDS-tiled form (Eq. 2 right; Eq. 3; prior art: Alg. 2's staging of a dY row on chip).
//
// Every other backward kernel here fetches, per stored entry, the cache lines of a dY row that the destination's k
// columns fall into: about 1 KB of 128-byte lines per entry at hidden width 256 for 4k useful bytes, and the L2 -> L1
// path (64 bytes per clock per CU) is what they wait for.  This kernel turns the traffic round: a workgroup OWNS a set
// of D destination nodes, keeps their D x k accumulators in LDS for its whole life, and streams the source rows of dY
// through LDS in tiles of 16 rows with full, coalesced 16-byte loads.  A tile is used by every entry (i -> j) with i in
// the tile and j in the set, so a row of dY is fetched once per destination set instead of once per entry:
// (N / D) * N * dim * 4 bytes in all.  The sampled reads dY[i, sp_index[j, t]] and the read-add-write of the accumulators
// are LDS traffic.  The workgroups of an XCD that sweep the same source range (a "pack") are kept within a few dozen
// tiles of each other by progress marks, so the rows come from that XCD's L2.
//
// Work assignment inside a workgroup (16 wavefronts):
//   - wavefronts 11..14 only load: each keeps a register queue of the next four tiles' rows (plain 16-byte loads; the
//     queue depth is what hides the L2 latency) and writes one tile per step into one of two LDS row buffers;
//   - wavefronts 0..10 only accumulate.  A "visit" is one (tile, destination) pair with at least one entry; k/4 lanes
//     work on it, four CBSR positions each, so a wave instruction covers a "set" of 64/(k/4) visits.  The visits of a
//     tile have distinct destinations, so the sets of one tile can be worked on by different wavefronts at the same
//     time without two lanes ever touching one accumulator; set s of the workgroup's list goes to wavefront s % 11,
//     counted through the whole list, so each wavefront walks an arithmetic progression of sets and fetches its
//     records eight sets ahead; a directory (one scalar load per tile) tells where a tile's sets end.  Eleven, not
//     eight: a tile holds about four sets, and a wavefront whose next set falls into the very next tile has to
//     prepare it (records, LDS addresses) on that tile's critical path instead of in a tile of its own;
//     A visit's first entry sits in the visit record, the second and third in a parallel 16-byte slot; further ones
//     (rare) are not worked on tile by tile at all: the workgroup adds them at the end, straight from dY;
//   - wavefront 15 touches cache lines of the tiles further ahead so that they are in L2 when the loaders ask, and
//     paces the workgroup against the others of its pack.
//   One workgroup barrier per tile hands a row buffer from the loaders to the accumulators and orders the
//   accumulator updates of consecutive tiles.
//
// The visit lists are built once per (D, k/4) by sorting the entries of A^T by (destination set, tile, destination,
// source); every tile's list is padded to whole sets.  When there are more CUs than destination sets, the source rows
// are cut into ranges, one workgroup per (range, set), and the partial sums are added to dXs with fp32 atomics.
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

#include "common.hpp"

namespace maxk {
namespace {

constexpr int kAccWaves = 11;       // accumulating wavefronts
constexpr int kLoadWaves = 4;       // loading wavefronts
constexpr int kTiledThreads = (kAccWaves + kLoadWaves + 1) * kWave;  // + one wavefront that prefetches
constexpr int kLdsBytes = 160 * 1024;
constexpr int kRecAhead = 8;        // sets between the fetch of a visit record and its use
constexpr int kIdxAhead = 4;        // sets between the fetch of a visit's CBSR columns and their use
constexpr int kPrefetchAheadRows = 512;  // rows between the L2 prefetch and the loads that use it
constexpr int kPrefetchGroupRows = 256;  // rows covered by one round of prefetch instructions
// progress marks: one per (XCD, source range, destination set of the XCD); at most 32 ranges
constexpr int kMarkStride = 32;  // uint32 per mark: one 128-byte line each
inline int64_t kMaxUnits(int n_dsets) { return (int64_t)8 * ((n_dsets + 7) / 8) * 32; }
constexpr int kPaceWindow = 32;           // tiles a workgroup may lead the slowest one of its pack by before it naps
constexpr int kPaceNap = 2;               // naps of 1024 clocks in one unit of waiting (a round is about 15,000 clocks)

// second word of a visit record: accumulator row (in units of four floats), source row within the tile, flags
constexpr uint32_t kVisitAccMask = 0x3FFFu;
constexpr uint32_t kVisitSrcShift = 14;                  // 6 bits
constexpr uint32_t kVisitHasExtra = 1u << 20;
constexpr uint32_t kVisitNull = 1u << 21;                // padding slot
// second word of an extra entry: source row within the tile, chain position of the next one, "another one follows"
constexpr uint32_t kExtraMore = 1u << 31;

// ------------------------------------------------------------------ table build ----

// key = ((set * n_tiles + tile) << 18) | dest_local << 6 | src_local, one per in-entry of A^T
__global__ __launch_bounds__(256) void tiled_keys_kernel(const int32_t* __restrict__ csc_ptr,
                                                         const int32_t* __restrict__ csc_src, int64_t N, int64_t nnz,
                                                         int32_t D, int32_t tile_rows, int32_t n_tiles,
                                                         uint64_t* __restrict__ key)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
        int64_t lo = 0, hi = N;  // largest j with csc_ptr[j] <= p
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if ((int64_t)csc_ptr[mid] <= p) lo = mid; else hi = mid;
        }
        const int32_t j = (int32_t)lo, i = csc_src[p];
        const int32_t d = j / D, jl = j - d * D;
        const int32_t tile = i / tile_rows, il = i - tile * tile_rows;
        const uint64_t group = (uint64_t)d * (uint64_t)n_tiles + (uint64_t)tile;
        key[p] = (group << 18) | ((uint64_t)jl << 6) | (uint64_t)il;
    }
}

// head[p] = entry p opens a visit; late[p] = entry p is the fourth or a later one of its visit (it goes to the chain)
__global__ __launch_bounds__(256) void tiled_flags_kernel(const uint64_t* __restrict__ key, int64_t nnz,
                                                          uint32_t* __restrict__ head, uint32_t* __restrict__ late)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
        const uint64_t v = key[p] >> 6;
        head[p] = (p == 0 || (key[p - 1] >> 6) != v) ? 1u : 0u;
        late[p] = (p >= 3 && (key[p - 3] >> 6) == v) ? 1u : 0u;  // sorted: then p-1 and p-2 are of this visit too
    }
}

// sets[g] = wave instructions that the visits of group g need; first_visit[g] = visits before group g
__global__ __launch_bounds__(256) void tiled_groups_kernel(const uint64_t* __restrict__ key,
                                                           const uint32_t* __restrict__ rank, int64_t nnz,
                                                           int64_t n_groups, int32_t E, uint32_t n_visits,
                                                           uint32_t* __restrict__ first_visit,
                                                           uint32_t* __restrict__ sets)
{
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g > n_groups) return;
    auto lower = [&](uint64_t bound) {  // first entry whose key is >= bound
        int64_t lo = 0, hi = nnz;
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (key[mid] < bound) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    auto visits_before = [&](int64_t pos) { return pos < nnz ? rank[pos] - 1u : n_visits; };
    const uint32_t fv = visits_before(lower((uint64_t)g << 18));
    first_visit[g] = fv;
    if (g < n_groups) {
        const uint32_t nv = visits_before(lower((uint64_t)(g + 1) << 18)) - fv;
        sets[g] = (nv + (uint32_t)E - 1u) / (uint32_t)E;
    } else {
        sets[g] = 0;
    }
}

__global__ __launch_bounds__(256) void tiled_fill_null_kernel(uint2* __restrict__ rec, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) rec[i] = make_uint2(0u, kVisitNull);
}

__global__ __launch_bounds__(256) void tiled_records_kernel(const uint64_t* __restrict__ key,
                                                            const float* __restrict__ val,
                                                            const uint32_t* __restrict__ head,
                                                            const uint32_t* __restrict__ rank,
                                                            const uint32_t* __restrict__ late,
                                                            const uint32_t* __restrict__ chain_pos, int64_t nnz,
                                                            int32_t E, int32_t LPV, int32_t n_tiles, int32_t tile_rows,
                                                            int32_t n_ranges, int32_t tiles_per_range, int32_t n_owners,
                                                            const uint32_t* __restrict__ first_visit,
                                                            const uint32_t* __restrict__ dir_sets,
                                                            uint2* __restrict__ rec, uint4* __restrict__ extra,
                                                            uint4* __restrict__ ovf, uint64_t* __restrict__ ovf_key)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
        const uint64_t kp = key[p];
        const uint32_t il = (uint32_t)(kp & 63u);
        if (head[p]) {
            const bool more = p + 1 < nnz && !head[p + 1];
            const uint64_t g = kp >> 18;
            const uint32_t v = rank[p] - 1u;
            const int64_t slot = (int64_t)dir_sets[g] * E + (int64_t)(v - first_visit[g]);
            const uint32_t jl = (uint32_t)((kp >> 6) & 0xFFFu);
            rec[slot] = make_uint2(__float_as_uint(val[p]),
                                   (jl * (uint32_t)LPV) | (il << kVisitSrcShift) | (more ? kVisitHasExtra : 0u));
            if (more) {
                const bool more2 = p + 2 < nnz && !head[p + 2];
                const uint32_t il1 = (uint32_t)(key[p + 1] & 63u);
                const uint32_t il2 = more2 ? (uint32_t)(key[p + 2] & 63u) : 0u;
                extra[slot] = make_uint4(__float_as_uint(val[p + 1]), il1 | (more2 ? kExtraMore : 0u),
                                         more2 ? __float_as_uint(val[p + 2]) : 0u,
                                         il2);
            }
        } else if (late[p]) {
            // fourth and later entries of a visit (rare) are not worked on tile by tile: the kernel adds them at the end,
            // straight from dY.  {weight, source row, destination within the set}; they are then sorted by
            // (workgroup = destination set and source range, owner = the lane group that adds them, destination)
            const uint64_t g = kp >> 18;
            const uint32_t tile = (uint32_t)(g % (uint64_t)n_tiles), dset = (uint32_t)(g / (uint64_t)n_tiles);
            const uint32_t jl = (uint32_t)((kp >> 6) & 0xFFFu);
            const uint32_t range = tile / (uint32_t)tiles_per_range, tl = tile - range * (uint32_t)tiles_per_range;
            const uint64_t bucket = ((uint64_t)dset * (uint64_t)n_ranges + range) * (uint64_t)n_owners + jl % (uint32_t)n_owners;
            ovf[chain_pos[p]] = make_uint4(__float_as_uint(val[p]), tile * (uint32_t)tile_rows + il, jl, 0u);
            ovf_key[chain_pos[p]] = (bucket << 32) | ((uint64_t)jl << 20) | (uint64_t)(((tl << 6) | il) & 0xFFFFFu);
        }
    }
}

__global__ __launch_bounds__(256) void tiled_iota_kernel(uint32_t* __restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = (uint32_t)i;
}

__global__ __launch_bounds__(256) void tiled_ovf_gather_kernel(const uint32_t* __restrict__ order,
                                                               const uint4* __restrict__ in, int64_t n,
                                                               uint4* __restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = in[order[i]];
}

// dir[b] = overflow entries in buckets below b (b = 0 .. n_buckets)
__global__ __launch_bounds__(256) void tiled_ovf_dir_kernel(const uint64_t* __restrict__ key, int64_t n, int64_t n_buckets,
                                                            uint32_t* __restrict__ dir)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b > n_buckets) return;
    int64_t lo = 0, hi = n;  // first entry whose bucket is >= b
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)(key[mid] >> 32) < b) lo = mid + 1; else hi = mid;
    }
    dir[b] = (uint32_t)lo;
}

// ----------------------------------------------------------------------- kernel ----

struct TiledArgs {
    const float* dY;
    const void* sp_index;
    float* dXs;
    const uint32_t* dir_sets;  // [n_dsets * n_tiles + 1] first set of every (destination set, tile)
    const uint2* rec;          // [total_sets * E] visit records
    const uint4* extra;        // [total_sets * E] second and third entry of a visit, where it has them
    const uint4* ovf;          // fourth and later entries of a visit: {weight, source row, destination within its set}
    const uint32_t* ovf_dir;   // [(n_dsets * R) * lane groups + 1] overflow entries before every (workgroup, lane group)
    int64_t N;
    int32_t dim, k;
    int32_t D, n_dsets, n_tiles;
    int32_t G, R, tiles_per_range;  // destination sets per XCD, source ranges, tiles per range
    uint32_t* progress;             // [8 * G * R] tiles swept so far by every workgroup (0 = not started, ~0 = done)
    int32_t window;                 // tiles a workgroup may be ahead of the slowest one of its pack; 0 = no pacing
    int32_t atomic_out;
    int32_t ovf_by_bucket;  // how the overflow entries are added at the end (see there)
    int32_t range_per_xcd;  // workgroup-to-(range, destination set) mapping (see the kernel's first lines)
};

// PPL (= 4) consecutive sp_index entries, fetched with one load
template <typename IdxT, int PPL>
struct IdxVec;
template <>
struct IdxVec<uint8_t, 4> {
    uint32_t w;
    __device__ __forceinline__ void load(const void* p) { w = *reinterpret_cast<const uint32_t*>(p); }
    __device__ __forceinline__ uint32_t get(int i) const { return (w >> (8 * i)) & 0xFFu; }
};
template <>
struct IdxVec<uint16_t, 4> {
    uint2 w;
    __device__ __forceinline__ void load(const void* p) { w = *reinterpret_cast<const uint2*>(p); }
    __device__ __forceinline__ uint32_t get(int i) const { return ((i < 2 ? w.x : w.y) >> (16 * (i & 1))) & 0xFFFFu; }
};
template <>
struct IdxVec<int32_t, 4> {
    uint4 w;
    __device__ __forceinline__ void load(const void* p) { w = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ uint32_t get(int i) const { return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w; }
};

// TR: source rows per tile (16 is what the launcher uses: 32 and 48 were measured slower);
// DIMC: hidden width when known at compile time (LDS and row offsets become immediates), 0 = a.dim;
// RC: 256-column chunks that cover a dY row (dim <= RC * 256); PPL: CBSR positions per lane (4; 8 was measured slower)
//
// A wavefront on its own issues at most one instruction every four clocks or so, and a tile's few sets are each one
// wavefront's work, so the instruction count per tile and per set is what this kernel's time follows: addresses are kept as a uniform base (scalar registers, advanced with scalar adds) plus a fixed 32-bit lane
// offset, the lists are padded so that reading ahead needs no clamping, and nothing is recomputed per tile.
template <int TR, int DIMC, int RC, int PPL, typename IdxT>
__global__ __launch_bounds__(kTiledThreads) void bwd_tiled_kernel(const TiledArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int dim = DIMC ? DIMC : a.dim, k = a.k, D = a.D;
    constexpr bool FULL = DIMC == RC * 256;

    // Workgroup b runs on XCD b % 8.  Destination set d belongs to XCD d % 8, and an XCD takes its (source range,
    // destination set) units range by range, so the 32 workgroups that are resident on it together sweep the same
    // one or two source ranges at the same pace, and a dY row is pulled into that XCD's L2 once per range.
    const int b = blockIdx.x, xcd = b & 7, m = b >> 3;
    // Two ways from (XCD, position m on it) to (source range, destination set).  When all workgroups are resident at
    // once and R divides 8 (`range_per_xcd`), an XCD sweeps ONE range - XCD x takes range x % R and every (8/R)-th
    // destination set - so its 32 workgroups share one stream of rows through its L2 instead of R streams.
    // Otherwise the XCD takes its G destination sets range after range.  `pack_slot` of `pack_size`: this
    // workgroup among those that sweep its range on its XCD.
    int range, d, pack_slot, pack_size, pack_id;
    if (a.range_per_xcd) {
        const int per = 8 / a.R;
        range = xcd % a.R;
        d = xcd / a.R + per * m;
        pack_slot = m; pack_size = a.G * a.R; pack_id = xcd;
    } else {
        range = m / a.G;
        pack_slot = m - range * a.G;
        d = xcd + 8 * pack_slot;
        pack_size = a.G; pack_id = range * 8 + xcd;
    }
    const int gi = pack_slot;
    if (range >= a.R || d >= a.n_dsets) return;
    const int t0 = range * a.tiles_per_range, t1 = min(a.n_tiles, t0 + a.tiles_per_range);
    if (t0 >= t1) return;
    const int64_t dest0 = (int64_t)d * D;
    const int Dn = (int)min((int64_t)D, a.N - dest0);

    const int acc_floats = (D * k + 3) & ~3;
    float* __restrict__ acc = lds;
    float* __restrict__ rows = lds + acc_floats;  // two buffers of TR rows
    for (int i = tid; i < acc_floats / 4; i += kTiledThreads) reinterpret_cast<float4*>(acc)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    // Barrier protocol: barrier number t (t = t0 .. t1-1) is passed by the loaders after they have written tile t and
    // by the accumulators before they start on tile t, i.e. after they have finished tile t-1.  Every wavefront
    // executes exactly t1 - t0 of them, whatever its role.
    if (wave == kAccWaves + kLoadWaves) {
        // ---- prefetching wavefront ----
        // The workgroups of an XCD that sweep one source range move as a pack: whoever is first takes the miss to
        // memory, the others hit L2 and catch up, so the pack would advance at the rate one CU can miss (its
        // loads in flight / memory latency).  Instead every workgroup of the pack touches its 1/G share of the
        // cache lines of the tiles kPrefetchAhead ahead (one dword per 128-byte line), which pulls them into L2 with
        // G times as many misses in flight.  The loaded values are not used.
        constexpr int PG = kPrefetchGroupRows / TR > 0 ? kPrefetchGroupRows / TR : 1;  // tiles per prefetch round
        constexpr int PA = kPrefetchAheadRows / TR;                                     // tiles ahead
        const int pack = min(pack_size, 32);  // workgroups that share the lines of a round
        const int64_t row_bytes = (int64_t)dim * 4, total_bytes = a.N * row_bytes;
        const int64_t lines_per_group = (PG * TR * row_bytes + 127) / 128;
        const int pf_loads = pack >= 8 ? (int)min((int64_t)4, (lines_per_group / pack + kWave - 1) / kWave) : 0;
        uint32_t got[4] = {0u, 0u, 0u, 0u};
        // Pacing.  The workgroups of a pack (same XCD, same source range) share the rows they sweep through that
        // XCD's L2 only while they are within a few dozen tiles of each other, and left alone they drift apart by
        // thousands (their destination sets differ in work by 10-30 %).  So every workgroup publishes how far it
        // is once per round, reads the others' marks one round later, and the ones that are more than `window`
        // tiles ahead of the slowest nap here, ahead of the barrier, which holds their whole workgroup.  The naps are
        // bounded whatever the others do, so every wavefront reaches the end.
        // (a mark has a cache line to itself: with several in one line, the writers of the others hold up every reader)
        uint32_t* const my_mark = a.progress + ((int64_t)pack_id * pack_size + pack_slot) * kMarkStride;
        const uint32_t* const pack_marks = a.progress + (int64_t)pack_id * pack_size * kMarkStride;
        // lane l looks at the workgroup in slot l of the pack (if that slot has a destination set at all)
        const bool member = lane < pack_size && (a.range_per_xcd ? xcd / a.R + (8 / a.R) * lane : xcd + 8 * lane) < a.n_dsets;
        const uint32_t* const my_view = pack_marks + (member ? lane : gi) * kMarkStride;  // every lane loads, so that no branch (and
        uint32_t seen_next = 0xFFFFFFFFu;                                   // no conservative wait) surrounds the load
        int countdown = 0;
        for (int tile = t0; tile < t1; ++tile) {
            if (countdown == 0) {
                // One round in PG tiles.  Everything that is waited for here was issued a round ago, and everything
                // that is issued here is left in flight until the next round: this wavefront is on the critical path
                // of the tile like any other, and a wait for a fresh load or store would hold the whole workgroup.
#pragma unroll
                for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(got[j]));  // the previous round has landed
                if (a.window > 0) {
                    // How far ahead of the slowest mark (read a round ago)?  One, two or four windows: nap for one, two
                    // or four units.  No loads in here and no loop around loads: the compiler then keeps its waits
                    // exact, and the naps are bounded whatever the marks say.
                    const uint32_t cur = (uint32_t)(tile - t0);
                    const uint32_t seen = member ? seen_next : 0xFFFFFFFFu;
                    const uint32_t w = (uint32_t)a.window;
                    int naps = 0;
                    const bool running = seen != 0u && seen != 0xFFFFFFFFu;  // neither waiting for a CU nor done
                    if (__builtin_amdgcn_ballot_w64(running && seen + w < cur) != 0) naps = 1;
                    if (__builtin_amdgcn_ballot_w64(running && seen + 2 * w < cur) != 0) naps = 2;
                    if (__builtin_amdgcn_ballot_w64(running && seen + 4 * w < cur) != 0) naps = 4;
                    for (int i = 0; i < naps * kPaceNap; ++i) __builtin_amdgcn_s_sleep(16);  // 16 * 64 clocks each
                }
                if (pf_loads) {
                    const int64_t base = (int64_t)(tile + PA) * TR * row_bytes;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int64_t off = base + ((int64_t)(j * kWave + lane) * pack + gi % pack) * 128;
                        if (j < pf_loads && off + 4 <= total_bytes && tile + PA < t1)
                            got[j] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(a.dY) + off);
                    }
                }
                if (a.window > 0) {
                    if (lane == 0) __hip_atomic_store(my_mark, (uint32_t)(tile - t0 + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    seen_next = __hip_atomic_load(my_view, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                countdown = PG;
            }
            --countdown;
            __syncthreads();
        }
        if (a.window > 0 && lane == 0) __hip_atomic_store(my_mark, 0xFFFFFFFFu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(got[j]));
    } else if (wave >= kAccWaves) {
        // ---- loading wavefronts: tile t -> row buffer t & 1 ----
        constexpr int RP = TR / kLoadWaves;                    // rows per wavefront and tile
        constexpr int Q = (TR == 16 && RC == 1) ? 4 : 2;        // tiles this wavefront keeps in flight
        static_assert(TR % kLoadWaves == 0 && Q * RP * RC * 4 <= 96, "the row queue must fit the register budget");
        const int lw = wave - kAccWaves;
        float4 q0[RP][RC], q1[RP][RC], q2[RP][RC], q3[RP][RC];  // named, not indexed: they must stay in registers
        const uint32_t lane_bytes = (uint32_t)lane * 16u;
        bool col_ok[RC];
#pragma unroll
        for (int cc = 0; cc < RC; ++cc) col_ok[cc] = FULL || cc * 256 + lane * 4 < dim;
        const uint32_t row_bytes = (uint32_t)dim * 4u;
        const int64_t tile_bytes = (int64_t)TR * row_bytes;
        // uniform address of this wavefront's first row of tile 0
        const char* const src0 = reinterpret_cast<const char*>(a.dY) + (int64_t)(lw * RP) * row_bytes;
        char* const dst0 = reinterpret_cast<char*>(rows) + lw * RP * row_bytes + lane_bytes;
        const int last_full = (int)(a.N / TR);  // tiles below this one have all their rows
        const int t1m = min(t1, last_full);     // the queue handles the full tiles [t0, t1m)
        // A step stores the oldest tile of the queue and issues the tile Q ahead.  Tiles past the last full one
        // are replaced by the last full one (loaded, never used), so that every step issues the same loads and the
        // compiler can wait for exactly the oldest tile in the queue.
#define MAXK_TILED_ISSUE(QQ, TILE)                                                                            \
    {                                                                                                         \
        const char* const src = src0 + (int64_t)min((TILE), last_full - 1) * tile_bytes;                      \
        _Pragma("unroll") for (int rr = 0; rr < RP; ++rr)                                                     \
            _Pragma("unroll") for (int cc = 0; cc < RC; ++cc)                                                 \
                if (col_ok[cc])                                                                               \
                    QQ[rr][cc] = *reinterpret_cast<const float4*>(src + (rr * row_bytes + cc * 1024u + lane_bytes)); \
    }
#define MAXK_TILED_STORE(QQ, TILE)                                                                            \
    {                                                                                                         \
        char* const dst = dst0 + ((TILE) & 1) * (TR * row_bytes);                                             \
        _Pragma("unroll") for (int rr = 0; rr < RP; ++rr)                                                     \
            _Pragma("unroll") for (int cc = 0; cc < RC; ++cc)                                                 \
                if (col_ok[cc]) *reinterpret_cast<float4*>(dst + rr * row_bytes + cc * 1024u) = QQ[rr][cc];   \
    }
#pragma unroll
        for (int rr = 0; rr < RP; ++rr)
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) q0[rr][cc] = q1[rr][cc] = q2[rr][cc] = q3[rr][cc] = make_float4(0.f, 0.f, 0.f, 0.f);
        int base = t0;
        if (t0 < t1m) {
            MAXK_TILED_ISSUE(q0, t0)
            MAXK_TILED_ISSUE(q1, t0 + 1)
            if constexpr (Q == 4) {
                MAXK_TILED_ISSUE(q2, t0 + 2)
                MAXK_TILED_ISSUE(q3, t0 + 3)
            }
#define MAXK_TILED_STEP(QQ, TILE) \
    MAXK_TILED_STORE(QQ, TILE)    \
    MAXK_TILED_ISSUE(QQ, (TILE) + Q) \
    __syncthreads();
            for (; base + Q <= t1m; base += Q) {
                MAXK_TILED_STEP(q0, base)
                MAXK_TILED_STEP(q1, base + 1)
                if constexpr (Q == 4) {
                    MAXK_TILED_STEP(q2, base + 2)
                    MAXK_TILED_STEP(q3, base + 3)
                }
            }
#undef MAXK_TILED_STEP
            if (base < t1m) { MAXK_TILED_STORE(q0, base) __syncthreads(); }
            if constexpr (Q == 4) {
                if (base + 1 < t1m) { MAXK_TILED_STORE(q1, base + 1) __syncthreads(); }
                if (base + 2 < t1m) { MAXK_TILED_STORE(q2, base + 2) __syncthreads(); }
            }
        }
        if (t1m < t1) {
            // the one tile that is cut short by the end of dY: loaded directly, row by row
            const int tile = t1m;
#pragma unroll
            for (int rr = 0; rr < RP; ++rr) {
                const int64_t row = (int64_t)tile * TR + lw * RP + rr;
#pragma unroll
                for (int cc = 0; cc < RC; ++cc) {
                    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (row < a.N && col_ok[cc])
                        x = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(a.dY) + row * row_bytes + cc * 1024u + lane_bytes);
                    q0[rr][cc] = x;
                }
            }
            MAXK_TILED_STORE(q0, tile)
            __syncthreads();
        }
#undef MAXK_TILED_ISSUE
#undef MAXK_TILED_STORE
    } else {
        // ---- accumulating wavefronts ----
        constexpr int NQ = PPL / 4;  // float4 pieces of a lane's accumulators
        const int LPV = k / PPL, E = kWave / LPV;
        const int g = lane / LPV, q = lane - g * LPV;
        const bool lane_on = g < E;
        const int gs = lane_on ? g : 0;
        // The directory is read through the constant address space: it does not change while the kernel runs, its
        // addresses are wave-uniform, and so the reads become scalar loads, which do not queue behind the vector
        // loads in flight (a vector load here would have to wait for all of them at every tile).
        typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;
        const const_u32_ptr dt = (const_u32_ptr)(a.dir_sets + (int64_t)d * a.n_tiles);
        // Set s of the workgroup's list goes to wavefront s % kAccWaves, whatever tile it belongs to: this wavefront's
        // sets are first + kAccWaves * i, i = 0 .. n_it - 1
        const uint32_t u0 = dt[t0], u1 = dt[t1];
        const uint32_t first = u0 + ((uint32_t)wave + (uint32_t)kAccWaves - u0 % (uint32_t)kAccWaves) % (uint32_t)kAccWaves;
        const int n_it = first >= u1 ? 0 : (int)((u1 - first + kAccWaves - 1) / kAccWaves);
        int tile = t0;
        uint32_t s_end = dt[t0 + 1];                 // first set past `tile`
        uint32_t s_end_next = dt[t0 + 2];            // (the directory has three spare entries at its end)
        uint32_t s_end_after = dt[t0 + 3];           // read one tile before it is looked at: the scalar load has a
        const_u32_ptr dt_next = dt + (t0 + 4);       // whole tile to arrive, cache miss or not
        // uniform bases + fixed lane offsets (bytes)
        const int64_t set_bytes = (int64_t)E * 8;                               // one set of records
        const int64_t step_bytes = set_bytes * kAccWaves;                       // from one of this wavefront's sets to the next
        const uint32_t rec_lane = (uint32_t)gs * 8u;
        const char* rec_at = reinterpret_cast<const char*>(a.rec) + (int64_t)first * set_bytes;      // set being fetched
        const char* ext_at = reinterpret_cast<const char*>(a.extra) + (int64_t)first * set_bytes * 2;  // set whose columns are fetched
        const char* const idx_at = reinterpret_cast<const char*>(a.sp_index) + dest0 * k * (int64_t)sizeof(IdxT);
        const uint32_t idx_lane = (uint32_t)q * (uint32_t)(PPL * sizeof(IdxT));
        // LDS addresses are worked out as 32-bit numbers ahead of the barrier and used as they are after it
        typedef __attribute__((address_space(3))) char lds_char;
        typedef __attribute__((address_space(3))) float lds_float;
        typedef float vec4 __attribute__((ext_vector_type(4)));  // a plain vector type: it can be read through an LDS pointer
        typedef __attribute__((address_space(3))) vec4 lds_vec4;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)lds;
        const uint32_t acc_lane_off = lds0 + (uint32_t)q * (uint32_t)(4 * PPL);  // the accumulators come first
        const uint32_t rows_off = lds0 + (uint32_t)acc_floats * 4u;
        const uint32_t row_bytes = (uint32_t)dim * 4u, buf_bytes = TR * row_bytes;
        __syncthreads();  // barrier t0: the rows of tile t0 are in buffer t0 & 1

        if (n_it > 0) {
            static_assert(kRecAhead == 8 && kIdxAhead == 4, "the queues below are written out for these depths");
            uint2 rq0, rq1, rq2, rq3, rq4, rq5, rq6, rq7;  // named, not indexed: they must stay in registers
            IdxVec<IdxT, PPL> iq0, iq1, iq2, iq3;
            uint4 xq0, xq1, xq2, xq3;
            // the record arrays end with kRecAhead * 8 padding sets, so fetching ahead of the list needs no clamp
#define MAXK_TILED_FETCH_REC(RQ)                                   \
    RQ = *reinterpret_cast<const uint2*>(rec_at + rec_lane);       \
    rec_at += step_bytes;
// the second-entry array is read for every set, whether a visit has a second entry or not (lanes without one read
// the set's first slot): a load that is issued only sometimes would keep the compiler from counting the loads in
// flight, and it would then wait for younger ones than it needs
#define MAXK_TILED_FETCH_IDX(RQ, IQ, XQ)                                                                              \
    IQ.load(idx_at + ((RQ.y & kVisitAccMask) * (uint32_t)(PPL * sizeof(IdxT)) + idx_lane));                          \
    XQ = *reinterpret_cast<const uint4*>(ext_at + ((RQ.y & kVisitHasExtra) ? 2u * rec_lane : 0u));                    \
    ext_at += 2 * step_bytes;
            MAXK_TILED_FETCH_REC(rq0) MAXK_TILED_FETCH_REC(rq1) MAXK_TILED_FETCH_REC(rq2) MAXK_TILED_FETCH_REC(rq3)
            MAXK_TILED_FETCH_REC(rq4) MAXK_TILED_FETCH_REC(rq5) MAXK_TILED_FETCH_REC(rq6) MAXK_TILED_FETCH_REC(rq7)
            xq0 = xq1 = xq2 = xq3 = make_uint4(0u, 0u, 0u, 0u);
            MAXK_TILED_FETCH_IDX(rq0, iq0, xq0) MAXK_TILED_FETCH_IDX(rq1, iq1, xq1)
            MAXK_TILED_FETCH_IDX(rq2, iq2, xq2) MAXK_TILED_FETCH_IDX(rq3, iq3, xq3)
            // One set.  What a wavefront does between leaving a barrier and reaching the next one is on the critical
            // path of that tile, so as much as possible is done in tiles where the wavefront has no set of its own
            // (its sets are eleven apart in the list, a tile holds about four): it first crosses into the tile BEFORE
            // the set's tile, there takes the oldest queue entries, refills the queues (the same loads every time, so
            // that the compiler can count them) and works out every LDS address - pinned in registers by the empty asm
            // statements, which the compiler may not move across the barrier - and only then crosses into the set's
            // tile, where nothing is left but LDS reads, multiply-adds and the LDS write.
#define MAXK_TILED_PIN(X) asm volatile("" : "+v"(X));
#define MAXK_TILED_CROSS                                                         \
    {                                                                            \
        ++tile;                                                                  \
        s_end = s_end_next;                                                      \
        s_end_next = s_end_after;                                                \
        __syncthreads();                                                         \
        s_end_after = *dt_next++; /* asked for after the barrier */              \
    }
#define MAXK_TILED_SET(RQ, RQ_AHEAD, IQ, XQ, IT)                                                                      \
    {                                                                                                                 \
        const uint32_t my_set = first + (uint32_t)(IT) * kAccWaves;                                                   \
        while (my_set >= s_end_next) MAXK_TILED_CROSS /* now the set is in this tile or the next one */               \
        const uint2 cur = RQ;                                                                                         \
        const IdxVec<IdxT, PPL> ci = IQ;                                                                              \
        const uint4 cx = XQ;                                                                                          \
        MAXK_TILED_FETCH_REC(RQ)                                                                                      \
        MAXK_TILED_FETCH_IDX(RQ_AHEAD, IQ, XQ)                                                                        \
        const bool cross = my_set >= s_end;                                                                           \
        const bool live = lane_on && !(cur.y & kVisitNull);                                                           \
        const bool two = live && (cur.y & kVisitHasExtra) != 0u;                                                      \
        uint32_t acc_at = acc_lane_off + (cur.y & kVisitAccMask) * (uint32_t)(4 * PPL);                               \
        const uint32_t buf_at = rows_off + (((uint32_t)tile + (cross ? 1u : 0u)) & 1u) * buf_bytes;                   \
        const uint32_t row1 = buf_at + __umul24((cur.y >> kVisitSrcShift) & 63u, row_bytes);                          \
        const uint32_t row2 = buf_at + __umul24(cx.y & 63u, row_bytes);                                               \
        float w1 = __uint_as_float(cur.x), w2 = two ? __uint_as_float(cx.x) : 0.f; /* no second entry: slot unset */  \
        uint32_t at1[PPL], at2[PPL]; /* LDS byte addresses of the sampled elements */                                 \
        _Pragma("unroll") for (int i = 0; i < PPL; ++i) {                                                             \
            at1[i] = row1 + ci.get(i) * 4u;                                                                           \
            at2[i] = row2 + ci.get(i) * 4u;                                                                           \
            MAXK_TILED_PIN(at1[i]) MAXK_TILED_PIN(at2[i])                                                             \
        }                                                                                                             \
        MAXK_TILED_PIN(acc_at) MAXK_TILED_PIN(w1) MAXK_TILED_PIN(w2)                                                  \
        if (cross) MAXK_TILED_CROSS                                                                                   \
        if (live) {                                                                                                   \
            lds_vec4* const ap = (lds_vec4*)(uintptr_t)acc_at;                                                        \
            vec4 av[NQ];                                                                                              \
            float x1[PPL], x2[PPL];                                                                                   \
            _Pragma("unroll") for (int n = 0; n < NQ; ++n) av[n] = ap[n];                                             \
            _Pragma("unroll") for (int i = 0; i < PPL; ++i) x1[i] = *(const lds_float*)(uintptr_t)at1[i];             \
            _Pragma("unroll") for (int i = 0; i < PPL; ++i) x2[i] = 0.f;                                              \
            if (two) {                                                                                                \
                _Pragma("unroll") for (int i = 0; i < PPL; ++i) x2[i] = *(const lds_float*)(uintptr_t)at2[i];         \
            }                                                                                                         \
            _Pragma("unroll") for (int n = 0; n < NQ; ++n) {                                                          \
                av[n].x = fmaf(w2, x2[4 * n], fmaf(w1, x1[4 * n], av[n].x)); /* two multiply-adds per element */      \
                av[n].y = fmaf(w2, x2[4 * n + 1], fmaf(w1, x1[4 * n + 1], av[n].y));                                  \
                av[n].z = fmaf(w2, x2[4 * n + 2], fmaf(w1, x1[4 * n + 2], av[n].z));                                  \
                av[n].w = fmaf(w2, x2[4 * n + 3], fmaf(w1, x1[4 * n + 3], av[n].w));                                  \
            }                                                                                                         \
            if (two && (cx.y & kExtraMore)) { /* a third entry, from the same slot (2 visits in 1000 on the dense workload) */ \
                const float v = __uint_as_float(cx.z);                                                                \
                const uint32_t row = buf_at + __umul24(cx.w & 63u, row_bytes);                                        \
                _Pragma("unroll") for (int n = 0; n < NQ; ++n) {                                                      \
                    av[n].x += v * *(const lds_float*)(uintptr_t)(row + ci.get(4 * n) * 4u);                          \
                    av[n].y += v * *(const lds_float*)(uintptr_t)(row + ci.get(4 * n + 1) * 4u);                      \
                    av[n].z += v * *(const lds_float*)(uintptr_t)(row + ci.get(4 * n + 2) * 4u);                      \
                    av[n].w += v * *(const lds_float*)(uintptr_t)(row + ci.get(4 * n + 3) * 4u);                      \
                }                                                                                                     \
            }                                                                                                         \
            _Pragma("unroll") for (int n = 0; n < NQ; ++n) ap[n] = av[n];                                             \
        }                                                                                                             \
    }
            int ib = 0;
            for (; ib + kRecAhead <= n_it; ib += kRecAhead) {
                MAXK_TILED_SET(rq0, rq4, iq0, xq0, ib)
                MAXK_TILED_SET(rq1, rq5, iq1, xq1, ib + 1)
                MAXK_TILED_SET(rq2, rq6, iq2, xq2, ib + 2)
                MAXK_TILED_SET(rq3, rq7, iq3, xq3, ib + 3)
                MAXK_TILED_SET(rq4, rq0, iq0, xq0, ib + 4)
                MAXK_TILED_SET(rq5, rq1, iq1, xq1, ib + 5)
                MAXK_TILED_SET(rq6, rq2, iq2, xq2, ib + 6)
                MAXK_TILED_SET(rq7, rq3, iq3, xq3, ib + 7)
            }
            if (ib < n_it) MAXK_TILED_SET(rq0, rq4, iq0, xq0, ib)
            if (ib + 1 < n_it) MAXK_TILED_SET(rq1, rq5, iq1, xq1, ib + 1)
            if (ib + 2 < n_it) MAXK_TILED_SET(rq2, rq6, iq2, xq2, ib + 2)
            if (ib + 3 < n_it) MAXK_TILED_SET(rq3, rq7, iq3, xq3, ib + 3)
            if (ib + 4 < n_it) MAXK_TILED_SET(rq4, rq0, iq0, xq0, ib + 4)
            if (ib + 5 < n_it) MAXK_TILED_SET(rq5, rq1, iq1, xq1, ib + 5)
            if (ib + 6 < n_it) MAXK_TILED_SET(rq6, rq2, iq2, xq2, ib + 6)
#undef MAXK_TILED_FETCH_REC
#undef MAXK_TILED_FETCH_IDX
#undef MAXK_TILED_SET
#undef MAXK_TILED_CROSS
#undef MAXK_TILED_PIN
        }
        while (tile < t1 - 1) {
            ++tile;
            __syncthreads();
        }
    }
    __syncthreads();
    {
        // Overflow entries of this (source range, destination set): fourth and later entries of a visit.  They are few
        // (1 visit in 8,000 on the dense workload has any), so they are not chained behind their visit, where the
        // dependent load would sit on a tile's critical path, but added here, sampled straight from dY.  They come
        // sorted into one bucket per lane group (k/4 lanes, as in a set), a destination always in the same bucket, so
        // a lane group can add its entries one after the other with plain LDS read-add-writes and nobody else touches
        // those accumulators (LDS atomics retire about one lane in 3 clocks here); which of the two ways below is
        // taken is decided when the lists are built, from the number of entries and the longest bucket.
        const int LPV = k / PPL, E = kWave / LPV, g = lane / LPV, q = lane - g * LPV;
        const int n_owners = (kTiledThreads / kWave) * E;
        const int64_t bucket0 = ((int64_t)d * a.R + range) * n_owners;
        const IdxT* const ib = reinterpret_cast<const IdxT*>(a.sp_index) + (dest0 * (int64_t)k + q * PPL);
        if (g < E && a.ovf_by_bucket) {
            // Mode 1 (many overflow entries, spread evenly: small dense graphs): every lane group adds its own bucket.
            const uint32_t b0 = a.ovf_dir[bucket0 + (wave * E + g)], b1 = a.ovf_dir[bucket0 + (wave * E + g) + 1];
            if (b0 < b1) {
                // two stages ahead of the adds: the next record, and the next destination's columns (reads past the
                // end are clamped to the last entry and dropped)
                const uint32_t last = b1 - 1;
                uint4 r0 = a.ovf[b0], r1 = a.ovf[min(b0 + 1, last)];
                IdxVec<IdxT, PPL> i0;
                i0.load(ib + (int64_t)r0.z * k);
                for (uint32_t e = b0; e < b1; ++e) {
                    const uint4 r2 = a.ovf[min(e + 2, last)];
                    IdxVec<IdxT, PPL> i1;
                    i1.load(ib + (int64_t)r1.z * k);
                    const float w = __uint_as_float(r0.x);
                    const float* __restrict__ row = a.dY + (int64_t)r0.y * dim;
                    float x[PPL];
#pragma unroll
                    for (int c = 0; c < PPL; ++c) x[c] = row[i0.get(c)];
                    float4* const ap = reinterpret_cast<float4*>(acc + (r0.z * k + q * PPL));
                    float4 av = *ap;
                    av.x += w * x[0]; av.y += w * x[1]; av.z += w * x[2]; av.w += w * x[3];
                    *ap = av;
                    r0 = r1; r1 = r2; i0 = i1;
                }
            }
        } else if (g < E) {
            // Mode 2 (few overflow entries, but hub destinations with hundreds of them in one bucket: large graphs):
            // the workgroup's entries are dealt to the lane groups in turn and added with LDS atomics.
            const uint32_t o0 = a.ovf_dir[bucket0], o1 = a.ovf_dir[bucket0 + n_owners];
            if (o0 < o1) {
                const uint32_t stride = (uint32_t)n_owners, last = o1 - 1;
                uint32_t e = o0 + (uint32_t)(wave * E + g);
                uint4 r0 = a.ovf[min(e, last)], r1 = a.ovf[min(e + stride, last)];
                IdxVec<IdxT, PPL> i0;
                i0.load(ib + (int64_t)r0.z * k);
                for (; e < o1; e += stride) {
                    const uint4 r2 = a.ovf[min(e + 2 * stride, last)];
                    IdxVec<IdxT, PPL> i1;
                    i1.load(ib + (int64_t)r1.z * k);
                    const float w = __uint_as_float(r0.x);
                    const float* __restrict__ row = a.dY + (int64_t)r0.y * dim;
                    float x[PPL];
#pragma unroll
                    for (int c = 0; c < PPL; ++c) x[c] = row[i0.get(c)];
#pragma unroll
                    for (int c = 0; c < PPL; ++c) atomicAdd(&acc[r0.z * k + q * PPL + c], w * x[c]);
                    r0 = r1; r1 = r2; i0 = i1;
                }
            }
        }
    }
    __syncthreads();
    float* __restrict__ out = a.dXs + dest0 * k;
    const int n_out = Dn * k;
    if (a.atomic_out) {
        for (int i = tid; i < n_out; i += kTiledThreads) unsafeAtomicAdd(out + i, acc[i]);
    } else {
        for (int i = tid; i < n_out; i += kTiledThreads) out[i] = acc[i];
    }
}

template <int TR, int DIMC, int RC, int PPL, typename IdxT>
maxk_status launch_tiled_t(const TiledArgs& a, size_t lds_bytes, hipStream_t s)
{
    static bool attr_set = false;  // per instantiation; the attribute is idempotent
    if (!attr_set) {
        MAXK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_tiled_kernel<TR, DIMC, RC, PPL, IdxT>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
        attr_set = true;
    }
    const int64_t grid = (int64_t)8 * a.G * a.R;
    if (grid > 0x7FFFFFFFll) return MAXK_UNSUPPORTED;
    hipLaunchKernelGGL((bwd_tiled_kernel<TR, DIMC, RC, PPL, IdxT>), dim3((unsigned)grid), dim3(kTiledThreads), lds_bytes, s, a);
    MAXK_LAUNCH_CHECK();
    return MAXK_OK;
}

}  // namespace

// CBSR positions one lane works on.  Eight (where k allows) were measured no faster than four on the dense workload
// (2.20 / 3.82 / 7.3 ms against 2.17 / 3.54 / 6.65 ms at k = 8 / 16 / 32): half as many wave instructions, each
// nearly twice as long.
int tiled_positions_per_lane(int) { return 4; }

void free_tiled(TiledSet& T)
{
    (void)hipFree(T.d_dir_sets);
    (void)hipFree(T.d_rec);
    (void)hipFree(T.d_extra);
    (void)hipFree(T.d_ovf);
    (void)hipFree(T.d_ovf_dir);
    (void)hipFree(T.d_progress);
    T = TiledSet();
}

// Destination-set size for (N, dim, k): as many nodes as LDS holds accumulators for beside two row buffers, rounded
// so that the number of sets is a power of two (the 32 CUs of an XCD then hold whole groups of sets).  Tiles of 16
// rows: taller ones (32, 48 rows, with correspondingly smaller sets) were measured slower at every k.
bool tiled_shape(int64_t N, int dim, int k, TiledShape& sh)
{
    if (N < 1 || k % 4 != 0 || k < 4 || k > 256 || dim % 4 != 0 || dim > 512) return false;
    const int tr = 16;
    const int64_t row_bytes = 2ll * tr * dim * 4;
    const int64_t dmax = std::min<int64_t>((kLdsBytes - row_bytes - 256) / (4ll * k), 4096);
    if (dmax < 64) return false;
    int64_t S = 8;
    while ((N + S - 1) / S > dmax) S *= 2;
    const int64_t D = (N + S - 1) / S;
    const int64_t n_dsets = (N + D - 1) / D;
    if (n_dsets > 65536) return false;
    sh.D = (int)D;
    sh.TR = tr;
    sh.n_dsets = (int)n_dsets;
    return true;
}

// Builds the visit lists for destination sets of D nodes and k/4 lanes per visit.  Synchronises the device.
// An XCD holds G destination sets and runs 32 workgroups at a time; the source rows are cut into R ranges so that
// its G * R workgroups fill whole rounds of 32 (as nearly as a small R allows).
void tiled_ranges(int n_dsets, int n_tiles, int& G, int& R, int& tiles_per_range)
{
    G = (n_dsets + 7) / 8;
    int best_r = 1;
    double best_fill = 0.0;
    for (int r = 1; r <= 32; ++r) {
        const int units = G * r;
        const double fill = (double)units / (32.0 * ((units + 31) / 32));
        if (fill > best_fill + 0.02) { best_fill = fill; best_r = r; }
    }
    R = std::min<int>(best_r, std::max<int>(1, n_tiles / 8));
    tiles_per_range = (n_tiles + R - 1) / R;
    R = (n_tiles + tiles_per_range - 1) / tiles_per_range;
}

maxk_status build_tiled(TiledSet& T, int64_t N, int64_t nnz, const int32_t* d_csc_ptr, const int32_t* d_csc_src,
                        const float* d_csc_val, int D, int TR, int k)
{
    const int LPV = k / tiled_positions_per_lane(k), E = kWave / LPV;
    MAXK_HIP_TRY(hipDeviceSynchronize());
    const int64_t n_dsets = (N + D - 1) / D, n_tiles = (N + TR - 1) / TR;
    const int64_t n_groups = n_dsets * n_tiles;
    if (n_groups + 1 > ((int64_t)1 << 28) || nnz < 1 || (int64_t)D * LPV > (int64_t)kVisitAccMask + 1) return MAXK_UNSUPPORTED;
    hipStream_t s = nullptr;
    uint64_t *d_key = nullptr, *d_key_sorted = nullptr;
    float* d_val_sorted = nullptr;
    uint32_t *d_head = nullptr, *d_rank = nullptr, *d_late = nullptr, *d_chain_pos = nullptr, *d_first_visit = nullptr,
             *d_sets = nullptr, *d_ovf_order = nullptr, *d_ovf_order_sorted = nullptr;
    uint64_t *d_ovf_key = nullptr, *d_ovf_key_sorted = nullptr;
    uint4* d_ovf_unsorted = nullptr;
    void* d_tmp = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(d_key); (void)hipFree(d_key_sorted); (void)hipFree(d_val_sorted); (void)hipFree(d_head);
        (void)hipFree(d_rank); (void)hipFree(d_late); (void)hipFree(d_chain_pos); (void)hipFree(d_first_visit);
        (void)hipFree(d_sets); (void)hipFree(d_tmp); (void)hipFree(d_ovf_order); (void)hipFree(d_ovf_order_sorted);
        (void)hipFree(d_ovf_key); (void)hipFree(d_ovf_key_sorted); (void)hipFree(d_ovf_unsorted);
    };
#define MAXK_TRY_CLEAN(expr)                                                           \
    do {                                                                               \
        hipError_t _e = (expr);                                                        \
        if (_e != hipSuccess) { cleanup(); free_tiled(T); return hip_fail(_e); }       \
    } while (0)
    const unsigned blocks = (unsigned)std::min<int64_t>((nnz + 255) / 256, 65536);
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_key, sizeof(uint64_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_key_sorted, sizeof(uint64_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_val_sorted, sizeof(float) * (size_t)nnz));
    hipLaunchKernelGGL(tiled_keys_kernel, dim3(blocks), dim3(256), 0, s, d_csc_ptr, d_csc_src, N, nnz, D, TR,
                       (int32_t)n_tiles, d_key);
    MAXK_TRY_CLEAN(hipGetLastError());
    int end_bit = 19;
    while (end_bit < 64 && ((uint64_t)1 << (end_bit - 18)) < (uint64_t)n_groups) ++end_bit;
    size_t tmp_bytes = 0;
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(nullptr, tmp_bytes, d_key, d_key_sorted, d_csc_val, d_val_sorted, (size_t)nnz,
                                             0, (unsigned)end_bit, s));
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(d_tmp, tmp_bytes, d_key, d_key_sorted, d_csc_val, d_val_sorted, (size_t)nnz,
                                             0, (unsigned)end_bit, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    (void)hipFree(d_tmp); d_tmp = nullptr;
    (void)hipFree(d_key); d_key = nullptr;

    MAXK_TRY_CLEAN(hipMalloc((void**)&d_head, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_rank, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_late, sizeof(uint32_t) * (size_t)nnz));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_chain_pos, sizeof(uint32_t) * (size_t)nnz));
    hipLaunchKernelGGL(tiled_flags_kernel, dim3(blocks), dim3(256), 0, s, d_key_sorted, nnz, d_head, d_late);
    MAXK_TRY_CLEAN(hipGetLastError());
    tmp_bytes = 0;
    MAXK_TRY_CLEAN(rocprim::inclusive_scan(nullptr, tmp_bytes, d_head, d_rank, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    size_t tmp2 = 0;
    MAXK_TRY_CLEAN(rocprim::exclusive_scan(nullptr, tmp2, d_late, d_chain_pos, 0u, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    tmp_bytes = std::max(tmp_bytes, tmp2);
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::inclusive_scan(d_tmp, tmp_bytes, d_head, d_rank, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    MAXK_TRY_CLEAN(rocprim::exclusive_scan(d_tmp, tmp2, d_late, d_chain_pos, 0u, (size_t)nnz, rocprim::plus<uint32_t>(), s));
    uint32_t n_visits = 0, last_late = 0, last_chain = 0;
    MAXK_TRY_CLEAN(hipMemcpyAsync(&n_visits, d_rank + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipMemcpyAsync(&last_late, d_late + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipMemcpyAsync(&last_chain, d_chain_pos + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    (void)hipFree(d_tmp); d_tmp = nullptr;
    const int64_t n_chain = (int64_t)last_chain + last_late;

    MAXK_TRY_CLEAN(hipMalloc((void**)&d_first_visit, sizeof(uint32_t) * (size_t)(n_groups + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_sets, sizeof(uint32_t) * (size_t)(n_groups + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_dir_sets, sizeof(uint32_t) * (size_t)(n_groups + 4)));
    MAXK_TRY_CLEAN(hipMemsetAsync(T.d_dir_sets + n_groups, 0xFF, sizeof(uint32_t) * 4, s));  // spare entries: read, never used
    hipLaunchKernelGGL(tiled_groups_kernel, dim3((unsigned)((n_groups + 1 + 255) / 256)), dim3(256), 0, s, d_key_sorted,
                       d_rank, nnz, n_groups, E, n_visits, d_first_visit, d_sets);
    MAXK_TRY_CLEAN(hipGetLastError());
    tmp_bytes = 0;
    MAXK_TRY_CLEAN(rocprim::exclusive_scan(nullptr, tmp_bytes, d_sets, T.d_dir_sets, 0u, (size_t)(n_groups + 1),
                                           rocprim::plus<uint32_t>(), s));
    MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
    MAXK_TRY_CLEAN(rocprim::exclusive_scan(d_tmp, tmp_bytes, d_sets, T.d_dir_sets, 0u, (size_t)(n_groups + 1),
                                           rocprim::plus<uint32_t>(), s));
    uint32_t total_sets = 0;
    MAXK_TRY_CLEAN(hipMemcpyAsync(&total_sets, T.d_dir_sets + n_groups, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    // the set count is a 32-bit sum: refuse graphs where it could have wrapped
    if ((int64_t)n_visits > (int64_t)total_sets * E ||
        (int64_t)total_sets > (int64_t)n_visits) {
        cleanup(); free_tiled(T); return MAXK_UNSUPPORTED;
    }
    // padding sets at the end: the kernel fetches kRecAhead of a wavefront's sets ahead without clamping
    const int64_t n_slots = ((int64_t)total_sets + (kRecAhead + 1) * kAccWaves) * E;
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_rec, sizeof(uint2) * (size_t)std::max<int64_t>(n_slots, 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_extra, sizeof(uint4) * (size_t)std::max<int64_t>(n_slots, 1)));
    // overflow entries: written in visit order, then sorted into one bucket per (workgroup, lane group of the workgroup)
    int G = 0, R = 0, tiles_per_range = 0;
    tiled_ranges((int)n_dsets, (int)n_tiles, G, R, tiles_per_range);
    const int n_owners = (kTiledThreads / kWave) * E;
    const int64_t n_buckets = n_dsets * R * (int64_t)n_owners;
    if (n_buckets + 1 > ((int64_t)1 << 31)) { cleanup(); free_tiled(T); return MAXK_UNSUPPORTED; }
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_ovf, sizeof(uint4) * (size_t)(n_chain + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_ovf_unsorted, sizeof(uint4) * (size_t)(n_chain + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&d_ovf_key, sizeof(uint64_t) * (size_t)(n_chain + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_ovf_dir, sizeof(uint32_t) * (size_t)(n_buckets + 1)));
    MAXK_TRY_CLEAN(hipMalloc((void**)&T.d_progress, sizeof(uint32_t) * (size_t)(kMaxUnits((int)n_dsets) * kMarkStride)));  // (T.n_dsets is set below)
    hipLaunchKernelGGL(tiled_fill_null_kernel, dim3((unsigned)std::min<int64_t>((n_slots + 255) / 256 + 1, 65536)), dim3(256),
                       0, s, T.d_rec, n_slots);
    hipLaunchKernelGGL(tiled_records_kernel, dim3(blocks), dim3(256), 0, s, d_key_sorted, d_val_sorted, d_head, d_rank,
                       d_late, d_chain_pos, nnz, E, LPV, (int32_t)n_tiles, TR, R, tiles_per_range, n_owners, d_first_visit,
                       T.d_dir_sets, T.d_rec, T.d_extra, d_ovf_unsorted, d_ovf_key);
    MAXK_TRY_CLEAN(hipGetLastError());
    if (n_chain > 0) {
        MAXK_TRY_CLEAN(hipMalloc((void**)&d_ovf_key_sorted, sizeof(uint64_t) * (size_t)n_chain));
        MAXK_TRY_CLEAN(hipMalloc((void**)&d_ovf_order, sizeof(uint32_t) * (size_t)n_chain));
        MAXK_TRY_CLEAN(hipMalloc((void**)&d_ovf_order_sorted, sizeof(uint32_t) * (size_t)n_chain));
        hipLaunchKernelGGL(tiled_iota_kernel, dim3((unsigned)std::min<int64_t>((n_chain + 255) / 256, 65536)), dim3(256), 0, s,
                           d_ovf_order, n_chain);
        MAXK_TRY_CLEAN(hipGetLastError());
        (void)hipFree(d_tmp); d_tmp = nullptr;
        tmp_bytes = 0;
        MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(nullptr, tmp_bytes, d_ovf_key, d_ovf_key_sorted, d_ovf_order,
                                                 d_ovf_order_sorted, (size_t)n_chain, 0, 64, s));
        MAXK_TRY_CLEAN(hipMalloc(&d_tmp, tmp_bytes ? tmp_bytes : 16));
        MAXK_TRY_CLEAN(rocprim::radix_sort_pairs(d_tmp, tmp_bytes, d_ovf_key, d_ovf_key_sorted, d_ovf_order,
                                                 d_ovf_order_sorted, (size_t)n_chain, 0, 64, s));
        hipLaunchKernelGGL(tiled_ovf_gather_kernel, dim3((unsigned)std::min<int64_t>((n_chain + 255) / 256, 65536)), dim3(256),
                           0, s, d_ovf_order_sorted, d_ovf_unsorted, n_chain, T.d_ovf);
        MAXK_TRY_CLEAN(hipGetLastError());
    }
    hipLaunchKernelGGL(tiled_ovf_dir_kernel, dim3((unsigned)((n_buckets + 1 + 255) / 256)), dim3(256), 0, s,
                       n_chain > 0 ? d_ovf_key_sorted : d_ovf_key, n_chain, n_buckets, T.d_ovf_dir);
    MAXK_TRY_CLEAN(hipGetLastError());
    MAXK_TRY_CLEAN(hipStreamSynchronize(s));
    int ovf_by_bucket = 0;
    if (n_chain > 0 && n_buckets <= ((int64_t)1 << 24)) {
        // bucket by bucket costs about one memory round trip (~1500 clocks) per entry of the longest bucket, the
        // atomics about 3 clocks per element of a workgroup's share
        try {
            std::vector<uint32_t> h_dir((size_t)n_buckets + 1);
            MAXK_TRY_CLEAN(hipMemcpy(h_dir.data(), T.d_ovf_dir, sizeof(uint32_t) * h_dir.size(), hipMemcpyDeviceToHost));
            uint32_t longest = 0;
            for (int64_t b2 = 0; b2 < n_buckets; ++b2) longest = std::max(longest, h_dir[(size_t)b2 + 1] - h_dir[(size_t)b2]);
            const double by_bucket = 1500.0 * longest, by_atomics = 3.0 * k * (double)n_chain / (double)(n_dsets * R);
            ovf_by_bucket = by_bucket < by_atomics ? 1 : 0;
        } catch (const std::bad_alloc&) {
            ovf_by_bucket = 0;  // the atomics need no look at the buckets
        }
    }
#undef MAXK_TRY_CLEAN
    cleanup();
    T.ovf_by_bucket = ovf_by_bucket;
    T.D = D;
    T.TR = TR;
    T.E = E;
    T.LPV = LPV;
    T.n_dsets = (int32_t)n_dsets;
    T.n_tiles = (int32_t)n_tiles;
    T.total_sets = total_sets;
    T.n_visits = n_visits;
    T.n_chain = n_chain;
    T.G = G;
    T.R = R;
    T.tiles_per_range = tiles_per_range;
    return MAXK_OK;
}

bool tiled_supports(const void* dY, int value_type, const void* sp_index, int index_bytes, int dim, int k)
{
    return value_type == MAXK_VALUE_F32 && k % 4 == 0 && k >= 4 && k <= 256 && dim % 4 == 0 && dim <= 512 &&
           aligned(dY, 16) && aligned(sp_index, std::min<size_t>(16, (size_t)tiled_positions_per_lane(k) * index_bytes));
}

maxk_status launch_bwd_tiled(const TiledSet& T, const void* dY, int value_type, const void* sp_index, int index_bytes,
                             int64_t N, int dim, int k, float* dXs, hipStream_t s)
{
    if (!tiled_supports(dY, value_type, sp_index, index_bytes, dim, k) || T.LPV != k / tiled_positions_per_lane(k) || T.TR != 16) return MAXK_UNSUPPORTED;
    TiledArgs a;
    a.dY = (const float*)dY;
    a.sp_index = sp_index;
    a.dXs = dXs;
    a.dir_sets = T.d_dir_sets;
    a.rec = T.d_rec;
    a.extra = T.d_extra;
    a.ovf = T.d_ovf;
    a.ovf_dir = T.d_ovf_dir;
    a.ovf_by_bucket = T.ovf_by_bucket;
    a.N = N;
    a.dim = dim;
    a.k = k;
    a.D = T.D;
    a.n_dsets = T.n_dsets;
    a.n_tiles = T.n_tiles;
    a.G = T.G;  // fixed when the lists were built: the overflow entries are sorted by workgroup
    a.R = T.R;
    a.tiles_per_range = T.tiles_per_range;
    a.atomic_out = a.R > 1;
    a.range_per_xcd = (a.R > 1 && 8 % a.R == 0 && a.G * a.R <= 32) ? 1 : 0;
    if (a.atomic_out) {
        const maxk_status st = launch_fill_zero(dXs, N * (int64_t)k, s);
        if (st != MAXK_OK) return st;
    }
    a.progress = T.d_progress;
    // Pacing window: 32 tiles (0.5 MB of dY at hidden width 256) measured best of 16..256 on the dense workload at
    // k = 8, 16, 32: 3-5 % faster than without pacing, with a quarter of the L2 fills.  Calls that run at the same
    // time on one handle share the marks; that can only make them nap at the wrong moments.
    // Only when every workgroup has a CU from the start (256 CUs): otherwise the running ones are not one pack.
    a.window = (int64_t)8 * a.G * a.R <= 256 ? kPaceWindow : 0;
    if (!T.d_progress || (int64_t)8 * a.G * a.R > kMaxUnits(T.n_dsets)) a.window = 0;
    if (a.window > 0) {
        const maxk_status st = launch_fill_zero(reinterpret_cast<float*>(T.d_progress), (int64_t)8 * a.G * a.R * kMarkStride, s);
        if (st != MAXK_OK) return st;
    }
    const size_t lds_bytes = sizeof(float) * ((size_t)((T.D * k + 3) & ~3) + 2 * (size_t)T.TR * dim);
    if (lds_bytes > (size_t)kLdsBytes) return MAXK_UNSUPPORTED;
#define MAXK_TILED_I(TR, DIMC, RC, PPL)                                                                           \
    (index_bytes == 1 ? launch_tiled_t<TR, DIMC, RC, PPL, uint8_t>(a, lds_bytes, s)                               \
     : index_bytes == 2 ? launch_tiled_t<TR, DIMC, RC, PPL, uint16_t>(a, lds_bytes, s)                            \
                        : launch_tiled_t<TR, DIMC, RC, PPL, int32_t>(a, lds_bytes, s))
    const maxk_status st = dim == 256 ? MAXK_TILED_I(16, 256, 1, 4) : dim < 256 ? MAXK_TILED_I(16, 0, 1, 4) : MAXK_TILED_I(16, 0, 2, 4);
#undef MAXK_TILED_I
    return st;
}

}  // namespace maxk
