// Host-side launch of the query stage: picks the kernel variant for (d, d_bin, K).
#pragma once
#include "fg_query.hpp"
#include "fg_query_tile.hpp"
#include "fg_query_list.hpp"

namespace fg {

// ---- tile order: heaviest tiles first --------------------------------------------------------
// Tiles differ in cost by more than an order of magnitude (a tile inside a dense cluster scans thousands of
// candidates per query) and the hardware hands out workgroups in index order, so a heavy tile that starts late
// sets the kernel's end: measured on the 1M-point clustered workload the tile kernel took 1.2 ms for 0.73 ms of
// evenly spread work, the last third of it with most of the chip idle.  The tiles are therefore ranked by an
// estimate of their work, in 64 classes of half a power of two, heaviest class first.
// tile_order: [0, T) the order, [T, 2T) class of each tile (bit 6: uneven, see k_tile_work), [2T, 2T+64) class
// histogram, [2T+64, 2T+128) cursors.
constexpr int kTileClasses = 64;

static __global__ void k_reset_query_scratch(int32_t* work_count, int32_t* tile_counters)
{
    if (threadIdx.x == 0) *work_count = 0;
    if (tile_counters && threadIdx.x < 2 * kTileClasses) tile_counters[threadIdx.x] = 0;
}

// The work list of the list kernel from the tiles' hand-over marks: blocks of 1024 tiles, the queries of a block in
// tile order (a block's place in the list comes from one atomic add, so blocks may swap, 65 536 queries each).
static __global__ void __launch_bounds__(1024) k_list_compact(const uint64_t* __restrict__ handed, int32_t n_tiles,
                                                              int32_t* __restrict__ work_list, int32_t* __restrict__ work_count)
{
    __shared__ int32_t wave_tot[16];
    __shared__ int32_t block_base;
    const int32_t t = blockIdx.x * 1024 + threadIdx.x;
    const uint64_t m = t < n_tiles ? handed[t] : 0ull;
    const int32_t c = __popcll(m);
    int32_t incl = c;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int o = 1; o < 64; o <<= 1) {
        const int32_t up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int j = 0; j < 16; ++j) {
        const int32_t w = wave_tot[j];
        if (j < wv) before += w;
        total += w;
    }
    if (threadIdx.x == 0) block_base = total > 0 ? atomicAdd(work_count, total) : 0;
    __syncthreads();
    int32_t at = block_base + before + incl - c;
    for (uint64_t rest = m; rest; rest &= rest - 1)
        work_list[at++] = t * kQueryBlock + (__ffsll((unsigned long long)rest) - 1);
}

__device__ __forceinline__ int32_t tile_class(int32_t work)
{
    if (work < 2) return work < 1 ? 0 : 1;
    const int32_t lg = 31 - __clz(work);
    const int32_t c = 2 * lg + ((work >> (lg - 1)) & 1);
    return c < kTileClasses ? c : kTileClasses - 1;
}

constexpr int kTilesPerWave = 16;

// Work estimate of a tile: what the first two shells cost it without any pruning, i.e. for every column of the
// 3 x ... x 3 neighbourhood the longest candidate run any of its queries has there (the tile kernel scans a
// column for as long as its busiest lane needs), summed over the columns.  Taken over 8 of the tile's 64 queries
// (every ninth: consecutive queries mostly share their bins), 8 tiles per wavefront at a time: with all 64 the
// gathers of the bin boundaries made this kernel cost 73 us per million points.
constexpr int kTileSamples = 8;
constexpr int kFlatLaneUsePct = 60;   // below this estimated lane use (per cent) a tile takes the flattened scan
static_assert(kTileClasses == (1 << kTileFlatBit), "the flag sits above the class bits");

// maximum / sum over each aligned group of 8 lanes, returned in all 8 (DPP: swap inside pairs, swap pairs, mirror the half row)
__device__ __forceinline__ int32_t oct_max_i32(int32_t v)
{
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xb1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4e, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false));   // row_half_mirror
    return v;
}
__device__ __forceinline__ int32_t oct_sum_i32(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(v, v, 0xb1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(v, v, 0x4e, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false);
    return v;
}

template <int DB>
static __global__ void __launch_bounds__(256) k_tile_work(QueryArgs a, int32_t n_tiles)
{
    __shared__ int32_t hist[kTileClasses];
    if (threadIdx.x < kTileClasses) hist[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int sample = lane & (kTileSamples - 1);
    const int32_t wave_t0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kTilesPerWave;
    int32_t ncols = 1;
#pragma unroll
    for (int c = 0; c < DB - 1; ++c) ncols *= 3;
    for (int32_t tb = wave_t0; tb < wave_t0 + kTilesPerWave; tb += kQueryBlock / kTileSamples) {
        const int32_t t = tb + (lane >> 3);
        const int32_t p = t * kQueryBlock + sample * 9;            // queries 0, 9, ..., 63 of the tile
        const bool live = t < n_tiles && p < a.n;
        int32_t cc[DB], seg_cell0 = 0;
        {
            const int32_t row = live ? __float_as_int(reinterpret_cast<const float*>(a.rec)[(int64_t)p * (rec_vecs(a.d) * 4) + a.d]) : 0;
            const int32_t b = live ? a.bin_idx[row] : 0;
            int32_t r = b % a.cells_per_segment;
            seg_cell0 = b - r;
            // the flat number counts slices of the last dimension (2^sub_shift per bin)
            const int32_t nz = a.n_bins << a.sub_shift;
            cc[DB - 1] = (r % nz) >> a.sub_shift;
            r /= nz;
#pragma unroll
            for (int c = DB - 2; c >= 0; --c) { cc[c] = r % a.n_bins; r /= a.n_bins; }
        }
        int32_t work = 0, around = 0, longest = 0, total = 0;
        for (int32_t col = 0; col < ncols; ++col) {
            int32_t rem = col, flat = 0;
            bool ok = live;
#pragma unroll
            for (int c = 0; c < DB - 1; ++c) {     // digit c of col -> offset -1, 0, +1 in dimension c
                const int32_t j = cc[c] + rem % 3 - 1;
                rem /= 3;
                ok = ok && j >= 0 && j < a.n_bins;
                flat = flat * a.n_bins + j;
            }
            int32_t len = 0;
            if (ok) {
                const int32_t cz = cc[DB - 1];
                const int32_t za = cz > 0 ? cz - 1 : 0, zb = cz < a.n_bins - 1 ? cz + 1 : a.n_bins - 1;
                const int32_t row = flat * a.n_bins;
                len = a.bounds[seg_cell0 + ((row + zb + 1) << a.sub_shift)] - a.bounds[seg_cell0 + ((row + za) << a.sub_shift)];
            }
            around += len;
            const int32_t col_max = oct_max_i32(len);
            work += col_max >> 2;                  // in passes of four; keeps the sum small
            longest += col_max;
            total += oct_sum_i32(len);
        }
        // A query with few points around it will not be certified after shell 1 (the k-th neighbour of a query at
        // the centre of its bin lies inside the inscribed ball of the 3-bin cube, about a sixth of its volume, only
        // if the cube holds some 6 K points); where more such queries than the tile kernel hands over are expected,
        // the tile will go on to shell 2: 5 x ... x 5 columns of 5-bin runs.
        const bool lonely = live && around < 4 * (a.slot0 + a.k_list);
        const bool goes_on = oct_sum_i32(lonely ? 1 : 0) * (kQueryBlock / kTileSamples) > a.defer_lanes;
        if (__any(goes_on)) {
            int32_t ncols2 = 1;
#pragma unroll
            for (int c = 0; c < DB - 1; ++c) ncols2 *= 5;
            for (int32_t col = 0; col < ncols2; ++col) {
                int32_t rem = col, flat = 0;
                bool ok = lonely && goes_on;
#pragma unroll
                for (int c = 0; c < DB - 1; ++c) {
                    const int32_t j = cc[c] + rem % 5 - 2;
                    rem /= 5;
                    ok = ok && j >= 0 && j < a.n_bins;
                    flat = flat * a.n_bins + j;
                }
                int32_t len = 0;
                if (ok) {
                    const int32_t cz = cc[DB - 1];
                    const int32_t za = cz > 1 ? cz - 2 : 0, zb = cz < a.n_bins - 2 ? cz + 2 : a.n_bins - 1;
                    const int32_t row = flat * a.n_bins;
                    len = a.bounds[seg_cell0 + ((row + zb + 1) << a.sub_shift)] - a.bounds[seg_cell0 + ((row + za) << a.sub_shift)];
                }
                work += oct_max_i32(len) >> 2;
            }
        }
        if (sample == 0 && t < n_tiles) {
            const int32_t cls = tile_class(work);
            // Uneven tile: over these columns its queries' runs average less than kFlatLaneUsePct of the longest
            // one, so a direct scan (every column as long as its busiest lane) leaves most lanes idle and the
            // flattened scan, at about twice the cost per pass, still comes out ahead.  Pruning, which this
            // estimate does not see, only widens the spread.
            const bool uneven = total * 100 < longest * kTileSamples * kFlatLaneUsePct;
            a.tile_order[n_tiles + t] = cls | ((uneven ? 1 : 0) << kTileFlatBit);
            atomicAdd(&hist[cls], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x < kTileClasses && hist[threadIdx.x] > 0)
        atomicAdd(&a.tile_order[2 * n_tiles + threadIdx.x], hist[threadIdx.x]);
}

// Position of every tile: classes in descending order; inside a class roughly the bin order (blocks of 256
// consecutive tiles reserve their places with one atomic per class, and a block's tiles keep the order in which
// its waves arrive), so that tiles running at the same time still share their neighbourhoods in the L2 cache.
static __global__ void __launch_bounds__(256) k_tile_rank(int32_t* __restrict__ order, int32_t n_tiles)
{
    __shared__ int32_t local[kTileClasses];   // this block's tiles per class, then the block's first position in the class
    __shared__ int32_t first[kTileClasses];   // position of the class's first tile: all heavier classes before it
    if (threadIdx.x < kTileClasses) {
        local[threadIdx.x] = 0;
        int32_t s = 0;
        for (int c = threadIdx.x + 1; c < kTileClasses; ++c) s += order[2 * n_tiles + c];
        first[threadIdx.x] = s;
    }
    __syncthreads();
    const int32_t t = blockIdx.x * 256 + threadIdx.x;
    int32_t cls = 0, mine = 0, uneven = 0;
    if (t < n_tiles) {
        const int32_t word = order[n_tiles + t];
        cls = word & (kTileClasses - 1);
        uneven = (word >> kTileFlatBit) & 1;
        mine = atomicAdd(&local[cls], 1);
    }
    __syncthreads();
    if (threadIdx.x < kTileClasses && local[threadIdx.x] > 0)
        local[threadIdx.x] = atomicAdd(&order[2 * n_tiles + kTileClasses + threadIdx.x], local[threadIdx.x]);
    __syncthreads();
    if (t < n_tiles) order[first[cls] + local[cls] + mine] = t | (uneven << kOrderFlagBit);
}

template <typename K>
static void allow_lds(K kernel, size_t bytes)
{
    if (bytes > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// One pass of the fast path: tile kernel + list kernel for a.k_list <= 64 neighbours per query.
template <int D, int DB, bool COUNT, bool LOWER>
static void launch_query_pass(const QueryArgs& a_in, hipStream_t stream)
{
    QueryArgs a = a_in;
    const int grid = (a.n + kQueryBlock - 1) / kQueryBlock;
    const bool ordered = a.tile_order && a.bin_idx && grid > 1024;    // a few waves per SIMD: nothing to reorder
    hipLaunchKernelGGL(k_reset_query_scratch, dim3(1), dim3(2 * kTileClasses), 0, stream, a.work_count,
                       ordered ? a.tile_order + 2 * grid : nullptr);
    if (ordered) {
        hipLaunchKernelGGL(k_tile_work<DB>, dim3((grid + 4 * kTilesPerWave - 1) / (4 * kTilesPerWave)), dim3(256), 0, stream, a, grid);
        hipLaunchKernelGGL(k_tile_rank, dim3((grid + 255) / 256), dim3(256), 0, stream, a.tile_order, grid);
    } else {
        a.tile_order = nullptr;
    }
    const int32_t cap = a.k_list;
    if (cap <= 16) {
        const size_t lds = tile_sorted_lds_bytes<16, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 16, COUNT, LOWER>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 32) {
        const size_t lds = tile_sorted_lds_bytes<32, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 32, COUNT, LOWER>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 48) {
        const size_t lds = tile_sorted_lds_bytes<48, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 48, COUNT, LOWER>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else {
        const size_t lds = tile_sorted_lds_bytes<64, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 64, COUNT, LOWER>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    }
    hipLaunchKernelGGL(k_list_compact, dim3((grid + 1023) / 1024), dim3(1024), 0, stream, a.handed, grid, a.work_list, a.work_count);
    // one query per wavefront; four times the wave slots of the chip: the queries differ widely in cost, and with
    // more, shorter workgroups the hardware dispatcher evens them out (cursors in memory cost more than they gained)
    const int list_grid = a.n < 32768 ? a.n : 32768;
    hipLaunchKernelGGL((k_query_list_wave<D, DB, COUNT>), dim3(list_grid), dim3(kQueryBlock), 0, stream, a);
}

// Lists of more than 64 neighbours (K - 1 up to 127) take two passes: the first finds the 64 nearest, the second
// the rest, counting only keys above the 64th (keys are unique, so the split is exact).  A sorted list of more
// than 64 keys does not fit the 256 architectural registers of a wavefront next to everything else: held partly
// in accumulation registers it ran at one wavefront per SIMD with a copy at every use, 2.8x slower per query at
// K = 70 than at K = 65.
template <int D, int DB, bool COUNT>
static hipError_t launch_query_impl(const QueryArgs& a_in, hipStream_t stream)
{
    QueryArgs a = a_in;
    if (a.algo == 1) {
        const int grid = (a.n + kQueryBlock - 1) / kQueryBlock;
        const size_t heap_bytes = (size_t)(a.k > 1 ? a.k - 1 : 1) * kQueryBlock * sizeof(uint64_t);
        allow_lds(k_query_shell<D, DB, COUNT>, heap_bytes);
        hipLaunchKernelGGL((k_query_shell<D, DB, COUNT>), dim3(grid), dim3(kQueryBlock), heap_bytes, stream, a);
        return hipGetLastError();
    }
    const int32_t cap = a.k - 1;
    a.slot0 = 0;
    a.k_list = cap < 64 ? cap : 64;
    launch_query_pass<D, DB, COUNT, false>(a, stream);
    if (cap > 64) {
        a.slot0 = 64;
        a.k_list = cap - 64;
        launch_query_pass<D, DB, COUNT, true>(a, stream);
    }
    return hipGetLastError();
}

template <int D, int DB>
static hipError_t launch_query_shell(const QueryArgs& a, hipStream_t stream)
{
    return a.out_cand ? launch_query_impl<D, DB, true>(a, stream) : launch_query_impl<D, DB, false>(a, stream);
}

template <int D>
static hipError_t dispatch_query_dbin(const QueryArgs& a, int32_t d_bin, hipStream_t stream)
{
    switch (d_bin) {
        case 2: return launch_query_shell<D, 2>(a, stream);
        case 3: if constexpr (D >= 3) return launch_query_shell<D, 3>(a, stream); break;
        case 4: if constexpr (D >= 4) return launch_query_shell<D, 4>(a, stream); break;
        case 5: if constexpr (D >= 5) return launch_query_shell<D, 5>(a, stream); break;
        default: break;
    }
    return hipErrorInvalidValue;
}

}  // namespace fg
