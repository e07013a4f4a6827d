// Spatial partition + counting sort (paper Section 3: bin assignment per row split, points
// sorted by bin, cumulative bin boundaries).  gfx950, wave64.
//
// Stages, all enqueued on one stream:
//   prepare   zero the bin counters, reset the bounding-box keys
//   bbox      per row split, min/max of the first d_bin coordinates (register, wave and block
//             reduction, one atomic pair per block and dimension on an order-preserving key)
//   assign    per (row split, dim) the grid geometry (lower edge, cells per unit length, cell width,
//             rounding slack: computed from the bounding box where needed, the records written
//             for the query kernels); flat cell of every point + its arrival rank inside the cell
//             (LDS-privatised histogram per block, one returning global atomic per distinct cell
//             and block; issuing a thread's atomics back to back instead of one round trip at a
//             time changed nothing: the kernel runs at the rate of the memory-side atomics).
//             A cell is a bin, or one of the 2^sub_shift slices a bin is cut into along the last
//             binning dimension
//   scan      exclusive prefix over the counters (per-chunk totals, then apply; a pass over the
//             totals in between only when there are many chunks)
//   scatter   sorted position = bounds[cell] + rank: one record per point (coordinates, original row)
#include "fg_internal.hpp"

namespace fg {

constexpr int kBlock = 256;
constexpr int kScanItems = 16;                    // counters per thread in the scan kernels
constexpr int kScanChunk = kBlock * kScanItems;   // counters per block

__device__ __forceinline__ uint32_t float_to_key(float f)
{
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k)
{
    uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(b);
}

__global__ void __launch_bounds__(kBlock)
k_prepare(int32_t* __restrict__ counters, int64_t n_counters, uint32_t* __restrict__ bbox_keys, int32_t n_keys)
{
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int64_t step = (int64_t)gridDim.x * kBlock;
    for (int64_t j = i; j < n_counters; j += step) counters[j] = 0;
    // keys: [S][d_bin] minima then [S][d_bin] maxima
    for (int64_t j = i; j < 2 * (int64_t)n_keys; j += step) bbox_keys[j * kKeyStride] = (j < n_keys) ? 0xffffffffu : 0u;
}

__device__ __forceinline__ float wave_min(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// One block per chunk of kBboxChunk consecutive points.  A chunk that lies inside one row split
// (the common case) is reduced in registers, then across the wave, then across the block, and
// issues one atomic pair per dimension; a chunk straddling a split boundary falls back to
// per-wave or per-lane atomics.  Same-address atomics serialise, so their number matters.
constexpr int kBboxItems = 4;     // few points per thread: the launch needs well over 256 blocks to keep loads in flight
constexpr int kBboxChunk = kBlock * kBboxItems;

template <int DB>
__global__ void __launch_bounds__(kBlock)
k_bbox(const float* __restrict__ coords, const int32_t* __restrict__ row_splits, int32_t n, int32_t d,
       int32_t n_segments, uint32_t* __restrict__ bbox_keys)
{
    __shared__ float red[2][kBlock / 64][DB];
    const int64_t base = (int64_t)blockIdx.x * kBboxChunk;
    const int32_t last = (int32_t)(base + kBboxChunk < n ? base + kBboxChunk : n) - 1;
    uint32_t* kmin = bbox_keys;
    uint32_t* kmax = bbox_keys + (int64_t)n_segments * DB * kKeyStride;
    const int32_t s_first = segment_of(row_splits, n_segments, (int32_t)base);
    const int32_t s_last = segment_of(row_splits, n_segments, last);
    if (s_first == s_last) {
        float mn[DB], mx[DB];
#pragma unroll
        for (int c = 0; c < DB; ++c) { mn[c] = 3.4028235e38f; mx[c] = -3.4028235e38f; }
        for (int it = 0; it < kBboxItems; ++it) {
            const int64_t i = base + it * kBlock + threadIdx.x;
            if (i <= last) {
#pragma unroll
                for (int c = 0; c < DB; ++c) {
                    const float x = coords[i * d + c];
                    mn[c] = fminf(mn[c], x);
                    mx[c] = fmaxf(mx[c], x);
                }
            }
        }
        const int wv = threadIdx.x >> 6;
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            const float a = wave_min(mn[c]), b = wave_max(mx[c]);
            if ((threadIdx.x & 63) == 0) { red[0][wv][c] = a; red[1][wv][c] = b; }
        }
        __syncthreads();
        if (threadIdx.x < DB) {
            const int c = threadIdx.x;
            float a = red[0][0][c], b = red[1][0][c];
#pragma unroll
            for (int w = 1; w < kBlock / 64; ++w) { a = fminf(a, red[0][w][c]); b = fmaxf(b, red[1][w][c]); }
            atomicMin(&kmin[(s_first * DB + c) * kKeyStride], float_to_key(a));
            atomicMax(&kmax[(s_first * DB + c) * kKeyStride], float_to_key(b));
        }
        return;
    }
    for (int it = 0; it < kBboxItems; ++it) {
        const int64_t i = base + it * kBlock + threadIdx.x;
        const bool live = i <= last;
        const int32_t ii = live ? (int32_t)i : last;
        const int32_t s = segment_of(row_splits, n_segments, ii);
        const int32_t s0 = __shfl(s, 0, 64);
        const bool uniform = __all(s == s0);
        const float* p = coords + (int64_t)ii * d;
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            const float x = p[c];
            if (uniform) {
                const float a = wave_min(x), b = wave_max(x);   // dead lanes duplicate the chunk's last point: harmless
                if ((threadIdx.x & 63) == 0) {
                    atomicMin(&kmin[(s * DB + c) * kKeyStride], float_to_key(a));
                    atomicMax(&kmax[(s * DB + c) * kKeyStride], float_to_key(b));
                }
            } else if (live) {
                atomicMin(&kmin[(s * DB + c) * kKeyStride], float_to_key(x));
                atomicMax(&kmax[(s * DB + c) * kKeyStride], float_to_key(x));
            }
        }
    }
}

// geom[s][c] = { lo, inv_w, w, slack }.
//   inv_w = n_bins / (hi - lo) bins per unit length; 0 marks a dimension in which every point of
//           the row split lands in bin 0 (zero, denormal-small or non-finite extent, empty split).
//   slack  bounds |true bin threshold - (lo + j*w)| from above: the float32 evaluation of
//           floor((x-lo)*inv_w) and of lo + j*w together err by < 2^-21 * max(|lo|,|hi|,hi-lo).
struct DimGeom { float lo, inv_w, w, slack; };

__device__ __forceinline__ DimGeom dim_geometry(const uint32_t* __restrict__ bbox_keys, int32_t n_keys, int32_t t, int32_t n_bins)
{
    float lo = key_to_float(bbox_keys[(int64_t)t * kKeyStride]);
    const float hi = key_to_float(bbox_keys[(int64_t)(n_keys + t) * kKeyStride]);
    const float ext = hi - lo;
    float inv_w = 0.0f, w = 0.0f, slack = 0.0f;
    if (ext >= 1e-30f && ext <= 3.0e38f) {          // false for NaN and for the empty-split sentinels
        const float iw = (float)n_bins / ext;
        if (iw <= 3.0e38f) {
            inv_w = iw;
            w = ext / (float)n_bins;
            slack = 9.5367431640625e-07f * fmaxf(fmaxf(fabsf(lo), fabsf(hi)), ext);   // 2^-20
        }
    }
    if (!(lo >= -3.0e38f && lo <= 3.0e38f)) lo = 0.0f;   // empty split: keep the record finite
    return DimGeom{lo, inv_w, w, slack};
}

// Bin of every point and its arrival rank inside the bin.  The rank comes from an atomic add on
// the bin's counter; atomics on one address serialise, and skewed data put a large share of all
// points into a few bins.  So a block first counts its kAssignChunk points per bin in an
// LDS-privatised histogram (an open-addressing table keyed by bin, LDS atomics give the rank
// inside the block), then adds each distinct bin's block total to the global counter once, and
// finally hands every point the block's base plus its local rank.  A point that finds no table
// slot within kAssignProbes probes takes the global atomic directly.
constexpr int kAssignItems = 4;
constexpr int kAssignChunk = kBlock * kAssignItems;
constexpr int kAssignSlots = 2048;
constexpr int kAssignProbes = 8;

template <int DB>
__global__ void __launch_bounds__(kBlock)
k_assign(const float* __restrict__ coords, const int32_t* __restrict__ row_splits, int32_t n, int32_t d,
         int32_t n_segments, int32_t n_bins, int32_t sub_shift, int32_t cells_per_segment, int32_t morton_bits,
         const uint32_t* __restrict__ bbox_keys, float* __restrict__ geom, int32_t* __restrict__ bin_idx,
         int32_t* __restrict__ rank, int32_t* __restrict__ counters)
{
    // the geometry records the query kernels read: written here by the first blocks; the bins below are
    // computed from the same bounding-box keys with the same arithmetic
    const int32_t n_keys = n_segments * DB;
    for (int32_t t = blockIdx.x * kBlock + threadIdx.x; t < n_keys; t += gridDim.x * kBlock) {
        const DimGeom r = dim_geometry(bbox_keys, n_keys, t, (t % DB == DB - 1) ? n_bins << sub_shift : n_bins);
        float* g = geom + (int64_t)t * kGeomStride;
        g[0] = r.lo; g[1] = r.inv_w; g[2] = r.w; g[3] = r.slack;
    }
    __shared__ int32_t keys[kAssignSlots];
    __shared__ int32_t cnts[kAssignSlots];     // block-local population, then the block's base in the bin
    for (int i = threadIdx.x; i < kAssignSlots; i += kBlock) { keys[i] = -1; cnts[i] = 0; }
    __syncthreads();
    int32_t flat[kAssignItems], slot[kAssignItems], local[kAssignItems];
#pragma unroll
    for (int it = 0; it < kAssignItems; ++it) {
        const int64_t i = (int64_t)blockIdx.x * kAssignChunk + it * kBlock + threadIdx.x;
        flat[it] = -1; slot[it] = -1; local[it] = 0;
        if (i >= n) continue;
        const int32_t s = segment_of(row_splits, n_segments, (int32_t)i);
        const float* p = coords + i * d;
        int32_t cell[DB];
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            const int32_t nb_c = (c == DB - 1) ? n_bins << sub_shift : n_bins;    // the last dimension counts slices
            const DimGeom r = dim_geometry(bbox_keys, n_keys, s * DB + c, nb_c);
            cell[c] = cell_of(p[c], r.lo, r.inv_w, nb_c);
        }
        int32_t f = 0;
        if (morton_bits == 0) {                 // row-major, last dimension fastest (what the query kernels expect)
#pragma unroll
            for (int c = 0; c < DB; ++c) f = f * ((c == DB - 1) ? n_bins << sub_shift : n_bins) + cell[c];
        } else {                                // bit-interleaved: consecutive bins form compact blocks in space
            for (int b = 0; b < morton_bits; ++b) {
#pragma unroll
                for (int c = 0; c < DB; ++c) f |= ((cell[c] >> b) & 1) << (b * DB + (DB - 1 - c));
            }
        }
        f += s * cells_per_segment;
        flat[it] = f;
        bin_idx[i] = f;
        uint32_t h = ((uint32_t)f * 2654435761u) >> 21;              // 11 bits
#pragma unroll 1
        for (int probe = 0; probe < kAssignProbes; ++probe) {
            const int32_t prev = atomicCAS(&keys[h], -1, f);
            if (prev == -1 || prev == f) { slot[it] = (int32_t)h; local[it] = atomicAdd(&cnts[h], 1); break; }
            h = (h + 1) & (kAssignSlots - 1);
        }
        if (slot[it] < 0) local[it] = atomicAdd(&counters[f], 1);   // no slot: straight to memory
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kAssignSlots; i += kBlock) {
        const int32_t f = keys[i];
        if (f >= 0) cnts[i] = atomicAdd(&counters[f], cnts[i]);      // block total in, block base out
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kAssignItems; ++it) {
        const int64_t i = (int64_t)blockIdx.x * kAssignChunk + it * kBlock + threadIdx.x;
        if (i >= n) continue;
        rank[i] = slot[it] >= 0 ? cnts[slot[it]] + local[it] : local[it];
    }
}

// ---- exclusive scan over the counters, in place: counters[b] -> first sorted position of bin b.
__device__ __forceinline__ int32_t wave_incl_scan(int32_t v)
{
    int lane = threadIdx.x & 63;
    for (int o = 1; o < 64; o <<= 1) {
        int32_t t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// block-wide exclusive scan of one value per thread; returns the exclusive prefix, total in *total
__device__ __forceinline__ int32_t block_excl_scan(int32_t v, int32_t* total)
{
    __shared__ int32_t wave_tot[kBlock / 64];
    int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int32_t inc = wave_incl_scan(v);
    if (lane == 63) wave_tot[wv] = inc;
    __syncthreads();
    int32_t base = 0, tot = 0;
#pragma unroll
    for (int j = 0; j < kBlock / 64; ++j) {
        int32_t t = wave_tot[j];
        if (j < wv) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ void __launch_bounds__(kBlock)
k_scan_partials(const int32_t* __restrict__ counters, int64_t n_counters, int32_t* __restrict__ partials)
{
    int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int32_t sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        int64_t q = base + j;
        if (q < n_counters) sum += counters[q];
    }
    int32_t total;
    block_excl_scan(sum, &total);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// single block: exclusive scan of the per-chunk totals, in place
__global__ void __launch_bounds__(kBlock)
k_scan_tops(int32_t* __restrict__ partials, int32_t n_partials)
{
    int32_t carry = 0;
    for (int32_t b = 0; b < n_partials; b += kBlock) {
        int32_t q = b + threadIdx.x;
        int32_t v = q < n_partials ? partials[q] : 0;
        int32_t total;
        int32_t ex = block_excl_scan(v, &total);
        if (q < n_partials) partials[q] = carry + ex;
        carry += total;
    }
}

// partials hold exclusive prefixes (after k_scan_tops) or, with totals = true, the raw per-chunk totals, of
// which every block then sums those before its own (cheaper than a third launch while there are few chunks)
template <bool TOTALS>
__global__ void __launch_bounds__(kBlock)
k_scan_apply(int32_t* __restrict__ counters, int64_t n_counters, const int32_t* __restrict__ partials)
{
    int32_t chunk_base;
    if (TOTALS) {
        int32_t part = 0;
        for (int32_t q = threadIdx.x; q < (int32_t)blockIdx.x; q += kBlock) part += partials[q];
        block_excl_scan(part, &chunk_base);
    } else {
        chunk_base = partials[blockIdx.x];
    }
    int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int32_t v[kScanItems];
    int32_t sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        int64_t q = base + j;
        v[j] = q < n_counters ? counters[q] : 0;
        sum += v[j];
    }
    int32_t total;
    int32_t run = block_excl_scan(sum, &total) + chunk_base;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        int64_t q = base + j;
        if (q < n_counters) counters[q] = run;
        run += v[j];
    }
}

// Forward order: every point becomes one record (coordinates, original row, zero padding: whole 16-byte
// vectors) at its sorted position; that is one scattered 16-byte store per vector, where separate coordinate
// and permutation arrays took a scattered 4-byte store each (measured 103 MB written for a 16 MB payload).
// ROWS_ONLY (the backward's row order): only the permutation; for D = 3 the record area instead receives the
// rows in their original order padded to four floats, which the backward kernel gathers with one load per
// neighbour.
template <int D, bool ROWS_ONLY>
__global__ void __launch_bounds__(kBlock)
k_scatter(const float* __restrict__ coords, int32_t n, const int32_t* __restrict__ bin_idx,
          const int32_t* __restrict__ rank, const int32_t* __restrict__ bounds,
          int32_t* __restrict__ perm, float* __restrict__ rec)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const int32_t pos = bounds[bin_idx[i]] + rank[i];
    const float* p = coords + i * D;
    if constexpr (ROWS_ONLY) {
        perm[pos] = (int32_t)i;
        if constexpr (D == 3) reinterpret_cast<float4*>(rec)[i] = make_float4(p[0], p[1], p[2], 0.0f);
    } else {
        constexpr int NV = rec_vecs(D);
        float w[NV * 4];
#pragma unroll
        for (int c = 0; c < NV * 4; ++c) w[c] = 0.0f;
#pragma unroll
        for (int c = 0; c < D; ++c) w[c] = p[c];
        w[D] = __int_as_float((int32_t)i);
        float4* out = reinterpret_cast<float4*>(rec) + (int64_t)pos * NV;
#pragma unroll
        for (int v = 0; v < NV; ++v) out[v] = make_float4(w[4 * v], w[4 * v + 1], w[4 * v + 2], w[4 * v + 3]);
    }
}

template <int DB>
static void launch_bbox_assign(bool assign, const float* coords, const int32_t* row_splits, int32_t n, int32_t d,
                               int32_t n_segments, int32_t n_bins, int32_t sub_shift, int32_t cells_per_segment,
                               int32_t morton_bits, uint32_t* bbox_keys,
                               float* geom, int32_t* bin_idx, int32_t* rank, int32_t* counters,
                               hipStream_t stream)
{
    if (!assign)
        hipLaunchKernelGGL(k_bbox<DB>, dim3((unsigned)(((int64_t)n + kBboxChunk - 1) / kBboxChunk)), dim3(kBlock), 0, stream, coords,
                           row_splits, n, d, n_segments, bbox_keys);
    else
        hipLaunchKernelGGL(k_assign<DB>, dim3((unsigned)(((int64_t)n + kAssignChunk - 1) / kAssignChunk)), dim3(kBlock), 0, stream, coords,
                           row_splits, n, d, n_segments, n_bins, sub_shift, cells_per_segment, morton_bits, bbox_keys, geom,
                           bin_idx, rank, counters);
}

template <int D>
static void launch_scatter(bool rows_only, const float* coords, int32_t n, const int32_t* bin_idx, const int32_t* rank,
                           const int32_t* bounds, int32_t* perm, float* rec, hipStream_t stream)
{
    const unsigned grid = (unsigned)(((int64_t)n + kBlock - 1) / kBlock);
    if (rows_only)
        hipLaunchKernelGGL((k_scatter<D, true>), dim3(grid), dim3(kBlock), 0, stream, coords, n, bin_idx, rank, bounds,
                           perm, rec);
    else
        hipLaunchKernelGGL((k_scatter<D, false>), dim3(grid), dim3(kBlock), 0, stream, coords, n, bin_idx, rank, bounds,
                           perm, rec);
}

hipError_t launch_binning(const float* coords, const int32_t* row_splits, int32_t n, int32_t d,
                          int32_t n_segments, int32_t n_bins, int32_t d_bin, int32_t sub_shift, int64_t total_bins,
                          uint32_t* bbox_keys, float* geom, int32_t* bin_idx, int32_t* rank,
                          int32_t* perm, float* rec, int32_t* bounds,
                          int32_t* scan_partials, int32_t morton_bits, hipStream_t stream)
{
    const int64_t n_counters = total_bins + 1;
    const int32_t n_keys = n_segments * d_bin;
    const int32_t cells_per_segment = (int32_t)(total_bins / n_segments);
    {
        int64_t work = n_counters > 2 * (int64_t)n_keys ? n_counters : 2 * (int64_t)n_keys;
        int64_t grid = (work + kBlock - 1) / kBlock;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(k_prepare, dim3((unsigned)grid), dim3(kBlock), 0, stream, bounds, n_counters, bbox_keys,
                           n_keys);
    }
#define FG_DB_SWITCH(ASSIGN)                                                                                       \
    switch (d_bin) {                                                                                               \
        case 2: launch_bbox_assign<2>(ASSIGN, coords, row_splits, n, d, n_segments, n_bins, sub_shift, cells_per_segment, \
                                      morton_bits, bbox_keys, geom, bin_idx, rank, bounds, stream); break;                      \
        case 3: launch_bbox_assign<3>(ASSIGN, coords, row_splits, n, d, n_segments, n_bins, sub_shift, cells_per_segment, \
                                      morton_bits, bbox_keys, geom, bin_idx, rank, bounds, stream); break;                      \
        case 4: launch_bbox_assign<4>(ASSIGN, coords, row_splits, n, d, n_segments, n_bins, sub_shift, cells_per_segment, \
                                      morton_bits, bbox_keys, geom, bin_idx, rank, bounds, stream); break;                      \
        case 5: launch_bbox_assign<5>(ASSIGN, coords, row_splits, n, d, n_segments, n_bins, sub_shift, cells_per_segment, \
                                      morton_bits, bbox_keys, geom, bin_idx, rank, bounds, stream); break;                      \
        default: return hipErrorInvalidValue;                                                                      \
    }
    FG_DB_SWITCH(false)
    FG_DB_SWITCH(true)
#undef FG_DB_SWITCH
    {
        int64_t n_chunks = (n_counters + kScanChunk - 1) / kScanChunk;
        hipLaunchKernelGGL(k_scan_partials, dim3((unsigned)n_chunks), dim3(kBlock), 0, stream, bounds, n_counters,
                           scan_partials);
        if (n_chunks <= 2048) {
            hipLaunchKernelGGL(k_scan_apply<true>, dim3((unsigned)n_chunks), dim3(kBlock), 0, stream, bounds, n_counters,
                               scan_partials);
        } else {
            hipLaunchKernelGGL(k_scan_tops, dim3(1), dim3(kBlock), 0, stream, scan_partials, (int32_t)n_chunks);
            hipLaunchKernelGGL(k_scan_apply<false>, dim3((unsigned)n_chunks), dim3(kBlock), 0, stream, bounds, n_counters,
                               scan_partials);
        }
    }
    switch (d) {
        case 2: launch_scatter<2>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 3: launch_scatter<3>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 4: launch_scatter<4>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 5: launch_scatter<5>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 6: launch_scatter<6>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 7: launch_scatter<7>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 8: launch_scatter<8>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 9: launch_scatter<9>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        case 10: launch_scatter<10>(morton_bits > 0, coords, n, bin_idx, rank, bounds, perm, rec, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace fg
