// Internal declarations shared by the translation units of libfastgraph_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fastgraph.h"

namespace fg {

constexpr int kGeomStride = 4;   // floats per (segment, binning dim): lo, inv_w, w, slack
constexpr int kKeyStride = 16;   // words between two bounding-box keys: one 64-byte line each, so that the
                                 // atomics on different keys do not queue up behind one another in one L2 line

// Everything the query stage needs; plain device pointers.
struct QueryArgs {
    const float4* rec;         // [n][rec_vecs(d)] bin-ordered point records: coordinates, original row, padding
    const int32_t* bounds;     // [S*T+1], T counted in slices (see sub_shift)
    const float* geom;         // [S][d_bin][4]
    const int32_t* row_splits; // [S+1]
    const int32_t* dir;        // [n] direction flags in ORIGINAL row order, or nullptr
    int32_t* out_idx;          // [n][k]
    float* out_d2;             // [n][k]
    int32_t* out_cand;         // [n] or nullptr
    int32_t* work_list;        // [n] sorted positions of queries deferred by the tile kernel, in bin order
    int32_t* work_count;       // [1]
    uint64_t* handed;          // [ceil(n/64)] per tile: which of its 64 queries the tile kernel hands over
    const int32_t* bin_idx;    // [n] flat bin of each point, original row order
    int32_t* tile_order;       // [2*ceil(n/64) + 128]: tile order, tile classes, class histogram, class cursors
    int32_t n;
    int32_t d;                 // coordinates per point (the record length follows from it)
    int32_t n_segments;
    int32_t k;                 // slots per output row
    int32_t slot0;             // tile + list kernels: neighbours already placed by an earlier pass (0 or 64); this pass keeps only keys above the one in row slot `slot0`
    int32_t k_list;            // tile + list kernels: neighbours this pass finds (1..64, or 0 for K = 1); they go to row slots slot0+1 .. slot0+k_list
    int32_t n_bins;
    int32_t cells_per_segment; // T: bins of a row split times the slices per bin
    int32_t sub_shift;         // log2 of the slices every bin is cut into along the last binning dimension
    int32_t algo;              // 0: tile kernel + list kernel, 1: one lane per query for everything, 2: as 0 with the flattened scan on every tile
    int32_t defer_lanes;       // tile kernel: go on past shell 1 only while more lanes than this are unfinished
};

// Host-side launchers, one per translation unit.  Each returns hipGetLastError() of its launches.
hipError_t launch_binning(const float* coords, const int32_t* row_splits, int32_t n, int32_t d,
                          int32_t n_segments, int32_t n_bins, int32_t d_bin, int32_t sub_shift /* last binning dimension:
                          n_bins << sub_shift slices */, int64_t total_bins,
                          uint32_t* bbox_keys, float* geom, int32_t* bin_idx, int32_t* rank,
                          int32_t* perm, float* rec, int32_t* bounds,
                          int32_t* scan_partials,
                          int32_t morton_bits /* 0: row-major bins, the bin-ordered point records written to rec (perm unused);
                                                 b > 0 (the backward's row order): n_bins = 2^b, bit-interleaved bin order,
                                                 only perm is written, plus for d = 3 a copy of coords in the original
                                                 order padded to float4 in place of the records */,
                          hipStream_t stream);

// d = 2..10, d_bin = 2..min(d,5)
hipError_t launch_query(const QueryArgs& a, int32_t d, int32_t d_bin, hipStream_t stream);

// perm != nullptr: rows are taken in bin order (row of sorted position q = perm[q * perm_stride]: 1 for a plain
// permutation, the record length in words for the index field of the forward's point records) and combined in
// LDS; nullptr: plain atomic scatter.
// coords4 (d = 3 with perm only, else nullptr): coords padded to four floats per row.
hipError_t launch_backward(const float* grad_d2, const int32_t* idx, const float* coords, const float* coords4,
                           const int32_t* perm, int32_t perm_stride, int32_t n, int32_t d, int32_t k, float* grad_coords,
                           hipStream_t stream);

hipError_t launch_oc_helper(const int32_t* asso_idx, const int32_t* unique_idx, const int32_t* unique_rs_asso,
                            const int32_t* rs, int32_t n_vert, int32_t n_unique, int32_t n_splits, int32_t n_maxuq,
                            int32_t n_maxrs, int32_t calc_m_not, int32_t rot_block, int32_t* M, int32_t* M_not,
                            int32_t* counts /* workspace of oc_workspace_bytes(), or nullptr */, hipStream_t stream);
size_t oc_workspace_bytes(int64_t n_unique, int32_t n_maxrs);

// A bin-ordered point record: the d coordinates, then the original row index (its bits in a float), then zero
// padding up to a whole number of 16-byte vectors.  One scattered store per vector in the counting sort, one load
// per vector wherever a candidate is fetched.
constexpr int rec_vecs(int d) { return (d + 1 + 3) / 4; }
template <int D>
__device__ __forceinline__ void load_rec(const float4* __restrict__ rec, int64_t q, float (&x)[D], int32_t& row)
{
    constexpr int NV = rec_vecs(D);
    float w[NV * 4];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const float4 f = rec[q * NV + v];
        w[4 * v] = f.x; w[4 * v + 1] = f.y; w[4 * v + 2] = f.z; w[4 * v + 3] = f.w;
    }
#pragma unroll
    for (int c = 0; c < D; ++c) x[c] = w[c];
    row = __float_as_int(w[D]);
}
template <int D>
__device__ __forceinline__ int32_t rec_row(const float4* __restrict__ rec, int64_t q)
{
    return __float_as_int(reinterpret_cast<const float*>(rec)[q * (rec_vecs(D) * 4) + D]);
}

// Direction flags (paper Algorithm 2, useDir / dir[]): 0 or 2 = issues no query, 1 or 2 = is nobody's
// neighbour, anything else = both roles.
__device__ __forceinline__ bool dir_is_query(int32_t f) { return f != 0 && f != 2; }
__device__ __forceinline__ bool dir_is_neighbour(int32_t f) { return f != 1 && f != 2; }

// Key of an empty best-list slot: just above the bit pattern of +infinity, so every real key
// (finite or infinite squared distance) is below it and every NaN squared distance is not.
// Candidates excluded by a direction flag are staged with NaN coordinates and so can never be kept.
constexpr uint64_t kEmptyKey = 0x7f800001ull << 32;

// Segment of a (sorted or original) position: largest s with row_splits[s] <= p, skipping empty
// segments by construction (row_splits[s+1] > p).
__device__ __forceinline__ int32_t segment_of(const int32_t* __restrict__ row_splits,
                                              int32_t n_segments, int32_t p)
{
    int32_t lo = 0, hi = n_segments;   // invariant: row_splits[lo] <= p < row_splits[hi]
    while (hi - lo > 1) {
        int32_t mid = (lo + hi) >> 1;
        if (row_splits[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// Bin index of coordinate x in one dimension.  Monotone non-decreasing in x, which is what the
// search's lower bounds rely on.
__device__ __forceinline__ int32_t cell_of(float x, float lo, float inv_w, int32_t n_bins)
{
    float t = (x - lo) * inv_w;
    int32_t c = (int32_t)floorf(t);
    c = c < 0 ? 0 : c;
    return c > n_bins - 1 ? n_bins - 1 : c;
}

}  // namespace fg
