// Per-lane geometry shared by all query kernels, and the general shell-expanding walk with one
// lane per query (any shell radius).  The walk is the cross-check path (fg_query_options::algo = 1); the fast path is
// the tile kernel plus the one-query-per-wavefront list kernel.
//
// What it computes (paper Section 3, Algorithm 2): for every point, the K-1 nearest other
// points of its row split, found by scanning the bins on the surface of the hypercube of
// Chebyshev radius r = 0, 1, 2, ... around the query's bin (Algorithm 1) until the k-th best
// squared distance is certified smaller than anything unsearched.  Differences from the
// paper's kernel, none of which changes what "exact" means:
//   * the running best list is a max-heap of 64-bit keys (distance bits << 32 | original index)
//     in LDS, one column per lane, instead of an unsorted buffer with a linear max rescan; the
//     key order is the strict total order (d2, index), so the result does not depend on the
//     order candidates arrive in;
//   * the last binning dimension is walked as contiguous runs of bins (bins adjacent in the
//     last dimension are adjacent in the sorted point order);
//   * bins whose box lies farther than the current k-th best are skipped (a lower bound on the
//     distance to any point of the bin, per dimension, with rounding slack);
//   * the stop test uses the true distance from the query to the faces of the searched cube
//     instead of r times the first bin width, and stops at once when the cube covers the grid.
#pragma once
#include "fg_internal.hpp"

namespace fg {

constexpr int kQueryBlock = 64;                    // one wavefront per workgroup
constexpr int kStageChunk = 256;                   // most points staged through LDS per chunk (tile kernel)
constexpr float kBoundShrink = 0.99999618530273f;  // 1 - 2^-18: covers fp32 rounding of d2 and of the bound

// Per-lane geometry of one query: its coordinates, its bin, its row split's grid, and the
// current k-th best key `tau` (at or above kEmptyKey until K-1 candidates have been kept).
template <int D, int DB>
struct LaneGeom {
    float x[D];
    float glo[DB], gw[DB], gslack[DB];
    int32_t cc[DB], neff[DB];
    int32_t n_bins, seg_cell0;
    // The last binning dimension is cut finer than the others: every bin into 2^sub_shift slices, which are what
    // the counting sort orders by and what the bin boundaries count.  Shells, gaps and the stop test work in
    // whole bins (cc, neff; bin j starts at slice j << sub_shift); glo/gw/gslack of that dimension describe the
    // slices, slice_inv_w is slices per unit length and my_slice the query's own slice.
    int32_t sub_shift;
    float slice_inv_w;
    uint64_t tau;

    // lower edge of bin j in dimension c
    __device__ __forceinline__ float edge(int c, int32_t j) const
    {
        return glo[c] + (float)(c == DB - 1 ? j << sub_shift : j) * gw[c];
    }
    // first entry of the bin boundaries for bin z of the last dimension in the column of bins `col` (flat over
    // the first DB-1 dimensions)
    __device__ __forceinline__ int32_t bounds_at(int32_t col, int32_t z) const
    {
        return seg_cell0 + ((col * n_bins + z) << sub_shift);
    }

    __device__ __forceinline__ float tau_d2() const { return __uint_as_float((uint32_t)(tau >> 32)); }

    // true when no point of a box at squared lower-bound distance b2 can enter the best list
    __device__ __forceinline__ bool cannot_improve(float b2) const
    {
        return tau < kEmptyKey && b2 > 1e-30f && tau_d2() < b2 * kBoundShrink;
    }

    // lower bound (>= 0) on |x_c - y_c| for any point y whose bin index in dimension c is j = cc[c] + o
    __device__ __forceinline__ float gap(int c, int32_t j, int32_t o) const
    {
        if (o == 0) return 0.0f;
        float g = (o > 0) ? edge(c, j) - x[c] : x[c] - edge(c, j + 1);
        g -= gslack[c];
        return g > 0.0f ? g : 0.0f;
    }

    // The slices [lo_s, hi_s] of the last binning dimension that can still hold a point entering the best list,
    // for a column of bins whose squared lower-bound distance in the other binning dimensions is `partial`.
    // The ends are guessed from the radius the k-th best leaves in this dimension and then checked with the same
    // bound that prunes whole bins (slices below lo_s lie under the lower edge of slice lo_s, farther than the
    // gap to that edge); a guess that fails the check moves out by one slice, then gives way to the full range.
    __device__ __forceinline__ void slice_reach(float partial, int32_t& lo_s, int32_t& hi_s) const
    {
        constexpr int c = DB - 1;
        const int32_t n_slices = n_bins << sub_shift;
        lo_s = 0;
        hi_s = n_slices - 1;
        if (tau >= kEmptyKey) return;
        const float left = tau_d2() - partial;
        const float r = sqrtf(left > 0.0f ? left : 0.0f);
        auto below_out = [&](int32_t j) {       // true: no slice under j can improve the list
            const float g = x[c] - (glo[c] + (float)j * gw[c]) - gslack[c];
            return g > 0.0f && cannot_improve(partial + g * g);
        };
        auto above_out = [&](int32_t j) {       // true: no slice over j can improve the list
            const float g = (glo[c] + (float)(j + 1) * gw[c]) - x[c] - gslack[c];
            return g > 0.0f && cannot_improve(partial + g * g);
        };
        int32_t jl = cell_of(x[c] - r, glo[c], slice_inv_w, n_slices);
        if (jl > 0 && !below_out(jl)) {
            --jl;
            if (jl > 0 && !below_out(jl)) jl = 0;
        }
        int32_t jh = cell_of(x[c] + r, glo[c], slice_inv_w, n_slices);
        if (jh < n_slices - 1 && !above_out(jh)) {
            ++jh;
            if (jh < n_slices - 1 && !above_out(jh)) jh = n_slices - 1;
        }
        lo_s = jl;
        hi_s = jh;
    }

    // after shell r: true when the search may stop
    __device__ __forceinline__ bool certified(int32_t r) const
    {
        bool covered = true;
        float mingap = 3.0e38f;
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            int32_t jl = cc[c] - r, jh = cc[c] + r;
            if (jl > 0) {
                covered = false;
                float g = x[c] - edge(c, jl) - gslack[c];
                mingap = fminf(mingap, g > 0.0f ? g : 0.0f);
            }
            if (jh < neff[c] - 1) {
                covered = false;
                float g = edge(c, jh + 1) - x[c] - gslack[c];
                mingap = fminf(mingap, g > 0.0f ? g : 0.0f);
            }
        }
        if (covered) return true;
        return cannot_improve(mingap * mingap);
    }

    // p: sorted position of the query; returns its original row
    __device__ __forceinline__ int32_t init_geom(const QueryArgs& a, int32_t p)
    {
        n_bins = a.n_bins;
        sub_shift = a.sub_shift;
        tau = kEmptyKey;
        const int32_t seg = segment_of(a.row_splits, a.n_segments, p);
        seg_cell0 = seg * a.cells_per_segment;
        int32_t row;
        load_rec<D>(a.rec, p, x, row);
        const float* g = a.geom + (int64_t)seg * DB * kGeomStride;
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            const float inv_w = g[c * kGeomStride + 1];
            glo[c] = g[c * kGeomStride + 0];
            gw[c] = g[c * kGeomStride + 2];
            gslack[c] = g[c * kGeomStride + 3];
            if (c == DB - 1) {
                cc[c] = cell_of(x[c], glo[c], inv_w, a.n_bins << a.sub_shift) >> a.sub_shift;
                slice_inv_w = inv_w;
            } else {
                cc[c] = cell_of(x[c], glo[c], inv_w, a.n_bins);
            }
            neff[c] = inv_w > 0.0f ? a.n_bins : 1;
        }
        return row;
    }
};

template <int D, int DB, bool COUNT>
struct ShellSearch : LaneGeom<D, DB> {
    using G = LaneGeom<D, DB>;
    using G::x; using G::glo; using G::gw; using G::gslack; using G::cc; using G::neff;
    using G::n_bins; using G::seg_cell0; using G::tau; using G::bounds_at;
    using G::cannot_improve; using G::gap; using G::certified;
    uint64_t* heap;   // this lane's column: slot j lives at heap[j * kQueryBlock]
    const float4* __restrict__ rec;
    const int32_t* __restrict__ bounds;
    const int32_t* __restrict__ dir;
    int32_t self_pos, self_row, cap, filled, cand;

    __device__ __forceinline__ void sift_down(uint64_t key, int32_t size)
    {
        int32_t i = 0;
        for (;;) {
            int32_t l = 2 * i + 1;
            if (l >= size) break;
            uint64_t bk = heap[l * kQueryBlock];
            int32_t big = l;
            if (l + 1 < size) {
                uint64_t rk = heap[(l + 1) * kQueryBlock];
                if (rk > bk) { bk = rk; big = l + 1; }
            }
            if (bk <= key) break;
            heap[i * kQueryBlock] = bk;
            i = big;
        }
        heap[i * kQueryBlock] = key;
    }

    __device__ __forceinline__ void offer(uint64_t key)
    {
        if (filled < cap) {
            int32_t i = filled++;
            while (i > 0) {
                int32_t parent = (i - 1) >> 1;
                uint64_t pk = heap[parent * kQueryBlock];
                if (pk >= key) break;
                heap[i * kQueryBlock] = pk;
                i = parent;
            }
            heap[i * kQueryBlock] = key;
            if (filled == cap) tau = heap[0];
        } else if (key < tau) {
            sift_down(key, cap);
            tau = heap[0];
        }
    }

    // all points at sorted positions [a, b)
    __device__ __forceinline__ void scan_points(int32_t a, int32_t b)
    {
        for (int32_t q = a; q < b; ++q) {
            if (q == self_pos) continue;
            float y[D];
            int32_t row;
            load_rec<D>(rec, q, y, row);
            float diff = x[0] - y[0];
            float d2 = diff * diff;
#pragma unroll
            for (int c = 1; c < D; ++c) {
                diff = x[c] - y[c];
                d2 = d2 + diff * diff;
            }
            if (COUNT) ++cand;
            uint32_t bits = __float_as_uint(d2);
            if (bits > (uint32_t)(tau >> 32)) continue;
            if (dir && !dir_is_neighbour(dir[row])) continue;
            uint64_t key = ((uint64_t)bits << 32) | (uint32_t)row;
            offer(key);
        }
    }

    template <int LVL>
    __device__ __forceinline__ void visit(int32_t r, int32_t flat, float partial, bool surf)
    {
        const int32_t c0 = cc[LVL];
        if constexpr (LVL < DB - 1) {
            int32_t o_lo = -r < -c0 ? -c0 : -r;
            int32_t o_hi = r > neff[LVL] - 1 - c0 ? neff[LVL] - 1 - c0 : r;
            for (int32_t o = o_lo; o <= o_hi; ++o) {
                float g = gap(LVL, c0 + o, o);
                float p2 = partial + g * g;
                if (cannot_improve(p2)) continue;
                bool on = surf || o == r || o == -r;
                visit<LVL + 1>(r, flat * n_bins + c0 + o, p2, on);
            }
        } else {
            if (surf) {   // the whole run of the last dimension belongs to this shell
                int32_t za = c0 - r < 0 ? 0 : c0 - r;
                int32_t zb = c0 + r > neff[LVL] - 1 ? neff[LVL] - 1 : c0 + r;
                scan_points(bounds[bounds_at(flat, za)], bounds[bounds_at(flat, zb + 1)]);
            } else {      // only the two end bins of the run are on the surface
                if (c0 - r >= 0) {
                    float g = gap(LVL, c0 - r, -r);
                    if (!cannot_improve(partial + g * g)) scan_points(bounds[bounds_at(flat, c0 - r)], bounds[bounds_at(flat, c0 - r + 1)]);
                }
                if (c0 + r <= neff[LVL] - 1) {
                    float g = gap(LVL, c0 + r, r);
                    if (!cannot_improve(partial + g * g)) scan_points(bounds[bounds_at(flat, c0 + r)], bounds[bounds_at(flat, c0 + r + 1)]);
                }
            }
        }
    }

    __device__ __forceinline__ void run()
    {
        if (cap <= 0) return;
        for (int32_t r = 0;; ++r) {      // ends at the latest when the cube covers the grid (r = n_bins - 1)
            visit<0>(r, 0, 0.0f, r == 0);
            if (certified(r)) break;
        }
    }

    // heap -> ascending order in place
    __device__ __forceinline__ void sort_ascending()
    {
        for (int32_t m = filled - 1; m > 0; --m) {
            uint64_t top = heap[0];
            uint64_t last = heap[m * kQueryBlock];
            heap[m * kQueryBlock] = top;
            sift_down(last, m);
        }
    }
};

// ---- per-lane set-up and output, shared by both kernels ------------------------------------

template <int D, int DB, bool COUNT>
__device__ __forceinline__ void init_lane(ShellSearch<D, DB, COUNT>& s, const QueryArgs& a, int32_t p, uint64_t* heap)
{
    s.heap = heap;
    s.rec = a.rec; s.bounds = a.bounds; s.dir = a.dir;
    s.self_pos = p; s.cap = a.k - 1; s.filled = 0; s.cand = 0;
    s.self_row = s.init_geom(a, p);
}

// sort the lane's best list and write its output row (original row order)
template <int D, int DB, bool COUNT>
__device__ __forceinline__ void write_row(ShellSearch<D, DB, COUNT>& s, const QueryArgs& a, int32_t p, bool add_count)
{
    s.sort_ascending();
    const int32_t row = s.self_row;
    int32_t* oi = a.out_idx + (int64_t)row * a.k;
    float* od = a.out_d2 + (int64_t)row * a.k;
    oi[0] = (a.dir && !dir_is_query(a.dir[row])) ? -1 : row;    // a point that asks nothing gets an all-padding row
    od[0] = 0.0f;
    for (int32_t j = 0; j < s.cap; ++j) {
        if (j < s.filled) {
            uint64_t key = s.heap[j * kQueryBlock];
            oi[j + 1] = (int32_t)(uint32_t)key;
            od[j + 1] = __uint_as_float((uint32_t)(key >> 32));
        } else {
            oi[j + 1] = -1;
            od[j + 1] = 0.0f;
        }
    }
    if (COUNT) a.out_cand[row] = (add_count ? a.out_cand[row] : 0) + s.cand;
}

// Wave-wide min / max of one int per lane with DPP row shifts and row broadcasts (6 VALU
// operations and one readlane each); the result is uniform.
__device__ __forceinline__ int32_t wave_min_i32(int32_t v)
{
    const int32_t id = 0x7fffffff;
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x142, 0xa, 0xf, false));   // row_bcast:15 into rows 1 and 3
    v = min(v, __builtin_amdgcn_update_dpp(id, v, 0x143, 0xc, 0xf, false));   // row_bcast:31 into rows 2 and 3
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int32_t wave_sum_i32(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return __builtin_amdgcn_readlane(v, 63);
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int32_t wave_incl_scan_dpp_i32(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return v;
}
__device__ __forceinline__ int32_t wave_max_i32(int32_t v)
{
    const int32_t id = (int32_t)0x80000000;
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x111, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x112, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x114, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x118, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x142, 0xa, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(id, v, 0x143, 0xc, 0xf, false));
    return __builtin_amdgcn_readlane(v, 63);
}

// all queries through the one-lane-per-query walk (no tiles, no work list)
template <int D, int DB, bool COUNT>
__global__ void __launch_bounds__(kQueryBlock)
k_query_shell(QueryArgs a)
{
    extern __shared__ uint64_t lds64[];
    const int32_t p = blockIdx.x * kQueryBlock + threadIdx.x;
    if (p >= a.n) return;
    ShellSearch<D, DB, COUNT> s;
    init_lane(s, a, p, lds64 + threadIdx.x);
    if (!(a.dir && !dir_is_query(a.dir[s.self_row]))) s.run();
    write_row(s, a, p, false);
}

}  // namespace fg
