// List kernel: the queries the tile kernel hands over (isolated points, sparse regions) are
// searched ONE QUERY PER WAVEFRONT.
//
// Same algorithm as everywhere (paper Section 3, Algorithm 2: shells of growing radius, exact
// best K-1, certified stop), but the parallelism is across the shell instead of across queries:
//   * the column offsets of a shell (offsets in the first DB-1 binning dimensions) are spread
//     over the lanes, 64 at a time: one round trip fetches the bin boundaries of 64 columns;
//   * the candidates of those columns are flattened with a wave prefix sum and evaluated 64 per
//     pass, one per lane, straight from the bin-ordered coordinates (runs of consecutive
//     points, so the loads coalesce);
//   * candidates that beat the current k-th best are compacted (ballot + popcount) into a
//     pending array in LDS; 64 pending keys at a time are sorted across the lanes with a
//     shuffle-based bitonic network and merged into the best list, which lives one key per lane,
//     ascending by lane;
//   * the output row is written by the lanes that hold it: one contiguous store per row.
// A far-searching query therefore costs a few memory round trips per shell, not one per bin.
// The tile kernel has already searched the first shells of every query it hands over: its list so
// far sits in the query's output row and the first unsearched shell in slot 0 of the distance row,
// so the search resumes there with a k-th best that already prunes most of the new shell.
// A pass finds at most 64 neighbours; longer lists take two passes (see the launch code).
#pragma once
#include "fg_query.hpp"
#include "fg_sortnet.hpp"

namespace fg {

__device__ __forceinline__ uint64_t wave_sort_step(uint64_t v, int lane, int k, int j)
{
    const uint64_t other = __shfl_xor(v, j, 64);
    const bool keep_min = ((lane & k) == 0) == ((lane & j) == 0);
    return keep_min ? key_min(v, other) : key_max(v, other);
}

// ascending (by lane) bitonic sort of one key per lane
__device__ __forceinline__ uint64_t wave_sort64(uint64_t v, int lane)
{
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) v = wave_sort_step(v, lane, k, j);
    return v;
}

// keys form a bitonic sequence over the lanes -> ascending
__device__ __forceinline__ uint64_t wave_merge64(uint64_t v, int lane)
{
#pragma unroll
    for (int j = 32; j > 0; j >>= 1) v = wave_sort_step(v, lane, 64, j);
    return v;
}

constexpr int kListPend = 128;
constexpr int kListDirect = 12;   // accepted keys of one pass that are inserted one by one instead of sorted

// the key of the last lane, in every lane
__device__ __forceinline__ uint64_t wave_last_key(uint64_t v)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), kQueryBlock - 1) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, kQueryBlock - 1);
}

// value of the lane below (lane 0: zero), 64-bit: a wavefront shift by one lane, no trip through the LDS crossbar
__device__ __forceinline__ uint64_t wave_from_below(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, 0x138, 0xf, 0xf, false);          // wave_shr:1
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), 0x138, 0xf, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}

template <int D, int DB, bool COUNT>
__global__ void __launch_bounds__(kQueryBlock)
k_query_list_wave(QueryArgs a)
{
    __shared__ uint64_t pend[kListPend];
    __shared__ int32_t seg_excl[kQueryBlock], seg_a1[kQueryBlock], seg_len1[kQueryBlock], seg_a2[kQueryBlock];
    const int lane = threadIdx.x;
    const int32_t count = *a.work_count;
    const int32_t cap = a.k_list;                   // 1 <= cap <= 64
    const uint64_t lt_mask = (1ull << lane) - 1;

    for (int32_t item = blockIdx.x; item < count; item += gridDim.x) {
        const int32_t p = a.work_list[item];
        LaneGeom<D, DB> s;                          // identical in every lane
        const int32_t row = s.init_geom(a, p);
        int32_t* oi = a.out_idx + (int64_t)row * a.k;
        float* od = a.out_d2 + (int64_t)row * a.k;
        uint64_t best = 0ull;                       // ascending by lane; low lanes pinned
        if (lane >= kQueryBlock - cap) {
            const int32_t j = a.slot0 + lane - (kQueryBlock - cap) + 1;
            const int32_t bi = oi[j];
            best = bi < 0 ? kEmptyKey : (((uint64_t)__float_as_uint(od[j]) << 32) | (uint32_t)bi);
        }
        // second pass of a long list: only keys above the last one the first pass placed count
        uint64_t lower = 0;
        if (a.slot0 > 0) {
            const int32_t li = oi[a.slot0];
            lower = li < 0 ? kEmptyKey : (((uint64_t)__float_as_uint(od[a.slot0]) << 32) | (uint32_t)li);
        }
        const int32_t R0 = __float_as_int(od[0]);
        s.tau = wave_last_key(best);
        int32_t npend = 0, cand = 0;

        auto absorb64 = [&]() {                     // merges pend[0..min(npend,64)) into the best list
            const int32_t take = npend < kQueryBlock ? npend : kQueryBlock;
            uint64_t v = lane < take ? pend[lane] : kEmptyKey;
            uint64_t rest = (lane + kQueryBlock < npend) ? pend[lane + kQueryBlock] : 0ull;
            __syncthreads();
            if (lane + kQueryBlock < npend) pend[lane] = rest;
            npend -= take;
            v = wave_sort64(v, lane);
            const uint64_t rv = __shfl(v, kQueryBlock - 1 - lane, 64);
            best = key_min(rv, best);
            best = wave_merge64(best, lane);
            s.tau = wave_last_key(best);
            __syncthreads();
        };

        for (int32_t R = R0;; ++R) {   // ends at the latest when the cube covers the grid
            const int32_t side = 2 * R + 1;
            int32_t ncols = 1;
#pragma unroll
            for (int c = 0; c < DB - 1; ++c) ncols *= side;
            for (int32_t t0 = 0; t0 < ncols; t0 += kQueryBlock) {
                // this lane's column
                const int32_t t = t0 + lane;
                bool ok = t < ncols;
                bool surf = false;
                float partial = 0.0f;
                int32_t flat = 0;
                {
                    int32_t o[DB - 1];
                    int32_t rem = ok ? t : 0;
                    // digits of the column number in base `side`; up to 2^16 columns the quotient comes from a float
                    // reciprocal (the true quotient of rem + 1/2 lies at least 1/(2 side) from an integer, the
                    // product errs by less than a hundredth: exact), which saves two integer divisions per lane
                    const bool small = ncols <= 65536;
                    const float inv_side = 1.0f / (float)side;
#pragma unroll
                    for (int c = DB - 2; c >= 0; --c) {
                        const int32_t quo = small ? (int32_t)(((float)rem + 0.5f) * inv_side) : rem / side;
                        const int32_t v = rem - quo * side;
                        rem = quo;
                        o[c] = (v & 1) ? ((v + 1) >> 1) : -(v >> 1);
                        surf = surf || o[c] == R || o[c] == -R;
                    }
#pragma unroll
                    for (int c = 0; c < DB - 1; ++c) {
                        const int32_t j = s.cc[c] + o[c];
                        ok = ok && j >= 0 && j < s.neff[c];
                        const float g = s.gap(c, j, o[c]);
                        partial += g * g;
                        flat = flat * a.n_bins + j;
                    }
                }
                ok = ok && !s.cannot_improve(partial);
                int32_t a1 = 0, b1 = 0, a2 = 0, b2 = 0;
                if (ok) {
                    const int32_t cz = s.cc[DB - 1], nz = s.neff[DB - 1];
                    // every run ends at the slice of its bins that the k-th best still reaches
                    const int32_t sh = a.sub_shift;
                    const int32_t row0 = s.bounds_at(flat, 0);
                    int32_t s_lo = 0, s_hi = 0x7ffffffe;
                    if (sh > 0) s.slice_reach(partial, s_lo, s_hi);
                    auto cut_run = [&](int32_t z_first, int32_t z_last, int32_t& from, int32_t& to) {   // bins, inclusive
                        const int32_t fa = (z_first << sh) > s_lo ? (z_first << sh) : s_lo;
                        const int32_t fb = ((z_last + 1) << sh) < s_hi + 1 ? ((z_last + 1) << sh) : s_hi + 1;
                        if (fb > fa) { from = a.bounds[row0 + fa]; to = a.bounds[row0 + fb]; }
                    };
                    if (surf) {
                        int32_t za = cz - R < 0 ? 0 : cz - R;
                        int32_t zb = cz + R > nz - 1 ? nz - 1 : cz + R;
                        while (za < cz) {      // drop end bins of the run whose box is already too far
                            const float g = s.gap(DB - 1, za, za - cz);
                            if (!s.cannot_improve(partial + g * g)) break;
                            ++za;
                        }
                        while (zb > cz) {
                            const float g = s.gap(DB - 1, zb, zb - cz);
                            if (!s.cannot_improve(partial + g * g)) break;
                            --zb;
                        }
                        cut_run(za, zb, a1, b1);
                    } else {
                        if (cz - R >= 0) {
                            const float g = s.gap(DB - 1, cz - R, -R);
                            if (!s.cannot_improve(partial + g * g)) cut_run(cz - R, cz - R, a1, b1);
                        }
                        if (cz + R <= nz - 1) {
                            const float g = s.gap(DB - 1, cz + R, R);
                            if (!s.cannot_improve(partial + g * g)) cut_run(cz + R, cz + R, a2, b2);
                        }
                    }
                }
                const int32_t len1 = b1 - a1, len = len1 + (b2 - a2);
                const int32_t incl = wave_incl_scan_dpp_i32(len);
                const int32_t W = __builtin_amdgcn_readlane(incl, kQueryBlock - 1);
                __syncthreads();
                seg_excl[lane] = incl - len; seg_a1[lane] = a1; seg_len1[lane] = len1; seg_a2[lane] = a2;
                __syncthreads();
                for (int32_t f0 = 0; f0 < W; f0 += kQueryBlock) {
                    const int32_t f = f0 + lane;
                    const bool in = f < W;
                    // segment of candidate f: the largest j with seg_excl[j] <= f
                    int32_t j = 0;
#pragma unroll
                    for (int step = 32; step > 0; step >>= 1)
                        if (seg_excl[j + step] <= f) j += step;
                    const int32_t local = f - seg_excl[j];
                    const int32_t l1 = seg_len1[j];
                    int32_t q = local < l1 ? seg_a1[j] + local : seg_a2[j] + (local - l1);
                    q = in ? q : p;
                    float y[D];
                    int32_t src;
                    load_rec<D>(a.rec, q, y, src);
                    float diff = s.x[0] - y[0];
                    float d2 = diff * diff;
#pragma unroll
                    for (int c = 1; c < D; ++c) {
                        diff = s.x[c] - y[c];
                        d2 = d2 + diff * diff;
                    }
                    const bool live = in && q != p && !(a.dir && !dir_is_neighbour(a.dir[src]));
                    const uint64_t key = ((uint64_t)__float_as_uint(d2) << 32) | (uint32_t)src;
                    const bool acc = live && key < s.tau && (a.slot0 == 0 || key > lower);
                    if (COUNT) cand += __popcll(__ballot(live));
                    const uint64_t m = __ballot(acc);
                    if (m && __popcll(m) <= kListDirect) {
                        // A handed-over query arrives with a k-th best that already prunes most of the shell, so a
                        // pass rarely keeps more than a few keys.  Those go into the list one at a time: with the
                        // list ascending by lane, the new list is min(own, max(key, the lane below's)) in every
                        // lane (keys below the new one stay, the new one lands in the first lane holding a larger
                        // key, every larger key moves one lane up and the largest leaves): five instructions per
                        // key against some three hundred for a sorted merge of the pending array, and the k-th
                        // best tightens at once.  A key that no longer beats the k-th best changes nothing.
                        uint64_t mm = m;
                        do {
                            const int b = __ffsll((unsigned long long)mm) - 1;
                            mm &= mm - 1;
                            const uint64_t x = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(key >> 32), b) << 32) |
                                               (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)key, b);
                            best = key_min(best, key_max(x, wave_from_below(best)));
                        } while (mm);
                        s.tau = wave_last_key(best);
                    } else if (m) {
                        if (acc) pend[npend + __popcll(m & lt_mask)] = key;
                        npend += __popcll(m);
                        __syncthreads();
                        if (npend > kQueryBlock) absorb64();
                    }
                }
            }
            while (npend > 0) absorb64();
            if (s.certified(R)) break;
        }

        // output: slot 0 is the query itself, slot j >= 1 lives in lane 64 - cap + j - 1
        if (lane == 0) { oi[0] = row; od[0] = 0.0f; }
        if (lane >= kQueryBlock - cap) {
            const int32_t j = a.slot0 + lane - (kQueryBlock - cap) + 1;
            const bool real = best < kEmptyKey;
            oi[j] = real ? (int32_t)(uint32_t)best : -1;
            od[j] = real ? __uint_as_float((uint32_t)(best >> 32)) : 0.0f;
        }
        if (COUNT && lane == 0) a.out_cand[row] += cand;
        __syncthreads();
    }
}

}  // namespace fg
