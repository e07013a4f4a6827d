// Main query kernel: one wavefront per tile of 64 consecutive bin-ordered queries, worked as four
// sub-tiles of 16 queries (one DPP row each); the running best list of every lane is held SORTED
// IN REGISTERS.
//
// What it computes is Algorithm 2 of the paper (Section 3): shells of bins of growing Chebyshev
// radius around the query's bin, exact K-1 best others, stop once the k-th best is certified.
// How it is laid out for CDNA4:
//   * candidates are BROADCAST, not gathered: the 16 lanes of a row hold 16 candidates, one
//     each, and in step J every lane of the row evaluates candidate J, read from lane J's
//     registers by the DPP control row_newbcast:J folded into the subtraction itself.  A pair
//     costs its 3d-1 float operations, one move for the candidate's index and one compare; no
//     LDS read, no address arithmetic, every lane busy;
//   * what a row scans is therefore the UNION of what its 16 queries need: per shell R and per
//     column (a bin position in the first DB-1 binning dimensions; bins adjacent in the last one
//     are adjacent in memory) the interval of last-dimension bins spanned by the cubes of
//     radius R of the row's queries that reach the column.  The region scanned so far is, per
//     column, one interval that only grows, so a shell adds at most two runs of sorted points
//     per column, and no point is ever presented twice to a row;
//   * the columns of a shell are worked out 16 at a time by the lanes of the row (one column per
//     lane), their runs are laid end to end by a prefix sum, and lane L of the row fetches
//     candidate 16 c + L of that stream for chunk c (binary search over the 16 runs; the loads
//     of chunk c + 1 are issued before chunk c is evaluated);
//   * a candidate that beats the lane's current k-th best is appended to a small per-lane
//     pending buffer in LDS (one write, no ordering work).  When any lane's buffer is nearly
//     full, and at the end of every shell, all lanes absorb their pending keys into the sorted
//     register list with a fixed merging network (no data-dependent addressing);
//   * keys are 64-bit (distance bits << 32 | original index); slots beyond K-1 are pinned with
//     zero keys so that the last register is always the last wanted key (list sizes 16/32/48/64;
//     longer lists take a second pass that counts only keys above the first pass's last one);
//   * a tile that straddles row splits walks once per row split with the other lanes switched
//     off, so inside a walk the grid geometry is uniform;
//   * finished rows leave from the registers in 16-byte pieces when K equals the list size, else
//     through LDS so that each output row is written as contiguous bytes;
//   * lanes still uncertified when few are left are handed to the list kernel.
#pragma once
#include <type_traits>
#include "fg_query.hpp"
#include "fg_sortnet.hpp"

namespace fg {

// Waves per SIMD the register allocator aims at: the sorted list alone takes 2*KC registers.
template <int KC, int D> constexpr int tile_waves()
{
    return KC <= 16 ? 4 : (KC == 32 ? 3 : (KC == 48 ? (D <= 3 ? 3 : 2) : 2));
}
constexpr int kPend = 16;             // pending keys per lane between two merges
constexpr int kPendRows = kPend + 1;  // and one spare slot that takes the stores of candidates a lane does not keep
constexpr int kRow = 16;              // queries per sub-tile: one DPP row
constexpr int kRows = kQueryBlock / kRow;
constexpr int kStepGroup = 4;         // candidates evaluated between two checks of the pending buffers
constexpr int kSub = 2;               // candidates per lane in a chunk
constexpr int kChunk = kSub * kRow;   // candidates of a row in a chunk
constexpr int kMaxShellCols = 2048;   // columns a row may enumerate in one shell; beyond, its queries go to the list kernel

// row pitch of the output transposition in LDS: 65 words, so that the lanes writing one output row (consecutive
// slots of one query) read 65 words apart and spread over the banks instead of all landing in one
constexpr int kDumpStride = kQueryBlock + 1;

// ---- DPP helpers: all within one row of 16 lanes; every lane of the wave must be enabled -----------------
template <int J> __device__ __forceinline__ int32_t row_bcast_i32(int32_t v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + J, 0xf, 0xf, true);     // row_newbcast:J
}
template <int J> __device__ __forceinline__ float row_bcast_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x150 + J, 0xf, 0xf, true));
}
// reductions over the 16 lanes of a row, result in all of them: butterflies inside quads, across quads of a
// half row (half mirror), across the halves (mirror)
#define FG_ROW_REDUCE(NAME, T, OP)                                                                         \
    __device__ __forceinline__ T NAME(T v)                                                                 \
    {                                                                                                      \
        v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xb1, 0xf, 0xf, false)));  \
        v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4e, 0xf, 0xf, false)));  \
        v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, false))); \
        v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, false))); \
        return v;                                                                                          \
    }
__device__ __forceinline__ int32_t op_min_i32(int32_t a, int32_t b) { return a < b ? a : b; }
__device__ __forceinline__ int32_t op_max_i32(int32_t a, int32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t op_max_u32(uint32_t a, uint32_t b) { return a > b ? a : b; }
FG_ROW_REDUCE(row_min_i32, int32_t, op_min_i32)
FG_ROW_REDUCE(row_max_i32, int32_t, op_max_i32)
FG_ROW_REDUCE(row_max_u32, uint32_t, op_max_u32)
FG_ROW_REDUCE(row_min_f32, float, fminf)
FG_ROW_REDUCE(row_max_f32, float, fmaxf)
#undef FG_ROW_REDUCE
// inclusive prefix sum over the 16 lanes of a row
__device__ __forceinline__ int32_t row_incl_scan_i32(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    return v;
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// One whole output row from the lane that holds it: word 0 and the keys best[OFF ...], as 16-byte stores.
// The row has KC - OFF + 1 words, a multiple of four, and starts on a 16-byte boundary.
template <int KC, int OFF>
__device__ __forceinline__ void store_row_from_registers(const uint64_t (&best)[KC], int32_t* __restrict__ oi,
                                                         float* __restrict__ od, int32_t idx0, uint32_t d2_0)
{
    constexpr int WORDS = KC - OFF + 1;
    static_assert(WORDS % 4 == 0 && OFF >= 1, "whole 16-byte pieces");
#pragma unroll
    for (int c = 0; c < WORDS / 4; ++c) {
        int32_t wi[4];
        uint32_t wd[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = 4 * c + t;
            if (j == 0) { wi[t] = idx0; wd[t] = d2_0; continue; }
            const uint64_t key = best[OFF + j - 1];
            const bool real = key < kEmptyKey;
            wi[t] = real ? (int32_t)(uint32_t)key : -1;
            wd[t] = real ? (uint32_t)(key >> 32) : 0u;
        }
        reinterpret_cast<int4*>(oi)[c] = make_int4(wi[0], wi[1], wi[2], wi[3]);
        reinterpret_cast<uint4*>(od)[c] = make_uint4(wd[0], wd[1], wd[2], wd[3]);
    }
}

// LDS of a workgroup (one wavefront): the pending buffers (8 KB) and the run tables of the four rows (1 KB);
// at the end the same memory carries the output transposition.
constexpr size_t kPendBytes = (size_t)kPendRows * kQueryBlock * 8;
constexpr size_t kRunTableBytes = (size_t)kQueryBlock * 4 * 4;
template <int KC> constexpr size_t tile_lds_bytes()
{
    const size_t scan = kPendBytes + kRunTableBytes;
    const size_t out = (size_t)kQueryBlock * 4 * 2 + (size_t)KC * kDumpStride * 4;
    return scan > out ? scan : out;
}

// Evaluates candidate J of every row against the row's 16 queries and appends what a lane keeps to its
// pending buffer.  c[], ci: this lane's candidate (coordinates, original index); xq[]: this lane's query
// (NaN in a lane that must keep nothing); INTRA: the candidates are the row's own queries, lane J skips itself.
template <int J, int D, bool LOWER, bool INTRA>
__device__ __forceinline__ void scan_step(const float (&c)[D], int32_t ci, const float (&xq)[D], uint32_t tau_hi,
                                          uint64_t lower, uint32_t& pend_top, uint32_t spare, int rl)
{
    // (candidate - query) squared equals (query - candidate) squared bit for bit; summed left to right
    float diff = row_bcast_f32<J>(c[0]) - xq[0];
    float d2 = diff * diff;
#pragma unroll
    for (int k = 1; k < D; ++k) {
        diff = row_bcast_f32<J>(c[k]) - xq[k];
        d2 = d2 + diff * diff;
    }
    const uint32_t idx = (uint32_t)row_bcast_i32<J>(ci);
    const uint32_t bits = __float_as_uint(d2);
    // kept if its distance does not exceed the k-th best's (a tie on the distance may lose on the index: the
    // merge decides); NaN patterns (poisoned candidates, switched-off queries) lie above every bound
    // No branch and no change of the execution mask: every lane stores every candidate at its slot pointer, and
    // only a lane that keeps the candidate moves the pointer on, so what is not kept is overwritten by the next
    // store.  (Narrowing the mask per step made every step a chain of vector compare -> scalar mask -> store ->
    // scalar restore that three wavefronts per SIMD cannot hide.)  Index word and distance word are kPendRows
    // planes apart.
    static_assert(kPendRows == 17 && kQueryBlock * 4 == 0x100, "offsets below");
    if constexpr (!INTRA && !LOWER) {
        // A candidate that is not kept has a distance above the k-th best's, so it does no harm where it stays
        // if nothing overwrites it: the merge reads all kPend slots and drops it like any key above the k-th best
        // (slot kPend, beyond the last one the merge reads, takes the store of a lane whose buffer is full).
        asm volatile("ds_write2st64_b32 %0, %1, %2 offset1:17" : : "v"(pend_top), "v"(idx), "v"(bits));
        pend_top = bits <= tau_hi ? pend_top + 0x100u : pend_top;
    } else {
        // here a candidate can be turned down although it lies below the k-th best (the query itself, a key the
        // first pass of a long list has already placed): it must not stay in a slot the merge reads
        bool keep = bits <= tau_hi;
        if (INTRA) keep = keep && rl != J;
        if (LOWER) keep = keep && ((((uint64_t)bits << 32) | idx) > lower);
        const uint32_t addr = keep ? pend_top : spare;
        asm volatile("ds_write2st64_b32 %0, %1, %2 offset1:17" : : "v"(addr), "v"(idx), "v"(bits));
        pend_top = keep ? pend_top + 0x100u : pend_top;
    }
}

template <int D, int DB, int KC, bool COUNT, bool LOWER>
__global__ void __launch_bounds__(kQueryBlock) __attribute__((amdgpu_waves_per_eu(tile_waves<KC, D>(), tile_waves<KC, D>())))
k_query_tile(QueryArgs a)
{
    extern __shared__ uint64_t lds64[];
    // an entry of the order: the tile, heaviest first
    const int32_t tile = a.tile_order ? a.tile_order[blockIdx.x] : (int32_t)blockIdx.x;
    const int lane = threadIdx.x;
    const int rl = lane & (kRow - 1);
    const int row_lane0 = lane & ~(kRow - 1);
    // pending keys: index words [kPendRows][64], then distance words [kPendRows][64]
    uint32_t* const pend_lds = reinterpret_cast<uint32_t*>(lds64) + lane;
    constexpr int kPendHalf = kPendRows * kQueryBlock;
    // next free slot of this lane, kept as a plain LDS byte address so that an accepted candidate costs one
    // two-word store and one add
    using lds_word = __attribute__((address_space(3))) uint32_t;
    const uint32_t pend_base = (uint32_t)(uintptr_t)(lds_word*)pend_lds;
    uint32_t pend_top = pend_base;
    const uint32_t pend_full = pend_base + (kPend - kStepGroup) * kQueryBlock * 4;   // beyond this a group of steps may overflow
    const uint32_t pend_spare = pend_base + kPend * kQueryBlock * 4;
    // run tables of the four rows, one entry per column of the current batch of 16: offset of the column's
    // candidates in the row's stream, first run (start, length), start of the second run
    int32_t* const run_excl = reinterpret_cast<int32_t*>(lds64 + kPendRows * kQueryBlock) + row_lane0;
    int32_t* const run_a1 = run_excl + kQueryBlock;
    int32_t* const run_len1 = run_a1 + kQueryBlock;
    int32_t* const run_a2 = run_len1 + kQueryBlock;

    const int32_t cap = a.k_list;         // 0 <= cap <= KC
    const int32_t p = tile * kQueryBlock + lane;
    const bool valid = p < a.n;
    const int32_t pp = valid ? p : a.n - 1;   // dead lanes shadow the last point, never scan or write
    const int32_t my_row = a.perm[pp];
    const bool asks = !(a.dir && !dir_is_query(a.dir[my_row]));   // direction flag: does this point query at all
    const bool is_neighbour = !(a.dir && !dir_is_neighbour(a.dir[my_row]));
    bool active = valid && cap > 0 && asks;   // still searching (any row split)
    float x[D];
#pragma unroll
    for (int c = 0; c < D; ++c) x[c] = a.soa[(int64_t)c * a.soa_stride + pp];
    // second pass of a long list (more than 64 neighbours): the first pass has placed the 64 nearest; only keys
    // above the last of them count now (an empty slot there: the row split has no more points, nothing counts)
    uint64_t lower = 0;
    if (LOWER && active) {
        const int32_t li = a.out_idx[(int64_t)my_row * a.k + a.slot0];
        lower = li < 0 ? kEmptyKey : (((uint64_t)__float_as_uint(a.out_d2[(int64_t)my_row * a.k + a.slot0]) << 32) | (uint32_t)li);
    }

    uint64_t best[KC];
#pragma unroll
    for (int i = 0; i < KC; ++i) best[i] = (i < KC - cap) ? 0ull : kEmptyKey;
#pragma unroll
    for (int i = 0; i < kPend; ++i) pend_lds[kPendHalf + i * kQueryBlock] = (uint32_t)(kEmptyKey >> 32);   // all pending slots empty
    uint32_t tau_hi = (uint32_t)(best[KC - 1] >> 32);
    uint64_t tau = best[KC - 1];
    int32_t cand = 0;
    int32_t resume = 0;        // first shell the list kernel has to search for this lane, if it is handed over
    bool handed = false;

    auto absorb = [&]() {
        uint64_t pend[kPend];
        asm volatile("" : : : "memory");     // the stores of the steps above are issued before these reads
        // unused slots hold the empty key's distance word (refilled below), whatever their index word: such keys
        // lie at or above the empty key and sort behind every real one
        // (the sign bit of the distance word is cleared: a slot may hold a candidate that was not kept, whose
        // distance may be a NaN of either sign, and the networks order keys as non-negative doubles)
#pragma unroll
        for (int i = 0; i < kPend; ++i)
            pend[i] = ((uint64_t)(pend_lds[kPendHalf + i * kQueryBlock] & 0x7fffffffu) << 32) | pend_lds[i * kQueryBlock];
#pragma unroll
        for (int i = 0; i < kPend; ++i) pend_lds[kPendHalf + i * kQueryBlock] = (uint32_t)(kEmptyKey >> 32);
        net_sort<kPend>(pend);
        net_absorb<KC, kPend>(best, pend);
        pend_top = pend_base;
        tau = best[KC - 1];
        tau_hi = (uint32_t)(tau >> 32);
        asm volatile("" : : : "memory");     // and the refill above before the stores of the steps that follow
    };

    // the row splits this tile touches; each gets a walk of its own
    const int32_t p_last = tile * kQueryBlock + kQueryBlock - 1 < a.n - 1 ? tile * kQueryBlock + kQueryBlock - 1 : a.n - 1;
    const int32_t seg_first = segment_of(a.row_splits, a.n_segments, tile * kQueryBlock);
    const int32_t seg_last = segment_of(a.row_splits, a.n_segments, p_last);
    const float kNaN = __uint_as_float(0x7fc00000u);

    for (int32_t seg = seg_first; seg <= seg_last; ++seg) {
        const int32_t s0 = a.row_splits[seg], s1 = a.row_splits[seg + 1];
        const bool in_seg = valid && p >= s0 && p < s1;
        bool act = active && in_seg;                      // searching in this walk
        if (!__any(act)) continue;
        // grid of the row split (uniform over the wave), this lane's bin in it
        float glo[DB], gw[DB], gslack[DB];
        int32_t neff[DB], cc[DB];
        {
            const float* g = a.geom + (int64_t)seg * DB * kGeomStride;
#pragma unroll
            for (int c = 0; c < DB; ++c) {
                const float inv_w = g[c * kGeomStride + 1];
                glo[c] = g[c * kGeomStride + 0];
                gw[c] = g[c * kGeomStride + 2];
                gslack[c] = g[c * kGeomStride + 3];
                cc[c] = cell_of(x[c], glo[c], inv_w, a.n_bins);
                neff[c] = inv_w > 0.0f ? a.n_bins : 1;
            }
        }
        const int32_t seg_cell0 = seg * a.cells_per_segment;
        // true when no point of a box at squared lower-bound distance b2 can enter a list whose k-th best is t
        auto cannot_improve = [&](uint64_t t, float b2) -> bool {
            return t < kEmptyKey && b2 > 1e-30f && __uint_as_float((uint32_t)(t >> 32)) < b2 * kBoundShrink;
        };
        // after shell r: may this lane stop (the cube of radius r round its bin is searched)
        auto certified = [&](int32_t r) -> bool {
            bool covered = true;
            float mingap = 3.0e38f;
#pragma unroll
            for (int c = 0; c < DB; ++c) {
                const int32_t jl = cc[c] - r, jh = cc[c] + r;
                if (jl > 0) {
                    covered = false;
                    const float g = x[c] - (glo[c] + (float)jl * gw[c]) - gslack[c];
                    mingap = fminf(mingap, g > 0.0f ? g : 0.0f);
                }
                if (jh < neff[c] - 1) {
                    covered = false;
                    const float g = (glo[c] + (float)(jh + 1) * gw[c]) - x[c] - gslack[c];
                    mingap = fminf(mingap, g > 0.0f ? g : 0.0f);
                }
            }
            return covered || cannot_improve(tau, mingap * mingap);
        };
        // box of the row's queries of this walk in the binned coordinates: bounds every lane's distance to a bin from below
        float qmin[DB], qmax[DB];
#pragma unroll
        for (int c = 0; c < DB; ++c) {
            qmin[c] = row_min_f32(in_seg ? x[c] : 3.0e38f);
            qmax[c] = row_max_f32(in_seg ? x[c] : -3.0e38f);
        }
        float xq[D];   // what the scan sees as this lane's query
#pragma unroll
        for (int c = 0; c < D; ++c) xq[c] = act ? x[c] : kNaN;

        // ---- the row's own 16 points: every lane against the 15 others (they are left out of the streams below)
        {
            float cself[D];
            const bool offer = in_seg && is_neighbour;
#pragma unroll
            for (int c = 0; c < D; ++c) cself[c] = offer ? x[c] : kNaN;
            static_for<0, kRow>([&](auto J) {
                scan_step<decltype(J)::value, D, LOWER, true>(cself, my_row, xq, tau_hi, lower, pend_top, pend_spare, rl);
            });
            if (COUNT && act) cand += __popcll(__ballot(in_seg) & (0xffffull << row_lane0)) - 1;
            if (__any(pend_top > pend_full)) absorb();     // up to 15 kept per lane: make room for the first group of steps
        }
        const int32_t own0 = tile * kQueryBlock + row_lane0;                  // the row's own sorted positions
        const int32_t own1 = own0 + kRow;

        int32_t rdone = -1;    // last shell this lane took part in, in this walk
        bool give_up = false;  // this lane's row cannot enumerate its columns: to the list kernel
        int32_t R = 0;
        for (;; ++R) {   // ends at the latest at R = n_bins - 1, when every lane's cube covers its grid
            // who asks for columns in this shell: at shell 0 every point of the walk (so that the row's own points
            // are certainly inside the region, whatever their flags), afterwards the searching lanes
            const bool want = R == 0 ? in_seg : act;
            const int32_t ra = want ? R : -1;                             // radius this lane reaches now
            const int32_t rp = R == 0 ? -1 : (act ? R - 1 : rdone);       // radius this lane's columns were searched to
            // columns to enumerate: the box of the asking lanes' columns, widened by R, centre first
            int32_t c0[DB - 1], side[DB - 1];
            int32_t ncols = row_max_i32(act ? 1 : 0);    // a row without searching lanes has nothing to enumerate
            bool too_many = false;
#pragma unroll
            for (int c = 0; c < DB - 1; ++c) {
                const int32_t lo = row_min_i32(want ? cc[c] : 0x7fffffff);
                const int32_t hi = row_max_i32(want ? cc[c] : -1);
                const int32_t e = hi >= lo ? hi - lo : 0;
                c0[c] = (hi >= lo ? lo : 0) + (e >> 1);
                side[c] = 2 * (R + ((e + 1) >> 1)) + 1;
                if (hi < lo) ncols = 0;
                too_many = too_many || side[c] > kMaxShellCols || ncols * side[c] > kMaxShellCols;
                ncols = too_many ? 0 : ncols * side[c];
            }
            if (too_many) { give_up = give_up || act; ncols = 0; }
            const bool wants_now = want && !give_up;
            const int32_t ra_now = wants_now ? ra : -1;
            const uint64_t tau_row = ((uint64_t)row_max_u32(act ? (uint32_t)(tau >> 32) : 0u) << 32) | 0xffffffffu;   // no searching lane's k-th best is above this
            const int32_t max_cols = wave_max_i32(ncols);

            for (int32_t t0 = 0; t0 < max_cols; t0 += kRow) {
                // ---- this lane's column of its row: which bins of it are new in this shell
                const int32_t t = t0 + rl;
                bool ok = t < ncols;
                int32_t X[DB - 1];
                float partial = 0.0f;
                int32_t flat = 0;
                {
                    int32_t rem = ok ? t : 0;
#pragma unroll
                    for (int c = DB - 2; c >= 0; --c) {
                        // digit v of the column number maps to offset 0, +1, -1, +2, -2, ... from the centre
                        const int32_t q = (int32_t)(((float)rem + 0.5f) * (1.0f / (float)side[c]));   // exact: rem < 2^11 * side
                        const int32_t v = rem - q * side[c];
                        rem = q;
                        X[c] = c0[c] + ((v & 1) ? ((v + 1) >> 1) : -(v >> 1));
                    }
#pragma unroll
                    for (int c = 0; c < DB - 1; ++c) {
                        ok = ok && X[c] >= 0 && X[c] < neff[c];
                        // distance from the box of the row's queries to the bin, from below
                        const float below = qmin[c] - (glo[c] + (float)(X[c] + 1) * gw[c]) - gslack[c];
                        const float above = (glo[c] + (float)X[c] * gw[c]) - qmax[c] - gslack[c];
                        const float gp = fmaxf(fmaxf(below, above), 0.0f);
                        partial += gp * gp;
                        flat = snake_push(flat, ok ? X[c] : 0, a.n_bins);
                    }
                }
                // union over the row's queries that reach this column: what was searched before (plo..phi), what
                // this shell asks for (alo..ahi)
                int32_t plo = 0x7fffffff, phi = -0x7fffffff, alo = 0x7fffffff, ahi = -0x7fffffff;
                static_for<0, kRow>([&](auto J) {
                    constexpr int j = decltype(J)::value;
                    int32_t rmin = 0;
#pragma unroll
                    for (int c = 0; c < DB - 1; ++c) {
                        const int32_t dlt = row_bcast_i32<j>(cc[c]) - X[c];
                        rmin = op_max_i32(rmin, dlt < 0 ? -dlt : dlt);
                    }
                    const int32_t zj = row_bcast_i32<j>(cc[DB - 1]);
                    const int32_t rpj = row_bcast_i32<j>(rp);
                    const int32_t raj = row_bcast_i32<j>(ra_now);
                    if (rmin <= rpj) { plo = op_min_i32(plo, zj - rpj); phi = op_max_i32(phi, zj + rpj); }
                    if (rmin <= raj) { alo = op_min_i32(alo, zj - raj); ahi = op_max_i32(ahi, zj + raj); }
                });
                ok = ok && ahi >= alo && !cannot_improve(tau_row, partial);
                int32_t a1 = 0, b1 = 0, a2 = 0, b2 = 0;
                if (ok) {
                    const int32_t nz = neff[DB - 1];
                    // last-dimension bins new in this shell: below and above what was searched before
                    int32_t z1a, z1b, z2a, z2b;
                    if (phi < plo) { z1a = alo; z1b = ahi; z2a = 1; z2b = 0; }
                    else { z1a = alo; z1b = plo - 1; z2a = phi + 1; z2b = ahi; }
                    z1a = z1a < 0 ? 0 : z1a; z1b = z1b > nz - 1 ? nz - 1 : z1b;
                    z2a = z2a < 0 ? 0 : z2a; z2b = z2b > nz - 1 ? nz - 1 : z2b;
                    // drop end bins whose box is too far for every searching lane of the row
                    auto far_below = [&](int32_t z) {
                        const float g = fmaxf(qmin[DB - 1] - (glo[DB - 1] + (float)(z + 1) * gw[DB - 1]) - gslack[DB - 1], 0.0f);
                        return cannot_improve(tau_row, partial + g * g);
                    };
                    auto far_above = [&](int32_t z) {
                        const float g = fmaxf((glo[DB - 1] + (float)z * gw[DB - 1]) - qmax[DB - 1] - gslack[DB - 1], 0.0f);
                        return cannot_improve(tau_row, partial + g * g);
                    };
                    while (z1a <= z1b && far_below(z1a)) ++z1a;
                    if (phi < plo) { while (z1b >= z1a && far_above(z1b)) --z1b; }
                    while (z2b >= z2a && far_above(z2b)) --z2b;
                    int32_t f0, f1;
                    if (z1b >= z1a) { snake_run(flat, z1a, z1b, a.n_bins, &f0, &f1); a1 = a.bounds[seg_cell0 + f0]; b1 = a.bounds[seg_cell0 + f1 + 1]; }
                    if (z2b >= z2a) { snake_run(flat, z2a, z2b, a.n_bins, &f0, &f1); a2 = a.bounds[seg_cell0 + f0]; b2 = a.bounds[seg_cell0 + f1 + 1]; }
                    if (R == 0) {
                        // the row's own points are not streamed: cut them out of the (single) run
                        if (a1 < own1 && b1 > own0) {
                            a2 = own1 > a1 ? own1 : a1; b2 = b1;
                            b1 = own0 < b1 ? own0 : b1;
                            if (b2 < a2) b2 = a2;
                            if (b1 < a1) b1 = a1;
                        }
                    }
                }
                const int32_t len1 = b1 - a1, len = len1 + (b2 - a2);
                const int32_t incl = row_incl_scan_i32(len);
                const int32_t T = row_bcast_i32<kRow - 1>(incl);          // candidates of the row in this batch of columns
                __syncthreads();
                run_excl[rl] = incl - len; run_a1[rl] = a1; run_len1[rl] = len1; run_a2[rl] = a2;
                __syncthreads();
                const int32_t n_chunks = (wave_max_i32(T) + kChunk - 1) / kChunk;

                // A chunk is kSub candidates per lane (kSub x 16 per row): candidate (ch * kSub + u) * 16 + L of the
                // row's stream goes to register set u of lane L.  The loads of chunk ch + 1 are issued before chunk
                // ch is evaluated; they take well over a microsecond under load, which the kSub x 16 steps of a chunk
                // (with the other wavefronts of the SIMD) cover, and 16 steps do not.  All loads of a fetch are
                // independent and unconditional (slots beyond the end of the stream read a valid dummy position and
                // are poisoned afterwards): a load that waits for another one's result would expose a full memory
                // latency per chunk.
                struct Stage { float c[kSub][D]; int32_t ci[kSub]; };
                // this lane's place in the table: the run its last candidate came from and where that run ends in the
                // stream; candidates are taken in ascending order, so the next one is found by stepping forward
                int32_t cj = -1, c_end = 0, c_excl = 0;
                auto fetch = [&](int32_t ch, Stage& st) {
#pragma unroll
                    for (int u = 0; u < kSub; ++u) {
                        const int32_t f = (ch * kSub + u) * kRow + rl;
                        const bool in = f < T;
                        while (in && f >= c_end) {       // runs of length zero are stepped over; the last run ends at T > f
                            ++cj;
                            c_excl = c_end;
                            c_end = cj + 1 < kRow ? run_excl[cj + 1] : T;
                        }
                        const int32_t jj = cj < 0 ? 0 : cj;
                        const int32_t local = f - c_excl, l1 = run_len1[jj];
                        int32_t q = local < l1 ? run_a1[jj] + local : run_a2[jj] + (local - l1);
                        q = in ? q : pp;
                        // index of the candidate, or -1 if a direction flag says it is nobody's neighbour (a.perm_cand
                        // is a.perm where there are no flags)
                        st.ci[u] = a.perm_cand[q];
#pragma unroll
                        for (int c = 0; c < D; ++c) st.c[u][c] = a.soa[(int64_t)c * a.soa_stride + q];
                    }
                };
                Stage nxt, cur;
                if (n_chunks > 0) fetch(0, nxt);
                for (int32_t ch = 0; ch < n_chunks; ++ch) {
#pragma unroll
                    for (int u = 0; u < kSub; ++u) {
                        // a slot beyond the end of the stream, or a point that is nobody's neighbour: its coordinates
                        // become NaN (the loads were issued a chunk ago, unconditionally)
                        const int32_t f = (ch * kSub + u) * kRow + rl;
                        const bool real = f < T && nxt.ci[u] >= 0;
#pragma unroll
                        for (int c = 0; c < D; ++c) cur.c[u][c] = real ? nxt.c[u][c] : kNaN;
                        cur.ci[u] = nxt.ci[u];
                    }
                    if (COUNT && act) { const int32_t left = T - ch * kChunk; cand += left > kChunk ? kChunk : (left > 0 ? left : 0); }
                    fetch(ch + 1, nxt);          // beyond the last chunk: a harmless fetch of padding
#pragma unroll 1
                    for (int g = 0; g < kChunk / kStepGroup; ++g) {
                        static_for<0, kChunk / kStepGroup>([&](auto G) {
                            constexpr int gg = decltype(G)::value;
                            constexpr int u = gg / (kRow / kStepGroup), j0 = (gg % (kRow / kStepGroup)) * kStepGroup;
                            if (g == gg) {
                                static_for<j0, j0 + kStepGroup>([&](auto J) {
                                    scan_step<decltype(J)::value, D, LOWER, false>(cur.c[u], cur.ci[u], xq, tau_hi, lower, pend_top, pend_spare, rl);
                                });
                            }
                        });
                        if (__any(pend_top > pend_full)) absorb();
                    }
                }
            }
            if (__any(pend_top != pend_base)) absorb();
            // shell R is searched for every lane that asked and was not given up
            if (want && !give_up) rdone = R;
            if (act && give_up) { act = false; handed = true; resume = R; }
            if (act && certified(R)) act = false;
            if (!act) {
#pragma unroll
                for (int c = 0; c < D; ++c) xq[c] = kNaN;
            }
            const int32_t n_act = __popcll(__ballot(act));
            if (n_act == 0) break;
            // Go on to the next shell in this wave only while enough of its lanes still search: a shell costs the
            // whole wave the union of what its unfinished lanes need, and the list kernel takes a query from
            // where it stands for a few microseconds of one wavefront.
            if (R >= 1 && n_act <= a.defer_lanes) break;
        }
        // unfinished lanes of this walk go to the list kernel
        if (act) { handed = true; resume = R + 1; }
        active = active && !in_seg;
    }

    // handed-over lanes go to the work list (wave-aggregated append); their lists so far leave with the
    // finished rows, and the first shell still to search travels in slot 0 of the distance row
    const uint64_t mask = __ballot(handed);
    if (mask) {
        int32_t base = 0;
        const int leader = __ffsll((unsigned long long)mask) - 1;
        if (lane == leader) base = atomicAdd(a.work_count, __popcll(mask));
        base = __shfl(base, leader, 64);
        if (handed) a.work_list[base + __popcll(mask & ((1ull << lane) - 1))] = p;
    }
    const uint32_t resume_word = handed ? (uint32_t)resume : 0u;

    // Rows of exactly KC words (K = 16, 32, 48, 64) leave straight from the registers: every lane writes its own
    // row in 16-byte pieces (the pieces of a 128-byte line arrive within a few instructions of each other and are
    // joined in the L2 cache).  Rows that do not start on a 64-byte boundary (K = 40: 160 bytes) keep the
    // transposition.
    const bool direct_rows = a.slot0 == 0 && a.k == KC && cap == KC - 1 &&
                             (((uintptr_t)a.out_idx | (uintptr_t)a.out_d2) & 15) == 0;
    if (COUNT && valid) a.out_cand[my_row] = LOWER ? a.out_cand[my_row] + cand : cand;
    if (direct_rows) {
        if (valid) {
            int32_t* oi = a.out_idx + (int64_t)my_row * a.k;
            float* od = a.out_d2 + (int64_t)my_row * a.k;
            store_row_from_registers<KC, 1>(best, oi, od, asks ? my_row : -1, resume_word);
        }
        return;
    }
    // otherwise: registers -> LDS -> contiguous row writes
    __syncthreads();
    // two passes (indices, then distances) so the transposition needs KC x 64 words, not keys
    int32_t* rows_lds = reinterpret_cast<int32_t*>(lds64);
    uint32_t* resume_lds = reinterpret_cast<uint32_t*>(lds64) + kQueryBlock;
    uint32_t* dump = reinterpret_cast<uint32_t*>(lds64) + 2 * kQueryBlock;     // [KC][65] after the row and resume words
    rows_lds[lane] = valid ? (asks ? my_row : -2 - my_row) : -1;   // -1: nothing to write; <= -2: all-padding row
    resume_lds[lane] = resume_word;
    const int32_t k = a.k;
    const int32_t kk = cap + 1;                                         // words written per row: slot 0 and this pass's slots
    const int32_t per_iter = kk >= kQueryBlock ? 1 : kQueryBlock / kk;  // rows written per pass
    const int32_t sub = lane / kk;                                      // which of them this lane serves
    const int32_t j0 = lane - sub * kk;                                 // word inside the row
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads();
#pragma unroll
        for (int i = 0; i < KC; ++i) {
            const bool real = best[i] < kEmptyKey;
            const uint32_t word = pass == 0 ? (real ? (uint32_t)best[i] : 0xffffffffu)      // index or -1
                                            : (real ? (uint32_t)(best[i] >> 32) : 0u);       // distance bits or 0.0f
            dump[i * kDumpStride + lane] = word;
        }
        __syncthreads();
        for (int32_t r0 = 0; r0 < kQueryBlock; r0 += per_iter) {
            const int32_t ql = r0 + sub;
            if (sub >= per_iter || ql >= kQueryBlock) continue;
            const int32_t enc = rows_lds[ql];
            if (enc == -1) continue;
            const int32_t row = enc >= 0 ? enc : -2 - enc;
            for (int32_t j = j0; j < kk; j += kQueryBlock) {
                uint32_t word = pass == 0 ? (enc >= 0 ? (uint32_t)row : 0xffffffffu) : resume_lds[ql];   // slot 0: the row itself at distance 0, or where to resume
                if (j > 0) word = dump[(KC - cap + j - 1) * kDumpStride + ql];
                const int32_t slot = j > 0 ? a.slot0 + j : 0;
                if (pass == 0) a.out_idx[(int64_t)row * k + slot] = (int32_t)word;
                else a.out_d2[(int64_t)row * k + slot] = __uint_as_float(word);
            }
        }
    }
}

}  // namespace fg
