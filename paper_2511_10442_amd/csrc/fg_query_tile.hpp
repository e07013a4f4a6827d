// Main query kernel: one wavefront per tile of 64 consecutive bin-ordered queries, the running
// best list of every lane held SORTED IN REGISTERS.
//
// What it computes is Algorithm 2 of the paper (Section 3): shells of bins of growing Chebyshev
// radius around the query's bin, exact K-1 best others, stop once the k-th best is certified.
// How it is laid out for CDNA4:
//   * the shell walk is wave-uniform: all 64 lanes step through the same column offsets
//     (offsets in the first DB-1 binning dimensions) of the same shell together.  Queries of a
//     tile are consecutive in bin order, so the bins they need for one column offset form one
//     contiguous range of sorted points; it is staged through LDS in chunks (the point records
//     as the counting sort wrote them, 16-byte vectors), and each lane scans only its own
//     sub-range of the chunk: whole bins narrowed by the box bound, then cut to the slices of
//     the last binning dimension that the k-th best still reaches (direct scan); in tiles whose
//     lanes' sub-ranges differ widely the passes of all sub-ranges are dealt out evenly over the
//     lanes whichever query they belong to (flattened scan);
//   * a candidate that beats the lane's current k-th best is appended to a small per-lane
//     pending buffer in LDS (one write, no ordering work).  When any lane's buffer is full, and
//     at the end of every shell, all lanes absorb their pending keys into the sorted register
//     list with a fixed merging network (no data-dependent addressing, no LDS round trips);
//   * keys are 64-bit (distance bits << 32 | original index); slots beyond K-1 are pinned with
//     zero keys so that the last register is always the last wanted key (list sizes 16/32/48/64; longer
//     lists take a second pass that counts only keys above the first pass's last one);
//   * finished rows leave from the registers in 16-byte pieces when K equals the list size, else
//     through LDS so that each output row is written as contiguous bytes;
//   * the stage takes what the LDS budget of a workgroup leaves, and that budget is what lets as
//     many workgroups share a CU as the registers allow;
//   * lanes still uncertified after shell 1 (up to five dimensions; beyond, when few are left)
//     are handed to the list kernel.
#pragma once
#include "fg_query.hpp"
#include "fg_sortnet.hpp"

namespace fg {

// Waves per SIMD the register allocator aims at: the sorted list alone takes 2*KC registers.  Measured choices:
// KC = 32 at three (two are 18 % slower, four spill into the scan loop and are slower too); KC = 48 at three for
// d <= 3 (12 % faster than two although a few registers spill outside the loops; with d >= 4 a staged candidate
// takes two more vector registers per unrolled slot and three waves lose 8 %); 64 keys at two.
template <int KC, int D> constexpr int tile_waves()
{
    return KC <= 16 ? 4 : (KC == 32 ? 3 : (KC == 48 ? (D <= 3 ? 3 : 2) : 2));
}
constexpr int kPend = 16;   // pending keys per lane between two merges
constexpr int kContinueLanes = 48;   // unfinished lanes a wave needs to go on past shell 1 (more than 2 binning dims)
struct Ranges { int32_t a1, b1, a2, b2; };

// row pitch of the output transposition in LDS: 65 words, so that the lanes writing one output row (consecutive
// slots of one query) read 65 words apart and spread over the banks instead of all landing in one
constexpr int kDumpStride = kQueryBlock + 1;
constexpr int kUnroll = 4;  // candidates per lane per pass of the scan loop (independent LDS reads in flight)

// staged point = its D coordinates followed by its original index, padded to whole float4s
template <int D> constexpr int stage_vecs() { return (D + 1 + 3) / 4; }

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

constexpr int kTileFlatBit = 6;   // in a tile's class word: the ordering kernels found the tile uneven
constexpr int kOrderFlagBit = 30;  // the same flag in the tile's entry of the order (tiles number below 2^25)
// LDS of a workgroup (one wavefront): the pending buffers (8 KB), the stage, and for the flattened scan its tables.
// How many wavefronts a CU holds is set by the registers (tile_waves) only if 4 * tile_waves workgroups fit its
// 160 KB of LDS, so the stage is sized for that: 16 workgroups (lists of 16 keys) get 10 KB each, 12 get 12.5 KB
// (measured: 12.6 KB still gives 12, 13.1 KB gives 11), 8 get 20 KB.  With a fixed 256-point stage d >= 4 ran at
// 9 and d >= 8 at 7 wavefronts per CU instead of 12, and 16-key lists at 13 instead of 16: 1M uniform points,
// K = 32: d = 4 1.17 -> 0.95 ms, d = 5 2.80 -> 2.31 ms, d = 8 51 -> 41 ms; d = 3, K = 16: 0.31 -> 0.27 ms.
constexpr size_t kPendBytes = (size_t)kPend * kQueryBlock * 8;
constexpr size_t kFlatTables = (size_t)kQueryBlock * 4 * 3 + 8 + (size_t)kQueryBlock * 8;   // counters, runs, starts, lower bounds
template <int KC, int D> constexpr size_t tile_lds_budget()
{
    return tile_waves<KC, D>() >= 4 ? 10240 : (tile_waves<KC, D>() == 3 ? 12800 : 20480);
}
constexpr int chunk_that_fits(size_t bytes, int nv)    // points: a multiple of 16 in [64, 256], kUnroll more are padding
{
    const int room = (int)(bytes / ((size_t)nv * 16)) - kUnroll;
    const int chunk = room / 16 * 16;
    return chunk > kStageChunk ? kStageChunk : (chunk < 64 ? 64 : chunk);
}
template <int KC, int D> constexpr int direct_chunk() { return chunk_that_fits(tile_lds_budget<KC, D>() - kPendBytes, stage_vecs<D>()); }
// the flattened scan is compiled in where its tables leave room for a stage of at least 64 points
template <int KC, int D> constexpr bool tile_has_flat()
{
    return tile_lds_budget<KC, D>() >= kPendBytes + kFlatTables + (size_t)stage_vecs<D>() * 16 * (64 + kUnroll);
}
template <int KC, int D> constexpr int flat_chunk()
{
    return tile_has_flat<KC, D>() ? chunk_that_fits(tile_lds_budget<KC, D>() - kPendBytes - kFlatTables, stage_vecs<D>()) : 64;
}

template <int D, int DB, int KC, bool COUNT, bool LOWER, bool FLAT>
__device__ __forceinline__ void tile_body(const QueryArgs& a, const int32_t tile, uint64_t* lds64)
{
    constexpr int CHUNK = FLAT ? flat_chunk<KC, D>() : direct_chunk<KC, D>();
    // LDS: [pending kPend x 64 keys][stage: CHUNK + kUnroll points of NV float4s][tables of the flattened scan];
    //      re-used at the end as
    //      [rows 64 words][KC x 64 words of the sorted lists, indices first, distances second]
    const int lane = threadIdx.x;
    // pending keys: index words [kPend][64], then distance words [kPend][64]
    uint32_t* const pend_lds = reinterpret_cast<uint32_t*>(lds64) + lane;
    constexpr int kPendHalf = kPend * kQueryBlock;
    // next free slot of this lane, kept as a plain LDS byte address so that an accepted candidate costs one
    // two-word store and one add (a pointer relative to pend_lds cost a second add per candidate)
    using lds_word = __attribute__((address_space(3))) uint32_t;
    const uint32_t pend_base = (uint32_t)(uintptr_t)(lds_word*)pend_lds;
    uint32_t pend_top = pend_base;
    constexpr int NV = stage_vecs<D>();
    float4* stage = reinterpret_cast<float4*>(lds64 + kPend * kQueryBlock);   // [CHUNK + kUnroll][NV]
    // flattened scan only: after the stage, [64] pending counts, [64] run descriptors, [66] run starts in the
    // flattened order, [64] lower bounds
    uint32_t* const pend_cnt = reinterpret_cast<uint32_t*>(stage + (CHUNK + kUnroll) * NV);
    int32_t* const fl_info = reinterpret_cast<int32_t*>(pend_cnt + kQueryBlock);
    int32_t* const fl_start = fl_info + kQueryBlock;
    uint64_t* const qlower = reinterpret_cast<uint64_t*>(fl_start + kQueryBlock + 2);
    const uint64_t lt_mask = (1ull << lane) - 1;

    const int32_t cap = a.k_list;         // 0 <= cap <= KC
    const int32_t p = tile * kQueryBlock + lane;
    const bool valid = p < a.n;
    LaneGeom<D, DB> s;
    const int32_t my_row = s.init_geom(a, valid ? p : a.n - 1);  // dead lanes shadow the last point, never scan or write
    const bool asks = !(a.dir && !dir_is_query(a.dir[my_row]));   // direction flag: does this point query at all
    bool active = valid && cap > 0 && asks;
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
    if constexpr (FLAT) {
        pend_cnt[lane] = 0;
        fl_start[kQueryBlock] = 0x7fffffff;
        if (LOWER) qlower[lane] = lower;
    }
    int32_t cand = 0;
    int32_t useful = 0;   // candidates this lane evaluated
    int32_t passes = 0;   // scan passes of the wave (kUnroll lane slots each)

    auto absorb = [&]() {
        uint64_t pend[kPend];
        // unused slots hold the empty key's distance word (refilled below), whatever their index word: such keys
        // lie at or above the empty key and sort behind every real one
#pragma unroll
        for (int i = 0; i < kPend; ++i)
            pend[i] = ((uint64_t)pend_lds[kPendHalf + i * kQueryBlock] << 32) | pend_lds[i * kQueryBlock];
#pragma unroll
        for (int i = 0; i < kPend; ++i) pend_lds[kPendHalf + i * kQueryBlock] = (uint32_t)(kEmptyKey >> 32);
        net_sort<kPend>(pend);
        net_absorb<KC, kPend>(best, pend);
        pend_top = pend_base;
        s.tau = best[KC - 1];
        if constexpr (FLAT) {
            pend_cnt[lane] = 0;
            __syncthreads();
        }
    };

    int32_t R = 0;
    const uint32_t pend_full = pend_base + (kPend - kUnroll) * kQueryBlock * 4;   // beyond this a pass may overflow
    for (;; ++R) {   // ends at the latest at R = n_bins - 1, when every lane's cube covers its grid
        const int32_t side = 2 * R + 1;
        int32_t ncols = 1;
#pragma unroll
        for (int c = 0; c < DB - 1; ++c) ncols *= side;
        // this lane's candidate ranges for column t of shell R: up to two runs of sorted positions
        auto prepare = [&](int32_t t) -> Ranges {
            // column offsets, wave-uniform; digit v of t maps to 0, +1, -1, +2, -2, ... (centre first)
            int32_t o[DB - 1];
            bool surf = false;
            {
                int32_t rem = t;
#pragma unroll
                for (int c = DB - 2; c >= 0; --c) {
                    const int32_t v = rem % side;
                    rem /= side;
                    o[c] = (v & 1) ? ((v + 1) >> 1) : -(v >> 1);
                    surf = surf || o[c] == R || o[c] == -R;
                }
            }
            bool ok = active;
            float partial = 0.0f;
            int32_t flat = 0;
#pragma unroll
            for (int c = 0; c < DB - 1; ++c) {
                const int32_t j = s.cc[c] + o[c];
                ok = ok && j >= 0 && j < s.neff[c];
                const float g = s.gap(c, j, o[c]);
                partial += g * g;
                flat = flat * a.n_bins + j;
            }
            ok = ok && !s.cannot_improve(partial);
            int32_t a1 = 0, b1 = 0, a2 = 0, b2 = 0;
            if (ok) {
                const int32_t cz = s.cc[DB - 1], nz = s.neff[DB - 1];
                // runs are cut to the slices of their bins that the k-th best still reaches (from shell 1 on:
                // the query's own bin is scanned whole, around the query itself)
                const int32_t sh = a.sub_shift;
                const int32_t row0 = s.bounds_at(flat, 0);
                int32_t s_lo = 0, s_hi = 0x7ffffffe;
                if (R > 0 && sh > 0) s.slice_reach(partial, s_lo, s_hi);
                auto cut_run = [&](int32_t z_first, int32_t z_last, int32_t& from, int32_t& to) {   // bins, inclusive
                    const int32_t fa = (z_first << sh) > s_lo ? (z_first << sh) : s_lo;
                    const int32_t fb = ((z_last + 1) << sh) < s_hi + 1 ? ((z_last + 1) << sh) : s_hi + 1;
                    if (fb > fa) { from = a.bounds[row0 + fa]; to = a.bounds[row0 + fb]; }
                };
                if (surf) {
                    int32_t za = cz - R < 0 ? 0 : cz - R;
                    int32_t zb = cz + R > nz - 1 ? nz - 1 : cz + R;
                    // drop end bins of the run whose box is already too far
                    while (za < cz) {
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
                    if (R == 0) { a2 = p + 1; b2 = b1; b1 = p; }   // the query's own bin, the query itself left out
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
            return Ranges{a1, b1, a2, b2};
        };
        Ranges cur = prepare(0);
        for (int32_t t = 0; t < ncols; ++t) {
            // the next column's bin boundaries are requested before this column is scanned, so
            // their latency hides behind the scan (its pruning sees a k-th best one column old)
            Ranges nxt = Ranges{0, 0, 0, 0};
            if (t + 1 < ncols) nxt = prepare(t + 1);
            const int32_t a1 = cur.a1, b1 = cur.b1, a2 = cur.a2, b2 = cur.b2;
            cur = nxt;
            int32_t lo = 0x7fffffff, hi = 0;
            if (b1 > a1) { lo = a1; hi = b1; }
            if (b2 > a2) { lo = a2 < lo ? a2 : lo; hi = b2 > hi ? b2 : hi; }
            const int32_t PA = wave_min_i32(lo), PB = wave_max_i32(hi);
            for (int32_t base = PA; base < PB; base += CHUNK) {
                const int32_t cnt_pts = PB - base < CHUNK ? PB - base : CHUNK;
                __syncthreads();
                for (int32_t i = lane; i < cnt_pts; i += kQueryBlock) {
                    // the staged form of a point is its record as the counting sort wrote it
                    float w[NV * 4];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const float4 f = a.rec[(int64_t)(base + i) * NV + v];
                        w[4 * v] = f.x; w[4 * v + 1] = f.y; w[4 * v + 2] = f.z; w[4 * v + 3] = f.w;
                    }
                    const int32_t src = __float_as_int(w[D]);
                    if (a.dir && !dir_is_neighbour(a.dir[src])) {          // never a neighbour: poison its coordinates
#pragma unroll
                        for (int c = 0; c < D; ++c) w[c] = __uint_as_float(0x7fc00000u);
                    }
#pragma unroll
                    for (int v = 0; v < NV; ++v) stage[i * NV + v] = make_float4(w[4 * v], w[4 * v + 1], w[4 * v + 2], w[4 * v + 3]);
                }
                __syncthreads();
                if constexpr (!FLAT) {
                // this lane's two sub-ranges clipped to the chunk, walked one after the other
                const int32_t top = base + cnt_pts;
                int32_t q = a1 > base ? a1 : base, e = b1 < top ? b1 : top;
                int32_t q2 = a2 > base ? a2 : base, e2 = b2 < top ? b2 : top;
                useful += (e > q ? e - q : 0) + (e2 > q2 ? e2 - q2 : 0);
                const bool second_runs = __any(e2 > q2);      // only the centre column (and shell 0) has two runs per lane
                for (;;) {
                    if (second_runs) {
                        // a real branch on the wave-uniform flag: as selects, the switch to the second run cost four
                        // vector instructions in every pass of every column
                        asm volatile("");
                        if (q >= e && q2 < e2) { q = q2; e = e2; q2 = e2; }
                    }
                    const int32_t rem = e - q;
                    if (!__any(rem > 0)) break;
                    float w[kUnroll][NV * 4];
                    const uint32_t tau_hi = (uint32_t)(s.tau >> 32);
                    const int32_t i0 = rem > 0 ? q - base : 0;       // reads past the lane's range stay inside the padded chunk
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            const float4 f = stage[(i0 + u) * NV + v];
                            w[u][4 * v] = f.x; w[u][4 * v + 1] = f.y; w[u][4 * v + 2] = f.z; w[u][4 * v + 3] = f.w;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        float diff = s.x[0] - w[u][0];
                        float d2 = diff * diff;
#pragma unroll
                        for (int c = 1; c < D; ++c) {
                            diff = s.x[c] - w[u][c];
                            d2 = d2 + diff * diff;
                        }
                        const bool live = u < rem;
                        if (COUNT) cand += live;
                        // kept if its distance does not exceed the k-th best's (a tie on the distance may lose
                        // on the index: the merge decides); NaN (poisoned) patterns lie above every bound
                        const uint32_t bits = __float_as_uint(d2);
                        if (live && bits <= tau_hi && (!LOWER || (((uint64_t)bits << 32) | __float_as_uint(w[u][D])) > lower)) {
                            // index word and distance word kPend planes apart, then the slot pointer moves on:
                            // written out because the compiler spends a third instruction on a register copy
                            static_assert(kPendHalf * 4 == 16 * 256 && kQueryBlock * 4 == 0x100, "offsets below");
                            asm volatile("ds_write2st64_b32 %0, %1, %2 offset1:16\n\tv_add_u32 %0, 0x100, %0"
                                         : "+v"(pend_top) : "v"(__float_as_uint(w[u][D])), "v"(bits) : "memory");
                        }
                    }
                    q += kUnroll;
                    ++passes;
                    if (__any(pend_top > pend_full)) absorb();
                }
                } else {
                // Flattened scan: the work of this chunk is dealt out evenly over the lanes, whichever query it belongs
                // to.  Every query's clipped run is cut into passes of kUnroll candidates; the passes of all queries
                // are put in one order (prefix sum over the lanes) and lane L takes passes [L*C, (L+1)*C) of it.  What
                // a lane keeps goes to the pending buffer of the query the pass belongs to (slots from a counter in
                // LDS), and that query's lane merges it as before.
                const int32_t top = base + cnt_pts;
                const int32_t q = a1 > base ? a1 : base, e = b1 < top ? b1 : top;
                const int32_t q2 = a2 > base ? a2 : base, e2 = b2 < top ? b2 : top;
                const int32_t len1 = e > q ? e - q : 0, len2 = e2 > q2 ? e2 - q2 : 0;
                useful += len1 + len2;
                if (COUNT) cand += len1 + len2;
                const bool second_runs = __any(len2 > 0);      // only the centre column (and shell 0) has two runs per lane
                for (int run = 0; run < 2; ++run) {
                    if (run == 1 && !second_runs) break;
                    const int32_t len = run ? len2 : len1;
                    const uint64_t m = __ballot(len > 0);
                    if (m == 0) continue;
                    const int32_t nq = __popcll(m);
                    const int32_t ng = (len + kUnroll - 1) / kUnroll;          // passes this run takes
                    const int32_t incl = wave_incl_scan_dpp_i32(ng);
                    const int32_t TG = __builtin_amdgcn_readlane(incl, kQueryBlock - 1);
                    __syncthreads();
                    if (len > 0) {
                        const int32_t rank = __popcll(m & lt_mask);
                        fl_start[rank] = incl - ng;
                        static_assert(CHUNK <= 512, "run start and length are packed in 10 bits each");
                        fl_info[rank] = ((run ? q2 : q) - base) | (len << 10) | (lane << 20);
                    }
                    if (lane >= nq) fl_start[lane] = 0x7fffffff;
                    __syncthreads();
                    const int32_t C = (TG + kQueryBlock - 1) / kQueryBlock;
                    int32_t f = lane * C;
                    const int32_t f_end = f + C < TG ? f + C : TG;
                    int32_t j = 0;
#pragma unroll
                    for (int step = 32; step > 0; step >>= 1)
                        if (fl_start[j + step] <= f) j += step;
                    int32_t run_end = f, pos = 0, left = 0, owner = lane;
                    float xq[D];
                    uint32_t tau_hi = 0;
                    // The lane's place in run j: where the run's candidates sit in the stage, how many are left, and
                    // the query it belongs to, whose coordinates and k-th best are read from that query's lane
                    // (cross-lane reads return nothing from a lane that is switched off: every lane executes this,
                    // lanes without work with a harmless run number, and `take` says who keeps the result).
                    auto load_run = [&](bool take) {
                        const int32_t info = fl_info[j];
                        const int32_t first = fl_start[j], nxt_start = fl_start[j + 1];
                        const int32_t from = info >> 20;
                        float xo[D];
#pragma unroll
                        for (int c = 0; c < D; ++c) xo[c] = __shfl(s.x[c], from, 64);
                        const uint32_t to = (uint32_t)__shfl((int)(uint32_t)(s.tau >> 32), from, 64);
                        if (take) {
                            owner = from;
                            pos = (info & 0x3ff) + (f - first) * kUnroll;
                            left = ((info >> 10) & 0x3ff) - (f - first) * kUnroll;
                            run_end = nxt_start < f_end ? nxt_start : f_end;
#pragma unroll
                            for (int c = 0; c < D; ++c) xq[c] = xo[c];
                            tau_hi = to;
                        }
                    };
#pragma unroll
                    for (int c = 0; c < D; ++c) xq[c] = 0.0f;
                    load_run(f < f_end);
                    for (;;) {
                        const bool busy = f < run_end;
                        if (!__any(busy)) break;
                        const int32_t rem = busy ? left : 0;
                        float w[kUnroll][NV * 4];
                        const int32_t i0 = busy ? pos : 0;          // reads past the run stay inside the padded chunk
#pragma unroll
                        for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
                            for (int v = 0; v < NV; ++v) {
                                const float4 g = stage[(i0 + u) * NV + v];
                                w[u][4 * v] = g.x; w[u][4 * v + 1] = g.y; w[u][4 * v + 2] = g.z; w[u][4 * v + 3] = g.w;
                            }
                        }
                        uint32_t bits[kUnroll];
                        bool acc[kUnroll];
                        int32_t na = 0;
                        uint64_t low = 0;
                        if (LOWER) low = qlower[owner];
#pragma unroll
                        for (int u = 0; u < kUnroll; ++u) {
                            float diff = xq[0] - w[u][0];
                            float d2 = diff * diff;
#pragma unroll
                            for (int c = 1; c < D; ++c) {
                                diff = xq[c] - w[u][c];
                                d2 = d2 + diff * diff;
                            }
                            bits[u] = __float_as_uint(d2);
                            // kept if its distance does not exceed the k-th best's (a tie on the distance may lose on
                            // the index: the merge decides); NaN (poisoned) patterns lie above every bound
                            acc[u] = u < rem && bits[u] <= tau_hi &&
                                     (!LOWER || (((uint64_t)bits[u] << 32) | __float_as_uint(w[u][D])) > low);
                            na += acc[u] ? 1 : 0;
                        }
                        bool fail = false, hot = false;
                        if (na > 0) {
                            const int32_t s0 = (int32_t)atomicAdd(&pend_cnt[owner], (uint32_t)na);
                            fail = s0 + na > kPend;                 // no room: nothing is stored, the pass is repeated
                            hot = s0 + na > kPend - kUnroll;        // the next pass might not fit
                            if (!fail) {
                                static_assert(kPendHalf * 4 == 16 * 256 && kQueryBlock * 4 == 0x100, "offsets below");
                                uint32_t wptr = (pend_base - (uint32_t)lane * 4u) + (uint32_t)owner * 4u + (uint32_t)s0 * (kQueryBlock * 4u);
#pragma unroll
                                for (int u = 0; u < kUnroll; ++u) {
                                    if (acc[u]) {
                                        asm volatile("ds_write2st64_b32 %0, %1, %2 offset1:16\n\tv_add_u32 %0, 0x100, %0"
                                                     : "+v"(wptr) : "v"(__float_as_uint(w[u][D])), "v"(bits[u]) : "memory");
                                    }
                                }
                            }
                        }
                        if (busy && !fail) { ++f; pos += kUnroll; left -= kUnroll; }
                        ++passes;
                        const bool merge = __any(hot);
                        if (merge) { __syncthreads(); absorb(); }
                        const bool next_run = f >= run_end && f < f_end;
                        if (__any(next_run)) {
                            if (next_run) ++j;
                            load_run(next_run);
                        }
                        if (merge) tau_hi = (uint32_t)__shfl((int)(uint32_t)(s.tau >> 32), owner, 64);   // tightened by the merge
                    }
                }
                }
            }
        }
        // After shell 0 a lane can only be certified with a full list: where no lane has met as many candidates as its
        // list holds, the few pending keys wait for the first merge of shell 1 (the k-th best stays open either way).
        if (R == 0 && !__any(active && useful >= cap)) continue;
        if constexpr (FLAT) {
            __syncthreads();
            if (__any(pend_cnt[lane] != 0)) absorb();
        } else {
            if (__any(pend_top != pend_base)) absorb();
        }
        if (active && s.certified(R)) active = false;
        const int32_t n_active = __popcll(__ballot(active));
        if (n_active == 0) break;
        if (R >= 1) {
            // Go on to the next shell in this wave only if that is efficient.  Shell R + 1 costs the whole wave
            // (2R+3)^(DB-1) columns however few of its lanes still search, and the list kernel takes a query
            // from where it stands for a few microseconds of one wavefront: beyond two binning dimensions the
            // wave goes on only while most of its lanes (48 of 64) are unfinished (grids made for two shells, as
            // for d >= 6, or a fine grid on uniform data); measured on 1M uniform points, d = 5: 4.5 -> 3.5 ms,
            // d = 6: 14.2 -> 13.3 ms against the previous rule of 7 lanes.  With two binning dimensions the next
            // shell is a handful of long columns and 7 lanes are enough.  In either case the lanes must have
            // been evenly loaded so far (candidates evaluated vs lane slots spent): an uneven tile (sparse lanes
            // next to a dense cluster) keeps 64 lanes waiting for a few.
            if (n_active <= a.defer_lanes) break;
            if (DB > 2 && n_active < kContinueLanes) break;
            const int32_t spent = passes * kUnroll;
            if (wave_sum_i32(useful) * 5 < spent * kQueryBlock * 2) break;     // below 40 % lane use
        }
    }

    // unfinished lanes are marked for the work list, which a small kernel then writes in tile order, i.e. bin
    // order (appending here, in the order the tiles happen to finish, left neighbouring wavefronts of the list
    // kernel with unrelated queries); their lists so far leave with the finished rows, and the first shell still
    // to search travels in slot 0 of the distance row
    const uint64_t mask = __ballot(active);
    if (lane == 0) a.handed[tile] = mask;
    const uint32_t resume_word = (uint32_t)(R + 1);
    // Rows of exactly KC words (K = 16, 32, 48, 64) leave straight from the registers: every lane writes its own
    // row in 16-byte pieces (the pieces of a 128-byte line arrive within a few instructions of each other and are
    // joined in the L2 cache).  A sixteenth of the instructions of the transposition below: query stage -8 % at
    // K = 16, -4 % at K = 32, +-0 at K = 64.  Rows that do not start on a 64-byte boundary (K = 40: 160 bytes)
    // were 3 % slower this way and keep the transposition.
    const bool direct_rows = a.slot0 == 0 && a.k == KC && cap == KC - 1 &&
                             (((uintptr_t)a.out_idx | (uintptr_t)a.out_d2) & 15) == 0;
    if (direct_rows) {
        if (COUNT && valid) a.out_cand[my_row] = LOWER ? a.out_cand[my_row] + cand : cand;
        if (valid) {
            int32_t* oi = a.out_idx + (int64_t)my_row * a.k;
            float* od = a.out_d2 + (int64_t)my_row * a.k;
            const int32_t idx0 = asks ? my_row : -1;
            const uint32_t d2_0 = ((mask >> lane) & 1) ? resume_word : 0u;     // handed over: where to resume
            store_row_from_registers<KC, 1>(best, oi, od, idx0, d2_0);
        }
    } else {
    // otherwise: registers -> LDS -> contiguous row writes
    __syncthreads();
    // two passes (indices, then distances) so the transposition needs KC x 64 words, not keys
    int32_t* rows_lds = reinterpret_cast<int32_t*>(lds64);
    uint32_t* dump = reinterpret_cast<uint32_t*>(lds64) + kQueryBlock;     // [KC][64] after the 64 row words
    rows_lds[lane] = valid ? (asks ? my_row : -2 - my_row) : -1;   // -1: nothing to write; <= -2: all-padding row
    if (COUNT && valid) a.out_cand[my_row] = LOWER ? a.out_cand[my_row] + cand : cand;
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
                uint32_t word = pass == 0 ? (enc >= 0 ? (uint32_t)row : 0xffffffffu) : 0u;   // slot 0: the row itself at distance 0
                if (pass == 1 && ((mask >> ql) & 1)) word = resume_word;                     // handed over: where to resume
                if (j > 0) word = dump[(KC - cap + j - 1) * kDumpStride + ql];
                const int32_t slot = j > 0 ? a.slot0 + j : 0;
                if (pass == 0) a.out_idx[(int64_t)row * k + slot] = (int32_t)word;
                else a.out_d2[(int64_t)row * k + slot] = __uint_as_float(word);
            }
        }
    }
    }
}

// The kernel: one workgroup of one wavefront per tile.  Tiles the ordering kernels marked as uneven take the
// flattened scan, all others, and every tile of an unordered launch, the direct one.  One kernel with a branch,
// not two kernels: a tile alone takes ~0.1 ms from its first shell to its last row whatever runs beside it, so a
// second kernel for the uneven tiles adds its whole tail.  a.algo == 2 sends every tile to the flattened scan
// (tests).  The counting instantiation scans directly.
template <int D, int DB, int KC, bool COUNT, bool LOWER>
__global__ void __launch_bounds__(kQueryBlock) __attribute__((amdgpu_waves_per_eu(tile_waves<KC, D>(), tile_waves<KC, D>())))
k_query_tile_sorted(QueryArgs a)
{
    extern __shared__ uint64_t lds64[];
    // an entry of the order: the tile, heaviest first, and above it the flag of an uneven tile
    const int32_t entry = a.tile_order ? a.tile_order[blockIdx.x] : (int32_t)blockIdx.x;
    const int32_t tile = entry & ((1 << kOrderFlagBit) - 1);
    if constexpr (!COUNT && tile_has_flat<KC, D>()) {
        const bool uneven = a.algo == 2 || ((entry >> kOrderFlagBit) & 1);
        if (uneven) {
            tile_body<D, DB, KC, COUNT, LOWER, true>(a, tile, lds64);
            return;
        }
    }
    tile_body<D, DB, KC, COUNT, LOWER, false>(a, tile, lds64);
}

template <int KC, int D>
constexpr size_t tile_sorted_lds_bytes()
{
    const size_t flat = kPendBytes + (size_t)stage_vecs<D>() * 16 * (flat_chunk<KC, D>() + kUnroll) + kFlatTables;
    const size_t direct = kPendBytes + (size_t)stage_vecs<D>() * 16 * (direct_chunk<KC, D>() + kUnroll);
    const size_t out = (size_t)kQueryBlock * 4 + (size_t)KC * kDumpStride * 4;
    const size_t scan = (tile_has_flat<KC, D>() && flat > direct) ? flat : direct;
    return scan > out ? scan : out;
}

}  // namespace fg
