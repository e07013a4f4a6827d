// Tile kernel for six and more coordinates: the candidates of a tile are FILTERED on the matrix cores.
//
// From d = 6 on a grid prunes little (the paper's Section 4 shows the same for its own kernel): a query of 1M uniform
// points in 8 dimensions meets some 15 000 candidates, of which a few hundred ever enter its list, and the queries of
// a tile share most of them.  That is a dense contraction: for a chunk of staged candidates and the 64 queries of
// the tile, d2(q, c) = |q|^2 + |c|^2 - 2 q.c, the q.c of 32 candidates x 32 queries from one chain of
// v_mfma_f32_32x32x2_f32 (two coordinates per instruction).  The matrix result is NOT the distance of the definition
// (which is a left-to-right float32 sum of squared differences): it is used only to discard pairs that provably
// cannot enter the list,
//     |c|^2 - 2 q.c  >  kth * (1 + 2^-19) - |q|^2 + 2^-17 (|q|^2 + max |c|^2),
// all norms and products taken on coordinates centred on the tile's first query, so that the rounding errors of
// the expanded form (at most (d + 8) 2^-23 (|q|^2 + |c|^2), against the 2^-17 allowed for) scale with the size of
// the neighbourhood and not with the distance from the origin.  Every pair that survives is evaluated again exactly as
// the direct scan does it (original coordinates, separately rounded operations, the lane's own candidate ranges,
// the 32-bit compare with the k-th best), so the results are bit for bit those of the other kernels.
//
// Layout: one wavefront per tile of 64 bin-ordered queries, shells, columns, per-lane candidate ranges, the union
// range staged in chunks, pending buffers, the sorted register list and the hand-over exactly as in the direct
// kernel.  A chunk is staged as structure-of-arrays (one row of the chunk per coordinate, so that the 32 lanes of a
// matrix operand read consecutive words), with |c|^2 and the original row index beside it.  Candidates are the rows
// of the matrix product, queries its columns: a lane then holds 16 candidates of ONE query (lanes l and l + 32
// share query l mod 32), and compares them with that query's bound.  Survivors are queued in LDS as (candidate,
// query) codes and checked exactly 64 at a time, whichever query they belong to; what passes goes to the pending
// buffer of its query (slot from a per-query counter) and that query's lane merges it as before.
#pragma once
#include "fg_query_tile.hpp"

namespace fg {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMfmaQueue = 256;                                         // survivor codes waiting for the exact check
template <int D> constexpr int mfma_steps() { return (D + 1) / 2; }     // matrix instructions per product: 2 coordinates each
template <int D> constexpr int mfma_rows() { return 2 * mfma_steps<D>(); }   // coordinate rows of the stage (odd d: one of zeros)
constexpr size_t kMfmaLdsBudget = 20480;                                // two wavefronts per SIMD: eight workgroups per CU
// pending keys, counters, bounds, k-th bests, candidate ranges, survivor queue, lower bounds of a second pass
constexpr size_t kMfmaTables = kPendBytes + 3 * kQueryBlock * 4 + 4 * kQueryBlock * 4 + kMfmaQueue * 4 + kQueryBlock * 8;
template <int D> constexpr int mfma_chunk()
{
    const size_t room = kMfmaLdsBudget - kMfmaTables - (size_t)D * kQueryBlock * 4;   // the queries' coordinates
    const int c = (int)(room / ((size_t)(mfma_rows<D>() + 2) * 4)) / 32 * 32;
    return c > 224 ? 224 : c;
}
template <int KC, int D> constexpr size_t tile_mfma_lds_bytes()
{
    const size_t scan = kMfmaTables + (size_t)D * kQueryBlock * 4 + (size_t)(mfma_rows<D>() + 2) * 4 * mfma_chunk<D>();
    const size_t out = (size_t)kQueryBlock * 4 + (size_t)KC * kDumpStride * 4;
    return scan > out ? scan : out;
}

__device__ __forceinline__ float wave_max_f32(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <int D, int DB, int KC, bool COUNT, bool LOWER>
__global__ void __launch_bounds__(kQueryBlock) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_query_tile_mfma(QueryArgs a)
{
    extern __shared__ uint64_t lds64[];
    static_assert(D >= 6 && mfma_chunk<D>() >= 64 && mfma_chunk<D>() <= 256, "chunk positions are coded in 8 bits");
    constexpr int C = mfma_chunk<D>();
    constexpr int STEPS = mfma_steps<D>();
    constexpr int ROWS = mfma_rows<D>();
    const int32_t entry = a.tile_order ? a.tile_order[blockIdx.x] : (int32_t)blockIdx.x;
    const int32_t tile = entry & ((1 << kOrderFlagBit) - 1);
    const int lane = threadIdx.x;
    const int half = lane >> 5, col = lane & 31;
    const uint64_t lt_mask = (1ull << lane) - 1;

    // LDS: [pending kPend x 64 keys][counters][bounds][k-th bests][ranges 4 x 64][queue][lower bounds]
    //      [query coordinates D x 64][stage: ROWS x C coordinates, C norms, C row indices]
    uint32_t* const pend_lds = reinterpret_cast<uint32_t*>(lds64);          // index words [kPend][64], distance words [kPend][64]
    constexpr int kPendHalf = kPend * kQueryBlock;
    uint32_t* const pend_cnt = pend_lds + 2 * kPendHalf;
    float* const thr_base = reinterpret_cast<float*>(pend_cnt + kQueryBlock);
    uint32_t* const tau_tab = reinterpret_cast<uint32_t*>(thr_base + kQueryBlock);
    int32_t* const rng = reinterpret_cast<int32_t*>(tau_tab + kQueryBlock);   // [4][64]: a1, b1, a2, b2
    uint32_t* const queue = reinterpret_cast<uint32_t*>(rng + 4 * kQueryBlock);
    uint64_t* const qlower = reinterpret_cast<uint64_t*>(queue + kMfmaQueue);
    float* const xq = reinterpret_cast<float*>(qlower + kQueryBlock);         // [D][64] original coordinates
    float* const xs = xq + D * kQueryBlock;                                    // [ROWS][C] original coordinates
    float* const cn = xs + ROWS * C;                                           // [C] squared norms of the centred candidates
    int32_t* const idxs = reinterpret_cast<int32_t*>(cn + C);                  // [C] original rows

    const int32_t cap = a.k_list;
    const int32_t p = tile * kQueryBlock + lane;
    const bool valid = p < a.n;
    LaneGeom<D, DB> s;
    const int32_t my_row = s.init_geom(a, valid ? p : a.n - 1);
    const bool asks = !(a.dir && !dir_is_query(a.dir[my_row]));
    bool active = valid && cap > 0 && asks;
    uint64_t lower = 0;
    if (LOWER && active) {
        const int32_t li = a.out_idx[(int64_t)my_row * a.k + a.slot0];
        lower = li < 0 ? kEmptyKey : (((uint64_t)__float_as_uint(a.out_d2[(int64_t)my_row * a.k + a.slot0]) << 32) | (uint32_t)li);
    }
    uint64_t best[KC];
#pragma unroll
    for (int i = 0; i < KC; ++i) best[i] = (i < KC - cap) ? 0ull : kEmptyKey;
#pragma unroll
    for (int i = 0; i < kPend; ++i) pend_lds[kPendHalf + i * kQueryBlock + lane] = (uint32_t)(kEmptyKey >> 32);
    pend_cnt[lane] = 0;
    if (LOWER) qlower[lane] = lower;

    // origin of the centred coordinates: the tile's first query (lane 0 always holds a point)
    float org[ROWS];
#pragma unroll
    for (int c = 0; c < ROWS; ++c)
        org[c] = c < D ? __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s.x[c < D ? c : 0]))) : 0.0f;
    float qn = 0.0f;
#pragma unroll
    for (int c = 0; c < D; ++c) {
        xq[c * kQueryBlock + lane] = s.x[c];
        const float t = s.x[c] - org[c];
        qn = fmaf(t, t, qn);
    }
    // what the matrix result of a candidate has to stay under, but for the chunk's share of the error allowance
    auto publish = [&]() __attribute__((always_inline)) {
        float t = -__builtin_inff();                          // a lane that does not search keeps nothing
        if (active)                                           // a list still short of keys keeps everything
            t = s.tau < kEmptyKey ? s.tau_d2() * 1.0000019073486328f - qn + 7.62939453125e-06f * qn : __builtin_inff();
        thr_base[lane] = t;
        tau_tab[lane] = (uint32_t)(s.tau >> 32);
    };
    publish();
    __syncthreads();
    // this lane's operand of the queries' side: query 32 * b + col, coordinate 2 * step + half, centred
    float qb[2][STEPS];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int k0 = 2 * st, k1 = 2 * st + 1;
            const float v0 = xq[k0 * kQueryBlock + 32 * b + col] - org[k0];
            const float v1 = k1 < D ? xq[(k1 < D ? k1 : 0) * kQueryBlock + 32 * b + col] - org[k1] : 0.0f;
            qb[b][st] = half ? v1 : v0;
        }

    int32_t cand = 0;
    int32_t nq = 0;                  // survivor codes in the queue (wave-uniform)
    int32_t base = 0;                // first sorted position of the staged chunk

    auto absorb = [&]() __attribute__((always_inline)) {            // every lane merges its pending keys; counters, bounds and k-th bests renewed
        uint64_t pend[kPend];
#pragma unroll
        for (int i = 0; i < kPend; ++i)
            pend[i] = ((uint64_t)pend_lds[kPendHalf + i * kQueryBlock + lane] << 32) | pend_lds[i * kQueryBlock + lane];
#pragma unroll
        for (int i = 0; i < kPend; ++i) pend_lds[kPendHalf + i * kQueryBlock + lane] = (uint32_t)(kEmptyKey >> 32);
        net_sort<kPend>(pend);
        net_absorb<KC, kPend>(best, pend);
        s.tau = best[KC - 1];
        pend_cnt[lane] = 0;
        publish();
        __syncthreads();
    };

    // The exact check of the queued survivors, 64 at a time: the candidate must lie in one of its query's ranges for
    // this column, its distance as the definition computes it must not exceed the query's k-th best, and what passes
    // takes the next slot of the query's pending buffer.  A full buffer makes every lane merge; codes that found no
    // slot go back into the queue and are taken again afterwards.
    auto drain = [&]() __attribute__((always_inline)) {
        while (nq > 0) {
            const int32_t m = nq < kQueryBlock ? nq : kQueryBlock;
            const int32_t start = nq - m;
            const bool has = lane < m;
            const uint32_t code = has ? queue[start + lane] : 0u;
            const int32_t owner = (int32_t)(code >> 8), ci = (int32_t)(code & 255u);
            const int32_t pos = base + ci;
            const int32_t a1 = rng[owner], b1 = rng[kQueryBlock + owner], a2 = rng[2 * kQueryBlock + owner], b2 = rng[3 * kQueryBlock + owner];
            bool ok = has && ((pos >= a1 && pos < b1) || (pos >= a2 && pos < b2));
            float diff = xq[owner] - xs[ci];
            float d2 = diff * diff;
#pragma unroll
            for (int c = 1; c < D; ++c) {
                diff = xq[c * kQueryBlock + owner] - xs[c * C + ci];
                d2 = d2 + diff * diff;
            }
            const uint32_t bits = __float_as_uint(d2);
            const uint32_t src = (uint32_t)idxs[ci];
            ok = ok && bits <= tau_tab[owner];
            if (LOWER) ok = ok && (((uint64_t)bits << 32) | src) > qlower[owner];
            nq = start;
            int32_t slot = 0;
            if (ok) slot = (int32_t)atomicAdd(&pend_cnt[owner], 1u);
            const bool fail = ok && slot >= kPend;
            if (ok && !fail) {
                pend_lds[slot * kQueryBlock + owner] = src;
                pend_lds[kPendHalf + slot * kQueryBlock + owner] = bits;
            }
            const uint64_t mf = __ballot(fail);
            if (mf) {
                if (fail) queue[nq + __popcll(mf & lt_mask)] = code;
                nq += __popcll(mf);
            }
            if (__any(ok && slot >= kPend - 1)) {
                __syncthreads();
                absorb();
            }
        }
    };

    int32_t R = 0;
    for (;; ++R) {
        const int32_t side = 2 * R + 1;
        int32_t ncols = 1;
#pragma unroll
        for (int c = 0; c < DB - 1; ++c) ncols *= side;
        // this lane's candidate ranges for column t of shell R (as in the direct kernel: whole bins narrowed by the
        // box bound, cut to the slices the k-th best still reaches)
        auto prepare = [&](int32_t t) -> Ranges {
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
                const int32_t sh = a.sub_shift;
                const int32_t row0 = s.bounds_at(flat, 0);
                int32_t s_lo = 0, s_hi = 0x7ffffffe;
                if (R > 0 && sh > 0) s.slice_reach(partial, s_lo, s_hi);
                auto cut_run = [&](int32_t z_first, int32_t z_last, int32_t& from, int32_t& to) {
                    const int32_t fa = (z_first << sh) > s_lo ? (z_first << sh) : s_lo;
                    const int32_t fb = ((z_last + 1) << sh) < s_hi + 1 ? ((z_last + 1) << sh) : s_hi + 1;
                    if (fb > fa) { from = a.bounds[row0 + fa]; to = a.bounds[row0 + fb]; }
                };
                if (surf) {
                    int32_t za = cz - R < 0 ? 0 : cz - R;
                    int32_t zb = cz + R > nz - 1 ? nz - 1 : cz + R;
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
            Ranges nxt = Ranges{0, 0, 0, 0};
            if (t + 1 < ncols) nxt = prepare(t + 1);
            const int32_t a1 = cur.a1, b1 = cur.b1, a2 = cur.a2, b2 = cur.b2;
            cur = nxt;
            int32_t lo = 0x7fffffff, hi = 0;
            if (b1 > a1) { lo = a1; hi = b1; }
            if (b2 > a2) { lo = a2 < lo ? a2 : lo; hi = b2 > hi ? b2 : hi; }
            const int32_t PA = wave_min_i32(lo), PB = wave_max_i32(hi);
            if (PB <= PA) continue;
            if (COUNT) cand += (b1 > a1 ? b1 - a1 : 0) + (b2 > a2 ? b2 - a2 : 0);
            __syncthreads();
            rng[lane] = a1; rng[kQueryBlock + lane] = b1; rng[2 * kQueryBlock + lane] = a2; rng[3 * kQueryBlock + lane] = b2;
            for (base = PA; base < PB; base += C) {
                const int32_t cnt_pts = PB - base < C ? PB - base : C;
                const int32_t n_rb = (cnt_pts + 31) >> 5;
                __syncthreads();
                float cn_max = 0.0f;
                for (int32_t i = lane; i < n_rb * 32; i += kQueryBlock) {
                    constexpr int NV = rec_vecs(D);
                    float w[NV * 4];
                    int32_t src = -1;
                    float norm = __uint_as_float(0x7fc00000u);   // padding rows: not a number, under no bound
                    if (i < cnt_pts) {
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            const float4 f = a.rec[(int64_t)(base + i) * NV + v];
                            w[4 * v] = f.x; w[4 * v + 1] = f.y; w[4 * v + 2] = f.z; w[4 * v + 3] = f.w;
                        }
                        src = __float_as_int(w[D]);
                        if (a.dir && !dir_is_neighbour(a.dir[src])) {          // never a neighbour: poison its coordinates
#pragma unroll
                            for (int c = 0; c < D; ++c) w[c] = __uint_as_float(0x7fc00000u);
                        }
                        norm = 0.0f;
#pragma unroll
                        for (int c = 0; c < D; ++c) {
                            const float tc = w[c] - org[c];
                            norm = fmaf(tc, tc, norm);
                        }
                        if (norm < __builtin_inff()) cn_max = fmaxf(cn_max, norm);       // (false for a poisoned point)
                    } else {
#pragma unroll
                        for (int c = 0; c < D; ++c) w[c] = org[c];
                    }
#pragma unroll
                    for (int c = 0; c < D; ++c) xs[c * C + i] = w[c];
                    if (ROWS > D) xs[D * C + i] = 0.0f;
                    cn[i] = norm;
                    idxs[i] = src;
                }
                const float slack = 7.62939453125e-06f * wave_max_f32(cn_max);      // 2^-17 of the largest norm staged
                __syncthreads();
                for (int32_t rb = 0; rb < n_rb; ++rb) {
                    // the two blocks of 32 queries one after the other: 16 results live at a time (with both in flight
                    // the 64-key kernel spilled 230 registers)
                    uint32_t keep = 0;                 // bit 16 b + v: candidate v of query block b survives
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        floatx16 acc = {0};
#pragma unroll
                        for (int st = 0; st < STEPS; ++st) {
                            const float o0 = org[2 * st], o1 = org[2 * st + 1];
                            const float av = xs[(2 * st + half) * C + 32 * rb + col] - (half ? o1 : o0);
                            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, qb[b][st], acc, 0, 0, 0);
                        }
                        const float thr = thr_base[32 * b + col] + slack;
                        // A query whose list is still short of keys keeps everything: for it the candidates are cut to
                        // its own ranges here already (four consecutive positions per group against two intervals),
                        // or every candidate of the chunk would go through the exact check for every such query.
                        uint32_t allowed = 0xffffu;
                        if (__any(thr == __builtin_inff())) {
                            const int32_t q = 32 * b + col;
                            const int32_t r_a1 = rng[q], r_b1 = rng[kQueryBlock + q], r_a2 = rng[2 * kQueryBlock + q], r_b2 = rng[3 * kQueryBlock + q];
                            uint32_t inside = 0;
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                const int32_t pos0 = base + 32 * rb + 8 * g + 4 * half;
                                auto piece = [&](int32_t from, int32_t to) -> uint32_t {       // bits of pos0 .. pos0 + 3 inside [from, to)
                                    int32_t lo = from - pos0, hi = to - pos0;
                                    lo = lo < 0 ? 0 : (lo > 4 ? 4 : lo);
                                    hi = hi < 0 ? 0 : (hi > 4 ? 4 : hi);
                                    return ((1u << hi) - 1u) & ~((1u << lo) - 1u);
                                };
                                inside |= (piece(r_a1, r_b1) | piece(r_a2, r_b2)) << (4 * g);
                            }
                            if (thr == __builtin_inff()) allowed = inside;
                        }
                        // rows of this lane's 16 results: 8 g + 4 half + t, g, t = 0..3
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const float4 f = *reinterpret_cast<const float4*>(cn + 32 * rb + 8 * g + 4 * half);
                            if (fmaf(acc[4 * g], -2.0f, f.x) <= thr) keep |= 1u << (16 * b + 4 * g);
                            if (fmaf(acc[4 * g + 1], -2.0f, f.y) <= thr) keep |= 1u << (16 * b + 4 * g + 1);
                            if (fmaf(acc[4 * g + 2], -2.0f, f.z) <= thr) keep |= 1u << (16 * b + 4 * g + 2);
                            if (fmaf(acc[4 * g + 3], -2.0f, f.w) <= thr) keep |= 1u << (16 * b + 4 * g + 3);
                        }
                        keep &= (allowed << (16 * b)) | (b ? 0xffffu : 0xffff0000u);
                    }
                    while (__any(keep != 0)) {
                        const bool on = keep != 0;
                        const int32_t bit = on ? __ffs((int)keep) - 1 : 0;
                        keep &= keep - 1;
                        const int32_t v = bit & 15;
                        const uint32_t code = (uint32_t)(32 * rb + 8 * (v >> 2) + 4 * half + (v & 3)) |
                                              ((uint32_t)(32 * (bit >> 4) + col) << 8);
                        const uint64_t mq = __ballot(on);
                        if (on) queue[nq + __popcll(mq & lt_mask)] = code;
                        nq += __popcll(mq);
                        if (nq > kMfmaQueue - kQueryBlock) {
                            __syncthreads();
                            drain();
                        }
                    }
                }
                __syncthreads();
                drain();
            }
        }
        __syncthreads();
        if (__any(pend_cnt[lane] != 0)) absorb();
        if (active && s.certified(R)) {
            active = false;
            publish();
        }
        const int32_t n_active = __popcll(__ballot(active));
        if (n_active == 0) break;
        if (R >= 1) {
            // as in the direct kernel: the next shell costs the whole wave however few of its lanes still search
            if (n_active <= a.defer_lanes) break;
            if (DB > 2 && n_active < kContinueLanes) break;
        }
    }

    // hand-over and output: as in the direct kernel
    __syncthreads();
    const uint64_t mask = __ballot(active);
    if (mask) {
        int32_t wbase = 0;
        const int leader = __ffsll((unsigned long long)mask) - 1;
        if (lane == leader) wbase = atomicAdd(a.work_count, __popcll(mask));
        wbase = __shfl(wbase, leader, 64);
        if (active) a.work_list[wbase + __popcll(mask & lt_mask)] = p;
    }
    const uint32_t resume_word = (uint32_t)(R + 1);
    const bool direct_rows = a.slot0 == 0 && a.k == KC && cap == KC - 1 &&
                             (((uintptr_t)a.out_idx | (uintptr_t)a.out_d2) & 15) == 0;
    if (COUNT && valid) a.out_cand[my_row] = LOWER ? a.out_cand[my_row] + cand : cand;
    if (direct_rows) {
        if (valid) {
            int32_t* oi = a.out_idx + (int64_t)my_row * a.k;
            float* od = a.out_d2 + (int64_t)my_row * a.k;
            const int32_t idx0 = asks ? my_row : -1;
            const uint32_t d2_0 = ((mask >> lane) & 1) ? resume_word : 0u;
            store_row_from_registers<KC, 1>(best, oi, od, idx0, d2_0);
        }
        return;
    }
    int32_t* rows_lds = reinterpret_cast<int32_t*>(lds64);
    uint32_t* dump = reinterpret_cast<uint32_t*>(lds64) + kQueryBlock;
    rows_lds[lane] = valid ? (asks ? my_row : -2 - my_row) : -1;
    const int32_t k = a.k;
    const int32_t kk = cap + 1;
    const int32_t per_iter = kk >= kQueryBlock ? 1 : kQueryBlock / kk;
    const int32_t sub = lane / kk;
    const int32_t j0 = lane - sub * kk;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads();
#pragma unroll
        for (int i = 0; i < KC; ++i) {
            const bool real = best[i] < kEmptyKey;
            const uint32_t word = pass == 0 ? (real ? (uint32_t)best[i] : 0xffffffffu) : (real ? (uint32_t)(best[i] >> 32) : 0u);
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
                uint32_t word = pass == 0 ? (enc >= 0 ? (uint32_t)row : 0xffffffffu) : 0u;
                if (pass == 1 && ((mask >> ql) & 1)) word = resume_word;
                if (j > 0) word = dump[(KC - cap + j - 1) * kDumpStride + ql];
                const int32_t slot = j > 0 ? a.slot0 + j : 0;
                if (pass == 0) a.out_idx[(int64_t)row * k + slot] = (int32_t)word;
                else a.out_d2[(int64_t)row * k + slot] = __uint_as_float(word);
            }
        }
    }
}

}  // namespace fg
