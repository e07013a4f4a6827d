// Object-condensation index matrices (paper Section 5, Algorithm 3).
//
// For every object candidate k the vertices of its row split are walked from `tid` vertices
// into the window, wrapping round; members go to row k of M, non-members to row k of M_not,
// both padded with -1.  Entry `fill` of row k is stored at fill * n_unique + k (the paper's
// index macro), so neighbouring objects are neighbouring addresses.
//
// The paper runs one thread per object over its whole row split: with a few thousand objects
// that is a few dozen wavefronts, each a chain of 1e5 dependent steps.  Here the walk is cut
// into chunks so that (objects / 64) x (chunks) wavefronts run at once:
//   count    members of object k inside walk chunk c                    -> counts[c][k]
//   scan     exclusive prefix over the chunks of every object           -> members before chunk c, total
//   members  walk chunk c again and write the members at their final row of M; pad M with -1
//   others   for a block of 128 OUTPUT rows of M_not: find the chunk where the object's
//            non-member count reaches the block's first row (binary search in the prefix), walk
//            from there, emit 128 non-members.  In every step the 64 lanes (64 neighbouring
//            objects) write the same row: one contiguous 256-byte store.
// Lanes are objects throughout, so objects of one row split read neighbouring vertices.
// Integer-only; bound by the M_not write stream (n_unique x n_maxrs words).
// Without a workspace the single-kernel form of the paper is used.
#include "fg_internal.hpp"

namespace fg {

constexpr int kOcBlock = 64;
constexpr int kOcBatch = 8;       // independent loads kept in flight per lane
constexpr int kOcChunk = 128;     // walk positions per chunk, and output rows per block of the M_not kernel

struct OcWindow { int32_t uq, start, len, rot; };

__device__ __forceinline__ OcWindow oc_window(int32_t k, const int32_t* __restrict__ unique_idx,
                                              const int32_t* __restrict__ unique_rs_asso, const int32_t* __restrict__ rs,
                                              int32_t n_vert, int32_t n_splits, int32_t n_maxrs, int32_t rot_block)
{
    OcWindow w;
    w.uq = unique_idx[k];
    int32_t split = unique_rs_asso[k];
    split = split < 0 ? 0 : (split >= n_splits ? n_splits - 1 : split);    // out-of-range split: clamped, never read outside rs
    int32_t start = rs[split], end = rs[split + 1];
    start = start < 0 ? 0 : start;
    if (end > n_vert) end = n_vert;
    if (end - start > n_maxrs) end = start + n_maxrs;
    w.start = start;
    w.len = end > start ? end - start : 0;
    const int32_t tid = k % rot_block;
    w.rot = tid < w.len ? tid : 0;          // a start past the window means the window in order
    return w;
}

// vertex at walk position p (0 <= p < len)
__device__ __forceinline__ int32_t oc_vertex(const OcWindow& w, int32_t p)
{
    int32_t o = w.rot + p;
    if (o >= w.len) o -= w.len;
    return w.start + o;
}

// ---- single kernel, one lane per object (no workspace) ---------------------------------------
__global__ void __launch_bounds__(kOcBlock)
k_oc_helper(const int32_t* __restrict__ asso_idx, const int32_t* __restrict__ unique_idx,
            const int32_t* __restrict__ unique_rs_asso, const int32_t* __restrict__ rs, int32_t n_vert,
            int32_t n_unique, int32_t n_splits, int32_t n_maxuq, int32_t n_maxrs, int32_t calc_m_not,
            int32_t rot_block, int32_t* __restrict__ M, int32_t* __restrict__ M_not)
{
    const int32_t k = blockIdx.x * kOcBlock + threadIdx.x;
    if (k >= n_unique) return;
    const OcWindow w = oc_window(k, unique_idx, unique_rs_asso, rs, n_vert, n_splits, n_maxrs, rot_block);
    int32_t fill = 0, fill_not = 0;
    for (int32_t p = 0; p < w.len; ++p) {
        const int32_t i = oc_vertex(w, p);
        if (asso_idx[i] == w.uq) {
            if (fill < n_maxuq) { M[(int64_t)fill * n_unique + k] = i; ++fill; }
        } else if (calc_m_not) {
            M_not[(int64_t)fill_not * n_unique + k] = i;      // fill_not < len <= n_maxrs
            ++fill_not;
        }
    }
    for (; fill < n_maxuq; ++fill) M[(int64_t)fill * n_unique + k] = -1;
    if (calc_m_not)
        for (; fill_not < n_maxrs; ++fill_not) M_not[(int64_t)fill_not * n_unique + k] = -1;
}

// ---- chunked form ----------------------------------------------------------------------------
// grid (object groups, chunks); counts[c][k] = members of k at walk positions [c*C, (c+1)*C)
__global__ void __launch_bounds__(kOcBlock)
k_oc_count(const int32_t* __restrict__ asso_idx, const int32_t* __restrict__ unique_idx,
           const int32_t* __restrict__ unique_rs_asso, const int32_t* __restrict__ rs, int32_t n_vert, int32_t n_unique,
           int32_t n_splits, int32_t n_maxrs, int32_t rot_block, int32_t* __restrict__ counts)
{
    const int32_t k = blockIdx.x * kOcBlock + threadIdx.x;
    if (k >= n_unique) return;
    const OcWindow w = oc_window(k, unique_idx, unique_rs_asso, rs, n_vert, n_splits, n_maxrs, rot_block);
    const int32_t p0 = blockIdx.y * kOcChunk;
    const int32_t p1 = p0 + kOcChunk < w.len ? p0 + kOcChunk : w.len;
    int32_t c = 0;
    for (int32_t pb = p0; pb < p1; pb += kOcBatch) {       // loads of a batch are independent: all in flight at once
        int32_t v[kOcBatch];
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) v[u] = pb + u < p1 ? asso_idx[oc_vertex(w, pb + u)] : ~w.uq;
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) c += v[u] == w.uq;
    }
    counts[(int64_t)blockIdx.y * n_unique + k] = c;
}

// one lane per object: counts[c][k] -> members before chunk c; counts[n_chunks][k] = all members
__global__ void __launch_bounds__(kOcBlock)
k_oc_scan(int32_t* __restrict__ counts, int32_t n_unique, int32_t n_chunks)
{
    const int32_t k = blockIdx.x * kOcBlock + threadIdx.x;
    if (k >= n_unique) return;
    int32_t run = 0;
    for (int32_t cb = 0; cb < n_chunks; cb += kOcBatch) {
        int32_t t[kOcBatch];
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) t[u] = cb + u < n_chunks ? counts[(int64_t)(cb + u) * n_unique + k] : 0;
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) {
            if (cb + u < n_chunks) counts[(int64_t)(cb + u) * n_unique + k] = run;
            run += t[u];
        }
    }
    counts[(int64_t)n_chunks * n_unique + k] = run;
}

// grid (object groups, chunks + 1): chunk blocks write the members of their chunk at their final rows;
// the extra block pads the rows of M past the last member with -1
__global__ void __launch_bounds__(kOcBlock)
k_oc_members(const int32_t* __restrict__ asso_idx, const int32_t* __restrict__ unique_idx,
             const int32_t* __restrict__ unique_rs_asso, const int32_t* __restrict__ rs, int32_t n_vert, int32_t n_unique,
             int32_t n_splits, int32_t n_maxuq, int32_t n_maxrs, int32_t rot_block, int32_t n_chunks,
             const int32_t* __restrict__ counts, int32_t* __restrict__ M)
{
    const int32_t k = blockIdx.x * kOcBlock + threadIdx.x;
    if (k >= n_unique) return;
    if ((int32_t)blockIdx.y == n_chunks) {
        int32_t total = counts[(int64_t)n_chunks * n_unique + k];
        for (int32_t r = total < n_maxuq ? total : n_maxuq; r < n_maxuq; ++r) M[(int64_t)r * n_unique + k] = -1;
        return;
    }
    const OcWindow w = oc_window(k, unique_idx, unique_rs_asso, rs, n_vert, n_splits, n_maxrs, rot_block);
    const int32_t p0 = blockIdx.y * kOcChunk;
    const int32_t p1 = p0 + kOcChunk < w.len ? p0 + kOcChunk : w.len;
    int32_t fill = counts[(int64_t)blockIdx.y * n_unique + k];
    for (int32_t pb = p0; pb < p1 && fill < n_maxuq; pb += kOcBatch) {
        int32_t v[kOcBatch];
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) v[u] = pb + u < p1 ? asso_idx[oc_vertex(w, pb + u)] : ~w.uq;
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u)
            if (v[u] == w.uq && fill < n_maxuq) { M[(int64_t)fill * n_unique + k] = oc_vertex(w, pb + u); ++fill; }
    }
}

// grid (object groups, blocks of kOcChunk output rows of M_not)
__global__ void __launch_bounds__(kOcBlock)
k_oc_others(const int32_t* __restrict__ asso_idx, const int32_t* __restrict__ unique_idx,
            const int32_t* __restrict__ unique_rs_asso, const int32_t* __restrict__ rs, int32_t n_vert, int32_t n_unique,
            int32_t n_splits, int32_t n_maxrs, int32_t rot_block, int32_t n_chunks,
            const int32_t* __restrict__ counts, int32_t* __restrict__ M_not)
{
    const int32_t k = blockIdx.x * kOcBlock + threadIdx.x;
    if (k >= n_unique) return;
    const OcWindow w = oc_window(k, unique_idx, unique_rs_asso, rs, n_vert, n_splits, n_maxrs, rot_block);
    const int32_t r0 = blockIdx.y * kOcChunk;
    const int32_t r1 = r0 + kOcChunk < n_maxrs ? r0 + kOcChunk : n_maxrs;
    // largest chunk c whose start has at most r0 non-members before it: c*C - members_before(c) <= r0
    int32_t lo = 0, hi = n_chunks;           // invariant: others_before(lo) <= r0; chunks >= hi are too far (or hi = n_chunks)
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        const int32_t before = mid * kOcChunk - counts[(int64_t)mid * n_unique + k];
        if (before <= r0) lo = mid; else hi = mid;
    }
    int32_t p = lo * kOcChunk;
    int32_t fill = p - counts[(int64_t)lo * n_unique + k];      // non-members before walk position p
    // phase 1, no stores: advance to the walk position where this object's non-member count reaches r0.
    // Lanes need different numbers of steps here; keeping it apart from the emission lets the emission
    // run with every lane at the same output row.
    while (p < w.len && fill < r0) {
        int32_t v[kOcBatch];
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) v[u] = p + u < w.len ? asso_idx[oc_vertex(w, p + u)] : w.uq;
        int32_t adv = 0;
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) {
            if (fill < r0) { fill += v[u] != w.uq; ++adv; }
        }
        p += adv;
    }
    // phase 2: emit rows r0 .. r1-1; a lane falls one row behind its neighbours only when it meets a member
    int32_t r = r0;
    while (p < w.len && r < r1) {
        int32_t v[kOcBatch];
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) v[u] = p + u < w.len ? asso_idx[oc_vertex(w, p + u)] : w.uq;   // past the end: skipped like a member
#pragma unroll
        for (int u = 0; u < kOcBatch; ++u) {
            if (v[u] != w.uq && r < r1) { M_not[(int64_t)r * n_unique + k] = oc_vertex(w, p + u); ++r; }
        }
        p += kOcBatch;
    }
    for (; r < r1; ++r) M_not[(int64_t)r * n_unique + k] = -1;
}

size_t oc_workspace_bytes(int64_t n_unique, int32_t n_maxrs)
{
    const int64_t n_chunks = (n_maxrs + kOcChunk - 1) / kOcChunk;
    return (size_t)(n_chunks + 1) * (size_t)n_unique * sizeof(int32_t);
}

hipError_t launch_oc_helper(const int32_t* asso_idx, const int32_t* unique_idx, const int32_t* unique_rs_asso,
                            const int32_t* rs, int32_t n_vert, int32_t n_unique, int32_t n_splits, int32_t n_maxuq,
                            int32_t n_maxrs, int32_t calc_m_not, int32_t rot_block, int32_t* M, int32_t* M_not,
                            int32_t* counts, hipStream_t stream)
{
    const unsigned groups = (unsigned)((n_unique + kOcBlock - 1) / kOcBlock);
    const int32_t n_chunks = (n_maxrs + kOcChunk - 1) / kOcChunk;
    if (!counts || n_chunks + 1 > 65535) {
        hipLaunchKernelGGL(k_oc_helper, dim3(groups), dim3(kOcBlock), 0, stream, asso_idx, unique_idx, unique_rs_asso, rs,
                           n_vert, n_unique, n_splits, n_maxuq, n_maxrs, calc_m_not, rot_block, M, M_not);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_oc_count, dim3(groups, n_chunks), dim3(kOcBlock), 0, stream, asso_idx, unique_idx, unique_rs_asso,
                       rs, n_vert, n_unique, n_splits, n_maxrs, rot_block, counts);
    hipLaunchKernelGGL(k_oc_scan, dim3(groups), dim3(kOcBlock), 0, stream, counts, n_unique, n_chunks);
    hipLaunchKernelGGL(k_oc_members, dim3(groups, n_chunks + 1), dim3(kOcBlock), 0, stream, asso_idx, unique_idx,
                       unique_rs_asso, rs, n_vert, n_unique, n_splits, n_maxuq, n_maxrs, rot_block, n_chunks, counts, M);
    if (calc_m_not)
        hipLaunchKernelGGL(k_oc_others, dim3(groups, n_chunks), dim3(kOcBlock), 0, stream, asso_idx, unique_idx,
                           unique_rs_asso, rs, n_vert, n_unique, n_splits, n_maxrs, rot_block, n_chunks, counts, M_not);
    return hipGetLastError();
}

}  // namespace fg
