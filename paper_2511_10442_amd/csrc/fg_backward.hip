// Backward of the returned squared distances (paper Section 3, last paragraph).
//   d2(v,u) = sum_c (x[v][c]-x[u][c])^2, so each graph entry (v, j) with u = idx[v][j] >= 0 and
//   upstream gradient g adds t_c = 2 g (x[v][c]-x[u][c]) to grad[v][c] and -t_c to grad[u][c].
// Plain variant (no workspace): 16 lanes cooperate on one row v (lane l takes entries j = l, l+16, ...), so a wave
// covers 4 rows and reads grad_d2/idx in 64-byte pieces.  The row's own sum is reduced with
// wave shuffles and added once; the neighbour side is scattered with float32 atomics.
#include "fg_internal.hpp"

namespace fg {

constexpr int kBwdBlock = 256;
constexpr int kLanesPerRow = 16;

__global__ void __launch_bounds__(kBwdBlock)
k_fill_zero(float* __restrict__ p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * kBwdBlock + threadIdx.x;
    int64_t step = (int64_t)gridDim.x * kBwdBlock;
    for (; i < n; i += step) p[i] = 0.0f;
}

template <int D>
__global__ void __launch_bounds__(kBwdBlock)
k_backward(const float* __restrict__ grad_d2, const int32_t* __restrict__ idx, const float* __restrict__ coords,
           int32_t n, int32_t k, float* __restrict__ grad_coords)
{
    const int64_t t = (int64_t)blockIdx.x * kBwdBlock + threadIdx.x;
    const int64_t v = t / kLanesPerRow;
    const int32_t l = (int32_t)(t % kLanesPerRow);
    const bool live = v < n;               // whole 16-lane groups are live or dead together
    float xv[D], acc[D];
#pragma unroll
    for (int c = 0; c < D; ++c) { xv[c] = live ? coords[(int64_t)v * D + c] : 0.0f; acc[c] = 0.0f; }
    if (live) {
        for (int32_t j = l; j < k; j += kLanesPerRow) {
            const int32_t u = idx[(int64_t)v * k + j];
            if (u < 0 || u >= n || u == v) continue;   // padding / out of range: ignored; self contributes exactly 0
            const float g2 = 2.0f * grad_d2[(int64_t)v * k + j];
#pragma unroll
            for (int c = 0; c < D; ++c) {
                const float tc = g2 * (xv[c] - coords[(int64_t)u * D + c]);
                acc[c] += tc;
                atomicAdd(&grad_coords[(int64_t)u * D + c], -tc);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < D; ++c) {
        float s = acc[c];
        for (int o = kLanesPerRow / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (live && l == 0) atomicAdd(&grad_coords[(int64_t)v * D + c], s);
    }
}

// lanes 16r .. 16r+15 of a wave: afterwards lane 16r+15 holds their sum
__device__ __forceinline__ float row16_sum_to_last(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x111, 0xf, 0xf, false));   // row_shr:1
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x112, 0xf, 0xf, false));   // row_shr:2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, false));   // row_shr:4
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, false));   // row_shr:8
    return v;
}

// ---- tiled variant: rows taken in bin order, neighbour-side contributions combined in LDS ----
//
// Device-scope float atomics are the bottleneck of the plain kernel (every one costs the same,
// however local its address).  Rows that are adjacent in bin order are adjacent in space and
// share most of their neighbours, so a block that takes a tile of consecutive bin-ordered rows
// first adds all its contributions into an open-addressing hash table in LDS keyed by the
// destination row, and only then issues one global atomic per distinct destination and dimension.
// The table accumulates in double precision: measured on gfx950 the LDS atomic add on doubles runs
// about nine times faster than the one on floats (which handles about one lane every three cycles
// per CU), and the sums come out more accurate as well.  Entries that find no slot within kBwdProbes
// probes go straight to global memory, so the table size bounds nothing but speed.
// Sizes, all measured on the 1M-point d = 3 K = 32 workload: 1024 threads per block and two blocks per CU (the
// kernel waits on chains of dependent loads, row -> index -> coordinates, and on LDS round trips, so it wants
// every wave slot filled: 256-thread blocks with the same table were 35 % slower); eight table slots per row
// (a tile's rows reach two to three distinct destinations each, and a table a third full settles nearly every
// entry in the first probing round; with four slots per row the larger tile saved memory-side requests in
// the flush but lost more in probing rounds: 0.378 against 0.355 ms).
constexpr int kBwdProbes = 12;
constexpr int kBwdBatch = 4;          // (row, piece) pairs in flight per lane
constexpr int kBwdThreads = 1024;
constexpr int kBwdLdsKb = 56;         // LDS budget of a block's table: two blocks per CU
constexpr int kBwdSlotsPerRow = 8;
template <int D> constexpr int bwd_block() { return kBwdThreads; }
constexpr int pow2_floor(int v) { int p = 1; while (2 * p <= v) p *= 2; return p; }
// table slots: the largest power of two whose keys (4 bytes) and D double sums fit the LDS budget of a block
template <int D> constexpr int bwd_slots() { return pow2_floor(kBwdLdsKb * 1024 / (4 + 8 * D)); }
template <int D> constexpr int bwd_rows() { return bwd_slots<D>() / kBwdSlotsPerRow; }
constexpr int ilog2(int v) { int b = 0; while ((1 << b) < v) ++b; return b; }

// Adds NE entries of one lane to the table (key u[e], D values each; u[e] < 0: nothing to add).
// Open addressing with linear probing, in two phases.  First every entry finds its slot: rounds of
// compare-and-swaps, those of one round issued back to back so that their round trips through the LDS
// overlap, and an entry whose lanes are all settled issues nothing more.  Then the sums are added, one
// instruction per entry and dim for the whole wave.  The LDS pipeline is what bounds this kernel and it
// is paid per instruction, however few lanes take part: with the adds inside the probing rounds (issued
// again in every round for the few lanes that settled in it) the kernel spent 2.3 times the LDS
// instructions.
template <int D, int NE>
__device__ __forceinline__ void bwd_insert_batch(int32_t* keys, double* vals, const int32_t (&u)[NE],
                                                 const float (&t)[NE][D], float* __restrict__ grad_coords)
{
    constexpr int SLOTS = bwd_slots<D>();
    uint32_t h[NE];
    bool open[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        h[e] = ((uint32_t)u[e] * 2654435761u) >> (32 - ilog2(SLOTS));
        open[e] = u[e] >= 0;
    }
#pragma unroll 1
    for (int probe = 0; probe < kBwdProbes; ++probe) {
        bool any_open = false;
#pragma unroll
        for (int e = 0; e < NE; ++e) any_open = any_open || open[e];
        if (!__any(any_open)) break;
        int32_t prev[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            prev[e] = 0;
            if (__any(open[e])) prev[e] = open[e] ? atomicCAS(&keys[h[e]], -1, u[e]) : 0;
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (!open[e]) continue;
            if (prev[e] == -1 || prev[e] == u[e]) open[e] = false;
            else h[e] = (h[e] + 1) & (SLOTS - 1);
        }
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        if (u[e] < 0) continue;
        if (!open[e]) {
#pragma unroll
            for (int c = 0; c < D; ++c) atomicAdd(&vals[c * SLOTS + h[e]], (double)t[e][c]);
        } else {       // no slot within kBwdProbes probes: straight to global memory
#pragma unroll
            for (int c = 0; c < D; ++c) atomicAdd(&grad_coords[(int64_t)u[e] * D + c], t[e][c]);
        }
    }
}

// value of lane l + N of the same 16-lane row (lanes past the row's end keep their own)
template <int N>
__device__ __forceinline__ float row16_from_above(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), 0x100 + N, 0xf, 0xf, false));   // row_shl:N
}

// One point's coordinates with as few load instructions as its row allows: the gathers of the
// neighbours' coordinates are a third of this kernel's time when issued one float at a time.
// VEC promises a 16-byte aligned coords pointer.  For D = 3 the rows come from a copy padded to
// four floats (coords4), made while the rows were binned.
template <int D, bool VEC>
__device__ __forceinline__ void load_point(const float* __restrict__ coords, const float4* __restrict__ coords4,
                                           int64_t r, float (&out)[D])
{
    if constexpr (D == 3) {
        if (coords4) {
            const float4 f = coords4[r];
            out[0] = f.x; out[1] = f.y; out[2] = f.z;
            return;
        }
    }
    if constexpr (VEC && D % 4 == 0) {
        const float4* p = reinterpret_cast<const float4*>(coords) + r * (D / 4);
#pragma unroll
        for (int q = 0; q < D / 4; ++q) { const float4 f = p[q]; out[4 * q] = f.x; out[4 * q + 1] = f.y; out[4 * q + 2] = f.z; out[4 * q + 3] = f.w; }
    } else if constexpr (VEC && D % 2 == 0) {
        const float2* p = reinterpret_cast<const float2*>(coords) + r * (D / 2);
#pragma unroll
        for (int q = 0; q < D / 2; ++q) { const float2 f = p[q]; out[2 * q] = f.x; out[2 * q + 1] = f.y; }
    } else {
#pragma unroll
        for (int c = 0; c < D; ++c) out[c] = coords[r * D + c];
    }
}

template <int D, bool VEC>
__global__ void __launch_bounds__(bwd_block<D>())
k_backward_tiled(const float* __restrict__ grad_d2, const int32_t* __restrict__ idx, const float* __restrict__ coords,
                 const float4* __restrict__ coords4, const int32_t* __restrict__ perm, int32_t perm_stride, int32_t n,
                 int32_t k, float* __restrict__ grad_coords)
{
    constexpr int SLOTS = bwd_slots<D>();
    constexpr int ROWS = bwd_rows<D>();
    __shared__ int32_t keys[SLOTS];
    __shared__ double vals[D * SLOTS];
    __shared__ int32_t rows_v[ROWS];       // the tile's rows (original indices), -1 past the end
    const int64_t tile0 = (int64_t)blockIdx.x * ROWS;
    for (int i = threadIdx.x; i < SLOTS; i += bwd_block<D>()) keys[i] = -1;
    for (int i = threadIdx.x; i < D * SLOTS; i += bwd_block<D>()) vals[i] = 0.0;
    for (int i = threadIdx.x; i < ROWS; i += bwd_block<D>()) rows_v[i] = tile0 + i < n ? perm[(tile0 + i) * perm_stride] : -1;
    __syncthreads();

    // A group of 16 lanes owns rows tile0 + sub, tile0 + sub + G, ... (G groups per block); lane l of the
    // group takes entries j = l, l + 16, ... of each.  The (row, 16-entry piece) pairs of a group are walked
    // kBwdBatch at a time.  The chain row -> index -> neighbour coordinates is three dependent trips to memory
    // and one chain at a time left the kernel waiting on them: the rows come from LDS, the indices and upstream
    // gradients of a batch are requested while the batch before it is worked on, and all coordinate loads of a
    // batch are issued before any of its LDS work.
    constexpr int G = bwd_block<D>() / kLanesPerRow;
    constexpr int ROWS_PER_GROUP = ROWS / G;
    static_assert(ROWS_PER_GROUP >= 1 && ROWS_PER_GROUP * G == ROWS, "a tile is a whole number of rows per 16-lane group");
    const int l = threadIdx.x % kLanesPerRow;
    const int sub = threadIdx.x / kLanesPerRow;
    const int32_t pieces = (k + kLanesPerRow - 1) / kLanesPerRow;
    const int32_t n_it = ROWS_PER_GROUP * pieces;
    int32_t v_next[kBwdBatch], u_next[kBwdBatch];
    float g_next[kBwdBatch];
    auto request = [&](int32_t it0) {
#pragma unroll
        for (int e = 0; e < kBwdBatch; ++e) {
            const int32_t it = it0 + e;
            const int32_t ri = it / pieces;
            const int32_t j = (it - ri * pieces) * kLanesPerRow + l;
            v_next[e] = it < n_it ? rows_v[ri * G + sub] : -1;      // whole 16-lane groups are live or dead together
            const bool has = v_next[e] >= 0 && j < k;
            u_next[e] = has ? idx[(int64_t)v_next[e] * k + j] : -1;
            g_next[e] = has ? grad_d2[(int64_t)v_next[e] * k + j] : 0.0f;
        }
    };
    request(0);
    for (int32_t it0 = 0; it0 < n_it; it0 += kBwdBatch) {
        int32_t v[kBwdBatch], u[kBwdBatch];
        float g2[kBwdBatch];
#pragma unroll
        for (int e = 0; e < kBwdBatch; ++e) {
            v[e] = v_next[e];
            u[e] = u_next[e];
            g2[e] = 2.0f * g_next[e];
            if (u[e] >= n || u[e] == v[e]) u[e] = -1;    // out of range: ignored; self contributes exactly 0
        }
        float xv[kBwdBatch][D], xu[kBwdBatch][D];
#pragma unroll
        for (int e = 0; e < kBwdBatch; ++e) {
            load_point<D, VEC>(coords, coords4, v[e] < 0 ? 0 : v[e], xv[e]);
            load_point<D, VEC>(coords, coords4, u[e] < 0 ? 0 : u[e], xu[e]);
        }
        request(it0 + kBwdBatch);
        // One insertion for the neighbour side of the whole batch and the rows' own side.  Own side: each piece
        // summed over its 16 lanes (one DPP row: four shifted adds leave the total in the row's last lane, no
        // trip through the LDS crossbar); pieces of one row are added up first; then the batch's own sums move
        // from the last lane to lanes 15, 14, ... of the row, one per lane, so that they are a single table
        // entry per lane instead of kBwdBatch entries with a sixteenth of the lanes each.
        static_assert(kBwdBatch <= 4, "own sums are spread over the last four lanes of a row");
        int32_t key[kBwdBatch + 1];
        float t[kBwdBatch + 1][D];
        float own[kBwdBatch][D];
        bool own_live[kBwdBatch];
#pragma unroll
        for (int e = 0; e < kBwdBatch; ++e) {
            key[e] = u[e];
#pragma unroll
            for (int c = 0; c < D; ++c) {
                t[e][c] = u[e] >= 0 ? g2[e] * (xu[e][c] - xv[e][c]) : 0.0f;
                own[e][c] = -t[e][c];
            }
            own_live[e] = v[e] >= 0;
        }
#pragma unroll
        for (int e = 1; e < kBwdBatch; ++e) {
            if (v[e] >= 0 && v[e] == v[e - 1]) {      // next piece of the same row (the same in all 16 lanes)
#pragma unroll
                for (int c = 0; c < D; ++c) own[e][c] += own[e - 1][c];
                own_live[e - 1] = false;
            }
        }
        key[kBwdBatch] = -1;
#pragma unroll
        for (int c = 0; c < D; ++c) t[kBwdBatch][c] = 0.0f;
#pragma unroll
        for (int e = 0; e < kBwdBatch; ++e) {
            float moved[D];
#pragma unroll
            for (int c = 0; c < D; ++c) {
                const float total = row16_sum_to_last(own[e][c]);
                moved[c] = e == 0 ? total : e == 1 ? row16_from_above<1>(total) : e == 2 ? row16_from_above<2>(total)
                                                                                         : row16_from_above<3>(total);
            }
            if (l == kLanesPerRow - 1 - e) {
                key[kBwdBatch] = own_live[e] ? v[e] : -1;
#pragma unroll
                for (int c = 0; c < D; ++c) t[kBwdBatch][c] = moved[c];
            }
        }
        bwd_insert_batch<D, kBwdBatch + 1>(keys, vals, key, t, grad_coords);
    }
    __syncthreads();
    // flush: the D sums of a destination go out from neighbouring lanes, so that they reach the memory side as
    // one request per destination row instead of one per float
    constexpr int LPS = D <= 2 ? 2 : (D <= 4 ? 4 : (D <= 8 ? 8 : 16));   // lanes per slot
    for (int i = threadIdx.x; i < SLOTS * LPS; i += bwd_block<D>()) {
        const int slot = i / LPS, c = i % LPS;
        const int32_t u = keys[slot];
        if (u >= 0 && c < D)
            atomicAdd(&grad_coords[(int64_t)u * D + c], (float)vals[c * SLOTS + slot]);
    }
}

template <int D>
static void launch_bwd_tiled(const float* grad_d2, const int32_t* idx, const float* coords, const float4* coords4,
                             const int32_t* perm, int32_t perm_stride, int32_t n, int32_t k, float* grad_coords,
                             hipStream_t stream)
{
    unsigned grid = (unsigned)(((int64_t)n + bwd_rows<D>() - 1) / bwd_rows<D>());
    if (((uintptr_t)coords % 16) == 0)
        hipLaunchKernelGGL((k_backward_tiled<D, true>), dim3(grid), dim3(bwd_block<D>()), 0, stream, grad_d2, idx, coords,
                           coords4, perm, perm_stride, n, k, grad_coords);
    else
        hipLaunchKernelGGL((k_backward_tiled<D, false>), dim3(grid), dim3(bwd_block<D>()), 0, stream, grad_d2, idx, coords,
                           coords4, perm, perm_stride, n, k, grad_coords);
}

template <int D>
static void launch_bwd(const float* grad_d2, const int32_t* idx, const float* coords, int32_t n, int32_t k,
                       float* grad_coords, hipStream_t stream)
{
    int64_t threads = (int64_t)n * kLanesPerRow;
    unsigned grid = (unsigned)((threads + kBwdBlock - 1) / kBwdBlock);
    hipLaunchKernelGGL(k_backward<D>, dim3(grid), dim3(kBwdBlock), 0, stream, grad_d2, idx, coords, n, k, grad_coords);
}

hipError_t launch_backward(const float* grad_d2, const int32_t* idx, const float* coords, const float* coords4,
                           const int32_t* perm, int32_t perm_stride, int32_t n, int32_t d, int32_t k, float* grad_coords,
                           hipStream_t stream)
{
    {
        int64_t total = (int64_t)n * d;
        int64_t grid = (total + kBwdBlock - 1) / kBwdBlock;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)grid), dim3(kBwdBlock), 0, stream, grad_coords, total);
    }
    if (perm) {
        switch (d) {
            case 2: launch_bwd_tiled<2>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 3: launch_bwd_tiled<3>(grad_d2, idx, coords, reinterpret_cast<const float4*>(coords4), perm, perm_stride, n, k, grad_coords, stream); break;
            case 4: launch_bwd_tiled<4>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 5: launch_bwd_tiled<5>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 6: launch_bwd_tiled<6>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 7: launch_bwd_tiled<7>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 8: launch_bwd_tiled<8>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 9: launch_bwd_tiled<9>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            case 10: launch_bwd_tiled<10>(grad_d2, idx, coords, nullptr, perm, perm_stride, n, k, grad_coords, stream); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    switch (d) {
        case 2: launch_bwd<2>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 3: launch_bwd<3>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 4: launch_bwd<4>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 5: launch_bwd<5>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 6: launch_bwd<6>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 7: launch_bwd<7>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 8: launch_bwd<8>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 9: launch_bwd<9>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        case 10: launch_bwd<10>(grad_d2, idx, coords, n, k, grad_coords, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace fg
