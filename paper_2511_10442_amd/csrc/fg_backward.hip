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

// ---- tiled variant: rows taken in bin order, neighbour-side contributions combined in LDS ----
//
// Device-scope float atomics are the bottleneck of the plain kernel (every one costs the same,
// however local its address).  Rows that are adjacent in bin order are adjacent in space and
// share most of their neighbours, so a block that takes kBwdRows consecutive bin-ordered rows
// first adds all its contributions into an open-addressing hash table in LDS keyed by the
// destination row (LDS float atomics), and only then issues one global atomic per distinct
// destination and dimension.  Entries that find no slot within kBwdProbes probes go straight
// to global memory, so the table size bounds nothing but speed.
constexpr int kBwdProbes = 12;
template <int D> constexpr int bwd_slots() { return D <= 4 ? 2048 : 1024; }
template <int D> constexpr int bwd_rows() { return D <= 4 ? 256 : 128; }

template <int D>
__device__ __forceinline__ void bwd_insert(int32_t* keys, float* vals, int32_t u, const float (&t)[D],
                                           float* __restrict__ grad_coords)
{
    constexpr int SLOTS = bwd_slots<D>();
    uint32_t h = ((uint32_t)u * 2654435761u) >> (32 - (SLOTS == 2048 ? 11 : 10));
#pragma unroll 1
    for (int probe = 0; probe < kBwdProbes; ++probe) {
        const int32_t prev = atomicCAS(&keys[h], -1, u);
        if (prev == -1 || prev == u) {
#pragma unroll
            for (int c = 0; c < D; ++c) atomicAdd(&vals[c * SLOTS + h], t[c]);
            return;
        }
        h = (h + 1) & (SLOTS - 1);
    }
#pragma unroll
    for (int c = 0; c < D; ++c) atomicAdd(&grad_coords[(int64_t)u * D + c], t[c]);
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
__global__ void __launch_bounds__(kBwdBlock)
k_backward_tiled(const float* __restrict__ grad_d2, const int32_t* __restrict__ idx, const float* __restrict__ coords,
                 const float4* __restrict__ coords4, const int32_t* __restrict__ perm, int32_t n, int32_t k,
                 float* __restrict__ grad_coords)
{
    constexpr int SLOTS = bwd_slots<D>();
    constexpr int ROWS = bwd_rows<D>();
    __shared__ int32_t keys[SLOTS];
    __shared__ float vals[D * SLOTS];
    for (int i = threadIdx.x; i < SLOTS; i += kBwdBlock) keys[i] = -1;
    for (int i = threadIdx.x; i < D * SLOTS; i += kBwdBlock) vals[i] = 0.0f;
    __syncthreads();

    const int l = threadIdx.x % kLanesPerRow;
    const int sub = threadIdx.x / kLanesPerRow;
    const int64_t tile0 = (int64_t)blockIdx.x * ROWS;
    for (int r0 = 0; r0 < ROWS; r0 += kBwdBlock / kLanesPerRow) {
        const int64_t pos = tile0 + r0 + sub;
        const bool live = pos < n;                   // whole 16-lane groups are live or dead together
        const int32_t v = live ? perm[pos] : 0;
        float xv[D], acc[D];
        load_point<D, VEC>(coords, coords4, v, xv);     // dead groups read row 0: harmless
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] = 0.0f;
        if (live) {
            for (int32_t j = l; j < k; j += kLanesPerRow) {
                const int32_t u = idx[(int64_t)v * k + j];
                if (u < 0 || u >= n || u == v) continue;   // padding / out of range: ignored; self contributes exactly 0
                const float g2 = 2.0f * grad_d2[(int64_t)v * k + j];
                float t[D], xu[D];
                load_point<D, VEC>(coords, coords4, u, xu);
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const float tc = g2 * (xv[c] - xu[c]);
                    acc[c] += tc;
                    t[c] = -tc;
                }
                bwd_insert<D>(keys, vals, u, t, grad_coords);
            }
        }
#pragma unroll
        for (int c = 0; c < D; ++c) {
            float s = acc[c];
            for (int o = kLanesPerRow / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
            acc[c] = s;
        }
        if (live && l == 0) bwd_insert<D>(keys, vals, v, acc, grad_coords);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < SLOTS; i += kBwdBlock) {
        const int32_t u = keys[i];
        if (u >= 0) {
#pragma unroll
            for (int c = 0; c < D; ++c) atomicAdd(&grad_coords[(int64_t)u * D + c], vals[c * SLOTS + i]);
        }
    }
}

template <int D>
static void launch_bwd_tiled(const float* grad_d2, const int32_t* idx, const float* coords, const float4* coords4,
                             const int32_t* perm, int32_t n, int32_t k, float* grad_coords, hipStream_t stream)
{
    unsigned grid = (unsigned)((n + bwd_rows<D>() - 1) / bwd_rows<D>());
    if (((uintptr_t)coords % 16) == 0)
        hipLaunchKernelGGL((k_backward_tiled<D, true>), dim3(grid), dim3(kBwdBlock), 0, stream, grad_d2, idx, coords,
                           coords4, perm, n, k, grad_coords);
    else
        hipLaunchKernelGGL((k_backward_tiled<D, false>), dim3(grid), dim3(kBwdBlock), 0, stream, grad_d2, idx, coords,
                           coords4, perm, n, k, grad_coords);
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
                           const int32_t* perm, int32_t n, int32_t d, int32_t k, float* grad_coords, hipStream_t stream)
{
    {
        int64_t total = (int64_t)n * d;
        int64_t grid = (total + kBwdBlock - 1) / kBwdBlock;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)grid), dim3(kBwdBlock), 0, stream, grad_coords, total);
    }
    if (perm) {
        switch (d) {
            case 2: launch_bwd_tiled<2>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 3: launch_bwd_tiled<3>(grad_d2, idx, coords, reinterpret_cast<const float4*>(coords4), perm, n, k, grad_coords, stream); break;
            case 4: launch_bwd_tiled<4>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 5: launch_bwd_tiled<5>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 6: launch_bwd_tiled<6>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 7: launch_bwd_tiled<7>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 8: launch_bwd_tiled<8>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 9: launch_bwd_tiled<9>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
            case 10: launch_bwd_tiled<10>(grad_d2, idx, coords, nullptr, perm, n, k, grad_coords, stream); break;
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
