// Backward of the returned squared distances (paper Section 3, last paragraph).
//   d2(v,u) = sum_c (x[v][c]-x[u][c])^2, so each graph entry (v, j) with u = idx[v][j] >= 0 and
//   upstream gradient g adds t_c = 2 g (x[v][c]-x[u][c]) to grad[v][c] and -t_c to grad[u][c].
// Layout: 16 lanes cooperate on one row v (lane l takes entries j = l, l+16, ...), so a wave
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

template <int D>
static void launch_bwd(const float* grad_d2, const int32_t* idx, const float* coords, int32_t n, int32_t k,
                       float* grad_coords, hipStream_t stream)
{
    int64_t threads = (int64_t)n * kLanesPerRow;
    unsigned grid = (unsigned)((threads + kBwdBlock - 1) / kBwdBlock);
    hipLaunchKernelGGL(k_backward<D>, dim3(grid), dim3(kBwdBlock), 0, stream, grad_d2, idx, coords, n, k, grad_coords);
}

hipError_t launch_backward(const float* grad_d2, const int32_t* idx, const float* coords, int32_t n,
                           int32_t d, int32_t k, float* grad_coords, hipStream_t stream)
{
    {
        int64_t total = (int64_t)n * d;
        int64_t grid = (total + kBwdBlock - 1) / kBwdBlock;
        if (grid > 4096) grid = 4096;
        hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)grid), dim3(kBwdBlock), 0, stream, grad_coords, total);
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
