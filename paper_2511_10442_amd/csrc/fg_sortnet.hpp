// Data-independent sorting / merging networks over 64-bit keys held in registers.
// Every index is a compile-time constant after unrolling, so the arrays never leave the
// register file.  Keys are (squared-distance bits << 32) | index: an unsigned compare is the
// strict total order (d2, index).
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace fg {

__host__ __device__ __forceinline__ void cmp_swap(uint64_t& lo, uint64_t& hi)
{
    const bool sw = hi < lo;
    const uint64_t a = sw ? hi : lo;
    const uint64_t b = sw ? lo : hi;
    lo = a;
    hi = b;
}

// ascending bitonic sort of v[0..N), N a power of two
template <int N>
__host__ __device__ __forceinline__ void net_sort(uint64_t (&v)[N])
{
#pragma unroll
    for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                const int l = i ^ j;
                if (l > i) {
                    if ((i & k) == 0) cmp_swap(v[i], v[l]);
                    else cmp_swap(v[l], v[i]);
                }
            }
        }
    }
}

// v[OFF..OFF+N) is bitonic -> ascending
template <int N, int OFF, int M>
__host__ __device__ __forceinline__ void net_merge(uint64_t (&v)[M])
{
#pragma unroll
    for (int j = N >> 1; j > 0; j >>= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int l = i ^ j;
            if (l > i) cmp_swap(v[OFF + i], v[OFF + l]);
        }
    }
}

constexpr int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

// best[0..KC) ascending, pend[0..P) ascending, P <= KC, P a power of two, KC a multiple of P:
// afterwards best holds the KC smallest of the union, ascending.
template <int KC, int P>
__host__ __device__ __forceinline__ void net_absorb(uint64_t (&best)[KC], const uint64_t (&pend)[P])
{
    // the P largest slots against the reversed newcomers: keeps the P smallest of the two, as a bitonic run
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const uint64_t a = best[KC - 1 - i], b = pend[i];
        best[KC - 1 - i] = b < a ? b : a;
    }
    if (KC == P) {
        net_merge<KC, 0>(best);
    } else {
        net_merge<P, KC - P>(best);          // tail ascending
        // head ascending + reversed tail is bitonic: merge on a renamed copy.  When KC is not a
        // power of two the copy is padded in the middle with all-ones keys up to the next power
        // of two (ascending head, plateau of maxima, descending tail is still bitonic); the
        // padding is a compile-time constant, so every comparator that meets it folds away.
        constexpr int N = next_pow2(KC);
        uint64_t w[N];
#pragma unroll
        for (int i = 0; i < KC - P; ++i) w[i] = best[i];
#pragma unroll
        for (int i = KC - P; i < N - P; ++i) w[i] = ~0ull;
#pragma unroll
        for (int i = 0; i < P; ++i) w[N - P + i] = best[KC - 1 - i];
        net_merge<N, 0>(w);
#pragma unroll
        for (int i = 0; i < KC; ++i) best[i] = w[i];
    }
}

}  // namespace fg
