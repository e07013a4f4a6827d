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

// Batcher's odd-even merge: the N keys v[LO], v[LO+R], v[LO+2R], ... whose first and second halves are each
// ascending become ascending.  N a power of two.  (N/2) log2(N) - N/2 + 1 comparators, fewer than the bitonic
// merge's (N/2) log2(N).
template <int LO, int N, int R, int M>
__host__ __device__ __forceinline__ void net_oe_merge(uint64_t (&v)[M])
{
    if constexpr (N > 2) {
        net_oe_merge<LO, N / 2, 2 * R>(v);
        net_oe_merge<LO + R, N / 2, 2 * R>(v);
#pragma unroll
        for (int i = 1; i + 1 < N; i += 2) cmp_swap(v[LO + i * R], v[LO + (i + 1) * R]);
    } else {
        cmp_swap(v[LO], v[LO + R]);
    }
}

template <int LO, int N, int M>
__host__ __device__ __forceinline__ void net_oe_sort(uint64_t (&v)[M])
{
    if constexpr (N > 1) {
        net_oe_sort<LO, N / 2>(v);
        net_oe_sort<LO + N / 2, N / 2>(v);
        net_oe_merge<LO, N, 1>(v);
    }
}

// ascending sort of v[0..N), N a power of two (odd-even merge sort: 63 comparators for 16 keys)
template <int N>
__host__ __device__ __forceinline__ void net_sort(uint64_t (&v)[N])
{
    net_oe_sort<0, N>(v);
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
        constexpr int N = next_pow2(KC);
        if constexpr (KC - P <= N / 2) {
            // head and tail each ascending: odd-even merge of [head, padding | tail, padding], padded with
            // all-ones keys up to the next power of two.  The padding is a compile-time constant, so every
            // comparator that meets it folds away (65 comparators remain for 16 + 16 keys, 113 for 32 + 16).
            uint64_t w[N];
#pragma unroll
            for (int i = 0; i < N; ++i) w[i] = ~0ull;
#pragma unroll
            for (int i = 0; i < KC - P; ++i) w[i] = best[i];
#pragma unroll
            for (int i = 0; i < P; ++i) w[N / 2 + i] = best[KC - P + i];
            net_oe_merge<0, N, 1>(w);
#pragma unroll
            for (int i = 0; i < KC; ++i) best[i] = w[i];
        } else {
            // head ascending + reversed tail is bitonic: merge on a renamed copy.  When KC is not a
            // power of two the copy is padded in the middle with all-ones keys (ascending head, plateau
            // of maxima, descending tail is still bitonic); the padding folds away as above.
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
}

}  // namespace fg
