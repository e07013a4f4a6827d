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
#if defined(__HIP_DEVICE_COMPILE__)
    // On the device the comparator is a double-precision min / max pair: every key that reaches a network
    // (zero pins, real keys, the empty key 0x7f800001 << 32) has a sign bit of 0 and an exponent field below
    // 0x7ff, so as an IEEE double it is finite and non-negative, and finite non-negative doubles order like
    // their bit patterns.  Denormal patterns (squared distance 0: the key is just the index) pass through
    // unchanged because kernels run with double-precision denormals enabled.  Two instructions instead of a
    // 64-bit compare and four selects.
    const double a = __longlong_as_double((long long)lo), b = __longlong_as_double((long long)hi);
    double mn, mx;
    asm("v_min_f64 %0, %1, %2" : "=v"(mn) : "v"(a), "v"(b));
    asm("v_max_f64 %0, %1, %2" : "=v"(mx) : "v"(a), "v"(b));
    lo = (uint64_t)__double_as_longlong(mn);
    hi = (uint64_t)__double_as_longlong(mx);
#else
    const bool sw = hi < lo;
    const uint64_t a = sw ? hi : lo;
    const uint64_t b = sw ? lo : hi;
    lo = a;
    hi = b;
#endif
}

// smaller of two keys (same reasoning as cmp_swap)
__host__ __device__ __forceinline__ uint64_t key_min(uint64_t x, uint64_t y)
{
#if defined(__HIP_DEVICE_COMPILE__)
    double mn;
    asm("v_min_f64 %0, %1, %2" : "=v"(mn) : "v"(__longlong_as_double((long long)x)), "v"(__longlong_as_double((long long)y)));
    return (uint64_t)__double_as_longlong(mn);
#else
    return y < x ? y : x;
#endif
}

// larger of two keys
__host__ __device__ __forceinline__ uint64_t key_max(uint64_t x, uint64_t y)
{
#if defined(__HIP_DEVICE_COMPILE__)
    double mx;
    asm("v_max_f64 %0, %1, %2" : "=v"(mx) : "v"(__longlong_as_double((long long)x)), "v"(__longlong_as_double((long long)y)));
    return (uint64_t)__double_as_longlong(mx);
#else
    return y < x ? x : y;
#endif
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

// blocks B and B+1 (P keys each, each ascending) are merged in place, then block B-1 with B, down to block 0
template <int KC, int P, int B>
__host__ __device__ __forceinline__ void net_sink(uint64_t (&best)[KC])
{
    if constexpr (B >= 0) {
        net_oe_merge<B * P, 2 * P, 1>(best);
        net_sink<KC, P, B - 1>(best);
    }
}

// best[0..KC) ascending, pend[0..P) ascending, P a power of two, KC a multiple of P:
// afterwards best holds the KC smallest of the union, ascending.
template <int KC, int P>
__host__ __device__ __forceinline__ void net_absorb(uint64_t (&best)[KC], const uint64_t (&pend)[P])
{
    static_assert(KC % P == 0, "list size must be a multiple of the pending block");
    // the P largest slots against the reversed newcomers: keeps the P smallest of the two (the P largest of
    // the union drop out here), as a bitonic run, which a bitonic merge puts in order
#pragma unroll
    for (int i = 0; i < P; ++i) best[KC - 1 - i] = key_min(best[KC - 1 - i], pend[i]);
    net_merge<P, KC - P>(best);
    // the block of P now sinks through the blocks below it: an odd-even merge with the next lower block
    // leaves that pair in order; its upper half is final (everything further down is no larger than the
    // lower block's old minimum, which the upper half cannot go below), its lower half goes on sinking
    net_sink<KC, P, KC / P - 2>(best);
}

}  // namespace fg
