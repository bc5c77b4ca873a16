// Batcher's odd-even merge sort as a compile-time list of compare-exchanges, applied to an
// array that lives in the registers of one lane (v_max_u32 / v_min_u32 pairs, no branches).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fast_dct.hip.h"   // static_for

namespace deto {

// The network for N keys, descending.  For N that is not a power of two it is the network of
// the next power of two P with every compare-exchange that touches a position >= N left out:
// think of those positions as holding the smallest possible key; a compare-exchange (i, j),
// i < j, leaves the larger key at i, so such a key at j never moves and the exchange does
// nothing.
template <int N>
struct SortNet {
    static constexpr int pow2() {
        int p = 1;
        while (p < N) p *= 2;
        return p;
    }
    static constexpr int P = pow2();
    static constexpr int kCap = P * 12;   // P log^2 P / 4 compare-exchanges fit up to P = 128
    static_assert(P <= 128, "capacity");
    int a[kCap];
    int b[kCap];
    int n;
    constexpr SortNet() : a{}, b{}, n(0) { sort(0, P); }
    constexpr void add(int i, int j) {
        if (j < N) {
            a[n] = i;
            b[n] = j;
            ++n;
        }
    }
    constexpr void merge(int lo, int len, int r) {
        const int m = r * 2;
        if (m < len) {
            merge(lo, len, m);
            merge(lo + r, len, m);
            for (int i = lo + r; i + r < lo + len; i += m) add(i, i + r);
        } else {
            add(lo, lo + r);
        }
    }
    constexpr void sort(int lo, int len) {
        if (len > 1) {
            const int m = len / 2;
            sort(lo, m);
            sort(lo + m, m);
            merge(lo, len, 1);
        }
    }
};

template <int N>
struct SortNetHolder {
    static constexpr SortNet<N> net{};
};

// sort k[OFF .. OFF+N) descending, in registers
template <int N, int OFF = 0, int M>
__device__ __forceinline__ void sort_desc_range(uint32_t (&k)[M]) {
    static_assert(OFF + N <= M, "range inside the array");
    constexpr int cnt = SortNetHolder<N>::net.n;
    static_for<0, cnt>([&](auto I) {
        constexpr int i = OFF + SortNetHolder<N>::net.a[I];
        constexpr int j = OFF + SortNetHolder<N>::net.b[I];
        const uint32_t hi = max(k[i], k[j]);
        const uint32_t lo = min(k[i], k[j]);
        k[i] = hi;
        k[j] = lo;
    });
}

template <int N>
__device__ __forceinline__ void sort_desc(uint32_t (&k)[N]) {
    sort_desc_range<N, 0>(k);
}

// Sort the first N entries, a bitonic sequence (first falling then rising, or the reverse),
// into descending order.
template <int N, int M>
__device__ __forceinline__ void bitonic_merge_desc(uint32_t (&x)[M]) {
    static_assert((N & (N - 1)) == 0 && N <= M, "power of two");
#pragma unroll
    for (int d = N / 2; d >= 1; d /= 2) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & d) == 0) {
                const uint32_t hi = max(x[i], x[i + d]);
                const uint32_t lo = min(x[i], x[i + d]);
                x[i] = hi;
                x[i + d] = lo;
            }
        }
    }
}

// The TOP largest of the N keys, descending, in k[0 .. TOP); the other entries become zero
// (the smallest key).  Whoever only needs the k-th largest for some k <= TOP does not need
// the full order: groups of TOP are sorted (the last one may be shorter), and each further
// group is folded into the first with one row of maxima against its mirror image (the TOP
// largest of the two groups, as a bitonic sequence; a short group counts as filled up with
// zeros, which change nothing) and a bitonic merge.  N = 64: 340 / 528 / 744 / 956
// instructions for TOP = 4 / 8 / 16 / 32 against 1,086 for the full sort.
template <int N, int TOP>
__device__ __forceinline__ void sort_top_desc(uint32_t (&k)[N]) {
    static_assert(TOP <= N && (TOP & (TOP - 1)) == 0, "a power of two");
    constexpr int kFull = N / TOP, kRest = N % TOP;
    static_for<0, kFull>([&](auto g) { sort_desc_range<TOP, g * TOP>(k); });
    if constexpr (kRest > 0) sort_desc_range<kRest, kFull * TOP>(k);
    static_for<1, kFull>([&](auto g) {
        static_for<0, TOP>([&](auto i) { k[i] = max(k[i], k[g * TOP + TOP - 1 - i]); });
        bitonic_merge_desc<TOP>(k);
    });
    if constexpr (kRest > 0) {
        // mirror image of the short group: its entry j faces position TOP - 1 - j
        static_for<0, kRest>([&](auto j) {
            k[TOP - 1 - j] = max(k[TOP - 1 - j], k[kFull * TOP + j]);
        });
        bitonic_merge_desc<TOP>(k);
    }
#pragma unroll
    for (int i = TOP; i < N; ++i) k[i] = 0u;
}

}  // namespace deto
