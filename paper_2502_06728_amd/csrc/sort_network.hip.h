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

// sort descending, in registers
template <int N>
__device__ __forceinline__ void sort_desc(uint32_t (&k)[N]) {
    constexpr int cnt = SortNetHolder<N>::net.n;
    static_for<0, cnt>([&](auto I) {
        constexpr int i = SortNetHolder<N>::net.a[I];
        constexpr int j = SortNetHolder<N>::net.b[I];
        const uint32_t hi = max(k[i], k[j]);
        const uint32_t lo = min(k[i], k[j]);
        k[i] = hi;
        k[j] = lo;
    });
}

}  // namespace deto
