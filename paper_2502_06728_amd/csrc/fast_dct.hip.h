// Register-resident fast cosine transforms, fully unrolled at compile time.
//
// One lane owns one chunk: its N values live in N VGPRs and the whole transform is
// straight-line VALU code with literal twiddles, no cross-lane traffic.  The orthonormal
// DCT-II of the paper's ExtractFastComponents step is  coef[k] = a_k * dct2(x)[k]  and its
// inverse  x = dct3(a_k * coef[k]).
//
// Factorisation (all butterflies and plane rotations, so errors do not grow beyond
// O(log N) roundings; about 9 flops per point for N = 64 instead of 64):
//   dct2_N : u = x[n] + x[N-1-n], v = x[n] - x[N-1-n]
//            even outputs = dct2_{N/2}(u), odd outputs = dct4_{N/2}(v)
//   dct4_N : rotate the pairs (x[j], x[N-1-j]) by (2j+1)pi/(4N) into a[j], b[j],
//            A = dct2_{N/2}(a), B = dct2_{N/2}((-1)^j b),
//            y[0] = A[0], y[2l] = A[l] + B[N/2-l], y[2l+1] = A[l+1] - B[N/2-l-1],
//            y[N-1] = -B[0]
//   dct3_N : the transpose of dct2_N (dct4 is its own transpose)
// The recursion ends at N = 1, or at N = 3 (direct 3-point transforms) for sizes 3 * 2^a
// such as the chunk size 96 of the paper's Appendix B.
// Definitions (unnormalised):
//   dct2(x)[k] = sum_n x[n] cos(pi (2n+1) k / (2N))
//   dct4(x)[k] = sum_n x[n] cos(pi (2n+1)(2k+1) / (4N))
//   dct3(X)[n] = sum_k X[k] cos(pi (2n+1) k / (2N))
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

namespace deto {

// f(integral_constant<int, i>) for i = B .. E-1, in order.  Long ranges go in blocks of 64 so
// that the template recursion stays shallow (a sorting network has over a thousand steps).
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (E - B > 64) {
        static_for<B, B + 64>(f);
        static_for<B + 64, E>(f);
    } else if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// ---- compile-time sine/cosine for |x| <= pi/4 (Taylor series in double)
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double ct_sin(double x) {
    double term = x, sum = x;
    for (int i = 1; i < 14; ++i) {
        term *= -x * x / ((2 * i) * (2 * i + 1));
        sum += term;
    }
    return sum;
}

constexpr double ct_cos(double x) {
    double term = 1.0, sum = 1.0;
    for (int i = 1; i < 14; ++i) {
        term *= -x * x / ((2 * i - 1) * (2 * i));
        sum += term;
    }
    return sum;
}

// rotation angle of pair j in dct4_N: (2j+1) pi / (4N), always below pi/4
template <int N, int J>
struct Rot {
    static constexpr float c = static_cast<float>(ct_cos((2 * J + 1) * kPi / (4.0 * N)));
    static constexpr float s = static_cast<float>(ct_sin((2 * J + 1) * kPi / (4.0 * N)));
};

constexpr float kCosPi4 = 0.70710678118654752440f;
constexpr float kCosPi6 = 0.86602540378443864676f;    // cos(pi/6)
constexpr float kCosPi12 = 0.96592582628906828675f;   // cos(pi/12)
constexpr float kCos5Pi12 = 0.25881904510252076235f;  // cos(5 pi/12)

template <int N>
struct FastDct {
    static constexpr int H = N / 2;

    static __device__ __forceinline__ void dct2(float (&x)[N]) {
        if constexpr (N == 1) {
            return;
        } else if constexpr (N == 3) {
            // cos(pi (2n+1) k / 6): rows (1, 1, 1), (c, 0, -c), (1/2, -1, 1/2), c = cos(pi/6)
            const float a = x[0], b = x[1], d = x[2];
            x[0] = a + b + d;
            x[1] = kCosPi6 * (a - d);
            x[2] = fmaf(0.5f, a + d, -b);
        } else {
            float u[H], v[H];
            static_for<0, H>([&](auto i) {
                u[i] = x[i] + x[N - 1 - i];
                v[i] = x[i] - x[N - 1 - i];
            });
            FastDct<H>::dct2(u);
            FastDct<H>::dct4(v);
            static_for<0, H>([&](auto i) {
                x[2 * i] = u[i];
                x[2 * i + 1] = v[i];
            });
        }
    }

    static __device__ __forceinline__ void dct4(float (&x)[N]) {
        if constexpr (N == 1) {
            x[0] *= kCosPi4;
        } else if constexpr (N == 3) {
            // cos(pi (2n+1)(2k+1) / 12) with p = cos(pi/12), q = cos(pi/4), r = cos(5 pi/12):
            // rows (p, q, r), (q, -q, -q), (r, -q, p)
            const float a = x[0], b = x[1], d = x[2];
            x[0] = fmaf(kCosPi12, a, fmaf(kCosPi4, b, kCos5Pi12 * d));
            x[1] = kCosPi4 * (a - b - d);
            x[2] = fmaf(kCos5Pi12, a, fmaf(-kCosPi4, b, kCosPi12 * d));
        } else {
            float a[H], b[H];
            static_for<0, H>([&](auto j) {
                constexpr float c = Rot<N, j>::c, s = Rot<N, j>::s;
                const float p = x[j], q = x[N - 1 - j];
                a[j] = fmaf(p, c, q * s);
                const float bj = fmaf(q, c, -(p * s));
                b[j] = (j % 2) ? -bj : bj;
            });
            FastDct<H>::dct2(a);
            FastDct<H>::dct2(b);
            x[0] = a[0];
            static_for<1, H>([&](auto l) { x[2 * l] = a[l] + b[H - l]; });
            static_for<0, H - 1>([&](auto l) { x[2 * l + 1] = a[l + 1] - b[H - l - 1]; });
            x[N - 1] = -b[0];
        }
    }

    static __device__ __forceinline__ void dct3(float (&x)[N]) {
        if constexpr (N == 1) {
            return;
        } else if constexpr (N == 3) {
            // transpose of the 3-point dct2: columns (1, c, 1/2), (1, 0, -1), (1, -c, 1/2)
            const float a = x[0], b = kCosPi6 * x[1], d = x[2];
            x[0] = a + b + 0.5f * d;
            x[1] = a - d;
            x[2] = a - b + 0.5f * d;
        } else {
            float u[H], v[H];
            static_for<0, H>([&](auto i) {
                u[i] = x[2 * i];
                v[i] = x[2 * i + 1];
            });
            FastDct<H>::dct3(u);
            FastDct<H>::dct4(v);
            static_for<0, H>([&](auto i) {
                x[i] = u[i] + v[i];
                x[N - 1 - i] = u[i] - v[i];
            });
        }
    }
};

}  // namespace deto
