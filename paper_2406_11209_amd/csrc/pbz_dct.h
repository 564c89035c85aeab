// In-register orthonormal DCT-II / DCT-III of power-of-two length with compile-time constants.
//
// Forward (Sec. III-A, Appendix A):  X[q] = a_q sum_m x[m] cos(pi (2m+1) q / (2n)),  a_0 = sqrt(1/n), a_q = sqrt(2/n).
// Inverse:                            x[m] = sum_q a_q X[q] cos(pi (2m+1) q / (2n)).
//
// Both use the even/odd split: with s[m] = x[m] + x[n-1-m] and d[m] = x[m] - x[n-1-m] (m < n/2), the even
// outputs are 1/sqrt(2) times the length-n/2 transform of s and the odd outputs are a dense (n/2 x n/2)
// product with d.  Recursing costs 12 / 36 / 116 multiply-adds for n = 4 / 8 / 16 instead of the dense
// 16 / 64 / 256.  Everything is unrolled at compile time so that the data stays in registers; the scale
// factors are folded into the constants.  The functions also compile for the host, where a test runs them
// against an independent construction of the transform matrices.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

namespace pbz {
namespace dct {

// compile-time loop: f(std::integral_constant<int, i>) for i = 0 .. N-1, so that i can index constexpr tables
template <int I, int N, typename F>
__host__ __device__ __forceinline__ void static_for_impl(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for_impl<I + 1, N>(f);
  }
}
template <int N, typename F>
__host__ __device__ __forceinline__ void static_for(F&& f) {
  static_for_impl<0, N>(f);
}

constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double cx_sqrt(double x) {
  double g = x > 1.0 ? x : 1.0;
  for (int i = 0; i < 64; ++i) g = 0.5 * (g + x / g);
  return g;
}

// Taylor series on [0, pi/4]
constexpr double cx_cos_small(double x) {
  double term = 1.0, sum = 1.0;
  for (int k = 1; k <= 12; ++k) {
    term *= -x * x / double((2 * k - 1) * (2 * k));
    sum += term;
  }
  return sum;
}
constexpr double cx_sin_small(double x) {
  double term = x, sum = x;
  for (int k = 1; k <= 12; ++k) {
    term *= -x * x / double((2 * k) * (2 * k + 1));
    sum += term;
  }
  return sum;
}

// cos(k pi / (2n)) for integers k >= 0, n >= 1, reduced exactly in integer arithmetic
constexpr double cos_frac(long long k, long long n) {
  const long long period = 4 * n;  // k pi / (2n) has period 4n in k
  k %= period;
  if (k > 2 * n) k = period - k;           // cos(2 pi - t) = cos t      -> k in [0, 2n]
  double sign = 1.0;
  if (k > n) {                             // cos(pi - t) = -cos t       -> k in [0, n]
    k = 2 * n - k;
    sign = -1.0;
  }
  // angle t = k pi / (2n) in [0, pi/2]
  if (2 * k <= n) return sign * cx_cos_small(kPi * double(k) / double(2 * n));
  return sign * cx_sin_small(kPi * double(n - k) / double(2 * n));   // cos t = sin(pi/2 - t)
}

// entry [p][m] of the odd-part matrix of the length-n transform: sqrt(2/n) cos(pi (2m+1)(2p+1) / (2n))
constexpr double odd_coef(int n, int p, int m) {
  return cx_sqrt(2.0 / double(n)) * cos_frac((long long)(2 * m + 1) * (2 * p + 1), n);
}

constexpr double kInvSqrt2 = 0.70710678118654752440084436210484904;

// g as a compile-time rational power of 1/sqrt(2): the scale after `halvings` even splits is 2^(-halvings/2)
constexpr double scale_of(int halvings) {
  double g = 1.0;
  for (int i = 0; i < halvings; ++i) g *= kInvSqrt2;
  return g;
}

// Forward transform of v[0], v[S], ..., v[(n-1)S] in place; result is scale_of(H) * DCT_n.
template <typename T, int n, int S, int H>
struct Fwd {
  static __host__ __device__ __forceinline__ void run(T* v) {
    constexpr int h = n / 2;
    T s[h], d[h];
#pragma unroll
    for (int m = 0; m < h; ++m) {
      s[m] = v[m * S] + v[(n - 1 - m) * S];
      d[m] = v[m * S] - v[(n - 1 - m) * S];
    }
    Fwd<T, h, 1, H + 1>::run(s);
    static_for<h>([&](auto pc) {
      constexpr int p = decltype(pc)::value;
      v[(2 * p) * S] = s[p];
      constexpr T c0 = T(scale_of(H) * odd_coef(n, p, 0));
      T acc = c0 * d[0];
      static_for<h - 1>([&](auto mc) {
        constexpr int m = decltype(mc)::value + 1;
        constexpr T c = T(scale_of(H) * odd_coef(n, p, m));
        acc += c * d[m];
      });
      v[(2 * p + 1) * S] = acc;
    });
  }
};
template <typename T, int S, int H>
struct Fwd<T, 1, S, H> {
  static __host__ __device__ __forceinline__ void run(T* v) {
    if (H != 0) v[0] *= T(scale_of(H));
  }
};
template <typename T, int S, int H>
struct Fwd<T, 2, S, H> {
  static __host__ __device__ __forceinline__ void run(T* v) {
    T a = v[0], b = v[S];
    v[0] = (a + b) * T(scale_of(H + 1));
    v[S] = (a - b) * T(scale_of(H + 1));
  }
};

// Inverse transform in place; input entries with index >= K are known to be zero and are not read.
// Result is scale_of(H) * IDCT_n.
template <typename T, int n, int S, int H, int K>
struct Inv {
  static __host__ __device__ __forceinline__ void run(T* v) {
    constexpr int h = n / 2;
    constexpr int Ke = (K + 1) / 2;  // non-zero even-indexed inputs
    constexpr int Ko = K / 2;        // non-zero odd-indexed inputs
    T e[h], o[h];
#pragma unroll
    for (int p = 0; p < h; ++p) e[p] = p < Ke ? v[(2 * p) * S] : T(0);
    Inv<T, h, 1, H + 1, (Ke < h ? Ke : h)>::run(e);
    static_for<h>([&](auto mc) {
      constexpr int m = decltype(mc)::value;
      T acc = T(0);
      if constexpr (Ko > 0) {
        constexpr T c0 = T(scale_of(H) * odd_coef(n, 0, m));
        acc = c0 * v[1 * S];
        static_for<Ko - 1>([&](auto pc) {
          constexpr int p = decltype(pc)::value + 1;
          constexpr T c = T(scale_of(H) * odd_coef(n, p, m));
          acc += c * v[(2 * p + 1) * S];
        });
      }
      o[m] = acc;
    });
#pragma unroll
    for (int m = 0; m < h; ++m) {
      v[m * S] = e[m] + o[m];
      v[(n - 1 - m) * S] = e[m] - o[m];
    }
  }
};
template <typename T, int S, int H, int K>
struct Inv<T, 1, S, H, K> {
  static __host__ __device__ __forceinline__ void run(T* v) {
    if (K == 0)
      v[0] = T(0);
    else if (H != 0)
      v[0] *= T(scale_of(H));
  }
};
template <typename T, int S, int H, int K>
struct Inv<T, 2, S, H, K> {
  static __host__ __device__ __forceinline__ void run(T* v) {
    T a = K > 0 ? v[0] * T(scale_of(H + 1)) : T(0);
    T b = K > 1 ? v[S] * T(scale_of(H + 1)) : T(0);
    v[0] = a + b;
    v[S] = a - b;
  }
};

template <typename T, int n, int S>
__host__ __device__ __forceinline__ void forward(T* v) {
  Fwd<T, n, S, 0>::run(v);
}
template <typename T, int n, int S, int K>
__host__ __device__ __forceinline__ void inverse(T* v) {
  Inv<T, n, S, 0, K>::run(v);
}

}  // namespace dct
}  // namespace pbz
