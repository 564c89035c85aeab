// In-register orthonormal Haar wavelet transform of power-of-two length, the alternative to the DCT that
// Sec. III-A names (end of "Orthonormal transform").  Sequency order: coefficient 0 is the sum of the samples
// over sqrt(n); coefficient 2^p + j (0 <= j < 2^p) is supported on the n / 2^p samples starting at j n / 2^p,
// +sqrt(2^p / n) on the first half of that support and -sqrt(2^p / n) on the second.
//
// Forward: a cascade of pairwise sums and differences, scaled once on output (n - 1 additions, n - 1
// subtractions, n multiplications).  Inverse: every input is multiplied by its amplitude, then each level
// splits a node value v into v + d and v - d; inputs known to be zero (index >= K) cost nothing.
#pragma once

#include <hip/hip_runtime.h>

#include "pbz_dct.h"

namespace pbz {
namespace haar {

// v[0], v[S], ..., v[(n-1)S] in place
template <typename T, int n, int S>
__host__ __device__ __forceinline__ void forward(T* v) {
  T cur[n];
#pragma unroll
  for (int m = 0; m < n; ++m) cur[m] = v[m * S];
  double scale = 1.0;
#pragma unroll
  for (int len = n; len > 1; len >>= 1) {
    scale *= dct::kInvSqrt2;
    const int h = len >> 1;
#pragma unroll
    for (int k = 0; k < h; ++k) {
      const T a = cur[2 * k], b = cur[2 * k + 1];
      v[(h + k) * S] = (a - b) * T(scale);
      cur[k] = a + b;          // k <= 2k: entries still to be read are not overwritten
    }
  }
  v[0] = cur[0] * T(scale);
}

// inverse in place; inputs with index >= K are zero and are not read
template <typename T, int n, int S, int K>
__host__ __device__ __forceinline__ void inverse(T* v) {
  double amp = 1.0;
#pragma unroll
  for (int len = n; len > 1; len >>= 1) amp *= dct::kInvSqrt2;     // sqrt(1 / n)
  T u[n], w[n];
  u[0] = K > 0 ? v[0] * T(amp) : T(0);
#pragma unroll
  for (int count = 1; count < n; count <<= 1) {
#pragma unroll
    for (int j = 0; j < count; ++j) {
      if (count + j < K) {
        const T d = v[(count + j) * S] * T(amp);
        w[2 * j] = u[j] + d;
        w[2 * j + 1] = u[j] - d;
      } else {
        w[2 * j] = u[j];
        w[2 * j + 1] = u[j];
      }
    }
#pragma unroll
    for (int j = 0; j < 2 * count; ++j) u[j] = w[j];
    amp *= 1.41421356237309504880168872420969808;
  }
#pragma unroll
  for (int m = 0; m < n; ++m) v[m * S] = u[m];
}

}  // namespace haar

// transform selector used by the kernels: kTf = 0 the DCT, 1 the Haar transform
constexpr int kTfDct = 0, kTfHaar = 1;
template <int kTf, typename T, int n, int S>
__host__ __device__ __forceinline__ void tf_forward(T* v) {
  if constexpr (kTf == kTfHaar) haar::forward<T, n, S>(v);
  else dct::forward<T, n, S>(v);
}
template <int kTf, typename T, int n, int S, int K>
__host__ __device__ __forceinline__ void tf_inverse(T* v) {
  if constexpr (kTf == kTfHaar) haar::inverse<T, n, S, K>(v);
  else dct::inverse<T, n, S, K>(v);
}

}  // namespace pbz
