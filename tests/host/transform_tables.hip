// Prints what the kernels' in-register transforms (pbz_dct.h, pbz_haar.h) compute on the host: for every length
// n and both precisions, the image of each unit vector under the forward transform and under the inverse
// transform (all inputs, and with only the first n/2 inputs declared non-zero).  A test compares the rows with
// transform matrices built independently of this code.  Built for the host only; nothing here runs on a GPU.
#include <cstdio>

#include "pbz_dct.h"
#include "pbz_haar.h"

using namespace pbz;

template <int TF, typename T, int n>
void dump(const char* tf, const char* type) {
  for (int m = 0; m < n; ++m) {
    T v[n];
    for (int i = 0; i < n; ++i) v[i] = T(i == m ? 1 : 0);
    tf_forward<TF, T, n, 1>(v);
    std::printf("fwd %s %s %d %d", tf, type, n, m);
    for (int i = 0; i < n; ++i) std::printf(" %.17g", double(v[i]));
    std::printf("\n");
  }
  for (int q = 0; q < n; ++q) {
    T v[n];
    for (int i = 0; i < n; ++i) v[i] = T(i == q ? 1 : 0);
    tf_inverse<TF, T, n, 1, n>(v);
    std::printf("inv %s %s %d %d", tf, type, n, q);
    for (int i = 0; i < n; ++i) std::printf(" %.17g", double(v[i]));
    std::printf("\n");
  }
  if (n > 1) {
    for (int q = 0; q < n / 2; ++q) {     // inputs n/2 and above are declared zero and must not be read
      T v[n];
      for (int i = 0; i < n; ++i) v[i] = T(i == q ? 1 : (i >= n / 2 ? 1e30 : 0));
      tf_inverse<TF, T, n, 1, (n > 1 ? n / 2 : 1)>(v);
      std::printf("half %s %s %d %d", tf, type, n, q);
      for (int i = 0; i < n; ++i) std::printf(" %.17g", double(v[i]));
      std::printf("\n");
    }
  }
}

template <int TF>
void all(const char* tf) {
  dump<TF, float, 1>(tf, "f32");  dump<TF, double, 1>(tf, "f64");
  dump<TF, float, 2>(tf, "f32");  dump<TF, double, 2>(tf, "f64");
  dump<TF, float, 4>(tf, "f32");  dump<TF, double, 4>(tf, "f64");
  dump<TF, float, 8>(tf, "f32");  dump<TF, double, 8>(tf, "f64");
  dump<TF, float, 16>(tf, "f32"); dump<TF, double, 16>(tf, "f64");
  dump<TF, float, 32>(tf, "f32"); dump<TF, double, 32>(tf, "f64");
}

int main() {
  all<kTfDct>("dct");
  all<kTfHaar>("haar");
  return 0;
}
