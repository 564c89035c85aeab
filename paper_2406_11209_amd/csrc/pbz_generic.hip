// Fully general codec kernels: any dimensionality up to 8, any power-of-two block shape within the
// limits, any mask, any supported types.  One workgroup works on G whole blocks at a time, held in LDS;
// the transform is the dense contraction with the matrices H_d (Sec. III-A, Appendix A), one dimension
// per pass, ping-ponging between two LDS buffers.  Correct everywhere, tuned nowhere: the specialised
// kernels take the shapes that matter for throughput.
#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace {

constexpr int kThreads = 256;

// Blocks per workgroup iteration: a power of two, so that threads-per-block (kThreads / G) is integral.
int blocks_per_group(int vol) {
  int g = 1024 / vol;
  if (g < 1) g = 1;
  if (g > kThreads) g = kThreads;
  return g;
}

__device__ __forceinline__ void decode_element(const Geom& g, int64_t k, int j, int64_t* offset, bool* inside) {
  // block index k -> block coordinates, intra-block index j -> intra coordinates (both row-major)
  int64_t off = 0;
  bool in = true;
  for (int d = g.ndim - 1; d >= 0; --d) {
    int64_t kb = k % g.grid[d];
    k /= g.grid[d];
    int jd = j % g.block[d];
    j /= g.block[d];
    int64_t coord = kb * g.block[d] + jd;
    in = in && (coord < g.shape[d]);
    off += coord * g.stride[d];
  }
  *offset = off;
  *inside = in;
}

// One contraction pass over dimension d for every element of the G-block tile.
// forward:  out[.., q, ..] = sum_m in[.., m, ..] H[m][q];  inverse: out[.., m, ..] = sum_q in[.., q, ..] H[m][q]
template <typename T, bool kForward>
__device__ __forceinline__ void contract_dim(const T* in, T* out, int total, int n, int inner, const double* H) {
  for (int e = threadIdx.x; e < total; e += kThreads) {
    int o = (e / inner) % n;               // output index along this dimension
    int base = e - o * inner;              // element with index 0 along this dimension
    T acc = T(0);
    for (int a = 0; a < n; ++a) {
      T h = kForward ? T(H[a * n + o]) : T(H[o * n + a]);
      acc += in[base + a * inner] * h;
    }
    out[e] = acc;
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_compress_generic(Geom g, int G, const void* __restrict__ x, int xtype,
                                                               void* __restrict__ N, int ntype, void* __restrict__ F,
                                                               int itype, double r, const double* __restrict__ H,
                                                               const int32_t* __restrict__ kept_pos) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int total = G * g.vol;
  T* bufA = reinterpret_cast<T*>(smem);
  T* bufB = bufA + total;
  T* red = bufB + total;  // kThreads entries
  const int tpb = kThreads / G;  // threads per block for the max reduction
  const int64_t n_groups = (g.n_blocks + G - 1) / G;

  for (int64_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x) {
    // 1. gather G blocks, zero padded, converted to the compute type
    for (int e = threadIdx.x; e < total; e += kThreads) {
      int64_t k = grp * G + e / g.vol;
      T v = T(0);
      if (k < g.n_blocks) {
        int64_t off;
        bool in;
        decode_element(g, k, e % g.vol, &off, &in);
        if (in) v = load_float<T>(x, xtype, off);
      }
      bufA[e] = v;
    }
    __syncthreads();
    // 2. one pass per dimension
    T* src = bufA;
    T* dst = bufB;
    int inner = g.vol;
    for (int d = 0; d < g.ndim; ++d) {
      int n = g.block[d];
      inner /= n;
      if (n == 1) continue;
      contract_dim<T, true>(src, dst, total, n, inner, H + g.h_offset[d]);
      __syncthreads();
      T* tmp = src;
      src = dst;
      dst = tmp;
    }
    // 3. per-block max |C|
    {
      int b = threadIdx.x / tpb, l = threadIdx.x % tpb;
      T m = T(0);
      for (int j = l; j < g.vol; j += tpb) m = fmax(m, fabs(src[b * g.vol + j]));
      red[threadIdx.x] = m;
      __syncthreads();
      for (int s = tpb >> 1; s > 0; s >>= 1) {
        if (l < s) red[threadIdx.x] = fmax(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
      }
    }
    // 4. bin, prune, store
    for (int e = threadIdx.x; e < total; e += kThreads) {
      int b = e / g.vol, j = e % g.vol;
      int64_t k = grp * G + b;
      if (k >= g.n_blocks) continue;
      T nk = red[b * tpb];
      if (j == 0) store_float(N, ntype, k, nk);
      int pos = kept_pos[j];
      if (pos < 0) continue;
      T t = nk > T(0) ? (T(r) * src[e]) / nk : T(0);
      t = rint(t);
      t = fmin(fmax(t, T(-r)), T(r));
      store_index(F, itype, k * g.kept + pos, int64_t(t));
    }
    __syncthreads();
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_decompress_generic(Geom g, int G, const void* __restrict__ N, int ntype,
                                                                 const void* __restrict__ F, int itype, double r,
                                                                 void* __restrict__ y, int ytype,
                                                                 const double* __restrict__ H,
                                                                 const int32_t* __restrict__ kept_pos) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int total = G * g.vol;
  T* bufA = reinterpret_cast<T*>(smem);
  T* bufB = bufA + total;
  const int64_t n_groups = (g.n_blocks + G - 1) / G;

  for (int64_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x) {
    // 1. specified coefficients N F / r at the mask positions, zeros elsewhere (Algorithm 3)
    for (int e = threadIdx.x; e < total; e += kThreads) {
      int64_t k = grp * G + e / g.vol;
      T v = T(0);
      if (k < g.n_blocks) {
        int pos = kept_pos[e % g.vol];
        if (pos >= 0) {
          T nk = load_float<T>(N, ntype, k);
          v = (nk * T(load_index(F, itype, k * g.kept + pos))) / T(r);
        }
      }
      bufA[e] = v;
    }
    __syncthreads();
    // 2. inverse passes
    T* src = bufA;
    T* dst = bufB;
    int inner = g.vol;
    for (int d = 0; d < g.ndim; ++d) {
      int n = g.block[d];
      inner /= n;
      if (n == 1) continue;
      contract_dim<T, false>(src, dst, total, n, inner, H + g.h_offset[d]);
      __syncthreads();
      T* tmp = src;
      src = dst;
      dst = tmp;
    }
    // 3. merge blocks, crop, convert
    for (int e = threadIdx.x; e < total; e += kThreads) {
      int64_t k = grp * G + e / g.vol;
      if (k >= g.n_blocks) continue;
      int64_t off;
      bool in;
      decode_element(g, k, e % g.vol, &off, &in);
      if (in) store_float(y, ytype, off, src[e]);
    }
    __syncthreads();
  }
}

int grid_for(int64_t n_groups) {
  int64_t cap = 256 * 8;
  return int(n_groups < cap ? n_groups : cap);
}

}  // namespace

int launch_compress_generic(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* x, int xtype,
                            void* N, void* F, hipStream_t s) {
  const int G = blocks_per_group(c->vol);
  const int64_t n_groups = (g.n_blocks + G - 1) / G;
  const int total = G * c->vol;
  if (c->compute_f64) {
    size_t lds = sizeof(double) * (size_t(2 * total) + kThreads);
    hipLaunchKernelGGL(k_compress_generic<double>, dim3(grid_for(n_groups)), dim3(kThreads), lds, s, g, G, x, xtype, N,
                       int(c->ftype), F, int(c->itype), c->r, t->H, t->kept_pos);
  } else {
    size_t lds = sizeof(float) * (size_t(2 * total) + kThreads);
    hipLaunchKernelGGL(k_compress_generic<float>, dim3(grid_for(n_groups)), dim3(kThreads), lds, s, g, G, x, xtype, N,
                       int(c->ftype), F, int(c->itype), c->r, t->H, t->kept_pos);
  }
  return hip_status(hipGetLastError());
}

int launch_decompress_generic(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* N, const void* F,
                              void* y, int ytype, hipStream_t s) {
  const int G = blocks_per_group(c->vol);
  const int64_t n_groups = (g.n_blocks + G - 1) / G;
  const int total = G * c->vol;
  if (c->compute_f64) {
    size_t lds = sizeof(double) * size_t(2 * total);
    hipLaunchKernelGGL(k_decompress_generic<double>, dim3(grid_for(n_groups)), dim3(kThreads), lds, s, g, G, N,
                       int(c->ftype), F, int(c->itype), c->r, y, ytype, t->H, t->kept_pos);
  } else {
    size_t lds = sizeof(float) * size_t(2 * total);
    hipLaunchKernelGGL(k_decompress_generic<float>, dim3(grid_for(n_groups)), dim3(kThreads), lds, s, g, G, N,
                       int(c->ftype), F, int(c->itype), c->r, y, ytype, t->H, t->kept_pos);
  }
  return hip_status(hipGetLastError());
}

}  // namespace pbz
