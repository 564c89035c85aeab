// Compressed-space operations (Sec. IV-A): negate, multiply by a scalar, add, and the reductions
// dot / norm / cosine similarity / mean / covariance / variance.
//
// All of them stream N and F once.  The streaming kernels view F as 16-byte vectors; they need
// kept * sizeof(index) to be a multiple of 16 bytes (every vector lies inside one block) and 16-byte
// aligned pointers.  Everything else takes the slower per-element kernels at the end of this file.
#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int ilog2_exact(int64_t v) {  // log2(v) when v is a power of two, else -1
  if (v < 1 || (v & (v - 1))) return -1;
  int s = 0;
  while ((int64_t(1) << s) < v) ++s;
  return s;
}

int stream_groups(int64_t items, int per_thread) {
  int64_t g = (items + int64_t(kThreads) * per_thread - 1) / (int64_t(kThreads) * per_thread);
  if (g < 1) g = 1;
  if (g > kReduceMaxGroups) g = kReduceMaxGroups;
  return int(g);
}

// ---------------------------------------------------------------------------------------------
// packed integer helpers on one dword
// ---------------------------------------------------------------------------------------------
template <int kIType>
__device__ __forceinline__ uint32_t negate_packed(uint32_t x) {
  if (kIType == PBZ_I8) {
    uint32_t y = ~x;
    return ((y & 0x7f7f7f7fu) + 0x01010101u) ^ (y & 0x80808080u);
  } else if (kIType == PBZ_I16) {
    uint32_t y = ~x;
    return ((y & 0x7fff7fffu) + 0x00010001u) ^ (y & 0x80008000u);
  } else {
    return uint32_t(-int32_t(x));
  }
}

typedef short short2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ short2v as_short2(uint32_t u) {
  short2v s;
  s.x = short(u & 0xffffu);
  s.y = short(u >> 16);
  return s;
}

// sum over the elements of one dword of a*b, as a double (exact)
template <int kIType>
__device__ __forceinline__ double dot_dword(uint32_t a, uint32_t b) {
  if (kIType == PBZ_I8) {
    return double(__builtin_amdgcn_sdot4(int(a), int(b), 0, false));
  } else if (kIType == PBZ_I16) {
    return double(__builtin_amdgcn_sdot2(as_short2(a), as_short2(b), 0, false));
  } else {
    return double(int32_t(a)) * double(int32_t(b));
  }
}

// exact integer dot product of two 16-byte vectors for 8- and 16-bit indices
template <int kIType>
__device__ __forceinline__ double dot_vec(const uint4& a, const uint4& b) {
  if (kIType == PBZ_I8) {
    int acc = __builtin_amdgcn_sdot4(int(a.x), int(b.x), 0, false);
    acc = __builtin_amdgcn_sdot4(int(a.y), int(b.y), acc, false);
    acc = __builtin_amdgcn_sdot4(int(a.z), int(b.z), acc, false);
    acc = __builtin_amdgcn_sdot4(int(a.w), int(b.w), acc, false);
    return double(acc);
  } else if (kIType == PBZ_I16) {
    // one dword: at most 2 * 32767^2 < 2^31; four of them need 64 bits
    long long acc = (long long)__builtin_amdgcn_sdot2(as_short2(a.x), as_short2(b.x), 0, false);
    acc += (long long)__builtin_amdgcn_sdot2(as_short2(a.y), as_short2(b.y), 0, false);
    acc += (long long)__builtin_amdgcn_sdot2(as_short2(a.z), as_short2(b.z), 0, false);
    acc += (long long)__builtin_amdgcn_sdot2(as_short2(a.w), as_short2(b.w), 0, false);
    return double(acc);
  } else {
    return dot_dword<PBZ_I32>(a.x, b.x) + dot_dword<PBZ_I32>(a.y, b.y) + dot_dword<PBZ_I32>(a.z, b.z) +
           dot_dword<PBZ_I32>(a.w, b.w);
  }
}

template <int kIType>
__device__ __forceinline__ int first_element(uint32_t x) {
  if (kIType == PBZ_I8) return int(int8_t(x & 0xffu));
  if (kIType == PBZ_I16) return int(int16_t(x & 0xffffu));
  return int(x);
}

template <int kIType>
__device__ __forceinline__ void unpack_dword(uint32_t x, double* out) {  // 4 / 2 / 1 elements
  if (kIType == PBZ_I8) {
    out[0] = double(int(int8_t(x & 0xffu)));
    out[1] = double(int(int8_t((x >> 8) & 0xffu)));
    out[2] = double(int(int8_t((x >> 16) & 0xffu)));
    out[3] = double(int(int8_t(x >> 24)));
  } else if (kIType == PBZ_I16) {
    out[0] = double(int(int16_t(x & 0xffffu)));
    out[1] = double(int(int16_t(x >> 16)));
  } else {
    out[0] = double(int32_t(x));
  }
}

template <int kIType>
__device__ __forceinline__ uint32_t pack_dword(const int* v) {
  if (kIType == PBZ_I8)
    return (uint32_t(v[0]) & 0xffu) | ((uint32_t(v[1]) & 0xffu) << 8) | ((uint32_t(v[2]) & 0xffu) << 16) |
           (uint32_t(v[3]) << 24);
  if (kIType == PBZ_I16) return (uint32_t(v[0]) & 0xffffu) | (uint32_t(v[1]) << 16);
  return uint32_t(v[0]);
}

// F1 N1 + F2 N2 with both products and the sum rounded separately (Algorithm 2 as printed): a fused
// multiply-add would skip one rounding and break A + (-A) == 0 when N has more than 37 significant bits.
__device__ __forceinline__ double unfused_sum_of_products(double f1, double n1, double f2, double n2) {
#pragma clang fp contract(off)
  const double p1 = f1 * n1;
  const double p2 = f2 * n2;
  return p1 + p2;
}

template <int kIType>
struct PerDword {
  static constexpr int value = kIType == PBZ_I8 ? 4 : kIType == PBZ_I16 ? 2 : 1;
};

// ---------------------------------------------------------------------------------------------
// Algorithm 1 (and the F part of Algorithm 5): F_out = sign * F_in over 16-byte vectors
// ---------------------------------------------------------------------------------------------
template <int kIType, int kSign>
__global__ __launch_bounds__(kThreads) void k_scale_sign_vec(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                             int64_t nvec) {
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t v = int64_t(blockIdx.x) * kThreads + threadIdx.x; v < nvec; v += nthreads) {
    uint4 a = make_uint4(0u, 0u, 0u, 0u);
    if (kSign != 0) a = in[v];
    if (kSign < 0) {
      a.x = negate_packed<kIType>(a.x);
      a.y = negate_packed<kIType>(a.y);
      a.z = negate_packed<kIType>(a.z);
      a.w = negate_packed<kIType>(a.w);
    }
    out[v] = a;
  }
}

__global__ __launch_bounds__(kThreads) void k_scale_sign_scalar(const void* __restrict__ in, void* __restrict__ out,
                                                                int itype, int sign, int64_t n) {
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t e = int64_t(blockIdx.x) * kThreads + threadIdx.x; e < n; e += nthreads)
    store_index(out, itype, e, sign == 0 ? 0 : sign * load_index(in, itype, e));
}

template <int kSign>
void launch_sign_vec(int itype, const void* in, void* out, int64_t nvec, hipStream_t s) {
  dim3 grid(stream_groups(nvec, 2)), block(kThreads);
  const uint4* i4 = static_cast<const uint4*>(in);
  uint4* o4 = static_cast<uint4*>(out);
  if (itype == PBZ_I8)
    hipLaunchKernelGGL((k_scale_sign_vec<PBZ_I8, kSign>), grid, block, 0, s, i4, o4, nvec);
  else if (itype == PBZ_I16)
    hipLaunchKernelGGL((k_scale_sign_vec<PBZ_I16, kSign>), grid, block, 0, s, i4, o4, nvec);
  else
    hipLaunchKernelGGL((k_scale_sign_vec<PBZ_I32, kSign>), grid, block, 0, s, i4, o4, nvec);
}

int scale_sign(const pbz_codec* c, int64_t n_blocks, const void* in, void* out, int sign, hipStream_t s) {
  if (sign > 0 && in == out) return PBZ_OK;
  const int64_t n = n_blocks * c->kept;
  const int64_t bytes = n * itype_bytes(c->itype);
  if (bytes % 16 == 0 && aligned16(in) && aligned16(out)) {
    if (sign > 0)
      launch_sign_vec<1>(c->itype, in, out, bytes / 16, s);
    else if (sign < 0)
      launch_sign_vec<-1>(c->itype, in, out, bytes / 16, s);
    else
      launch_sign_vec<0>(c->itype, in, out, bytes / 16, s);
  } else {
    hipLaunchKernelGGL(k_scale_sign_scalar, dim3(stream_groups(n, 4)), dim3(kThreads), 0, s, in, out, int(c->itype),
                       sign, n);
  }
  return hip_status(hipGetLastError());
}

// Algorithm 5, N part: N_out = N_in |x| rounded to the working type
__global__ __launch_bounds__(kThreads) void k_scale_N(const void* __restrict__ in, void* __restrict__ out, int ntype,
                                                      double ax, int64_t n) {
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t k = int64_t(blockIdx.x) * kThreads + threadIdx.x; k < n; k += nthreads)
    store_float(out, ntype, k, load_float<double>(in, ntype, k) * ax);
}

// ---------------------------------------------------------------------------------------------
// Algorithm 2: element-wise addition with rebinning, in FP64, exactly in the printed operation order:
// C = F1 N1 + F2 N2 (each product and the sum rounded separately), N = max|C| / r, F = rint(C / N).
// A block occupies kLanes consecutive lanes, 16 bytes of F per lane.
// ---------------------------------------------------------------------------------------------
template <int kIType>
__global__ __launch_bounds__(kThreads) void k_add_vec(const void* __restrict__ N1, const uint4* __restrict__ F1,
                                                      const void* __restrict__ N2, const uint4* __restrict__ F2,
                                                      void* __restrict__ Nout, uint4* __restrict__ Fout, int ntype,
                                                      double r, int64_t nvec, int lanes_shift) {
  constexpr int kPer = PerDword<kIType>::value;
  constexpr int kElems = 4 * kPer;
  const int lanes = 1 << lanes_shift;
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  // the loop bound is uniform over the wave so that the lane exchanges below are always convergent
  const int64_t first = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t wave_first = first - (threadIdx.x & 63);
  for (int64_t base = wave_first; base < nvec; base += nthreads) {
    const int64_t v = base + (threadIdx.x & 63);
    const bool live = v < nvec;
    const int64_t k = v >> lanes_shift;
    double c[kElems];
    double m = 0.0;
    if (live) {
      const uint4 a = F1[v], b = F2[v];
      const double n1 = load_float<double>(N1, ntype, k), n2 = load_float<double>(N2, ntype, k);
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        double fa[kPer], fb[kPer];
        unpack_dword<kIType>(aw[w], fa);
        unpack_dword<kIType>(bw[w], fb);
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
          double ce = unfused_sum_of_products(fa[e], n1, fb[e], n2);
          c[w * kPer + e] = ce;
          m = fmax(m, fabs(ce));
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < kElems; ++e) c[e] = 0.0;
    }
    for (int off = lanes >> 1; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
    if (live) {
      const double n = m / r;
      uint32_t ow[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        int q[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
          double t = n > 0.0 ? c[w * kPer + e] / n : 0.0;
          t = fmin(fmax(rint(t), -r), r);
          q[e] = int(t);
        }
        ow[w] = pack_dword<kIType>(q);
      }
      Fout[v] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
      if ((v & (lanes - 1)) == 0) store_float(Nout, ntype, k, n);
    }
  }
}

// one wave per block, any kept count, any alignment
__global__ __launch_bounds__(64) void k_add_generic(const void* __restrict__ N1, const void* __restrict__ F1,
                                                    const void* __restrict__ N2, const void* __restrict__ F2,
                                                    void* __restrict__ Nout, void* __restrict__ Fout, int ntype,
                                                    int itype, double r, int64_t n_blocks, int kept) {
  for (int64_t k = blockIdx.x; k < n_blocks; k += gridDim.x) {
    const double n1 = load_float<double>(N1, ntype, k), n2 = load_float<double>(N2, ntype, k);
    double m = 0.0;
    for (int j = threadIdx.x; j < kept; j += 64) {
      double ce = unfused_sum_of_products(double(load_index(F1, itype, k * kept + j)), n1,
                                          double(load_index(F2, itype, k * kept + j)), n2);
      m = fmax(m, fabs(ce));
    }
    for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
    const double n = m / r;
    // F_out may alias an operand: every lane re-reads only the entries it then overwrites
    for (int j = threadIdx.x; j < kept; j += 64) {
      double ce = unfused_sum_of_products(double(load_index(F1, itype, k * kept + j)), n1,
                                          double(load_index(F2, itype, k * kept + j)), n2);
      double t = n > 0.0 ? ce / n : 0.0;
      t = fmin(fmax(rint(t), -r), r);
      store_index(Fout, itype, k * kept + j, int64_t(t));
    }
    if (threadIdx.x == 0) store_float(Nout, ntype, k, n);
  }
}

// ---------------------------------------------------------------------------------------------
// Reductions (Algorithms 6-11).  One streaming pass produces five FP64 sums per workgroup,
//   S12 = sum_k N1_k N2_k sum_j F1_kj F2_kj     S11, S22 likewise     D1 = sum_k N1_k F1_k0   D2 likewise
// (integer block sums are exact; the scale 1/r or 1/r^2 is applied once at the end), a second tiny
// kernel adds the partials in a fixed order and evaluates the requested statistic.
// ---------------------------------------------------------------------------------------------
enum { kS12 = 0, kS11 = 1, kS22 = 2, kD1 = 3, kD2 = 4, kNumSums = 5 };

__device__ __forceinline__ void store_partials(double* sums, double* __restrict__ partials) {
  __shared__ double lds[kThreads / 64][kNumSums];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < kNumSums; ++i) {
    double t = wave_sum(sums[i]);
    if (lane == 0) lds[wave][i] = t;
  }
  __syncthreads();
  if (threadIdx.x < kNumSums) {
    double t = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) t += lds[w][threadIdx.x];
    partials[int64_t(blockIdx.x) * kReducePartialSlots + threadIdx.x] = t;
  }
}

template <int kIType, bool kTwo, bool kDC>
__global__ __launch_bounds__(kThreads) void k_reduce_vec(const void* __restrict__ N1, const uint4* __restrict__ F1,
                                                         const void* __restrict__ N2, const uint4* __restrict__ F2,
                                                         int ntype, int64_t nvec, int vpb_shift, int64_t vpb,
                                                         double* __restrict__ partials) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t v0 = int64_t(blockIdx.x) * kThreads + threadIdx.x; v0 < nvec; v0 += nthreads * kUnroll) {
    uint4 a[kUnroll], b[kUnroll];
    double n1[kUnroll], n2[kUnroll];
    bool head[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t v = v0 + u * nthreads;
      a[u] = make_uint4(0u, 0u, 0u, 0u);
      b[u] = a[u];
      n1[u] = n2[u] = 0.0;
      head[u] = false;
      if (v < nvec) {
        const int64_t k = vpb_shift >= 0 ? (v >> vpb_shift) : (v / vpb);
        head[u] = (v - k * vpb) == 0;
        a[u] = F1[v];
        n1[u] = load_float<double>(N1, ntype, k);
        if (kTwo) {
          b[u] = F2[v];
          n2[u] = load_float<double>(N2, ntype, k);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      sums[kS11] += dot_vec<kIType>(a[u], a[u]) * (n1[u] * n1[u]);
      if (kTwo) {
        sums[kS12] += dot_vec<kIType>(a[u], b[u]) * (n1[u] * n2[u]);
        sums[kS22] += dot_vec<kIType>(b[u], b[u]) * (n2[u] * n2[u]);
      }
      if (kDC && head[u]) {
        sums[kD1] += n1[u] * double(first_element<kIType>(a[u].x));
        if (kTwo) sums[kD2] += n2[u] * double(first_element<kIType>(b[u].x));
      }
    }
  }
  store_partials(sums, partials);
}

// thread per block, any kept count and alignment
__global__ __launch_bounds__(kThreads) void k_reduce_generic(const void* __restrict__ N1, const void* __restrict__ F1,
                                                             const void* __restrict__ N2, const void* __restrict__ F2,
                                                             int ntype, int itype, int64_t n_blocks, int kept,
                                                             int two, int dc, double* __restrict__ partials) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t k = int64_t(blockIdx.x) * kThreads + threadIdx.x; k < n_blocks; k += nthreads) {
    const double n1 = load_float<double>(N1, ntype, k);
    const double n2 = two ? load_float<double>(N2, ntype, k) : 0.0;
    double s11 = 0.0, s12 = 0.0, s22 = 0.0;
    for (int j = 0; j < kept; ++j) {
      const double f1 = double(load_index(F1, itype, k * kept + j));
      s11 += f1 * f1;
      if (two) {
        const double f2 = double(load_index(F2, itype, k * kept + j));
        s12 += f1 * f2;
        s22 += f2 * f2;
      }
    }
    sums[kS11] += s11 * (n1 * n1);
    sums[kS12] += s12 * (n1 * n2);
    sums[kS22] += s22 * (n2 * n2);
    if (dc) {
      sums[kD1] += n1 * double(load_index(F1, itype, k * kept));
      if (two) sums[kD2] += n2 * double(load_index(F2, itype, k * kept));
    }
  }
  store_partials(sums, partials);
}

// Algorithm 7 needs only N and the first kept index of every block
__global__ __launch_bounds__(kThreads) void k_reduce_dc(const void* __restrict__ N1, const void* __restrict__ F1,
                                                        int ntype, int itype, int64_t n_blocks, int kept,
                                                        double* __restrict__ partials) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t k = int64_t(blockIdx.x) * kThreads + threadIdx.x; k < n_blocks; k += nthreads)
    sums[kD1] += load_float<double>(N1, ntype, k) * double(load_index(F1, itype, k * kept));
  store_partials(sums, partials);
}

__global__ __launch_bounds__(kThreads) void k_reduce_final(const double* __restrict__ partials, int n_partials, int op,
                                                           double r, double n_blocks, double vol,
                                                           double* __restrict__ out) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  for (int p = threadIdx.x; p < n_partials; p += kThreads)
#pragma unroll
    for (int i = 0; i < kNumSums; ++i) sums[i] += partials[int64_t(p) * kReducePartialSlots + i];
  __shared__ double lds[kThreads / 64][kNumSums];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < kNumSums; ++i) {
    double t = wave_sum(sums[i]);
    if (lane == 0) lds[wave][i] = t;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  double s[kNumSums];
  for (int i = 0; i < kNumSums; ++i) {
    s[i] = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) s[i] += lds[w][i];
  }
  double res = 0.0;
  switch (op) {
    case kDot: res = s[kS12] / (r * r); break;
    case kNorm2: res = sqrt(s[kS11]) / r; break;
    case kCosine: res = s[kS12] / (sqrt(s[kS11]) * sqrt(s[kS22])); break;
    case kMean: res = (s[kD1] / r) / (n_blocks * sqrt(vol)); break;
    // centring the first coefficients by their mean removes (sum D1)(sum D2) / n_blocks from the raw sum
    case kCovariance: res = ((s[kS12] - s[kD1] * s[kD2] / n_blocks) / (r * r)) / (n_blocks * vol); break;
    case kVariance: res = ((s[kS11] - s[kD1] * s[kD1] / n_blocks) / (r * r)) / (n_blocks * vol); break;
    default: break;
  }
  *out = res;
}

template <int kIType>
void launch_reduce_vec(bool two, bool dc, dim3 grid, hipStream_t s, const void* N1, const void* F1, const void* N2,
                       const void* F2, int ntype, int64_t nvec, int shift, int64_t vpb, double* partials) {
  const uint4* a = static_cast<const uint4*>(F1);
  const uint4* b = static_cast<const uint4*>(F2);
  dim3 block(kThreads);
  if (two && dc)
    hipLaunchKernelGGL((k_reduce_vec<kIType, true, true>), grid, block, 0, s, N1, a, N2, b, ntype, nvec, shift, vpb, partials);
  else if (two)
    hipLaunchKernelGGL((k_reduce_vec<kIType, true, false>), grid, block, 0, s, N1, a, N2, b, ntype, nvec, shift, vpb, partials);
  else if (dc)
    hipLaunchKernelGGL((k_reduce_vec<kIType, false, true>), grid, block, 0, s, N1, a, N2, b, ntype, nvec, shift, vpb, partials);
  else
    hipLaunchKernelGGL((k_reduce_vec<kIType, false, false>), grid, block, 0, s, N1, a, N2, b, ntype, nvec, shift, vpb, partials);
}

}  // namespace

int launch_negate(const pbz_codec* c, int64_t n_blocks, const void* Fin, void* Fout, hipStream_t s) {
  return scale_sign(c, n_blocks, Fin, Fout, -1, s);
}

int launch_mul_scalar(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double x, void* Nout,
                      void* Fout, hipStream_t s) {
  hipLaunchKernelGGL(k_scale_N, dim3(stream_groups(n_blocks, 4)), dim3(kThreads), 0, s, Nin, Nout, int(c->ftype),
                     std::fabs(x), n_blocks);
  int st = hip_status(hipGetLastError());
  if (st != PBZ_OK) return st;
  return scale_sign(c, n_blocks, Fin, Fout, x > 0.0 ? 1 : (x < 0.0 ? -1 : 0), s);
}

int launch_add(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
               void* Nout, void* Fout, hipStream_t s) {
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  const int lanes_shift = bpb % 16 == 0 ? ilog2_exact(bpb / 16) : -1;
  if (lanes_shift >= 0 && lanes_shift <= 6 && aligned16(F1) && aligned16(F2) && aligned16(Fout)) {
    const int64_t nvec = n_blocks * (bpb / 16);
    dim3 grid(stream_groups(nvec, 1)), block(kThreads);
    const uint4* a = static_cast<const uint4*>(F1);
    const uint4* b = static_cast<const uint4*>(F2);
    uint4* o = static_cast<uint4*>(Fout);
    if (c->itype == PBZ_I8)
      hipLaunchKernelGGL(k_add_vec<PBZ_I8>, grid, block, 0, s, N1, a, N2, b, Nout, o, int(c->ftype), c->r, nvec, lanes_shift);
    else if (c->itype == PBZ_I16)
      hipLaunchKernelGGL(k_add_vec<PBZ_I16>, grid, block, 0, s, N1, a, N2, b, Nout, o, int(c->ftype), c->r, nvec, lanes_shift);
    else
      hipLaunchKernelGGL(k_add_vec<PBZ_I32>, grid, block, 0, s, N1, a, N2, b, Nout, o, int(c->ftype), c->r, nvec, lanes_shift);
  } else {
    int64_t g = n_blocks < 65536 ? n_blocks : 65536;
    hipLaunchKernelGGL(k_add_generic, dim3(int(g)), dim3(64), 0, s, N1, F1, N2, F2, Nout, Fout, int(c->ftype),
                       int(c->itype), c->r, n_blocks, c->kept);
  }
  return hip_status(hipGetLastError());
}

int launch_reduce(const pbz_codec* c, ReduceOp op, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                  const void* F2, double* out, void* workspace, hipStream_t s) {
  double* partials = static_cast<double*>(workspace);
  const bool two = (op == kDot || op == kCosine || op == kCovariance);
  const bool dc = (op == kCovariance || op == kVariance);
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  int groups;
  if (op == kMean) {
    groups = stream_groups(n_blocks, 4);
    hipLaunchKernelGGL(k_reduce_dc, dim3(groups), dim3(kThreads), 0, s, N1, F1, int(c->ftype), int(c->itype), n_blocks,
                       c->kept, partials);
  } else if (bpb % 16 == 0 && aligned16(F1) && (!two || aligned16(F2))) {
    const int64_t vpb = bpb / 16;
    const int64_t nvec = n_blocks * vpb;
    groups = stream_groups(nvec, kUnroll);
    dim3 grid(groups);
    const int shift = ilog2_exact(vpb);
    if (c->itype == PBZ_I8)
      launch_reduce_vec<PBZ_I8>(two, dc, grid, s, N1, F1, N2, F2, int(c->ftype), nvec, shift, vpb, partials);
    else if (c->itype == PBZ_I16)
      launch_reduce_vec<PBZ_I16>(two, dc, grid, s, N1, F1, N2, F2, int(c->ftype), nvec, shift, vpb, partials);
    else
      launch_reduce_vec<PBZ_I32>(two, dc, grid, s, N1, F1, N2, F2, int(c->ftype), nvec, shift, vpb, partials);
  } else {
    groups = stream_groups(n_blocks, 1);
    hipLaunchKernelGGL(k_reduce_generic, dim3(groups), dim3(kThreads), 0, s, N1, F1, N2, F2, int(c->ftype),
                       int(c->itype), n_blocks, c->kept, two ? 1 : 0, dc ? 1 : 0, partials);
  }
  int st = hip_status(hipGetLastError());
  if (st != PBZ_OK) return st;
  hipLaunchKernelGGL(k_reduce_final, dim3(1), dim3(kThreads), 0, s, partials, groups, int(op), c->r, double(n_blocks),
                     double(c->vol), out);
  return hip_status(hipGetLastError());
}

}  // namespace pbz
