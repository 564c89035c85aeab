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
constexpr int kReduceGroupsOneSegment = 1024;

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

// the low bytes (int8) or halves (int16) of 4 / 2 integers gathered into one dword by byte permutes
template <int kIType>
__device__ __forceinline__ uint32_t pack_dword(const int* v) {
  if (kIType == PBZ_I8) {
    const uint32_t lo = __builtin_amdgcn_perm(uint32_t(v[1]), uint32_t(v[0]), 0x0c0c0400u);   // v0.b0, v1.b0
    const uint32_t hi = __builtin_amdgcn_perm(uint32_t(v[3]), uint32_t(v[2]), 0x0c0c0400u);   // v2.b0, v3.b0
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
  }
  if (kIType == PBZ_I16) return __builtin_amdgcn_perm(uint32_t(v[1]), uint32_t(v[0]), 0x05040100u);
  return uint32_t(v[0]);
}

// rint(t) as an integer for |t| < 2^31: adding 1.5 * 2^52 rounds t to an integer in the current (nearest-even)
// mode and leaves that integer, in two's complement, in the low word of the sum
__device__ __forceinline__ int rint_to_int(double t) {
  return int(uint32_t(__builtin_bit_cast(uint64_t, t + 6755399441055744.0)));
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
__device__ __forceinline__ uint4 apply_sign(uint4 a) {
  if (kSign == 0) return make_uint4(0u, 0u, 0u, 0u);
  if (kSign < 0) {
    a.x = negate_packed<kIType>(a.x);
    a.y = negate_packed<kIType>(a.y);
    a.z = negate_packed<kIType>(a.z);
    a.w = negate_packed<kIType>(a.w);
  }
  return a;
}

// Each workgroup streams one contiguous run of kThreads * kUnroll vectors: kUnroll independent loads per thread
// (kThreads vectors apart), then the stores.  The element-wise kernels of this file may be called in place (an
// output aliasing the operand it replaces), so none of their pointers is declared __restrict__; every lane reads
// all it needs of an element before it writes that element.
template <int kIType, int kSign>
__device__ __forceinline__ void scale_sign_run(const uint4* in, uint4* out, int64_t nvec,
                                               int64_t group) {
  const int64_t base = group * (kThreads * kUnroll) + threadIdx.x;
  if (base + (kUnroll - 1) * kThreads < nvec) {
    uint4 a[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) a[u] = kSign != 0 ? in[base + u * kThreads] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) out[base + u * kThreads] = apply_sign<kIType, kSign>(a[u]);
  } else {
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t v = base + u * kThreads;
      if (v < nvec) out[v] = apply_sign<kIType, kSign>(kSign != 0 ? in[v] : make_uint4(0u, 0u, 0u, 0u));
    }
  }
}

template <int kIType, int kSign>
__global__ __launch_bounds__(kThreads) void k_scale_sign_vec(const uint4* in, uint4* out,
                                                             int64_t nvec) {
  scale_sign_run<kIType, kSign>(in, out, nvec, blockIdx.x);
}

// Algorithm 5 in one launch: the first f_groups workgroups write F_out = sign(x) F_in, the others N_out = |x| N_in
template <int kIType, int kSign>
__global__ __launch_bounds__(kThreads) void k_mul_scalar_vec(const uint4* Fin, uint4* Fout,
                                                             int64_t nvec, unsigned f_groups,
                                                             const void* Nin, void* Nout, int ntype, double ax,
                                                             int64_t n_blocks) {   // Nin may be Nout

  if (blockIdx.x < f_groups) {
    scale_sign_run<kIType, kSign>(Fin, Fout, nvec, blockIdx.x);
    return;
  }
  const int64_t nthreads = int64_t(gridDim.x - f_groups) * kThreads;
  for (int64_t k = int64_t(blockIdx.x - f_groups) * kThreads + threadIdx.x; k < n_blocks; k += nthreads)
    store_float(Nout, ntype, k, load_float<double>(Nin, ntype, k) * ax);
}

__global__ __launch_bounds__(kThreads) void k_scale_sign_scalar(const void* in, void* out,
                                                                int itype, int sign, int64_t n) {
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t e = int64_t(blockIdx.x) * kThreads + threadIdx.x; e < n; e += nthreads)
    store_index(out, itype, e, sign == 0 ? 0 : sign * load_index(in, itype, e));
}

template <int kSign>
void launch_sign_vec(int itype, const void* in, void* out, int64_t nvec, hipStream_t s) {
  const int64_t per_group = int64_t(kThreads) * kUnroll;
  dim3 grid(static_cast<unsigned>((nvec + per_group - 1) / per_group)), block(kThreads);
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
__global__ __launch_bounds__(kThreads) void k_scale_N(const void* in, void* out, int ntype,
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
// N comes in three widths: kNType = PBZ_F64, PBZ_F32, or kN16 for the two 16-bit types, which share a kernel:
// the 16-bit load is the same, both decodings are computed and `f16` (uniform) selects one, so that no branch
// surrounds a load.
constexpr int kN16 = PBZ_BF16;
constexpr int n_kernel_type(int ftype) { return ftype == PBZ_F64 ? PBZ_F64 : (ftype == PBZ_F32 ? PBZ_F32 : kN16); }

template <int kNType>
__device__ __forceinline__ double load_N(const void* N, int64_t k, bool f16 = false) {
  if (kNType == PBZ_F64) return static_cast<const double*>(N)[k];
  if (kNType == PBZ_F32) return double(static_cast<const float*>(N)[k]);
  const uint16_t h = static_cast<const uint16_t*>(N)[k];
  const float as_bf16 = bf16_bits_to_float(h);
  const float as_f16 = float(__builtin_bit_cast(_Float16, h));
  return double(f16 ? as_f16 : as_bf16);
}

template <int kNType>
__device__ __forceinline__ void store_N(void* N, int64_t k, double v, bool f16 = false) {
  if (kNType == PBZ_F64) {
    static_cast<double*>(N)[k] = v;
  } else if (kNType == PBZ_F32) {
    static_cast<float*>(N)[k] = float(v);
  } else {
    const uint16_t as_bf16 = double_to_bf16_bits(v);
    const uint16_t as_f16 = __builtin_bit_cast(uint16_t, double_to_f16(v));
    static_cast<uint16_t*>(N)[k] = f16 ? as_f16 : as_bf16;
  }
}

// a / b rounded to nearest from a correctly rounded reciprocal: one multiply, the exact remainder by fused
// multiply-add, one correction.  Agrees with the hardware division sequence except in rare double-rounding
// corner cases, at a sixth of its cost.
__device__ __forceinline__ double div_by(double a, double b, double inv_b) {
  const double q = a * inv_b;
  const double rem = fma(-q, b, a);
  return fma(rem, inv_b, q);
}

template <int kIType, int kNType>
__global__ __launch_bounds__(kThreads) void k_add_vec(const void* N1, const uint4* F1,
                                                      const void* N2, const uint4* F2,
                                                      void* Nout, uint4* Fout, double r,
                                                      double sign2, int64_t nvec, int lanes_shift, int n_f16) {
  constexpr int kPer = PerDword<kIType>::value;
  constexpr int kElems = 4 * kPer;
  constexpr bool kExactProducts = kNType != PBZ_F64 && kIType != PBZ_I32;
  const int lanes = 1 << lanes_shift;
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  // sign2 = -1 subtracts: F2 (-N2) is exactly (-F2) N2, so the result is bit for bit that of negate + add
  // the loop bound is uniform over the wave so that the lane exchanges below are always convergent
  const int64_t first = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t wave_first = first - (threadIdx.x & 63);
  for (int64_t base = wave_first; base < nvec; base += nthreads) {
    const int64_t v = base + (threadIdx.x & 63);
    const bool live = v < nvec;
    const int64_t vc = live ? v : nvec - 1;      // lanes past the end redo the last vector and store nothing
    const int64_t k = vc >> lanes_shift;
    const uint4 a = F1[vc], b = F2[vc];
    const double n1 = load_N<kNType>(N1, k, n_f16 != 0), n2 = sign2 * load_N<kNType>(N2, k, n_f16 != 0);
    double c[kElems];
    double m = 0.0;
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      double fa[kPer], fb[kPer];
      unpack_dword<kIType>(aw[w], fa);
      unpack_dword<kIType>(bw[w], fb);
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        // an FP32-valued N times an index of at most 16 bits is exact in FP64, so fusing the first product
        // rounds exactly as the printed order does; otherwise both products are rounded on their own
        const double ce = kExactProducts ? fma(fa[e], n1, fb[e] * n2) : unfused_sum_of_products(fa[e], n1, fb[e], n2);
        c[w * kPer + e] = ce;
        m = fmax(m, fabs(ce));
      }
    }
    for (int off = lanes >> 1; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
    const double n = m / r;
    // F = rint(C / N), the quotient from the correctly rounded reciprocal with one remainder correction
    const double inv = n > 0.0 ? 1.0 / n : 0.0;
    uint32_t ow[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      int q[kPer];
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        // an all-zero block has n = inv = 0 and every c = 0: the three steps then give 0 without a division.
        // |C / N| <= r (1 + 2^-52), which rounds to at most r, so no clamp is needed.
        q[e] = rint_to_int(div_by(c[w * kPer + e], n, inv));
      }
      ow[w] = pack_dword<kIType>(q);
    }
    if (live) {
      Fout[v] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
      if ((v & (lanes - 1)) == 0) store_N<kNType>(Nout, k, n, n_f16 != 0);
    }
  }
}

// one wave per block, any kept count, any alignment
__global__ __launch_bounds__(64) void k_add_generic(const void* N1, const void* F1,
                                                    const void* N2, const void* F2,
                                                    void* Nout, void* Fout, int ntype,
                                                    int itype, double r, double sign2, int64_t n_blocks, int kept) {
  for (int64_t k = blockIdx.x; k < n_blocks; k += gridDim.x) {
    const double n1 = load_float<double>(N1, ntype, k), n2 = sign2 * load_float<double>(N2, ntype, k);
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
// Algorithm 4: addition of a scalar.  C = N F / r, the first coefficient of every block moves by
// x prod(sqrt(i)), then N = max|C| (taken after the shift, so that no index can exceed r) and
// F = rint(C r / N).  Same lane layout as k_add_vec.
// ---------------------------------------------------------------------------------------------
template <int kIType, int kNType>
__global__ __launch_bounds__(kThreads) void k_add_scalar_vec(const void* N1, const uint4* F1,
                                                             void* Nout, uint4* Fout,
                                                             double r, double shift, int64_t nvec, int lanes_shift,
                                                             int n_f16) {
  constexpr int kPer = PerDword<kIType>::value;
  constexpr int kElems = 4 * kPer;
  const int lanes = 1 << lanes_shift;
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  const int64_t first = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t wave_first = first - (threadIdx.x & 63);
  const double inv_r = 1.0 / r;
  for (int64_t base = wave_first; base < nvec; base += nthreads) {
    const int64_t v = base + (threadIdx.x & 63);
    const bool live = v < nvec;
    const int64_t vc = live ? v : nvec - 1;
    const int64_t k = vc >> lanes_shift;
    const uint4 a = F1[vc];
    const double n1 = load_N<kNType>(N1, k, n_f16 != 0);
    const bool head = (vc & (lanes - 1)) == 0;
    double c[kElems];
    double m = 0.0;
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      double fa[kPer];
      unpack_dword<kIType>(aw[w], fa);
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        double ce = div_by(n1 * fa[e], r, inv_r);          // N F / r as printed
        if (w == 0 && e == 0 && head) ce += shift;
        c[w * kPer + e] = ce;
        m = fmax(m, fabs(ce));
      }
    }
    for (int off = lanes >> 1; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
    // F = rint(C r / N) in the printed order (exact ties are common here: when a small-index coefficient becomes
    // the block maximum, the others are simple fractions of r)
    const double inv_m = m > 0.0 ? 1.0 / m : 0.0;
    uint32_t ow[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      int q[kPer];
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        // an all-zero block has m = inv_m = 0 and every c = 0, which gives 0; |C r / N| <= r (1 + 2^-51) rounds to
        // at most r, so neither a special case nor a clamp is needed
        q[e] = rint_to_int(div_by(c[w * kPer + e] * r, m, inv_m));
      }
      ow[w] = pack_dword<kIType>(q);
    }
    if (live) {
      Fout[v] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
      if (head) store_N<kNType>(Nout, k, m, n_f16 != 0);
    }
  }
}

__global__ __launch_bounds__(64) void k_add_scalar_generic(const void* N1, const void* F1,
                                                           void* Nout, void* Fout, int ntype,
                                                           int itype, double r, double shift, int64_t n_blocks,
                                                           int kept) {
  for (int64_t k = blockIdx.x; k < n_blocks; k += gridDim.x) {
    const double n1 = load_float<double>(N1, ntype, k);
    double m = 0.0;
    for (int j = threadIdx.x; j < kept; j += 64) {
      double ce = (n1 * double(load_index(F1, itype, k * kept + j))) / r + (j == 0 ? shift : 0.0);
      m = fmax(m, fabs(ce));
    }
    for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
    for (int j = threadIdx.x; j < kept; j += 64) {
      double ce = (n1 * double(load_index(F1, itype, k * kept + j))) / r + (j == 0 ? shift : 0.0);
      double t = m > 0.0 ? (ce * r) / m : 0.0;
      store_index(Fout, itype, k * kept + j, int64_t(fmin(fmax(rint(t), -r), r)));
    }
    if (threadIdx.x == 0) store_float(Nout, ntype, k, m);
  }
}

// ---------------------------------------------------------------------------------------------
// Block-wise statistics (Sec. IV-A): one FP64 value per block.
//   mean_k = C_k0 / prod(sqrt(i));   covariance_k = (sum_j C1_kj C2_kj - C1_k0 C2_k0) / prod(i)
// (centring a block by its own mean zeroes its first coefficient); variance = covariance(A, A); std = sqrt.
// ---------------------------------------------------------------------------------------------
enum BlockwiseMode { kBwVariance = 0, kBwStd = 1, kBwCovariance = 2 };

__global__ __launch_bounds__(kThreads) void k_blockwise_mean(const void* __restrict__ N1, const void* __restrict__ F1,
                                                             int ntype, int itype, double scale, int64_t n_blocks,
                                                             int kept, double* __restrict__ out) {
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  for (int64_t k = int64_t(blockIdx.x) * kThreads + threadIdx.x; k < n_blocks; k += nthreads)
    out[k] = load_float<double>(N1, ntype, k) * double(load_index(F1, itype, k * kept)) * scale;
}

template <int kIType, int kNType, bool kTwo>
__global__ __launch_bounds__(kThreads) void k_blockwise_vec(const void* __restrict__ N1, const uint4* __restrict__ F1,
                                                            const void* __restrict__ N2, const uint4* __restrict__ F2,
                                                            double* __restrict__ out, double scale, int mode,
                                                            int64_t nvec, int lanes_shift, int n_f16) {
  const int lanes = 1 << lanes_shift;
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  const int64_t first = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t wave_first = first - (threadIdx.x & 63);
  for (int64_t base = wave_first; base < nvec; base += nthreads) {
    const int64_t v = base + (threadIdx.x & 63);
    const bool live = v < nvec;
    const int64_t vc = live ? v : nvec - 1;
    const int64_t k = vc >> lanes_shift;
    uint4 a = F1[vc];
    const uint4 b = kTwo ? F2[vc] : a;
    const double n1 = load_N<kNType>(N1, k, n_f16 != 0);
    const double n2 = kTwo ? load_N<kNType>(N2, k, n_f16 != 0) : n1;
    const bool head = (vc & (lanes - 1)) == 0;
    // the first coefficient is left out by clearing it in one operand (subtracting its product afterwards would
    // cancel, and with 32-bit indices, whose products exceed 53 bits, could leave a negative sum under a root)
    constexpr uint32_t kRest = kIType == PBZ_I8 ? 0xffffff00u : (kIType == PBZ_I16 ? 0xffff0000u : 0u);
    a.x = head ? (a.x & kRest) : a.x;
    double sum = dot_vec<kIType>(a, b);          // integer sum (exact for int8 / int16)
    for (int off = lanes >> 1; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (live && head) {
      double res = sum * (n1 * n2) * scale;
      if (mode == kBwStd) res = sqrt(res);
      out[k] = res;
    }
  }
}

__global__ __launch_bounds__(64) void k_blockwise_generic(const void* __restrict__ N1, const void* __restrict__ F1,
                                                          const void* __restrict__ N2, const void* __restrict__ F2,
                                                          int ntype, int itype, double* __restrict__ out, double scale,
                                                          int mode, int64_t n_blocks, int kept) {
  for (int64_t k = blockIdx.x; k < n_blocks; k += gridDim.x) {
    double sum = 0.0;
    for (int j = 1 + threadIdx.x; j < kept; j += 64)
      sum += double(load_index(F1, itype, k * kept + j)) * double(load_index(F2, itype, k * kept + j));
    sum = wave_sum(sum);
    if (threadIdx.x == 0) {
      double res = sum * (load_float<double>(N1, ntype, k) * load_float<double>(N2, ntype, k)) * scale;
      if (mode == kBwStd) res = sqrt(res);
      out[k] = res;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Reductions (Algorithms 6-11).  One streaming pass produces five FP64 sums per workgroup,
//   S12 = sum_k N1_k N2_k sum_j F1_kj F2_kj     S11, S22 likewise     D1 = sum_k N1_k F1_k0   D2 likewise
// (integer block sums are exact; the scale 1/r or 1/r^2 is applied once at the end) and writes them to the
// workspace; a second one-workgroup kernel adds the partials in index order and evaluates the requested
// statistic.  The result therefore does not depend on the order in which workgroups run.
// (A single launch in which the last workgroup to finish does the final sum was measured slower: the
// per-workgroup ticket increments serialise on one address across the chip.)
// ---------------------------------------------------------------------------------------------
enum { kS12 = 0, kS11 = 1, kS22 = 2, kD1 = 3, kD2 = 4, kNumSums = 5 };

struct ReduceTail {
  double* partials;
  double* out;
  int op;
  double r, n_blocks, vol;
  double s_l, s_c, w_l, w_c, w_s;   // Algorithm 12's stabilisers and weights
  int n_f16;                        // N is FP16 (as opposed to bfloat16) when it is 16 bits wide
  // Shifted first coefficients.  Variance and covariance centre the first coefficients N_k F_k0 by their mean
  // (Algorithms 8, 9); summing them and their squares raw and subtracting afterwards would cancel against the
  // square of the mean.  The passes that need them therefore sum d_k = N_k F_k0 - K, with K the first
  // coefficient of the segment's first block (a pilot value: exact centring needs the mean, which is not known
  // yet, but any K near it removes the cancellation), and put d_k^2, d1_k d2_k into S11, S22, S12 in place of
  // the raw squares and product.  pilot_n1 == nullptr: nothing is shifted (K = 0).
  const void* pilot_n1;
  const void* pilot_f1;
  const void* pilot_n2;
  const void* pilot_f2;
  int64_t seg_n_bytes, seg_f_bytes;  // distance between the segments' first N and F
  int ntype, itype;
};

// K of operand (N, F) in segment `segment`: the same expression wherever it is evaluated
__device__ __forceinline__ double pilot_value(const void* N, const void* F, const ReduceTail& t, int64_t segment) {
  if (!N) return 0.0;
  const char* n = static_cast<const char*>(N) + segment * t.seg_n_bytes;
  const char* f = static_cast<const char*>(F) + segment * t.seg_f_bytes;
  return load_float<double>(n, t.ntype, 0) * double(load_index(f, t.itype, 0));
}

// s: the five sums, with the first coefficients shifted by K1 / K2 where the pass shifts them (else K = 0)
__device__ __forceinline__ double finish_statistic(const double* s, const ReduceTail& t, double K1, double K2) {
  const double n = t.n_blocks;
  // the raw sums back from the shifted ones: sum (d + K) = D + n K, sum (d1 + K1)(d2 + K2) = S12 + K2 D1 + K1 D2 + n K1 K2
  const double D1 = s[kD1] + n * K1, D2 = s[kD2] + n * K2;
  const double S11 = s[kS11] + 2.0 * K1 * s[kD1] + n * K1 * K1;
  const double S22 = s[kS22] + 2.0 * K2 * s[kD2] + n * K2 * K2;
  const double S12 = s[kS12] + K2 * s[kD1] + K1 * s[kD2] + n * K1 * K2;
  switch (t.op) {
    case kDot: return S12 / (t.r * t.r);
    case kNorm2: return sqrt(S11) / t.r;
    case kDiffNorm2: return sqrt(s[kS11]) / t.r;    // S11 then holds sum (N1 F1 - N2 F2)^2
    case kCosine: return S12 / (sqrt(S11) * sqrt(S22));
    case kMean: return (D1 / t.r) / (n * sqrt(t.vol));
    // centring the first coefficients by their mean removes (sum d1)(sum d2) / n_blocks from the sum of products,
    // whatever constant they were shifted by
    case kCovariance: return ((s[kS12] - s[kD1] * s[kD2] / n) / (t.r * t.r)) / (n * t.vol);
    case kVariance: return ((s[kS11] - s[kD1] * s[kD1] / n) / (t.r * t.r)) / (n * t.vol);
    case kSsim: {   // Algorithm 12 from the means, variances and covariance of Algorithms 7-9
      const double scale = 1.0 / (t.r * n * sqrt(t.vol));
      const double mu_a = D1 * scale, mu_b = D2 * scale;
      const double per = 1.0 / (t.r * t.r * n * t.vol);
      // a difference inside the rounding of its two terms is the variance of a constant array: zero (its root
      // would turn 1e-16 into 1e-8)
      const double noise = 8.0 * 2.220446049250313e-16;
      double ca = s[kS11] - s[kD1] * s[kD1] / n, cb = s[kS22] - s[kD2] * s[kD2] / n;
      if (ca <= noise * s[kS11]) ca = 0.0;
      if (cb <= noise * s[kS22]) cb = 0.0;
      const double var_a = ca * per, var_b = cb * per;
      const double cov = (s[kS12] - s[kD1] * s[kD2] / n) * per;
      const double sd = sqrt(var_a) * sqrt(var_b);
      const double lum = (2.0 * mu_a * mu_b + t.s_l) / (mu_a * mu_a + mu_b * mu_b + t.s_l);
      const double con = (2.0 * sd + t.s_c) / (var_a + var_b + t.s_c);
      const double str = (cov + 0.5 * t.s_c) / (sd + 0.5 * t.s_c);
      return pow(lum, t.w_l) * pow(con, t.w_c) * pow(str, t.w_s);
    }
    default: return 0.0;
  }
}

// sum of `sums` over the workgroup, valid in threads 0 .. kNumSums-1 (thread i returns total i)
template <int kWaves = kThreads / 64>
__device__ __forceinline__ double group_total(const double* sums, double (*lds)[kNumSums]) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < kNumSums; ++i) {
    double t = wave_sum(sums[i]);
    if (lane == 0) lds[wave][i] = t;
  }
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x < kNumSums)
    for (int w = 0; w < kWaves; ++w) t += lds[w][threadIdx.x];
  return t;
}

// the requested statistic(s) of segment `segment` from its five sums
__device__ __forceinline__ void write_statistic(const double* fin, const ReduceTail& t, int64_t segment, double K1,
                                                double K2) {
  if (t.op == kStatistics) {            // mean, variance and norm2 of one array from the same two sums
    ReduceTail one = t;
    const int ops[3] = {kMean, kVariance, kNorm2};
    for (int i = 0; i < 3; ++i) {
      one.op = ops[i];
      t.out[segment * 3 + i] = finish_statistic(fin, one, K1, K2);
    }
  } else if (t.op == kPairStatistics) { // every statistic of a pair of arrays from the five sums of one pass
    ReduceTail one = t;
    const double swapped[kNumSums] = {fin[kS12], fin[kS22], fin[kS11], fin[kD2], fin[kD1]};   // the operands exchanged
    const int both[3] = {kDot, kCosine, kCovariance}, each[3] = {kMean, kVariance, kNorm2};
    for (int i = 0; i < 3; ++i) {
      one.op = both[i];
      t.out[segment * 9 + i] = finish_statistic(fin, one, K1, K2);
      one.op = each[i];
      t.out[segment * 9 + 3 + 2 * i] = finish_statistic(fin, one, K1, K2);
      t.out[segment * 9 + 4 + 2 * i] = finish_statistic(swapped, one, K2, K1);
    }
  } else {
    t.out[segment] = finish_statistic(fin, t, K1, K2);
  }
}

// grid y runs over the segments of a segmented reduction (1 otherwise).  A segment covered by a single
// workgroup (small arrays) is finished here and needs no second launch; the sums are the same either way.
// K1, K2: the pilot values the sums were shifted by (zero where the pass shifts nothing).  Every workgroup of a
// segment has the same ones; they travel in the partial record (slots kPilot1, kPilot2), so that the final kernel
// finds them in the records it reads anyway instead of fetching N and F of the segment's first block once more.
constexpr int kPilot1 = 5, kPilot2 = 6;
static_assert(kPilot2 < kReducePartialSlots, "record layout");

__device__ __forceinline__ void reduce_tail(double* sums, const ReduceTail& t, double K1, double K2) {
  __shared__ double lds[kThreads / 64][kNumSums];
  __shared__ double fin[kNumSums];
  const double total = group_total(sums, lds);
  if (gridDim.x == 1) {
    if (threadIdx.x < kNumSums) fin[threadIdx.x] = total;
    __syncthreads();
    if (threadIdx.x == 0) write_statistic(fin, t, blockIdx.y, K1, K2);
    return;
  }
  double* record = t.partials + (int64_t(blockIdx.y) * gridDim.x + blockIdx.x) * kReducePartialSlots;
  if (threadIdx.x < kNumSums) record[threadIdx.x] = total;
  if (threadIdx.x == kPilot1) record[kPilot1] = K1;
  if (threadIdx.x == kPilot2) record[kPilot2] = K2;
}

// one workgroup per segment: adds that segment's n_partials (<= kFinalMaxPartials) partial sums in a fixed order.
// Every thread first issues all its loads (a partial is one 64-byte record, read as four 16-byte pieces,
// kFinalRecords records per thread, from a clamped index: no branch around a load), then adds: the kernel's
// duration is one memory round trip.  The pilot values are those of the segment's first record, which thread 0 holds.
constexpr int kFinalThreads = 256;
constexpr int kFinalMaxPartials = kReduceGroupsOneSegment;
constexpr int kFinalRecords = kFinalMaxPartials / kFinalThreads;
static_assert(kFinalMaxPartials % kFinalThreads == 0 && kReducePartialSlots == 8, "record layout");

__global__ __launch_bounds__(kFinalThreads) void k_reduce_final(ReduceTail t, int n_partials) {
  __shared__ double lds[kFinalThreads / 64][kNumSums];
  __shared__ double fin[kNumSums];
  double acc[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const double2* mine = reinterpret_cast<const double2*>(t.partials + int64_t(blockIdx.x) * n_partials * kReducePartialSlots);
  double2 rec[kFinalRecords][4];
#pragma unroll
  for (int j = 0; j < kFinalRecords; ++j) {
    const int p = j * kFinalThreads + int(threadIdx.x);
    const int pc = p < n_partials ? p : 0;
#pragma unroll
    for (int q = 0; q < (j == 0 ? 4 : 3); ++q) rec[j][q] = mine[int64_t(pc) * 4 + q];
  }
  __builtin_amdgcn_sched_barrier(0);      // all loads requested before the first is waited for
  const double K1 = rec[0][2].y, K2 = rec[0][3].x;      // slots kPilot1, kPilot2 (of record 0 in thread 0)
#pragma unroll
  for (int j = 0; j < kFinalRecords; ++j)
    if (j * kFinalThreads + int(threadIdx.x) >= n_partials) rec[j][0] = rec[j][1] = rec[j][2] = make_double2(0.0, 0.0);
#pragma unroll
  for (int j = 0; j < kFinalRecords; ++j) {
    acc[0] += rec[j][0].x; acc[1] += rec[j][0].y;
    acc[2] += rec[j][1].x; acc[3] += rec[j][1].y;
    acc[4] += rec[j][2].x;
  }
  const double grand = group_total<kFinalThreads / 64>(acc, lds);
  if (threadIdx.x < kNumSums) fin[threadIdx.x] = grand;
  __syncthreads();
  if (threadIdx.x == 0) write_statistic(fin, t, blockIdx.x, K1, K2);
}

// per-tile records {S, D, K, count} left by a compress kernel (first coefficients shifted by the tile's own pilot
// value K) -> partial sums per workgroup relative to the pilot value of the segment's first tile, added in tile
// order; grid y runs over segments of n_tiles consecutive tiles
__global__ __launch_bounds__(kThreads) void k_reduce_tiles(const double2* __restrict__ tile_sums, int64_t n_tiles,
                                                           int64_t chunk, ReduceTail tail) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  tile_sums += int64_t(blockIdx.y) * n_tiles * 2;
  const double K = tile_sums[1].x;                   // the segment's first tile
  const int64_t begin = int64_t(blockIdx.x) * chunk;
  const int64_t end = begin + chunk < n_tiles ? begin + chunk : n_tiles;
  for (int64_t t = begin + threadIdx.x; t < end; t += kThreads) {
    const double2 sd = tile_sums[2 * t], kc = tile_sums[2 * t + 1];
    const double delta = kc.x - K;                   // sum (d + delta)^2 = S + 2 delta D + count delta^2
    sums[kS11] += sd.x + 2.0 * delta * sd.y + kc.y * delta * delta;
    sums[kD1] += sd.y + kc.y * delta;
  }
  reduce_tail(sums, tail, K, 0.0);
}

// kDiff: the coefficients of the two operands are subtracted element by element before squaring (their
// difference can be far smaller than either, so the block sums S11 - 2 S12 + S22 would cancel)
struct HeadTerms {          // see the kDC branch of accumulate_vec
  uint32_t first_mask, rest_mask;
  double K1, K2;
};
template <int kIType>
__device__ __forceinline__ HeadTerms head_terms(bool head, double K1, double K2) {
  constexpr uint32_t kRest = kIType == PBZ_I8 ? 0xffffff00u : (kIType == PBZ_I16 ? 0xffff0000u : 0u);
  HeadTerms h;
  h.first_mask = head ? 0xffffffffu : 0u;
  h.rest_mask = head ? kRest : 0xffffffffu;
  h.K1 = head ? K1 : 0.0;
  h.K2 = head ? K2 : 0.0;
  return h;
}

template <int kIType, bool kTwo, bool kDC, bool kDiff>
__device__ __forceinline__ void accumulate_vec(double* sums, const uint4& a, const uint4& b, double n1, double n2,
                                               const HeadTerms& head) {
  if (kDiff) {
    constexpr int kPer = kIType == PBZ_I8 ? 4 : (kIType == PBZ_I16 ? 2 : 1);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    double acc = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      double fa[4], fb[4];
      unpack_dword<kIType>(aw[w], fa);
      unpack_dword<kIType>(bw[w], fb);
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const double d = n1 * fa[e] - n2 * fb[e];
        acc += d * d;
      }
    }
    sums[kS11] += acc;
    return;
  }
  if (kDC) {
    // The block's first coefficient leaves the integer sums (cleared in the vector that holds it) and enters
    // shifted by the pilot value.  `head` says whether this vector starts a block: first_mask = all ones and
    // rest_mask = everything but the first element for such a vector, 0 and all ones otherwise; K1, K2 are
    // already zero for the other vectors.
    const double f0 = double(int(uint32_t(first_element<kIType>(a.x)) & head.first_mask));
    const double d1 = fma(n1, f0, -head.K1);
    uint4 ar = a, br = b;
    ar.x &= head.rest_mask;
    sums[kS11] = fma(d1, d1, fma(dot_vec<kIType>(ar, ar), n1 * n1, sums[kS11]));
    sums[kD1] += d1;
    if (kTwo) {
      const double g0 = double(int(uint32_t(first_element<kIType>(b.x)) & head.first_mask));
      const double d2 = fma(n2, g0, -head.K2);
      br.x &= head.rest_mask;
      sums[kS12] = fma(d1, d2, fma(dot_vec<kIType>(ar, br), n1 * n2, sums[kS12]));
      sums[kS22] = fma(d2, d2, fma(dot_vec<kIType>(br, br), n2 * n2, sums[kS22]));
      sums[kD2] += d2;
    }
    return;
  }
  sums[kS11] += dot_vec<kIType>(a, a) * (n1 * n1);
  if (kTwo) {
    sums[kS12] += dot_vec<kIType>(a, b) * (n1 * n2);
    sums[kS22] += dot_vec<kIType>(b, b) * (n2 * n2);
  }
}

// N is FP32 or FP64 (template), F is viewed as 16-byte vectors; vpb vectors per block (a power of two when
// vpb_shift >= 0).  Workgroup b streams the contiguous vectors [b * chunk, (b + 1) * chunk): per step every
// thread issues kUnroll loads per operand, kThreads vectors apart, with no branch between them.
constexpr int reduce_unroll(bool two) { return two ? kUnroll : 2 * kUnroll; }

// block that vector v belongs to: a shift when the vectors per block are a power of two (kGeneral = false)
template <bool kGeneral>
__device__ __forceinline__ int64_t block_of(int64_t v, int vpb_shift, int64_t vpb) {
  if constexpr (kGeneral) return vpb_shift >= 0 ? (v >> vpb_shift) : (v / vpb);
  else return v >> vpb_shift;
}

template <int kIType, int kNType, bool kTwo, bool kDC, bool kDiff = false, bool kAnyHeads = false>
__global__ __launch_bounds__(kThreads) void k_reduce_vec(const void* __restrict__ N1, const uint4* __restrict__ F1,
                                                         const void* __restrict__ N2, const uint4* __restrict__ F2,
                                                         int64_t nvec, int64_t chunk, int vpb_shift, int64_t vpb,
                                                         int64_t seg_blocks, ReduceTail tail) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  {  // segment blockIdx.y starts seg_blocks blocks (= nvec vectors) further on
    const int64_t nb = int64_t(blockIdx.y) * seg_blocks;
    constexpr int kNBytes = kNType == PBZ_F64 ? 8 : (kNType == PBZ_F32 ? 4 : 2);
    N1 = static_cast<const char*>(N1) + nb * kNBytes;
    F1 += int64_t(blockIdx.y) * nvec;
    if (kTwo) {
      N2 = static_cast<const char*>(N2) + nb * kNBytes;
      F2 += int64_t(blockIdx.y) * nvec;
    }
  }
  // the segment's pilot values (its first block's N F0, the expression of pilot_value): here N1 / F1 already point at
  // the segment and the types are the kernel's own, so the two loads carry no branch and no wait of their own
  const double K1 = kDC ? load_N<kNType>(N1, 0, tail.n_f16 != 0) * double(first_element<kIType>(F1[0].x)) : 0.0;
  const double K2 = kDC && kTwo ? load_N<kNType>(N2, 0, tail.n_f16 != 0) * double(first_element<kIType>(F2[0].x)) : 0.0;
  // Whether a thread's vector starts a block does not change from step to step when the vectors per block are a
  // power of two that divides the step (every workgroup starts at a multiple of it): its head terms are then
  // computed once, and a vector's block is a shift away.  The host launches the kAnyHeads variant (which works the
  // head terms out per vector, at the price of 30 more registers, and divides) for every other layout.  Keeping the
  // division out of the common variant matters beyond its cost: with the two alternatives behind a run-time test
  // the compiler put a full wait after each load of the 16-bit-index passes that carry first coefficients, eight
  // memory round trips per step instead of one.
  const HeadTerms fixed = head_terms<kIType>(kDC && (threadIdx.x & (vpb - 1)) == 0, K1, K2);
  const int64_t begin = int64_t(blockIdx.x) * chunk;
  const int64_t end = begin + chunk < nvec ? begin + chunk : nvec;
  constexpr int kLoads = reduce_unroll(kTwo);       // the same bytes in flight with one operand as with two
  constexpr int64_t kStep = int64_t(kThreads) * kLoads;
  int64_t base = begin;
  for (; base + kStep <= end; base += kStep) {
    uint4 a[kLoads], b[kTwo ? kLoads : 1];
    double n1[kLoads], n2[kLoads];
    int64_t k[kLoads];
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const int64_t v = base + u * kThreads + threadIdx.x;
      k[u] = block_of<kAnyHeads>(v, vpb_shift, vpb);
      a[u] = F1[v];
      if constexpr (kTwo) b[u] = F2[v];
    }
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      n1[u] = load_N<kNType>(N1, k[u], tail.n_f16 != 0);
      n2[u] = kTwo ? load_N<kNType>(N2, k[u], tail.n_f16 != 0) : 0.0;
    }
    // The passes that carry first coefficients request every load of the step before any of its arithmetic: left
    // to itself the instruction scheduler sinks their loads towards the first use to save registers, and the step
    // then takes one memory round trip per vector instead of one in all (workload 4: variance 57.6 -> 49 us,
    // covariance 111 -> 103.5 us).  The other passes are scheduled well as they are, and the fence costs them 0.5 us.
    if constexpr (kDC) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const int64_t v = base + u * kThreads + threadIdx.x;
      accumulate_vec<kIType, kTwo, kDC, kDiff>(
          sums, a[u], kTwo ? b[kTwo ? u : 0] : a[u], n1[u], n2[u],
          kAnyHeads ? head_terms<kIType>(kDC && (v - k[u] * vpb) == 0, K1, K2) : fixed);
    }
  }
  for (int64_t v = base + threadIdx.x; v < end; v += kThreads) {
    const int64_t k = block_of<kAnyHeads>(v, vpb_shift, vpb);
    const uint4 a = F1[v];
    const uint4 b = kTwo ? F2[v] : a;
    accumulate_vec<kIType, kTwo, kDC, kDiff>(sums, a, b, load_N<kNType>(N1, k, tail.n_f16 != 0),
                                             kTwo ? load_N<kNType>(N2, k, tail.n_f16 != 0) : 0.0,
                                             kAnyHeads ? head_terms<kIType>(kDC && (v - k * vpb) == 0, K1, K2) : fixed);
  }
  reduce_tail(sums, tail, K1, K2);
}

// thread per block, any kept count, alignment and N type
__global__ __launch_bounds__(kThreads) void k_reduce_generic(const void* __restrict__ N1, const void* __restrict__ F1,
                                                             const void* __restrict__ N2, const void* __restrict__ F2,
                                                             int ntype, int itype, int64_t n_blocks, int kept,
                                                             int two, int dc, int diff, ReduceTail tail) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  const int64_t k0 = int64_t(blockIdx.y) * n_blocks;     // first block of this segment
  const double K1 = dc ? pilot_value(tail.pilot_n1, tail.pilot_f1, tail, blockIdx.y) : 0.0;
  const double K2 = dc && two ? pilot_value(tail.pilot_n2, tail.pilot_f2, tail, blockIdx.y) : 0.0;
  for (int64_t kk = int64_t(blockIdx.x) * kThreads + threadIdx.x; kk < n_blocks; kk += nthreads) {
    const int64_t k = k0 + kk;
    const double n1 = load_float<double>(N1, ntype, k);
    const double n2 = two ? load_float<double>(N2, ntype, k) : 0.0;
    if (diff) {
      double acc = 0.0;
      for (int j = 0; j < kept; ++j) {
        const double d = n1 * double(load_index(F1, itype, k * kept + j)) - n2 * double(load_index(F2, itype, k * kept + j));
        acc += d * d;
      }
      sums[kS11] += acc;
      continue;
    }
    double s11 = 0.0, s12 = 0.0, s22 = 0.0;
    for (int j = dc ? 1 : 0; j < kept; ++j) {       // dc: the first coefficient enters shifted, below
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
      const double d1 = n1 * double(load_index(F1, itype, k * kept)) - K1;
      const double d2 = two ? n2 * double(load_index(F2, itype, k * kept)) - K2 : 0.0;
      sums[kS11] += d1 * d1;
      sums[kS12] += d1 * d2;
      sums[kS22] += d2 * d2;
      sums[kD1] += d1;
      sums[kD2] += d2;
    }
  }
  reduce_tail(sums, tail, K1, K2);
}

// Algorithm 7 needs only N and the first kept index of every block
__global__ __launch_bounds__(kThreads) void k_reduce_dc(const void* __restrict__ N1, const void* __restrict__ F1,
                                                        int ntype, int itype, int64_t n_blocks, int kept,
                                                        ReduceTail tail) {
  double sums[kNumSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
  const int64_t nthreads = int64_t(gridDim.x) * kThreads;
  const int64_t k0 = int64_t(blockIdx.y) * n_blocks;     // first block of this segment
  const double K1 = pilot_value(tail.pilot_n1, tail.pilot_f1, tail, blockIdx.y);
  for (int64_t kk = int64_t(blockIdx.x) * kThreads + threadIdx.x; kk < n_blocks; kk += nthreads)
    sums[kD1] += load_float<double>(N1, ntype, k0 + kk) * double(load_index(F1, itype, (k0 + kk) * kept)) - K1;
  reduce_tail(sums, tail, K1, 0.0);
}

template <int kIType, int kNType>
void launch_reduce_vec2(bool two, bool dc, bool diff, dim3 grid, hipStream_t s, const void* N1, const void* F1, const void* N2,
                        const void* F2, int64_t nvec, int64_t chunk, int shift, int64_t vpb, int64_t seg_blocks,
                        const ReduceTail& tail) {
  const uint4* a = static_cast<const uint4*>(F1);
  const uint4* b = static_cast<const uint4*>(F2);
  dim3 block(kThreads);
  const bool pow2 = shift >= 0;        // vectors per block a power of two: the variants without a division
#define PBZ_REDUCE(TWO, DC, DIFF, GENERAL) \
  hipLaunchKernelGGL((k_reduce_vec<kIType, kNType, TWO, DC, DIFF, GENERAL>), grid, block, 0, s, N1, a, N2, b, nvec, chunk, shift, vpb, seg_blocks, tail)
  if (diff) {
    if (pow2) PBZ_REDUCE(true, false, true, false);
    else PBZ_REDUCE(true, false, true, true);
  } else if (dc) {
    // does the same thread meet the first vector of a block at every step?
    const bool fixed_heads = pow2 && vpb <= kThreads;
    if (two && fixed_heads) PBZ_REDUCE(true, true, false, false);
    else if (two) PBZ_REDUCE(true, true, false, true);
    else if (fixed_heads) PBZ_REDUCE(false, true, false, false);
    else PBZ_REDUCE(false, true, false, true);
  } else if (two) {
    if (pow2) PBZ_REDUCE(true, false, false, false);
    else PBZ_REDUCE(true, false, false, true);
  } else {
    if (pow2) PBZ_REDUCE(false, false, false, false);
    else PBZ_REDUCE(false, false, false, true);
  }
#undef PBZ_REDUCE
}

template <int kIType>
void launch_reduce_vec(int ntype, bool two, bool dc, bool diff, dim3 grid, hipStream_t s, const void* N1, const void* F1,
                       const void* N2, const void* F2, int64_t nvec, int64_t chunk, int shift, int64_t vpb,
                       int64_t seg_blocks, const ReduceTail& tail) {
  if (ntype == PBZ_F64)
    launch_reduce_vec2<kIType, PBZ_F64>(two, dc, diff, grid, s, N1, F1, N2, F2, nvec, chunk, shift, vpb, seg_blocks, tail);
  else if (ntype == PBZ_F32)
    launch_reduce_vec2<kIType, PBZ_F32>(two, dc, diff, grid, s, N1, F1, N2, F2, nvec, chunk, shift, vpb, seg_blocks, tail);
  else
    launch_reduce_vec2<kIType, kN16>(two, dc, diff, grid, s, N1, F1, N2, F2, nvec, chunk, shift, vpb, seg_blocks, tail);
}

}  // namespace

int launch_negate(const pbz_codec* c, int64_t n_blocks, const void* Fin, void* Fout, hipStream_t s) {
  return scale_sign(c, n_blocks, Fin, Fout, -1, s);
}

template <int kSign>
static void launch_mul_scalar_vec(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double ax,
                                  void* Nout, void* Fout, int64_t nvec, hipStream_t s) {
  const int64_t per_group = int64_t(kThreads) * kUnroll;
  const unsigned f_groups = static_cast<unsigned>((nvec + per_group - 1) / per_group);
  dim3 grid(f_groups + unsigned(stream_groups(n_blocks, 4))), block(kThreads);
  const uint4* i4 = static_cast<const uint4*>(Fin);
  uint4* o4 = static_cast<uint4*>(Fout);
  if (c->itype == PBZ_I8)
    hipLaunchKernelGGL((k_mul_scalar_vec<PBZ_I8, kSign>), grid, block, 0, s, i4, o4, nvec, f_groups, Nin, Nout,
                       int(c->ftype), ax, n_blocks);
  else if (c->itype == PBZ_I16)
    hipLaunchKernelGGL((k_mul_scalar_vec<PBZ_I16, kSign>), grid, block, 0, s, i4, o4, nvec, f_groups, Nin, Nout,
                       int(c->ftype), ax, n_blocks);
  else
    hipLaunchKernelGGL((k_mul_scalar_vec<PBZ_I32, kSign>), grid, block, 0, s, i4, o4, nvec, f_groups, Nin, Nout,
                       int(c->ftype), ax, n_blocks);
}

int launch_mul_scalar(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double x, void* Nout,
                      void* Fout, hipStream_t s) {
  const int sign = x > 0.0 ? 1 : (x < 0.0 ? -1 : 0);
  const int64_t f_bytes = n_blocks * c->kept * itype_bytes(c->itype);
  const bool f_untouched = sign > 0 && Fin == Fout;
  if (!f_untouched && f_bytes % 16 == 0 && aligned16(Fin) && aligned16(Fout)) {
    if (sign > 0) launch_mul_scalar_vec<1>(c, n_blocks, Nin, Fin, std::fabs(x), Nout, Fout, f_bytes / 16, s);
    else if (sign < 0) launch_mul_scalar_vec<-1>(c, n_blocks, Nin, Fin, std::fabs(x), Nout, Fout, f_bytes / 16, s);
    else launch_mul_scalar_vec<0>(c, n_blocks, Nin, Fin, std::fabs(x), Nout, Fout, f_bytes / 16, s);
    return hip_status(hipGetLastError());
  }
  hipLaunchKernelGGL(k_scale_N, dim3(stream_groups(n_blocks, 4)), dim3(kThreads), 0, s, Nin, Nout, int(c->ftype),
                     std::fabs(x), n_blocks);
  int st = hip_status(hipGetLastError());
  if (st != PBZ_OK) return st;
  return scale_sign(c, n_blocks, Fin, Fout, sign, s);
}

int launch_add(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
               void* Nout, void* Fout, hipStream_t s, double sign2) {
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  const int lanes_shift = bpb % 16 == 0 ? ilog2_exact(bpb / 16) : -1;
  const int n_f16 = c->ftype == PBZ_F16 ? 1 : 0;     // which of the two 16-bit types N is, when it is one
  if (lanes_shift >= 0 && lanes_shift <= 6 && aligned16(F1) && aligned16(F2) && aligned16(Fout)) {
    const int64_t nvec = n_blocks * (bpb / 16);
    int64_t add_groups = (nvec + kThreads - 1) / kThreads;      // one vector per thread; the kernel loops beyond that
    if (add_groups > (int64_t(1) << 30)) add_groups = int64_t(1) << 30;
    dim3 grid(static_cast<unsigned>(add_groups)), block(kThreads);
    const uint4* a = static_cast<const uint4*>(F1);
    const uint4* b = static_cast<const uint4*>(F2);
    uint4* o = static_cast<uint4*>(Fout);
#define PBZ_ADD(IT, NT) hipLaunchKernelGGL((k_add_vec<IT, NT>), grid, block, 0, s, N1, a, N2, b, Nout, o, c->r, sign2, nvec, lanes_shift, n_f16)
    if (c->ftype == PBZ_F64) {
      if (c->itype == PBZ_I8) PBZ_ADD(PBZ_I8, PBZ_F64);
      else if (c->itype == PBZ_I16) PBZ_ADD(PBZ_I16, PBZ_F64);
      else PBZ_ADD(PBZ_I32, PBZ_F64);
    } else if (c->ftype == PBZ_F32) {
      if (c->itype == PBZ_I8) PBZ_ADD(PBZ_I8, PBZ_F32);
      else if (c->itype == PBZ_I16) PBZ_ADD(PBZ_I16, PBZ_F32);
      else PBZ_ADD(PBZ_I32, PBZ_F32);
    } else {
      if (c->itype == PBZ_I8) PBZ_ADD(PBZ_I8, kN16);
      else if (c->itype == PBZ_I16) PBZ_ADD(PBZ_I16, kN16);
      else PBZ_ADD(PBZ_I32, kN16);
    }
#undef PBZ_ADD
  } else {
    int64_t g = n_blocks < 65536 ? n_blocks : 65536;
    hipLaunchKernelGGL(k_add_generic, dim3(int(g)), dim3(64), 0, s, N1, F1, N2, F2, Nout, Fout, int(c->ftype),
                       int(c->itype), c->r, sign2, n_blocks, c->kept);
  }
  return hip_status(hipGetLastError());
}

// contiguous vectors per workgroup: whole steps of kThreads * kUnroll, as few as keep the grid within max_groups
static int64_t chunk_for(int64_t nvec, int max_groups, int* groups, bool two) {
  const int64_t step = int64_t(kThreads) * reduce_unroll(two);
  int64_t steps = (nvec + step * max_groups - 1) / (step * max_groups);
  if (steps < 1) steps = 1;
  int64_t chunk = steps * step;
  // up to four steps go to one workgroup, which then also finishes the statistic: cheaper than a second launch
  if (nvec <= 4 * step) chunk = 4 * step;
  *groups = int((nvec + chunk - 1) / chunk);
  return chunk;
}

// n_segments consecutive runs of n_blocks blocks each; one result per segment (n_segments == 1: the plain reductions)
int launch_reduce(const pbz_codec* c, ReduceOp op, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                  const void* F2, double* out, void* workspace, hipStream_t s, const double* ssim_params,
                  int64_t n_segments) {
  ReduceTail tail;
  tail.s_l = tail.s_c = 0.0;
  tail.w_l = tail.w_c = tail.w_s = 1.0;
  if (ssim_params) {
    tail.s_l = ssim_params[0]; tail.s_c = ssim_params[1];
    tail.w_l = ssim_params[2]; tail.w_c = ssim_params[3]; tail.w_s = ssim_params[4];
  }
  tail.partials = static_cast<double*>(workspace);
  tail.n_f16 = c->ftype == PBZ_F16 ? 1 : 0;
  tail.op = int(op);
  tail.r = c->r;
  tail.n_blocks = double(n_blocks);
  tail.vol = double(c->vol);
  const bool diff = (op == kDiffNorm2);
  const bool two = (op == kDot || op == kCosine || op == kCovariance || op == kSsim || op == kPairStatistics || diff);
  const bool dc = (op == kCovariance || op == kVariance || op == kSsim || op == kStatistics || op == kMean ||
                   op == kPairStatistics);
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  const int64_t n_stride = n_blocks * ftype_bytes(c->ftype), f_stride = n_blocks * bpb;   // bytes per segment

  // the workspace holds kReduceMaxGroups partial sums: segments are handled in batches of at most that many
  for (int64_t seg0 = 0; seg0 < n_segments; seg0 += kReduceMaxGroups) {
    const int batch = int(n_segments - seg0 < kReduceMaxGroups ? n_segments - seg0 : kReduceMaxGroups);
    // workgroups per segment.  Four per compute unit measured best for one segment (2048 and 4096: the final kernel
    // has more records to add and the streaming kernel's workgroups last one step; 512: too few waves for the
    // passes that carry first coefficients; workload 5 dot 0.035 -> 0.030 ms, workload 4 norm 0.059 -> 0.056 ms)
    const int max_groups = kReduceMaxGroups / batch < kReduceGroupsOneSegment ? kReduceMaxGroups / batch : kReduceGroupsOneSegment;
    const char* n1 = static_cast<const char*>(N1) + seg0 * n_stride;
    const char* f1 = static_cast<const char*>(F1) + seg0 * f_stride;
    const char* n2 = two ? static_cast<const char*>(N2) + seg0 * n_stride : nullptr;
    const char* f2 = two ? static_cast<const char*>(F2) + seg0 * f_stride : nullptr;
    tail.out = out + seg0 * (op == kStatistics ? 3 : (op == kPairStatistics ? 9 : 1));
    tail.pilot_n1 = dc ? n1 : nullptr;
    tail.pilot_f1 = dc ? f1 : nullptr;
    tail.pilot_n2 = dc && two ? n2 : nullptr;
    tail.pilot_f2 = dc && two ? f2 : nullptr;
    tail.seg_n_bytes = n_stride;
    tail.seg_f_bytes = f_stride;
    tail.ntype = int(c->ftype);
    tail.itype = int(c->itype);
    int groups;
    const bool vectors = bpb % 16 == 0 && aligned16(f1) && (!two || aligned16(f2)) && f_stride % 16 == 0;
    // Algorithm 7 needs one index per block, but memory is fetched in 128-byte lines: when a block's indices
    // fill at most one line, every line of F is fetched anyway, and streaming F with whole-KiB loads (the
    // variance pass) is faster than gathering one index per line (workload 4: 0.049 against 0.066 ms)
    if (op == kMean && !(vectors && bpb <= 128)) {
      groups = stream_groups(n_blocks, 4);
      if (groups > max_groups) groups = max_groups;
      hipLaunchKernelGGL(k_reduce_dc, dim3(groups, batch), dim3(kThreads), 0, s, n1, f1, int(c->ftype), int(c->itype),
                         n_blocks, c->kept, tail);
    } else if (vectors) {
      const int64_t vpb = bpb / 16;
      const int64_t nvec = n_blocks * vpb;
      const int64_t chunk = chunk_for(nvec, max_groups, &groups, two);
      dim3 grid(groups, batch);
      const int shift = ilog2_exact(vpb);
      if (c->itype == PBZ_I8)
        launch_reduce_vec<PBZ_I8>(int(c->ftype), two, dc, diff, grid, s, n1, f1, n2, f2, nvec, chunk, shift, vpb, n_blocks, tail);
      else if (c->itype == PBZ_I16)
        launch_reduce_vec<PBZ_I16>(int(c->ftype), two, dc, diff, grid, s, n1, f1, n2, f2, nvec, chunk, shift, vpb, n_blocks, tail);
      else
        launch_reduce_vec<PBZ_I32>(int(c->ftype), two, dc, diff, grid, s, n1, f1, n2, f2, nvec, chunk, shift, vpb, n_blocks, tail);
    } else {
      groups = stream_groups(n_blocks, 1);
      if (groups > max_groups) groups = max_groups;
      hipLaunchKernelGGL(k_reduce_generic, dim3(groups, batch), dim3(kThreads), 0, s, n1, f1, n2, f2, int(c->ftype),
                         int(c->itype), n_blocks, c->kept, two ? 1 : 0, dc ? 1 : 0, diff ? 1 : 0, tail);
    }
    int st = hip_status(hipGetLastError());
    if (st != PBZ_OK) return st;
    if (groups > 1) {          // a single workgroup per segment has already written the results
      hipLaunchKernelGGL(k_reduce_final, dim3(batch), dim3(kFinalThreads), 0, s, tail, groups);
      st = hip_status(hipGetLastError());
      if (st != PBZ_OK) return st;
    }
  }
  return PBZ_OK;
}

int launch_statistics_from_tiles(const pbz_codec* c, int64_t blocks_per_segment, const double* tile_sums,
                                 int64_t tiles_per_segment, int64_t n_segments, double* out, void* workspace,
                                 hipStream_t s) {
  ReduceTail tail;
  tail.s_l = tail.s_c = 0.0;
  tail.w_l = tail.w_c = tail.w_s = 1.0;
  tail.partials = static_cast<double*>(workspace);
  tail.n_f16 = 0;
  tail.op = int(kStatistics);
  tail.pilot_n1 = tail.pilot_f1 = tail.pilot_n2 = tail.pilot_f2 = nullptr;      // the pilot value comes from the tiles
  tail.seg_n_bytes = tail.seg_f_bytes = 0;
  tail.ntype = int(c->ftype);
  tail.itype = int(c->itype);
  tail.r = c->r;
  tail.n_blocks = double(blocks_per_segment);
  tail.vol = double(c->vol);
  for (int64_t seg0 = 0; seg0 < n_segments; seg0 += kReduceMaxGroups) {
    const int batch = int(n_segments - seg0 < kReduceMaxGroups ? n_segments - seg0 : kReduceMaxGroups);
    int max_groups = kReduceMaxGroups / batch;
    if (max_groups > kReduceGroupsOneSegment) max_groups = kReduceGroupsOneSegment;
    // four tiles per thread and workgroup unless that needs more workgroups than the workspace has slots for
    int64_t chunk = int64_t(kThreads) * 4;
    if ((tiles_per_segment + chunk - 1) / chunk > max_groups)
      chunk = ((tiles_per_segment + max_groups - 1) / max_groups + kThreads - 1) / kThreads * kThreads;
    const int groups = int((tiles_per_segment + chunk - 1) / chunk);
    tail.out = out + seg0 * 3;
    hipLaunchKernelGGL(k_reduce_tiles, dim3(groups, batch), dim3(kThreads), 0, s,
                       reinterpret_cast<const double2*>(tile_sums + seg0 * tiles_per_segment * 4), tiles_per_segment,
                       chunk, tail);
    int st = hip_status(hipGetLastError());
    if (st != PBZ_OK) return st;
    if (groups > 1) {          // a single workgroup per segment has already written the results
      hipLaunchKernelGGL(k_reduce_final, dim3(batch), dim3(kFinalThreads), 0, s, tail, groups);
      st = hip_status(hipGetLastError());
      if (st != PBZ_OK) return st;
    }
  }
  return PBZ_OK;
}

int launch_add_scalar(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double x, void* Nout,
                      void* Fout, hipStream_t s) {
  double root = 1.0;                       // prod(sqrt(i)), multiplied in dimension order
  for (int d = 0; d < c->ndim; ++d) root *= std::sqrt(double(c->block[d]));
  const double shift = x * root;
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  const int lanes_shift = bpb % 16 == 0 ? ilog2_exact(bpb / 16) : -1;
  const int n_f16 = c->ftype == PBZ_F16 ? 1 : 0;     // which of the two 16-bit types N is, when it is one
  if (lanes_shift >= 0 && lanes_shift <= 6 && aligned16(Fin) && aligned16(Fout)) {
    const int64_t nvec = n_blocks * (bpb / 16);
    int64_t groups = (nvec + kThreads - 1) / kThreads;
    if (groups > (int64_t(1) << 30)) groups = int64_t(1) << 30;
    dim3 grid(static_cast<unsigned>(groups)), block(kThreads);
    const uint4* a = static_cast<const uint4*>(Fin);
    uint4* o = static_cast<uint4*>(Fout);
#define PBZ_ADDS(IT, NT) hipLaunchKernelGGL((k_add_scalar_vec<IT, NT>), grid, block, 0, s, Nin, a, Nout, o, c->r, shift, nvec, lanes_shift, n_f16)
    if (c->ftype == PBZ_F64) {
      if (c->itype == PBZ_I8) PBZ_ADDS(PBZ_I8, PBZ_F64);
      else if (c->itype == PBZ_I16) PBZ_ADDS(PBZ_I16, PBZ_F64);
      else PBZ_ADDS(PBZ_I32, PBZ_F64);
    } else if (c->ftype == PBZ_F32) {
      if (c->itype == PBZ_I8) PBZ_ADDS(PBZ_I8, PBZ_F32);
      else if (c->itype == PBZ_I16) PBZ_ADDS(PBZ_I16, PBZ_F32);
      else PBZ_ADDS(PBZ_I32, PBZ_F32);
    } else {
      if (c->itype == PBZ_I8) PBZ_ADDS(PBZ_I8, kN16);
      else if (c->itype == PBZ_I16) PBZ_ADDS(PBZ_I16, kN16);
      else PBZ_ADDS(PBZ_I32, kN16);
    }
#undef PBZ_ADDS
  } else {
    int64_t g = n_blocks < 65536 ? n_blocks : 65536;
    hipLaunchKernelGGL(k_add_scalar_generic, dim3(int(g)), dim3(64), 0, s, Nin, Fin, Nout, Fout, int(c->ftype),
                       int(c->itype), c->r, shift, n_blocks, c->kept);
  }
  return hip_status(hipGetLastError());
}

int launch_blockwise_mean(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out,
                          hipStream_t s) {
  const double scale = 1.0 / (c->r * std::sqrt(double(c->vol)));
  hipLaunchKernelGGL(k_blockwise_mean, dim3(stream_groups(n_blocks, 1)), dim3(kThreads), 0, s, N, F, int(c->ftype),
                     int(c->itype), scale, n_blocks, c->kept, out);
  return hip_status(hipGetLastError());
}

// mode: 0 variance, 1 standard deviation, 2 covariance (N2 / F2 used only by the covariance)
int launch_blockwise(const pbz_codec* c, int mode, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                     const void* F2, double* out, hipStream_t s) {
  const bool two = mode == kBwCovariance;
  if (!two) {
    N2 = N1;
    F2 = F1;
  }
  const double scale = 1.0 / (c->r * c->r * double(c->vol));
  const int64_t bpb = int64_t(c->kept) * itype_bytes(c->itype);
  const int lanes_shift = bpb % 16 == 0 ? ilog2_exact(bpb / 16) : -1;
  const int n_f16 = c->ftype == PBZ_F16 ? 1 : 0;     // which of the two 16-bit types N is, when it is one
  if (lanes_shift >= 0 && lanes_shift <= 6 && aligned16(F1) && aligned16(F2)) {
    const int64_t nvec = n_blocks * (bpb / 16);
    int64_t groups = (nvec + kThreads - 1) / kThreads;
    if (groups > (int64_t(1) << 30)) groups = int64_t(1) << 30;
    dim3 grid(static_cast<unsigned>(groups)), block(kThreads);
    const uint4* a = static_cast<const uint4*>(F1);
    const uint4* b = static_cast<const uint4*>(F2);
#define PBZ_BW(IT, NT)                                                                                              \
  do {                                                                                                              \
    if (two)                                                                                                        \
      hipLaunchKernelGGL((k_blockwise_vec<IT, NT, true>), grid, block, 0, s, N1, a, N2, b, out, scale, mode, nvec,   \
                         lanes_shift, n_f16);                                                                       \
    else                                                                                                            \
      hipLaunchKernelGGL((k_blockwise_vec<IT, NT, false>), grid, block, 0, s, N1, a, N2, b, out, scale, mode, nvec,  \
                         lanes_shift, n_f16);                                                                       \
  } while (0)
    if (c->ftype == PBZ_F64) {
      if (c->itype == PBZ_I8) PBZ_BW(PBZ_I8, PBZ_F64);
      else if (c->itype == PBZ_I16) PBZ_BW(PBZ_I16, PBZ_F64);
      else PBZ_BW(PBZ_I32, PBZ_F64);
    } else if (c->ftype == PBZ_F32) {
      if (c->itype == PBZ_I8) PBZ_BW(PBZ_I8, PBZ_F32);
      else if (c->itype == PBZ_I16) PBZ_BW(PBZ_I16, PBZ_F32);
      else PBZ_BW(PBZ_I32, PBZ_F32);
    } else {
      if (c->itype == PBZ_I8) PBZ_BW(PBZ_I8, kN16);
      else if (c->itype == PBZ_I16) PBZ_BW(PBZ_I16, kN16);
      else PBZ_BW(PBZ_I32, kN16);
    }
#undef PBZ_BW
  } else {
    int64_t g = n_blocks < 65536 ? n_blocks : 65536;
    hipLaunchKernelGGL(k_blockwise_generic, dim3(int(g)), dim3(64), 0, s, N1, F1, N2, F2, int(c->ftype), int(c->itype),
                       out, scale, mode, n_blocks, c->kept);
  }
  return hip_status(hipGetLastError());
}

}  // namespace pbz
