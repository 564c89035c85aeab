// Shared pieces of the specialised codec kernels (pbz_fast_*.hip): launch geometry, element conversion, binning
// and index packing, streaming and 4-byte-aligned 16-byte accesses, lane trades, the per-wave statistic sums,
// the register-resident block transforms, and the host-side folding of an array into at most three dimensions.
// Everything here is inline or a template; each kernel family is a translation unit of its own.
#pragma once

#include <type_traits>

#include "pbz_dct.h"
#include "pbz_haar.h"
#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace fast {

struct FastGeom {
  int64_t Z, Y, X;        // array extents after folding
  int64_t gz, gy, gx;     // block grid
  uint32_t tiles_x;       // waves needed to cover the gx blocks of one block row
  uint32_t tiles_yx;      // gy * tiles_x: waves per z-slab of blocks
  int ntype;              // storage type of N (pbz_ftype): FP64, or FP32 / bfloat16 / FP16 for the kernels computing below FP64 width of N
  double r;
};

// Which tile does this wave own?  Grid x runs over the tiles of one z-slab (kWaves per workgroup), grid y / z
// over the slabs.  Everything here is uniform over the wave and 32-bit, so it compiles to a handful of
// scalar instructions instead of 64-bit vector divisions.
template <int kWaves>
__device__ __forceinline__ bool decode_tile(const FastGeom& g, int64_t& tx, int64_t& by, int64_t& bz) {
  const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t t = blockIdx.x * kWaves + w;
  const uint32_t slab = blockIdx.y + blockIdx.z * gridDim.y;
  if (t >= g.tiles_yx || slab >= g.gz) return false;
  const uint32_t row = t / g.tiles_x;
  tx = t - row * g.tiles_x;
  by = row;
  bz = slab;
  return true;
}

// launch geometry shared by all kernels; false when the tile counts do not fit the grid limits
inline bool tile_grid(FastGeom& g, int blocks_per_wave, int waves_per_group, dim3* grid) {
  const int64_t tiles_x = (g.gx + blocks_per_wave - 1) / blocks_per_wave;
  const int64_t tiles_yx = tiles_x * g.gy;
  if (tiles_yx >= (int64_t(1) << 31) || g.gz > int64_t(65535) * 65535) return false;
  g.tiles_x = uint32_t(tiles_x);
  g.tiles_yx = uint32_t(tiles_yx);
  const unsigned gy = unsigned(g.gz < 65535 ? g.gz : 65535);
  *grid = dim3(unsigned((tiles_yx + waves_per_group - 1) / waves_per_group), gy, unsigned((g.gz + gy - 1) / gy));
  return true;
}

// ---- element conversion ------------------------------------------------------------------------------
template <typename T, typename XT>
struct Unpack;   // 16 bytes of XT -> T[16 / sizeof(XT)]
template <typename T>
struct Unpack<T, float> {
  static constexpr int n = 4;
  static __device__ __forceinline__ void run(const uint4& u, T* o) {
    o[0] = T(__uint_as_float(u.x)); o[1] = T(__uint_as_float(u.y));
    o[2] = T(__uint_as_float(u.z)); o[3] = T(__uint_as_float(u.w));
  }
};
template <typename T>
struct Unpack<T, double> {
  static constexpr int n = 2;
  static __device__ __forceinline__ void run(const uint4& u, T* o) {
    o[0] = T(__longlong_as_double((long long)(((unsigned long long)u.y << 32) | u.x)));
    o[1] = T(__longlong_as_double((long long)(((unsigned long long)u.w << 32) | u.z)));
  }
};
struct bf16_t { uint16_t bits; };
template <typename T>
struct Unpack<T, bf16_t> {
  static constexpr int n = 8;
  static __device__ __forceinline__ void run(const uint4& u, T* o) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = T(__uint_as_float(w[i] << 16));
      o[2 * i + 1] = T(__uint_as_float(w[i] & 0xffff0000u));
    }
  }
};

struct f16_t { uint16_t bits; };
template <typename T>
struct Unpack<T, f16_t> {
  static constexpr int n = 8;
  static __device__ __forceinline__ void run(const uint4& u, T* o) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = T(float(__builtin_bit_cast(_Float16, uint16_t(w[i] & 0xffffu))));
      o[2 * i + 1] = T(float(__builtin_bit_cast(_Float16, uint16_t(w[i] >> 16))));
    }
  }
};

template <typename T, typename XT>
struct Pack;     // T[16 / sizeof(XT)] -> 16 bytes of XT, round to nearest even
template <typename T>
struct Pack<T, float> {
  static __device__ __forceinline__ uint4 run(const T* v) {
    return make_uint4(__float_as_uint(float(v[0])), __float_as_uint(float(v[1])), __float_as_uint(float(v[2])),
                      __float_as_uint(float(v[3])));
  }
};
template <typename T>
struct Pack<T, double> {
  static __device__ __forceinline__ uint4 run(const T* v) {
    unsigned long long a = (unsigned long long)__double_as_longlong(double(v[0]));
    unsigned long long b = (unsigned long long)__double_as_longlong(double(v[1]));
    return make_uint4(uint32_t(a), uint32_t(a >> 32), uint32_t(b), uint32_t(b >> 32));
  }
};
template <>
struct Pack<float, bf16_t> {
  static __device__ __forceinline__ uint4 run(const float* v) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = uint32_t(float_to_bf16_bits(v[2 * i])) | (uint32_t(float_to_bf16_bits(v[2 * i + 1])) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <>
struct Pack<float, f16_t> {
  static __device__ __forceinline__ uint4 run(const float* v) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = uint32_t(__builtin_bit_cast(uint16_t, _Float16(v[2 * i]))) |
             (uint32_t(__builtin_bit_cast(uint16_t, _Float16(v[2 * i + 1]))) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {   // hardware conversion, round to nearest even
  float2v f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// ---- binning and index packing ------------------------------------------------------------------------
// rint(t * inv) without a rounding and a conversion instruction: one fused multiply-add onto 1.5 * 2^23 (FP32;
// 1.5 * 2^52 in FP64) rounds the exact product to an integer in the nearest-even mode and leaves that integer,
// in two's complement, in the low bits of the sum's (low) word.  Valid for |t * inv| < 2^22; only the low 8 or
// 16 bits are used.
__device__ __forceinline__ uint32_t bin_bits(float t, float inv) {
  return __builtin_bit_cast(uint32_t, __builtin_fmaf(t, inv, 12582912.0f));
}
__device__ __forceinline__ uint32_t bin_bits(double t, double inv) {
  return uint32_t(__builtin_bit_cast(uint64_t, __builtin_fma(t, inv, 6755399441055744.0)));
}

// the low bytes / halves of `per` words gathered into one dword by byte permutes
template <typename IT>
struct IdxPack;   // kPer indices per dword
template <>
struct IdxPack<int8_t> {
  static constexpr int per = 4;
  static __device__ __forceinline__ uint32_t pack(const uint32_t* q) {
    const uint32_t lo = __builtin_amdgcn_perm(q[1], q[0], 0x0c0c0400u);    // q0.b0, q1.b0
    const uint32_t hi = __builtin_amdgcn_perm(q[3], q[2], 0x0c0c0400u);    // q2.b0, q3.b0
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
  }
  static __device__ __forceinline__ int get(uint32_t w, int i) { return int(int8_t((w >> (8 * i)) & 0xffu)); }
};
template <>
struct IdxPack<int16_t> {
  static constexpr int per = 2;
  static __device__ __forceinline__ uint32_t pack(const uint32_t* q) {
    return __builtin_amdgcn_perm(q[1], q[0], 0x05040100u);
  }
  static __device__ __forceinline__ int get(uint32_t w, int i) { return int(int16_t((w >> (16 * i)) & 0xffffu)); }
};

template <>
struct IdxPack<int32_t> {
  static constexpr int per = 1;
  static __device__ __forceinline__ uint32_t pack(const uint32_t* q) { return q[0]; }
  static __device__ __forceinline__ int get(uint32_t w, int) { return int(w); }
};

// ---- arrays whose last extent is not a multiple of the block's ------------------------------------------
// Rows then start at any multiple of the element size, so 16-byte accesses are only 4-byte aligned (the hardware
// takes them; the type tells the compiler), and the last block of every row is partial.  Kernels built with
// kTailX read every 16-byte piece from a start clamped to the row's last whole piece (always in bounds), which
// is already right for every block but the row's last; the lane that owns that block then re-reads its
// in-range elements one by one.  Stores: whole pieces that fit, single elements for the rest.
// The uncompressed arrays are touched once and are far larger than any cache: their loads and stores carry the
// non-temporal hint, which leaves the caches to the compressed arrays that the next operation reads again.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const u32x4 t = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store16_stream(void* p, const uint4& u) {
  const u32x4 t = {u.x, u.y, u.z, u.w};
  __builtin_nontemporal_store(t, static_cast<u32x4*>(p));
}

struct __attribute__((packed, aligned(4))) uint4_a4 { uint32_t x, y, z, w; };
__device__ __forceinline__ uint4 load16_a4(const void* p) {
  const uint4_a4 v = *static_cast<const uint4_a4*>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16_a4(void* p, const uint4& u) {
  uint4_a4 v;
  v.x = u.x; v.y = u.y; v.z = u.z; v.w = u.w;
  *static_cast<uint4_a4*>(p) = v;
}

__device__ __forceinline__ uint4 f4_bits(const float* v) {
  return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
}
__device__ __forceinline__ void bits_f4(const uint4& u, float* v) {
  v[0] = __uint_as_float(u.x); v[1] = __uint_as_float(u.y); v[2] = __uint_as_float(u.z); v[3] = __uint_as_float(u.w);
}

template <typename T>
struct ExchangeSlot;                                   // 16 bytes of a lane's values <-> one uint4 slot of an LDS exchange
template <>
struct ExchangeSlot<float> {
  static constexpr int n = 4;
  static __device__ __forceinline__ uint4 pack(const float* v) { return f4_bits(v); }
  static __device__ __forceinline__ void unpack(const uint4& u, float* v) { bits_f4(u, v); }
};
template <>
struct ExchangeSlot<double> {
  static constexpr int n = 2;
  static __device__ __forceinline__ uint4 pack(const double* v) {
    const uint64_t a = __builtin_bit_cast(uint64_t, v[0]), b = __builtin_bit_cast(uint64_t, v[1]);
    return make_uint4(uint32_t(a), uint32_t(a >> 32), uint32_t(b), uint32_t(b >> 32));
  }
  static __device__ __forceinline__ void unpack(const uint4& u, double* v) {
    v[0] = __builtin_bit_cast(double, uint64_t(u.x) | (uint64_t(u.y) << 32));
    v[1] = __builtin_bit_cast(double, uint64_t(u.z) | (uint64_t(u.w) << 32));
  }
};

// Four consecutive array elements as one piece: 16 bytes of FP32, 8 bytes of a 16-bit type.  kTailX: the piece
// is only known to start on a 4-byte boundary.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
struct __attribute__((packed, aligned(4))) U2A4 { uint32_t x, y; };
template <typename XT>
struct Quad4;
template <>
struct Quad4<float> {
  typedef uint4 raw_t;
  template <bool kTailX>
  static __device__ __forceinline__ raw_t load(const float* p) { return kTailX ? load16_a4(p) : load16_stream(p); }
  template <bool kTailX>
  static __device__ __forceinline__ void store(float* p, const raw_t& r) {
    if constexpr (kTailX) store16_a4(p, r); else store16_stream(p, r);
  }
  static __device__ __forceinline__ void keep(raw_t& r, uint32_t m) { r.x &= m; r.y &= m; r.z &= m; r.w &= m; }
  static __device__ __forceinline__ void unpack(const raw_t& r, float* v) { bits_f4(r, v); }
  static __device__ __forceinline__ raw_t pack(const float* v) { return f4_bits(v); }
};
template <typename XT>
struct Quad4Half {                      // XT = bf16_t or f16_t
  typedef uint2 raw_t;
  template <bool kTailX>
  static __device__ __forceinline__ raw_t load(const XT* p) {
    if constexpr (kTailX) {
      const U2A4 t = *reinterpret_cast<const U2A4*>(p);
      return make_uint2(t.x, t.y);
    } else {
      const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
      return make_uint2(t.x, t.y);
    }
  }
  template <bool kTailX>
  static __device__ __forceinline__ void store(XT* p, const raw_t& r) {
    if constexpr (kTailX) {
      U2A4 t;
      t.x = r.x; t.y = r.y;
      *reinterpret_cast<U2A4*>(p) = t;
    } else {
      const u32x2 t = {r.x, r.y};
      __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
    }
  }
  static __device__ __forceinline__ void keep(raw_t& r, uint32_t m) { r.x &= m; r.y &= m; }
  static __device__ __forceinline__ void unpack(const raw_t& r, float* v) {
    const uint32_t w[2] = {r.x, r.y};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if constexpr (std::is_same<XT, bf16_t>::value) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      } else {
        v[2 * i] = float(__builtin_bit_cast(_Float16, uint16_t(w[i] & 0xffffu)));
        v[2 * i + 1] = float(__builtin_bit_cast(_Float16, uint16_t(w[i] >> 16)));
      }
    }
  }
  static __device__ __forceinline__ raw_t pack(const float* v) {
    if constexpr (std::is_same<XT, bf16_t>::value) {
      return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    } else {
      uint32_t w[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        w[i] = uint32_t(__builtin_bit_cast(uint16_t, _Float16(v[2 * i]))) |
               (uint32_t(__builtin_bit_cast(uint16_t, _Float16(v[2 * i + 1]))) << 16);
      return make_uint2(w[0], w[1]);
    }
  }
};
template <> struct Quad4<bf16_t> : Quad4Half<bf16_t> {};
template <> struct Quad4<f16_t> : Quad4Half<f16_t> {};
struct U4x2 { uint4 lo, hi; };
template <>
struct Quad4<double> {                  // four FP64 elements: two 16-byte pieces
  typedef U4x2 raw_t;
  template <bool kTailX>
  static __device__ __forceinline__ raw_t load(const double* p) {
    raw_t r;
    if constexpr (kTailX) {
      r.lo = load16_a4(p);
      r.hi = load16_a4(p + 2);
    } else {
      // The two halves are requested one right after the other: no other memory instruction may be scheduled
      // across the barrier (everything else may).  Left alone, the compiler issued a strip's sixteen upper pieces
      // before its sixteen lower ones, and a line fetched with the non-temporal hint was gone by the time its
      // other half was asked for (counters, 1 GiB array: 1.8 GiB fetched; 1.17 GiB with plain loads in that order).
      r.lo = load16_stream(p);
      r.hi = load16_stream(p + 2);
      __builtin_amdgcn_sched_barrier(0x38f);
    }
    return r;
  }
  template <bool kTailX>
  static __device__ __forceinline__ void store(double* p, const raw_t& r) {
    if constexpr (kTailX) {
      store16_a4(p, r.lo);
      store16_a4(p + 2, r.hi);
    } else {
      // two pieces per lane, 32 bytes apart: plain stores, which the L2 merges into whole lines
      *reinterpret_cast<uint4*>(p) = r.lo;
      *reinterpret_cast<uint4*>(p + 2) = r.hi;
    }
  }
  static __device__ __forceinline__ void keep(raw_t& r, uint32_t m) {
    r.lo.x &= m; r.lo.y &= m; r.lo.z &= m; r.lo.w &= m;
    r.hi.x &= m; r.hi.y &= m; r.hi.z &= m; r.hi.w &= m;
  }
};
// four elements of the array as values of the arithmetic type T, and back (one rounding from T to XT)
template <typename T, typename XT>
__device__ __forceinline__ void quad4_unpack(const typename Quad4<XT>::raw_t& r, T* v) {
  if constexpr (sizeof(XT) == 8) {
    Unpack<T, double>::run(r.lo, v);
    Unpack<T, double>::run(r.hi, v + 2);
  } else {
    float f[4];
    Quad4<XT>::unpack(r, f);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = T(f[e]);
  }
}
template <typename T, typename XT>
__device__ __forceinline__ typename Quad4<XT>::raw_t quad4_pack(const T* v) {
  if constexpr (sizeof(XT) == 8) {
    typename Quad4<XT>::raw_t r;
    r.lo = Pack<T, double>::run(v);
    r.hi = Pack<T, double>::run(v + 2);
    return r;
  } else {
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = float(v[e]);
    return Quad4<XT>::pack(f);
  }
}

template <typename T, typename XT>
struct Elem {   // one element: float and double arrays
  static __device__ __forceinline__ T load(const XT* p) { return T(*p); }
  static __device__ __forceinline__ void store(XT* p, T v) { *p = XT(v); }
};
template <typename T>
struct Elem<T, bf16_t> {
  static __device__ __forceinline__ T load(const bf16_t* p) { return T(bf16_bits_to_float(p->bits)); }
  static __device__ __forceinline__ void store(bf16_t* p, T v) { p->bits = float_to_bf16_bits(float(v)); }
};

template <typename T>
struct Elem<T, f16_t> {
  static __device__ __forceinline__ T load(const f16_t* p) { return T(float(__builtin_bit_cast(_Float16, p->bits))); }
  static __device__ __forceinline__ void store(f16_t* p, T v) { p->bits = __builtin_bit_cast(uint16_t, _Float16(float(v))); }
};

template <typename T>
__device__ __forceinline__ T abs_t(T v) { return v < T(0) ? -v : v; }
template <>
__device__ __forceinline__ float abs_t<float>(float v) { return fabsf(v); }
template <>
__device__ __forceinline__ double abs_t<double>(double v) { return fabs(v); }

// Orders this wave's LDS writes before its later LDS reads.  LDS operations of one wave execute in
// order; the fences keep the compiler from moving accesses across, no workgroup barrier is involved.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- N in its storage type ---------------------------------------------------------------------------------
// N is written through store_float (one rounding from the compute type).  The value a later reader gets back:
template <typename T>
__device__ __forceinline__ double stored_N(T m, int ntype) {
  switch (ntype) {
    case PBZ_F64: return double(m);
    case PBZ_F32: return double(float(m));
    case PBZ_BF16: return double(bf16_bits_to_float(sizeof(T) == 8 ? double_to_bf16_bits(double(m)) : float_to_bf16_bits(float(m))));
    default: return double(float(sizeof(T) == 8 ? double_to_f16(double(m)) : _Float16(float(m))));
  }
}
// kCount values of N at once: one switch around all the loads, so that they are in flight together
template <int kCount, typename T>
__device__ __forceinline__ void load_N_many(const void* N, int ntype, const int64_t* idx, T* out) {
  switch (ntype) {
    case PBZ_F32:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = T(static_cast<const float*>(N)[idx[i]]);
      break;
    case PBZ_BF16:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = T(bf16_bits_to_float(static_cast<const uint16_t*>(N)[idx[i]]));
      break;
    case PBZ_F16:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = T(float(static_cast<const _Float16*>(N)[idx[i]]));
      break;
    default:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = T(static_cast<const double*>(N)[idx[i]]);
      break;
  }
}

// ---- statistics emitted while compressing ---------------------------------------------------------------
// With kStats a compress kernel also leaves, per wave, the two sums that the mean (Algorithm 7), the variance
// (Algorithm 9) and the L2 norm (Algorithm 10) of the array it has just compressed are made of:
//   S11 = sum_k N_k^2 sum_j F_kj^2   and   D1 = sum_k N_k F_k0   over the wave's blocks,
// N_k as stored, the integer sums exact, the first coefficients shifted by a pilot value (see emit_tile_sums).
// The record of tile t = bz * tiles_yx + by * tiles_x + tx starts at tile_sums[4 t]; a later kernel adds the
// records in index order.
typedef short short2s __attribute__((ext_vector_type(2)));

template <typename IT, int kWords>
__device__ __forceinline__ double sum_of_squares(const uint32_t* w) {   // of the indices packed in w[0 .. kWords)
  if constexpr (sizeof(IT) == 1) {
    static_assert(kWords * 4 * 127 * 127 < (1LL << 31), "fits 32 bits");
    int acc = 0;
#pragma unroll
    for (int k = 0; k < kWords; ++k) acc = __builtin_amdgcn_sdot4(int(w[k]), int(w[k]), acc, false);
    return double(acc);
  } else {
    static_assert(sizeof(IT) == 2, "exact integer sums: 8- and 16-bit indices only");
    long long acc = 0;      // one dword: 2 * 32767^2 < 2^31
#pragma unroll
    for (int k = 0; k < kWords; ++k) {
      short2s h;
      h.x = short(w[k] & 0xffffu);
      h.y = short(w[k] >> 16);
      acc += (long long)__builtin_amdgcn_sdot2(h, h, 0, false);
    }
    return double(acc);
  }
}

// The same sum without the first index of w[0] when `skip_first` (the statistics take a block's first coefficient
// separately, shifted by a pilot value).  8- and 16-bit indices: exact integer sum minus the exact square.  32-bit
// indices: squares reach 2^62, so the sum is taken in FP64 and the first index, usually by far the largest, is left
// out instead of being subtracted (the difference would cancel to nothing).
template <typename IT, int kWords>
__device__ __forceinline__ double sum_of_squares_rest(const uint32_t* w, bool skip_first) {
  if constexpr (sizeof(IT) == 4) {
    const double f0 = double(int32_t(w[0]));
    double acc = skip_first ? 0.0 : f0 * f0;
#pragma unroll
    for (int k = 1; k < kWords; ++k) {
      const double f = double(int32_t(w[k]));
      acc += f * f;
    }
    return acc;
  } else {
    const double f0 = skip_first ? double(IdxPack<IT>::get(w[0], 0)) : 0.0;
    return sum_of_squares<IT, kWords>(w) - f0 * f0;
  }
}

// One record of four doubles per tile: { S, D, K, count }.  `rest` is this lane's share of N_k^2 sum_j F_kj^2
// without the blocks' first coefficients; the lanes that hold a first coefficient N_k F_k0 of a block inside the
// array pass it as d (minus the pilot value K, the first coefficient of the tile's first block, which lane 0
// holds) in `shifted` and count it in `count`:  S = sum rest + sum (N_k F_k0 - K)^2,  D = sum (N_k F_k0 - K).
// Shifting keeps the later subtraction S - D^2 / n from cancelling against the square of the mean.
__device__ __forceinline__ double tile_pilot(double first_coefficient_of_lane) {
  return __shfl(first_coefficient_of_lane, 0, 64);
}
__device__ __forceinline__ void emit_tile_sums(double* __restrict__ tile_sums, const FastGeom& g, int64_t tx, int64_t by,
                                               int64_t bz, double rest, double shifted_squares, double shifted,
                                               double count, double K) {
  const double S = wave_sum(rest + shifted_squares);
  const double D = wave_sum(shifted);
  const double n = wave_sum(count);
  if ((threadIdx.x & 63) == 0) {
    const int64_t t = bz * int64_t(g.tiles_yx) + by * int64_t(g.tiles_x) + tx;
    tile_sums[4 * t] = S;
    tile_sums[4 * t + 1] = D;
    tile_sums[4 * t + 2] = K;
    tile_sums[4 * t + 3] = n;
  }
}


// forward transform of a register-resident [BZ][BY][BX] block, one dimension after the other
template <int TF, typename T, int BZ, int BY, int BX>
__device__ __forceinline__ void forward_block(T* v) {
  if constexpr (BX > 1) {
#pragma unroll
    for (int row = 0; row < BZ * BY; ++row) tf_forward<TF, T, BX, 1>(v + row * BX);
  }
  if constexpr (BY > 1) {
#pragma unroll
    for (int z = 0; z < BZ; ++z)
#pragma unroll
      for (int xx = 0; xx < BX; ++xx) tf_forward<TF, T, BY, BX>(v + z * BY * BX + xx);
  }
  if constexpr (BZ > 1) {
#pragma unroll
    for (int yx = 0; yx < BY * BX; ++yx) tf_forward<TF, T, BZ, BY * BX>(v + yx);
  }
}

// inverse transform; only the low-frequency box [KZ][KY][KX] of the input is non-zero
template <int TF, typename T, int BZ, int BY, int BX, int KZ, int KY, int KX>
__device__ __forceinline__ void inverse_block(T* v) {
  if constexpr (BZ > 1) {
#pragma unroll
    for (int y = 0; y < KY; ++y)
#pragma unroll
      for (int xx = 0; xx < KX; ++xx) tf_inverse<TF, T, BZ, BY * BX, KZ>(v + y * BX + xx);
  }
  if constexpr (BY > 1) {
#pragma unroll
    for (int z = 0; z < BZ; ++z)
#pragma unroll
      for (int xx = 0; xx < KX; ++xx) tf_inverse<TF, T, BY, BX, KY>(v + z * BY * BX + xx);
  }
  if constexpr (BX > 1) {
#pragma unroll
    for (int row = 0; row < BZ * BY; ++row) tf_inverse<TF, T, BX, 1, KX>(v + row * BX);
  }
}

// first <-> second: lanes 32-63 of `first` trade places with lanes 0-31 of `second` (all 64 lanes must be active)
__device__ __forceinline__ void swap_half_waves(uint32_t& first, uint32_t& second) {
  const auto r = __builtin_amdgcn_permlane32_swap(first, second, false, false);
  first = r[0];
  second = r[1];
}

// Rows 0-3 of 16 lanes each ("quarters"): afterwards piece k of quarter q is what was piece q of quarter k
// (a 4 x 4 transpose between the piece index and the quarter index, in two rounds of pairwise trades; all 64
// lanes must be active).  Its own inverse.
__device__ __forceinline__ void swap_odd_even_rows(uint32_t& first, uint32_t& second) {
  const auto r = __builtin_amdgcn_permlane16_swap(first, second, false, false);   // rows 1, 3 of first <-> rows 0, 2 of second
  first = r[0];
  second = r[1];
}
__device__ __forceinline__ void transpose_quarter_waves(uint4& p0, uint4& p1, uint4& p2, uint4& p3) {
  swap_half_waves(p0.x, p2.x); swap_half_waves(p0.y, p2.y); swap_half_waves(p0.z, p2.z); swap_half_waves(p0.w, p2.w);
  swap_half_waves(p1.x, p3.x); swap_half_waves(p1.y, p3.y); swap_half_waves(p1.z, p3.z); swap_half_waves(p1.w, p3.w);
  swap_odd_even_rows(p0.x, p1.x); swap_odd_even_rows(p0.y, p1.y); swap_odd_even_rows(p0.z, p1.z); swap_odd_even_rows(p0.w, p1.w);
  swap_odd_even_rows(p2.x, p3.x); swap_odd_even_rows(p2.y, p3.y); swap_odd_even_rows(p2.z, p3.z); swap_odd_even_rows(p2.w, p3.w);
}


// ---- host side --------------------------------------------------------------------------------------
struct Folded {
  bool ok;
  int bz, by, bx;     // block extents
  int kz, ky, kx;     // kept box (== block extents when nothing is pruned), 0 when the mask is not a box
  bool tail_x;        // the last extent is not a multiple of the block's: rows unaligned, last block of a row partial
  FastGeom g;
};

// NT = double: N is FP64; NT = float: N is FP32 or one of the 16-bit types (the kernels convert on load / store)
template <typename NT>
inline bool n_type_ok(int ftype) { return sizeof(NT) == 8 ? ftype == PBZ_F64 : ftype != PBZ_F64; }

// can a kernel whose 16-byte pieces hold `per16` elements of `elem_bytes` bytes take this geometry?
inline bool x_extent_ok(const Folded& f, int per16, int elem_bytes) {
  return !f.tail_x || (f.g.X >= per16 && (f.g.X * elem_bytes) % 4 == 0);
}

inline Folded fold(const pbz_codec* c, const Geom& geo) {
  Folded f{};
  f.ok = false;
  const int nd = c->ndim;
  int64_t ext[3] = {1, 1, 1};
  int blk[3] = {1, 1, 1}, box[3] = {1, 1, 1};
  // last three dimensions map to z, y, x; everything before must have block extent 1 and folds into z
  int lead = nd > 3 ? nd - 3 : 0;
  for (int d = lead; d < nd; ++d) {
    int slot = 3 - (nd - d);
    ext[slot] = geo.shape[d];
    blk[slot] = int(c->block[d]);
    box[slot] = c->box[0] ? c->box[d] : 0;
  }
  int64_t fold_count = 1;
  for (int d = 0; d < lead; ++d) {
    if (c->block[d] != 1) return f;
    fold_count *= geo.shape[d];
  }
  if (fold_count > 1) {
    if (blk[0] != 1 && ext[0] % blk[0] != 0) return f;
    ext[0] *= fold_count;
  }
  // a 3-D array whose slowest block extent is 1 is a batch of 2-D problems: nothing to do, z blocks of extent 1
  f.bz = blk[0]; f.by = blk[1]; f.bx = blk[2];
  f.kz = box[0]; f.ky = box[1]; f.kx = box[2];
  if (!c->box[0]) f.kz = f.ky = f.kx = 0;
  FastGeom& g = f.g;
  g.Z = ext[0]; g.Y = ext[1]; g.X = ext[2];
  g.gz = (g.Z + blk[0] - 1) / blk[0];
  g.gy = (g.Y + blk[1] - 1) / blk[1];
  g.gx = (g.X + blk[2] - 1) / blk[2];
  g.r = c->r;
  g.ntype = int(c->ftype);
  f.tail_x = g.X % blk[2] != 0;
  f.ok = true;
  return f;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename XT>
constexpr int xtype_code();
template <> constexpr int xtype_code<float>() { return PBZ_F32; }
template <> constexpr int xtype_code<double>() { return PBZ_F64; }
template <> constexpr int xtype_code<bf16_t>() { return PBZ_BF16; }
template <> constexpr int xtype_code<f16_t>() { return PBZ_F16; }
template <typename IT>
constexpr int itype_code();
template <> constexpr int itype_code<int8_t>() { return PBZ_I8; }
template <> constexpr int itype_code<int16_t>() { return PBZ_I16; }
template <> constexpr int itype_code<int32_t>() { return PBZ_I32; }

// A family's table of instantiations, tried in order.  compress / decompress: 0 when no instantiation matches
// (`*name` stays null), else the kernel's name in `*name` and 1 / a negative status (dry_run: 1 when the launch
// geometry fits, nothing launched).  tiles: waves that a compress launch would use, -1 when nothing matches.
#define PBZ_FAST_FAMILY(FAMILY)                                                                                       \
  int FAMILY##_compress(const pbz_codec* c, const Folded& f, int xtype, const void* x, void* N, void* F, hipStream_t s, \
                        bool dry_run, const char** name, double* tile_sums);                                          \
  int64_t FAMILY##_tiles(const pbz_codec* c, const Folded& f, int xtype);                                             \
  int FAMILY##_decompress(const pbz_codec* c, const Folded& f, int ytype, const void* N, const void* F, void* y,      \
                          hipStream_t s, bool dry_run, const char** name);
PBZ_FAST_FAMILY(lane)
PBZ_FAST_FAMILY(quad16)
PBZ_FAST_FAMILY(oct8)
PBZ_FAST_FAMILY(cube16)
#undef PBZ_FAST_FAMILY

// Defines the three functions of a family from its X-macro list FOR_EACH(X, TF, SUFFIX) of (type, name) rows,
// once for the DCT (plain names) and once for the Haar transform (names ending in _haar).
#define COMMA ,
#define PBZ_DEFINE_FAST_FAMILY(FAMILY, FOR_EACH)                                                                      \
  int FAMILY##_compress(const pbz_codec* c, const Folded& f, int xtype, const void* x, void* N, void* F, hipStream_t s, \
                        bool dry_run, const char** name, double* tile_sums) {                                         \
    FOR_EACH(PBZ_FAST_COMPRESS_ROW, kTfDct, "")                                                                       \
    FOR_EACH(PBZ_FAST_COMPRESS_ROW, kTfHaar, "_haar")                                                                 \
    return 0;                                                                                                         \
  }                                                                                                                   \
  int64_t FAMILY##_tiles(const pbz_codec* c, const Folded& f, int xtype) {                                            \
    FOR_EACH(PBZ_FAST_TILES_ROW, kTfDct, "")                                                                          \
    FOR_EACH(PBZ_FAST_TILES_ROW, kTfHaar, "_haar")                                                                    \
    return -1;                                                                                                        \
  }                                                                                                                   \
  int FAMILY##_decompress(const pbz_codec* c, const Folded& f, int ytype, const void* N, const void* F, void* y,      \
                          hipStream_t s, bool dry_run, const char** name) {                                           \
    FOR_EACH(PBZ_FAST_DECOMPRESS_ROW, kTfDct, "")                                                                     \
    FOR_EACH(PBZ_FAST_DECOMPRESS_ROW, kTfHaar, "_haar")                                                               \
    return 0;                                                                                                         \
  }
#define PBZ_FAST_COMPRESS_ROW(K, NAME)                                         \
  if (K::matches(c, f, xtype)) {                                               \
    *name = NAME;                                                              \
    return dry_run ? K::fits(f.g) : K::compress(f.g, x, N, F, tile_sums, s);   \
  }
#define PBZ_FAST_TILES_ROW(K, NAME) \
  if (K::matches(c, f, xtype)) return K::tiles(f.g);
#define PBZ_FAST_DECOMPRESS_ROW(K, NAME)                                 \
  if (K::matches(c, f, ytype)) {                                         \
    *name = NAME;                                                        \
    return dry_run ? K::fits(f.g) : K::decompress(f.g, N, F, y, s);      \
  }

}  // namespace fast
}  // namespace pbz
