// Specialised codec kernels for the block shapes that matter for throughput.
//
// Every kernel here is "wave autonomous": a 64-lane wave owns a run of consecutive blocks along the
// contiguous (last) array dimension, reads whole block rows straight from HBM with 16-byte loads (the
// lanes of a wave cover a contiguous span of every row, which measures at the same bandwidth as a
// linear copy on MI355X), transforms in registers with the even/odd-split DCT of pbz_dct.h or the Haar
// cascade of pbz_haar.h (template switch TF), and writes N and F.  There is no workgroup barrier in the
// compress kernels; LDS, where used, is private to a wave.
//
// Family "lane":   one lane owns one whole block (blocks of at most 64 elements: 8x8, 4x4x4).  Where a block
//                   row is two (four) 16-byte pieces the half-waves (quarter-waves) trade pieces, so that every
//                   load / store instruction of the array covers one contiguous KiB.  Indices leave through a wave-private
//                   LDS transpose when a block's F is 64 bytes or more, for the same reason.
// Family "quad16":  16x16 and 4x16x16 blocks of FP32 or 16-bit input, 16 planes of 16x16 per wave.  Each lane first holds a 16-row x
//                   4-column strip (the column transform runs in registers), the wave exchanges through LDS,
//                   then each lane holds four whole rows (row transform, and for 4x16x16 the transform across
//                   the four planes); rows leave as 16-byte pieces in linear order.
// Family "oct8":    8x8x8 blocks of bfloat16, FP16 or FP32 input, 8 blocks per wave.  Each lane first holds one z-plane of
//                   a block (x and y transforms), the wave exchanges through LDS, then each lane holds one
//                   y-row of all eight z-planes (z transform).  Decompression needs no exchange: every
//                   lane rebuilds its own z-plane from the block's few kept coefficients; wide arrays use a
//                   variant in which a wave owns one plane of 64 blocks and stores whole 1 KiB row pieces.
//
// Variants of every kernel: kRagged (the slower dimensions are not multiples of the block extents), kTailX
// (neither is the last one: rows start at any 4-byte boundary, the last block of a row is partial), kStats
// (compress also leaves the per-wave sums from which mean, variance and norm follow).  N is stored in the
// codec's working type, converted on load / store.
//
// Preconditions checked on the host (otherwise the call falls back to the general kernels): the array
// reduces to at most three dimensions (leading dimensions with block extent 1 fold into the slowest one),
// the block shape / types / mask box match an instantiation, rows are at least one 16-byte piece long and
// start on a 4-byte boundary.
#include "pbz_dct.h"
#include "pbz_haar.h"
#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace {

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
template <int kCount>
__device__ __forceinline__ void load_N_many(const void* N, int ntype, const int64_t* idx, float* out) {
  switch (ntype) {
    case PBZ_F32:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = static_cast<const float*>(N)[idx[i]];
      break;
    case PBZ_BF16:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = bf16_bits_to_float(static_cast<const uint16_t*>(N)[idx[i]]);
      break;
    case PBZ_F16:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = float(static_cast<const _Float16*>(N)[idx[i]]);
      break;
    default:
#pragma unroll
      for (int i = 0; i < kCount; ++i) out[i] = float(static_cast<const double*>(N)[idx[i]]);
      break;
  }
}

// ---- statistics emitted while compressing ---------------------------------------------------------------
// With kStats a compress kernel also leaves, per wave, the two sums that the mean (Algorithm 7), the variance
// (Algorithm 9) and the L2 norm (Algorithm 10) of the array it has just compressed are made of:
//   S11 = sum_k N_k^2 sum_j F_kj^2   and   D1 = sum_k N_k F_k0   over the wave's blocks,
// N_k as stored, the integer sums exact.  tile_sums[2 t], tile_sums[2 t + 1] belong to tile
// t = bz * tiles_yx + by * tiles_x + tx; a later kernel adds them in index order.
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

__device__ __forceinline__ void emit_tile_sums(double* __restrict__ tile_sums, const FastGeom& g, int64_t tx, int64_t by,
                                               int64_t bz, double s11, double d1) {
  s11 = wave_sum(s11);
  d1 = wave_sum(d1);
  if ((threadIdx.x & 63) == 0) {
    const int64_t t = bz * int64_t(g.tiles_yx) + by * int64_t(g.tiles_x) + tx;
    tile_sums[2 * t] = s11;
    tile_sums[2 * t + 1] = d1;
  }
}


// H[m][q] of the length-8 orthonormal DCT-II as a compile-time table (for lane-dependent rows)
struct Dct8Table {
  float h[8][8];
  constexpr Dct8Table() : h{} {
    for (int m = 0; m < 8; ++m)
      for (int q = 0; q < 8; ++q)
        h[m][q] = float((q == 0 ? dct::cx_sqrt(1.0 / 8.0) : dct::cx_sqrt(2.0 / 8.0)) *
                        dct::cos_frac((long long)(2 * m + 1) * q, 8));
  }
};
__constant__ Dct8Table c_dct8 = Dct8Table();

struct Haar8Table {       // the same for the length-8 orthonormal Haar transform
  float h[8][8];
  constexpr Haar8Table() : h{} {
    for (int m = 0; m < 8; ++m) h[m][0] = float(dct::cx_sqrt(1.0 / 8.0));
    int q = 1;
    for (int count = 1; count < 8; count *= 2) {
      const int width = 8 / count;
      for (int j = 0; j < count; ++j, ++q)
        for (int m = 0; m < width; ++m)
          h[j * width + m][q] = float((m < width / 2 ? 1.0 : -1.0) * dct::cx_sqrt(double(count) / 8.0));
    }
  }
};
__constant__ Haar8Table c_haar8 = Haar8Table();

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

// =====================================================================================================
// Family "lane": one lane = one block
// =====================================================================================================
// kRagged: the slow dimensions are not multiples of the block extents, so some block rows lie outside the
// array.  Such rows are still loaded (from a clamped, valid address: a branch around a load would make the
// compiler wait for all outstanding loads at the join) and zeroed afterwards.
template <int TF, typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX,
          bool kRagged, bool kStats, bool kTailX = false>
__global__ __launch_bounds__(256) void k_compress_lane(FastGeom g, const XT* __restrict__ x, void* __restrict__ N,
                                                       IT* __restrict__ F, double* __restrict__ tile_sums) {
  constexpr int VOL = BZ * BY * BX, ROWS = BZ * BY;
  constexpr int RV = BX * int(sizeof(XT)) / 16;       // 16-byte loads per block row
  constexpr int PER16 = Unpack<T, XT>::n;
  constexpr int KEPT = KZ * KY * KX;
  constexpr int KW = KEPT * int(sizeof(IT)) / 4;      // dwords of F per block
  static_assert(BX * sizeof(XT) % 16 == 0 && (KEPT * sizeof(IT)) % 16 == 0, "rows and F blocks are whole 16-byte vectors");

  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<4>(g, tx, by, bz)) return;
  const int64_t bx = tx * 64 + lane;
  const bool active = bx < g.gx;
  const int64_t bxc = active ? bx : g.gx - 1;   // lanes past the end re-read the last block and store nothing
  const bool whole_wave = tx * 64 + 64 <= g.gx; // uniform

  uint4 raw[ROWS * RV];
#pragma unroll
  for (int z = 0; z < BZ; ++z)
#pragma unroll
    for (int y = 0; y < BY; ++y) {
      int64_t zz = bz * BZ + z, yy = by * BY + y;
      if constexpr (kRagged) {
        zz = zz < g.Z ? zz : g.Z - 1;
        yy = yy < g.Y ? yy : g.Y - 1;
      }
      if constexpr (kTailX) {
        const XT* row = x + (zz * g.Y + yy) * g.X;
#pragma unroll
        for (int k = 0; k < RV; ++k) {
          const int64_t x0 = bxc * BX + k * PER16;
          raw[(z * BY + y) * RV + k] = load16_a4(row + (x0 + PER16 <= g.X ? x0 : g.X - PER16));
        }
      } else if (RV == 2 && whole_wave) {
        // two 16-byte pieces per block row: every load instruction reads one contiguous KiB (the rows of 32
        // blocks), and the half-waves then trade the pieces that belong to the other one
        const uint4* p = reinterpret_cast<const uint4*>(x + (zz * g.Y + yy) * g.X + tx * 64 * BX) + 2 * (lane & 31) + (lane >> 5);
        raw[(z * BY + y) * 2] = load16_stream(p);
        raw[(z * BY + y) * 2 + 1] = load16_stream(p + 64);
      } else if (RV == 4 && whole_wave) {
        // four pieces per block row: load j reads the rows of blocks 16j .. 16j+15 as one contiguous KiB (lane
        // (quarter q, i) takes piece q of block 16j + i); the quarter transpose below sorts the pieces out
        const uint4* p = reinterpret_cast<const uint4*>(x + (zz * g.Y + yy) * g.X + tx * 64 * BX) + 4 * (lane & 15) + (lane >> 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) raw[(z * BY + y) * RV + k] = load16_stream(p + 64 * k);
      } else {
        const uint4* p = reinterpret_cast<const uint4*>(x + (zz * g.Y + yy) * g.X + bxc * BX);
#pragma unroll
        for (int k = 0; k < RV; ++k) raw[(z * BY + y) * RV + k] = load16_stream(&p[k]);
      }
    }
  if constexpr (RV == 4 && !kTailX) {
    if (whole_wave) {
#pragma unroll
      for (int i = 0; i < ROWS; ++i) transpose_quarter_waves(raw[4 * i], raw[4 * i + 1], raw[4 * i + 2], raw[4 * i + 3]);
    }
  }
  if constexpr (RV == 2 && !kTailX) {
    if (whole_wave) {
#pragma unroll
      for (int i = 0; i < ROWS; ++i) {
        swap_half_waves(raw[2 * i].x, raw[2 * i + 1].x);
        swap_half_waves(raw[2 * i].y, raw[2 * i + 1].y);
        swap_half_waves(raw[2 * i].z, raw[2 * i + 1].z);
        swap_half_waves(raw[2 * i].w, raw[2 * i + 1].w);
      }
    }
  }
  if constexpr (kRagged) {
#pragma unroll
    for (int z = 0; z < BZ; ++z)
#pragma unroll
      for (int y = 0; y < BY; ++y) {
        const uint32_t keep = (bz * BZ + z < g.Z && by * BY + y < g.Y) ? 0xffffffffu : 0u;   // uniform over the wave
#pragma unroll
        for (int k = 0; k < RV; ++k) {
          uint4& u = raw[(z * BY + y) * RV + k];
          u.x &= keep; u.y &= keep; u.z &= keep; u.w &= keep;
        }
      }
  }
  T v[VOL];
#pragma unroll
  for (int i = 0; i < ROWS * RV; ++i) Unpack<T, XT>::run(raw[i], v + i * PER16);
  if constexpr (kTailX) {
    if ((bxc + 1) * BX > g.X) {        // the row's last, partial block: its in-range elements one by one, zeros beyond
#pragma unroll
      for (int z = 0; z < BZ; ++z)
#pragma unroll
        for (int y = 0; y < BY; ++y) {
          const int64_t zz = bz * BZ + z, yy = by * BY + y;
          const bool row_in = zz < g.Z && yy < g.Y;
          const XT* row = x + ((row_in ? zz : g.Z - 1) * g.Y + (row_in ? yy : g.Y - 1)) * g.X;
#pragma unroll
          for (int e = 0; e < BX; ++e) {
            const int64_t xi = bxc * BX + e;
            const T val = Elem<T, XT>::load(row + (xi < g.X ? xi : g.X - 1));
            v[(z * BY + y) * BX + e] = row_in && xi < g.X ? val : T(0);
          }
        }
    }
  }

  forward_block<TF, T, BZ, BY, BX>(v);

  T m = T(0);
#pragma unroll
  for (int i = 0; i < VOL; ++i) m = fmax(m, abs_t(v[i]));
  const T inv = m > T(0) ? T(g.r) / m : T(0);

  uint32_t w[KW];
  constexpr int PER = IdxPack<IT>::per;
#pragma unroll
  for (int kw = 0; kw < KW; ++kw) {
    uint32_t q[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = kw * PER + e;                         // position in F
      const int kx = j % KX, ky = (j / KX) % KY, kz = j / (KX * KY);
      q[e] = bin_bits(v[(kz * BY + ky) * BX + kx], inv);
    }
    w[kw] = IdxPack<IT>::pack(q);
  }
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * 64;   // first block of this wave
  if (active) store_float(N, g.ntype, block0 + lane, m);
  if constexpr (kStats) {
    const double n = active ? stored_N(m, g.ntype) : 0.0;
    emit_tile_sums(tile_sums, g, tx, by, bz, sum_of_squares<IT, KW>(w) * (n * n), n * double(IdxPack<IT>::get(w[0], 0)));
  }
  constexpr int P = KW / 4;                                   // 16-byte pieces of F per block
  if constexpr (P >= 4) {
    // Lane-strided 16-byte stores 64 bytes or more apart run at about half the write bandwidth of linear
    // ones, so the pieces are transposed through LDS first: lane l puts piece p at l*P + (p ^ (l % P)) (the XOR
    // spreads the lanes over the banks), then the wave reads the staging area linearly and stores every
    // piece to its place; the pieces one instruction stores are a permutation of one contiguous span.
    __shared__ uint4 stage[4][64 * P];
    uint4* st = stage[threadIdx.x >> 6];
#pragma unroll
    for (int p = 0; p < P; ++p)
      st[lane * P + (p ^ (lane & (P - 1)))] = make_uint4(w[4 * p], w[4 * p + 1], w[4 * p + 2], w[4 * p + 3]);
    wave_lds_sync();
    const int n_active = int(g.gx - tx * 64 < 64 ? g.gx - tx * 64 : 64);
    uint4* dst = reinterpret_cast<uint4*>(F + block0 * KEPT);
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const int idx = j * 64 + lane;
      const int src = idx / P, piece = (idx % P) ^ (src & (P - 1));
      if (src < n_active) dst[src * P + piece] = st[idx];
    }
  } else if (active) {
    uint4* dst = reinterpret_cast<uint4*>(F + (block0 + lane) * KEPT);
#pragma unroll
    for (int k = 0; k < P; ++k) dst[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
  }
}

template <int TF, typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX,
          bool kRagged, bool kTailX = false>
__global__ __launch_bounds__(256) void k_decompress_lane(FastGeom g, const void* __restrict__ N, const IT* __restrict__ F,
                                                         XT* __restrict__ y) {
  constexpr int VOL = BZ * BY * BX, ROWS = BZ * BY;
  constexpr int RV = BX * int(sizeof(XT)) / 16;
  constexpr int PER16 = Unpack<T, XT>::n;
  constexpr int KEPT = KZ * KY * KX;
  constexpr int KW = KEPT * int(sizeof(IT)) / 4;
  constexpr int PER = IdxPack<IT>::per;

  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<4>(g, tx, by, bz)) return;
  const int64_t bx = tx * 64 + lane;
  if (bx >= g.gx) return;
  const int64_t block = (bz * g.gy + by) * g.gx + bx;
  const bool whole_wave = tx * 64 + 64 <= g.gx;       // uniform: all 64 lanes hold a block

  uint32_t w[KW];
  const uint4* src = reinterpret_cast<const uint4*>(F + block * KEPT);
#pragma unroll
  for (int k = 0; k < KW / 4; ++k) {
    const uint4 u = src[k];
    w[4 * k] = u.x; w[4 * k + 1] = u.y; w[4 * k + 2] = u.z; w[4 * k + 3] = u.w;
  }
  const T scale = load_float<T>(N, g.ntype, block) / T(g.r);          // Algorithm 3: N F / r, the division hoisted per block

  T v[VOL];
#pragma unroll
  for (int i = 0; i < VOL; ++i) v[i] = T(0);
#pragma unroll
  for (int j = 0; j < KEPT; ++j) {
    const int kx = j % KX, ky = (j / KX) % KY, kz = j / (KX * KY);
    v[(kz * BY + ky) * BX + kx] = scale * T(IdxPack<IT>::get(w[j / PER], j % PER));
  }

  inverse_block<TF, T, BZ, BY, BX, KZ, KY, KX>(v);

#pragma unroll
  for (int z = 0; z < BZ; ++z)
#pragma unroll
    for (int yy0 = 0; yy0 < BY; ++yy0) {
      const int64_t zz = bz * BZ + z, yy = by * BY + yy0;
      if (!kRagged || (zz < g.Z && yy < g.Y)) {
        if constexpr (kTailX) {
          XT* row = y + (zz * g.Y + yy) * g.X;
#pragma unroll
          for (int k = 0; k < RV; ++k) {
            const int64_t x0 = bx * BX + k * PER16;
            const T* piece = v + ((z * BY + yy0) * RV + k) * PER16;
            if (x0 + PER16 <= g.X) {
              store16_a4(row + x0, Pack<T, XT>::run(piece));
            } else {
#pragma unroll
              for (int e = 0; e < PER16; ++e)
                if (x0 + e < g.X) Elem<T, XT>::store(row + x0 + e, piece[e]);
            }
          }
        } else if (RV == 2 && whole_wave) {
          // A block row is two 16-byte pieces, so a plain store instruction would write every other piece of a
          // 2 KiB span.  The two half-waves trade pieces instead (lanes 32-63 hand the first piece of their row
          // to lanes 0-31 and take those lanes' second piece): the first store then writes the rows of blocks
          // 0-31 as one contiguous KiB, the second those of blocks 32-63 (workload 4: 0.251 -> 0.240 ms; with
          // the non-temporal hint on top: 0.255 ms).  The compiler hoists every row's trade above the first store
          // (256 registers, two waves per SIMD): running the last transform pass row by row just before each
          // row's stores brought that to 160 registers and three waves, and was slower (0.252 ms): a wave's
          // 32 stores leaving back to back matter more than the third wave.
          uint4 h0 = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + 0) * PER16);
          uint4 h1 = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + 1) * PER16);
          swap_half_waves(h0.x, h1.x);
          swap_half_waves(h0.y, h1.y);
          swap_half_waves(h0.z, h1.z);
          swap_half_waves(h0.w, h1.w);
          uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + tx * 64 * BX) + 2 * (lane & 31) + (lane >> 5);
          p[0] = h0;
          p[64] = h1;
        } else if (RV == 4 && whole_wave) {
          // four pieces per block row: after the quarter transpose store j writes the rows of blocks
          // 16j .. 16j+15 as one contiguous KiB
          uint4 h[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) h[k] = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + k) * PER16);
          transpose_quarter_waves(h[0], h[1], h[2], h[3]);
          uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + tx * 64 * BX) + 4 * (lane & 15) + (lane >> 4);
#pragma unroll
          for (int k = 0; k < 4; ++k) p[64 * k] = h[k];
        } else {
          // plain stores: a lane's pieces alternate with its neighbours' within a line, which the L2 merges into
          // whole lines; with the non-temporal hint these 16-byte pieces reach memory singly (measured: twice as
          // slow), and passing the rows through LDS to store whole lines doubled the kernel's registers
          uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + bx * BX);
#pragma unroll
          for (int k = 0; k < RV; ++k) p[k] = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + k) * PER16);
        }
      }
    }
}


// =====================================================================================================
// Family "quad16": BZ x 16 x 16 blocks with BZ = 1 (2-D) or 4, FP32 / FP16 / bfloat16 arrays, FP32 arithmetic, int8 indices,
// nothing pruned
// =====================================================================================================
// A wave works on 16 planes of 16 x 16 samples: plane p = 4 j + s (j, s in 0..3).  For BZ = 1 these are 16
// consecutive blocks; for BZ = 4 they are the four z-planes (j) of four consecutive blocks (s), so that the lane
// which holds one row of planes j = 0..3 of block s after the exchange can transform along z in registers.
constexpr int kQuadRow = 65;   // uint4 per LDS row: 64 + 1 of padding so that column reads spread over the banks

template <int BZ>
struct QuadMap {
  static constexpr int kBlocksPerWave = BZ == 1 ? 16 : 4;
  // plane p of the wave: which block (relative to the wave's first) and which z-plane of it
  static __device__ __forceinline__ int block_of(int p) { return BZ == 1 ? p : (p & 3); }
  static __device__ __forceinline__ int plane_of(int p) { return BZ == 1 ? 0 : (p >> 2); }
};

template <int TF, typename XT, int BZ, bool kRagged, bool kStats, bool kTailX = false>
__global__ __launch_bounds__(128) void k_compress_quad16(FastGeom g, const XT* __restrict__ x, void* __restrict__ N,
                                                         int8_t* __restrict__ F, double* __restrict__ tile_sums) {
  using Q4 = Quad4<XT>;
  static_assert(BZ == 1 || BZ == 4, "one plane or four");
  using Map = QuadMap<BZ>;
  constexpr int BPW = Map::kBlocksPerWave;
  __shared__ uint4 lds[2][16 * kQuadRow];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<2>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];

  // phase A: lane = (plane p, column quarter q); strip of 16 rows x 4 columns; transform along y
  {
    const int p = lane >> 2, q = lane & 3;
    const int64_t bx = tx * BPW + Map::block_of(p);
    const int64_t bxc = bx < g.gx ? bx : g.gx - 1;
    int64_t zz = bz * BZ + Map::plane_of(p);
    uint32_t keep_z = 0xffffffffu;
    if constexpr (kRagged && BZ > 1) {
      keep_z = zz < g.Z ? 0xffffffffu : 0u;                   // planes past the end: load a valid one, zero it below
      zz = zz < g.Z ? zz : g.Z - 1;
    }
    float v[64];
    typename Q4::raw_t raw[16];
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      int64_t yy = by * 16 + yy0;
      if constexpr (kRagged) yy = yy < g.Y ? yy : g.Y - 1;     // rows past the end: load a valid row, zero it below
      int64_t x0 = bxc * 16 + q * 4;
      if constexpr (kTailX) x0 = x0 + 4 <= g.X ? x0 : g.X - 4;
      raw[yy0] = Q4::template load<kTailX>(x + (zz * g.Y + yy) * g.X + x0);
    }
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      if constexpr (kRagged) Q4::keep(raw[yy0], by * 16 + yy0 < g.Y ? keep_z : 0u);
      Q4::unpack(raw[yy0], v + yy0 * 4);
    }
    if constexpr (kTailX) {
      const int64_t x0 = bxc * 16 + q * 4;
      if (x0 + 4 > g.X) {              // a piece of the row's last, partial block: element by element, zeros beyond
#pragma unroll
        for (int yy0 = 0; yy0 < 16; ++yy0) {
          const int64_t yy = by * 16 + yy0;
          const bool row_in = yy < g.Y && keep_z != 0u;
          const XT* row = x + (zz * g.Y + (yy < g.Y ? yy : g.Y - 1)) * g.X;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int64_t xi = x0 + e;
            const float val = Elem<float, XT>::load(row + (xi < g.X ? xi : g.X - 1));
            v[yy0 * 4 + e] = row_in && xi < g.X ? val : 0.0f;
          }
        }
      }
    }
#pragma unroll
    for (int xl = 0; xl < 4; ++xl) tf_forward<TF, float, 16, 4>(v + xl);
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) st[yy0 * kQuadRow + lane] = f4_bits(v + yy0 * 4);
  }
  wave_lds_sync();
  // phase B: lane = (row yrow, s); four whole rows, row yrow of planes 4 j + s; transform along x (and z)
  const int yrow = lane & 15, bsub = lane >> 4;
  float u[64];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int xq = 0; xq < 4; ++xq) bits_f4(st[yrow * kQuadRow + (4 * j + bsub) * 4 + xq], u + j * 16 + xq * 4);
#pragma unroll
  for (int j = 0; j < 4; ++j) tf_forward<TF, float, 16, 1>(u + j * 16);
  if constexpr (BZ == 4) {
#pragma unroll
    for (int i = 0; i < 16; ++i) tf_forward<TF, float, 4, 16>(u + i);
  }

  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * BPW;
  double s11 = 0.0, d1 = 0.0;
  float m4 = 0.0f;                                     // BZ = 4: the block's maximum over its four planes
  if constexpr (BZ == 4) {
#pragma unroll
    for (int i = 0; i < 64; ++i) m4 = fmaxf(m4, fabsf(u[i]));
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) m4 = fmaxf(m4, __shfl_xor(m4, off, 64));
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float m = m4;
    if constexpr (BZ == 1) {
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(u[j * 16 + i]));
#pragma unroll
      for (int off = 1; off < 16; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));   // the 16 rows of the block
    }
    const float inv = m > 0.0f ? float(g.r) / m : 0.0f;
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      uint32_t q4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) q4[e] = bin_bits(u[j * 16 + k * 4 + e], inv);
      w[k] = IdxPack<int8_t>::pack(q4);
    }
    const int blk = Map::block_of(4 * j + bsub);
    if (tx * BPW + blk < g.gx) {
      // the wave's pieces of F are linear in the lane: 16 consecutive pieces per (plane, block)
      const int piece = BZ == 1 ? yrow : j * 16 + yrow;
      reinterpret_cast<uint4*>(F + (block0 + blk) * (BZ * 256))[piece] = make_uint4(w[0], w[1], w[2], w[3]);
      const bool first = yrow == 0 && (BZ == 1 || j == 0);
      if (first) store_float(N, g.ntype, block0 + blk, m);
      if constexpr (kStats) {
        const double n = stored_N(m, g.ntype);
        s11 += sum_of_squares<int8_t, 4>(w) * (n * n);
        if (first) d1 += n * double(IdxPack<int8_t>::get(w[0], 0));
      }
    }
  }
  if constexpr (kStats) emit_tile_sums(tile_sums, g, tx, by, bz, s11, d1);
}

template <int TF, typename XT, int BZ, bool kTailX = false>
__global__ __launch_bounds__(128) void k_decompress_quad16(FastGeom g, const void* __restrict__ N,
                                                           const int8_t* __restrict__ F, XT* __restrict__ y) {
  using Q4 = Quad4<XT>;
  using Map = QuadMap<BZ>;
  constexpr int BPW = Map::kBlocksPerWave;
  __shared__ uint4 lds[2][16 * kQuadRow];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<2>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * BPW;
  {
    const int yrow = lane & 15, bsub = lane >> 4;
    float u[64];
    int64_t blocks[4];
    uint4 fs[4];
    float ns[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t blk = Map::block_of(4 * j + bsub);
      if (tx * BPW + blk >= g.gx) blk = g.gx - 1 - tx * BPW;   // past the end: decode the last block again, stored nowhere
      blocks[j] = block0 + blk;
      const int piece = BZ == 1 ? yrow : j * 16 + yrow;
      fs[j] = reinterpret_cast<const uint4*>(F + blocks[j] * (BZ * 256))[piece];
    }
    load_N_many<4>(N, g.ntype, blocks, ns);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint4 f = fs[j];
      const float scale = ns[j] / float(g.r);
      const uint32_t w[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
      for (int i = 0; i < 16; ++i) u[j * 16 + i] = scale * float(IdxPack<int8_t>::get(w[i >> 2], i & 3));
    }
    if constexpr (BZ == 4) {
#pragma unroll
      for (int i = 0; i < 16; ++i) tf_inverse<TF, float, 4, 16, 4>(u + i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) tf_inverse<TF, float, 16, 1, 16>(u + j * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int xq = 0; xq < 4; ++xq) st[yrow * kQuadRow + (4 * j + bsub) * 4 + xq] = f4_bits(u + j * 16 + xq * 4);
  }
  wave_lds_sync();
  const int p = lane >> 2, q = lane & 3;
  const int64_t bx = tx * BPW + Map::block_of(p);
  const int64_t zz = bz * BZ + Map::plane_of(p);
  float v[64];
#pragma unroll
  for (int yy0 = 0; yy0 < 16; ++yy0) bits_f4(st[yy0 * kQuadRow + lane], v + yy0 * 4);
#pragma unroll
  for (int xl = 0; xl < 4; ++xl) tf_inverse<TF, float, 16, 4, 16>(v + xl);
  if (bx < g.gx && zz < g.Z) {
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      const int64_t yy = by * 16 + yy0;
      if (yy < g.Y) {
        if constexpr (kTailX) {
          XT* row = y + (zz * g.Y + yy) * g.X;
          const int64_t x0 = bx * 16 + q * 4;
          if (x0 + 4 <= g.X) {
            Q4::template store<true>(row + x0, Q4::pack(v + yy0 * 4));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (x0 + e < g.X) Elem<float, XT>::store(row + x0 + e, v[yy0 * 4 + e]);
          }
        } else {
          Q4::template store<false>(y + (zz * g.Y + yy) * g.X + bx * 16 + q * 4, Q4::pack(v + yy0 * 4));
        }
      }
    }
  }
}

// =====================================================================================================
// Family "oct8": 3-D 8x8x8 blocks, bfloat16, FP16 or FP32 arrays, FP32 arithmetic, int8 indices, low-frequency box kept
// =====================================================================================================
// LDS exchange, done in two rounds (left and right half of every 8-element row) so that a wave needs 8 KiB
// instead of 16 KiB and twice as many waves fit a CU (the kernel is latency-bound: halving its occupancy
// cost 40 %).  Per round block b occupies 64 sixteen-byte slots ordered [y][z]; the low four bits of the slot
// are XORed with 2b and a permutation of y so that both the plane-wise writes (lanes differ in z, b) and the
// row-wise reads (lanes differ in b, y) touch sixteen different bank groups per sixteen lanes.
__device__ __forceinline__ int oct_slot(int b, int yy, int z) {
  const int perm = ((yy >> 1) & 1) | (((yy >> 2) & 1) << 2);
  return b * 64 + ((yy * 8 + z) ^ (2 * b) ^ perm);
}

constexpr int kOctWaves = 4;   // waves per workgroup: neighbouring tiles, so that a workgroup reads 512-byte row pieces

template <int TF, typename XT, int KZ, int KY, int KX, bool kRagged, bool kStats, bool kTailX = false>
__global__ __launch_bounds__(kOctWaves * 64) void k_compress_oct8(FastGeom g, const XT* __restrict__ x,
                                                                  void* __restrict__ N, int8_t* __restrict__ F,
                                                                  double* __restrict__ tile_sums) {
  static_assert(KX == 4 || KX == 8, "a kept row is one or two dwords of int8");
  constexpr int KEPT = KZ * KY * KX;
  constexpr int PER16 = Unpack<float, XT>::n;     // elements per 16-byte piece: 8 (bfloat16) or 4 (FP32)
  constexpr int RV = 8 / PER16;                   // pieces per block row
  __shared__ uint4 lds[kOctWaves][8 * 64];
  // a wave that is fetching its tile goes ahead of the waves that are busy transforming theirs
  __builtin_amdgcn_s_setprio(3);
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<kOctWaves>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int z = lane >> 3, b = lane & 7;      // phase A: lane = (plane z, block b)
  const int bb = lane >> 3, j = lane & 7;     // phase B: lane = (block bb, row j)

  // phase A: one 8x8 z-plane per lane; transforms along x and y
  float v[64];
  {
    const int64_t bx = tx * 8 + b;
    const int64_t bxc = bx < g.gx ? bx : g.gx - 1;
    int64_t zz = bz * 8 + z;
    uint32_t keep_z = 0xffffffffu;
    if constexpr (kRagged) {
      keep_z = zz < g.Z ? 0xffffffffu : 0u;      // planes / rows past the end: load a valid row, zero it below
      zz = zz < g.Z ? zz : g.Z - 1;
    }
    uint4 raw[8 * RV];
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) {
      int64_t yy = by * 8 + yy0;
      if constexpr (kRagged) yy = yy < g.Y ? yy : g.Y - 1;
#pragma unroll
      for (int k = 0; k < RV; ++k) {
        const int64_t x0 = bxc * 8 + k * PER16;
        if constexpr (kTailX)
          raw[yy0 * RV + k] = load16_a4(x + (zz * g.Y + yy) * g.X + (x0 + PER16 <= g.X ? x0 : g.X - PER16));
        else
          raw[yy0 * RV + k] = load16_stream(x + (zz * g.Y + yy) * g.X + x0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) {
#pragma unroll
      for (int k = 0; k < RV; ++k) {
        uint4& piece = raw[yy0 * RV + k];
        if constexpr (kRagged) {
          const uint32_t keep = by * 8 + yy0 < g.Y ? keep_z : 0u;
          piece.x &= keep; piece.y &= keep; piece.z &= keep; piece.w &= keep;
        }
        Unpack<float, XT>::run(piece, v + yy0 * 8 + k * PER16);
      }
    }
    if constexpr (kTailX) {
      if (bxc * 8 + 8 > g.X) {         // the row's last, partial block: element by element, zeros beyond
#pragma unroll
        for (int yy0 = 0; yy0 < 8; ++yy0) {
          const int64_t yy = by * 8 + yy0;
          const bool row_in = yy < g.Y && keep_z != 0u;
          const XT* row = x + (zz * g.Y + (yy < g.Y ? yy : g.Y - 1)) * g.X;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int64_t xi = bxc * 8 + e;
            const float val = Elem<float, XT>::load(row + (xi < g.X ? xi : g.X - 1));
            v[yy0 * 8 + e] = row_in && xi < g.X ? val : 0.0f;
          }
        }
      }
    }
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) tf_forward<TF, float, 8, 1>(v + yy0 * 8);
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) tf_forward<TF, float, 8, 8>(v + xx);
  }
  // exchange: afterwards the lane holds the row y = j of all eight planes of block bb; transform along z
  float u[64];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) st[oct_slot(b, yy0, z)] = f4_bits(v + yy0 * 8 + h * 4);
    wave_lds_sync();
#pragma unroll
    for (int zz0 = 0; zz0 < 8; ++zz0) bits_f4(st[oct_slot(bb, j, zz0)], u + zz0 * 8 + h * 4);
    wave_lds_sync();
  }
#pragma unroll
  for (int xx = 0; xx < 8; ++xx) tf_forward<TF, float, 8, 8>(u + xx);

  float m = 0.0f;
#pragma unroll
  for (int i = 0; i < 64; ++i) m = fmaxf(m, fabsf(u[i]));
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));     // the 8 rows of the block
  const float inv = m > 0.0f ? float(g.r) / m : 0.0f;

  // kept entries of this lane: z < KZ, x < KX when j < KY; staged in LDS at their position in the wave's span of F
  static_assert(8 * KEPT <= 8 * 64 * 16, "the staged F of a tile fits the exchange buffer");
  uint32_t* st32 = reinterpret_cast<uint32_t*>(st);
  int squares = 0;            // of this lane's kept indices: at most 64 * 127^2
  uint32_t first = 0;         // the dword that starts with F_k0 (lanes with j == 0)
  if (j < KY) {
#pragma unroll
    for (int zq = 0; zq < KZ; ++zq)
#pragma unroll
      for (int k = 0; k < KX / 4; ++k) {
        uint32_t q4[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) q4[e] = bin_bits(u[zq * 8 + k * 4 + e], inv);
        const uint32_t pw = IdxPack<int8_t>::pack(q4);
        st32[(bb * KEPT + (zq * KY + j) * KX) / 4 + k] = pw;
        if constexpr (kStats) {
          squares = __builtin_amdgcn_sdot4(int(pw), int(pw), squares, false);
          if (zq == 0 && k == 0) first = pw;
        }
      }
  }
  if constexpr (kStats) {
    const double n = tx * 8 + bb < g.gx ? stored_N(m, g.ntype) : 0.0;
    emit_tile_sums(tile_sums, g, tx, by, bz, double(squares) * (n * n),
                   j == 0 ? n * double(IdxPack<int8_t>::get(first, 0)) : 0.0);
  }
  wave_lds_sync();
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * 8;
  constexpr int PIECES = 8 * KEPT / 16;            // 16-byte pieces of F per wave
  constexpr int PPB = KEPT / 16;                   // per block
  static_assert(KEPT % 16 == 0, "F blocks are whole 16-byte vectors");
#pragma unroll
  for (int p0 = 0; p0 < PIECES; p0 += 64) {
    const int p = p0 + lane;
    if (p < PIECES && tx * 8 + p / PPB < g.gx) reinterpret_cast<uint4*>(F + block0 * KEPT)[p] = st[p];
  }
  if (j == 0 && tx * 8 + bb < g.gx) store_float(N, g.ntype, block0 + bb, m);
}

// 16 bytes of an output row from FP32 values: bfloat16 through the hardware conversion
template <typename XT>
__device__ __forceinline__ uint4 oct_pack(const float* v) {
  if constexpr (std::is_same<XT, bf16_t>::value)
    return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  else
    return Pack<float, XT>::run(v);
}

// the eight values r8 of block bx's row at `row`: whole 16-byte pieces where they fit, single elements otherwise
template <typename XT, bool kTailX>
__device__ __forceinline__ void oct_store_row(const FastGeom& g, XT* row, int64_t bx, const float* r8) {
  constexpr int PER16 = Unpack<float, XT>::n;
#pragma unroll
  for (int k = 0; k < 8 / PER16; ++k) {
    const int64_t x0 = bx * 8 + k * PER16;
    if constexpr (kTailX) {
      if (x0 + PER16 <= g.X) {
        store16_a4(row + x0, oct_pack<XT>(r8 + k * PER16));
      } else {
#pragma unroll
        for (int e = 0; e < PER16; ++e)
          if (x0 + e < g.X) Elem<float, XT>::store(row + x0 + e, r8[k * PER16 + e]);
      }
    } else if constexpr (PER16 == 8) {
      store16_stream(row + x0, oct_pack<XT>(r8 + k * PER16));       // the lanes' pieces are contiguous: whole lines
    } else {
      // two pieces per lane, 32 bytes apart: plain stores, which the L2 merges into whole lines (with the
      // non-temporal hint such pieces reach memory singly)
      *reinterpret_cast<uint4*>(row + x0) = oct_pack<XT>(r8 + k * PER16);
    }
  }
}

template <int TF, typename XT, int KZ, int KY, int KX, bool kTailX = false>
__global__ __launch_bounds__(256) void k_decompress_oct8(FastGeom g, const void* __restrict__ N,
                                                         const int8_t* __restrict__ F, XT* __restrict__ y) {
  constexpr int KEPT = KZ * KY * KX;
  static_assert(KEPT % 16 == 0, "F blocks are whole 16-byte vectors");
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<4>(g, tx, by, bz)) return;
  const int z = lane >> 3, b = lane & 7;
  const int64_t bx = tx * 8 + b;
  const int64_t zz = bz * 8 + z;
  if (bx >= g.gx || zz >= g.Z) return;
  const int64_t block = (bz * g.gy + by) * g.gx + bx;

  uint32_t w[KEPT / 4];
#pragma unroll
  for (int k = 0; k < KEPT / 16; ++k) {
    const uint4 f = reinterpret_cast<const uint4*>(F + block * KEPT)[k];
    w[4 * k] = f.x; w[4 * k + 1] = f.y; w[4 * k + 2] = f.z; w[4 * k + 3] = f.w;
  }
  // this lane's plane z of the inverse z transform: sum_q (N / r) H[z][q] C[q][.][.]
  const float scale = load_float<float>(N, g.ntype, block) / float(g.r);
  float hz[KZ];
#pragma unroll
  for (int q = 0; q < KZ; ++q) hz[q] = scale * (TF == kTfHaar ? c_haar8.h[z][q] : c_dct8.h[z][q]);
  float v[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) v[i] = 0.0f;
#pragma unroll
  for (int yy0 = 0; yy0 < KY; ++yy0)
#pragma unroll
    for (int xx = 0; xx < KX; ++xx) {
      float acc = 0.0f;
#pragma unroll
      for (int q = 0; q < KZ; ++q) {
        const int jf = (q * KY + yy0) * KX + xx;
        acc += hz[q] * float(IdxPack<int8_t>::get(w[jf >> 2], jf & 3));
      }
      v[yy0 * 8 + xx] = acc;
    }
#pragma unroll
  for (int xx = 0; xx < KX; ++xx) tf_inverse<TF, float, 8, 8, KY>(v + xx);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) tf_inverse<TF, float, 8, 1, KX>(v + yy0 * 8);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) {
    const int64_t yy = by * 8 + yy0;
    if (yy < g.Y) oct_store_row<XT, kTailX>(g, y + (zz * g.Y + yy) * g.X, bx, v + yy0 * 8);
  }
}

// The same computation laid out for wide arrays: a workgroup of eight waves owns 64 consecutive blocks, wave z
// rebuilds plane z of all of them (lane = block), so that every store instruction writes one whole contiguous
// 1 KiB row piece (measured 6.6 TB/s for this store pattern against 5.7 TB/s for the 128-byte pieces above);
// the plane index is uniform over the wave, so its matrix row comes from scalar loads.
template <int TF, typename XT, int KZ, int KY, int KX, bool kTailX = false>
__global__ __launch_bounds__(512) void k_decompress_oct8_rows(FastGeom g, const void* __restrict__ N,
                                                              const int8_t* __restrict__ F, XT* __restrict__ y) {
  constexpr int KEPT = KZ * KY * KX;
  static_assert(KEPT % 16 == 0, "F blocks are whole 16-byte vectors");
  const int lane = threadIdx.x & 63;
  const int z = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t t = blockIdx.x;                               // tile of 64 blocks within the z-slab
  const uint32_t slab = blockIdx.y + blockIdx.z * gridDim.y;
  if (t >= g.tiles_yx || slab >= g.gz) return;
  const int64_t by = t / g.tiles_x, tx = t - uint32_t(by) * g.tiles_x, bz = slab;
  const int64_t bx = tx * 64 + lane;
  const int64_t zz = bz * 8 + z;
  if (bx >= g.gx || zz >= g.Z) return;
  const bool whole_wave = tx * 64 + 64 <= int64_t(g.gx);     // uniform: no lane has left
  const int64_t block = (bz * g.gy + by) * g.gx + bx;

  uint32_t w[KEPT / 4];
#pragma unroll
  for (int k = 0; k < KEPT / 16; ++k) {
    const uint4 f = reinterpret_cast<const uint4*>(F + block * KEPT)[k];
    w[4 * k] = f.x; w[4 * k + 1] = f.y; w[4 * k + 2] = f.z; w[4 * k + 3] = f.w;
  }
  // this lane's plane z of the inverse z transform: sum_q (N / r) H[z][q] C[q][.][.]
  const float scale = load_float<float>(N, g.ntype, block) / float(g.r);
  float hz[KZ];
#pragma unroll
  for (int q = 0; q < KZ; ++q) hz[q] = scale * (TF == kTfHaar ? c_haar8.h[z][q] : c_dct8.h[z][q]);
  float v[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) v[i] = 0.0f;
#pragma unroll
  for (int yy0 = 0; yy0 < KY; ++yy0)
#pragma unroll
    for (int xx = 0; xx < KX; ++xx) {
      float acc = 0.0f;
#pragma unroll
      for (int q = 0; q < KZ; ++q) {
        const int jf = (q * KY + yy0) * KX + xx;
        acc += hz[q] * float(IdxPack<int8_t>::get(w[jf >> 2], jf & 3));
      }
      v[yy0 * 8 + xx] = acc;
    }
#pragma unroll
  for (int xx = 0; xx < KX; ++xx) tf_inverse<TF, float, 8, 8, KY>(v + xx);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) tf_inverse<TF, float, 8, 1, KX>(v + yy0 * 8);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) {
    const int64_t yy = by * 8 + yy0;
    if (yy >= g.Y) continue;
    if constexpr (sizeof(XT) == 4 && !kTailX) {
      if (whole_wave) {
        // FP32 rows are two 16-byte pieces per block: the half-waves trade pieces so that each store writes one
        // contiguous KiB (the rows of 32 blocks)
        uint4 h0 = oct_pack<XT>(v + yy0 * 8), h1 = oct_pack<XT>(v + yy0 * 8 + 4);
        swap_half_waves(h0.x, h1.x);
        swap_half_waves(h0.y, h1.y);
        swap_half_waves(h0.z, h1.z);
        swap_half_waves(h0.w, h1.w);
        uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + tx * 64 * 8) + 2 * (lane & 31) + (lane >> 5);
        store16_stream(p, h0);
        store16_stream(p + 64, h1);
        continue;
      }
    }
    oct_store_row<XT, kTailX>(g, y + (zz * g.Y + yy) * g.X, bx, v + yy0 * 8);
  }
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

Folded fold(const pbz_codec* c, const Geom& geo) {
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

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

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

// One table row per instantiation.
template <int TF, typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX>
struct LaneKernel {
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->transform == TF && c->compute_f64 == (sizeof(T) == 8) && xtype == xtype_code<XT>() && int(c->itype) == itype_code<IT>() &&
           n_type_ok<NT>(int(c->ftype)) && f.bz == BZ && f.by == BY && f.bx == BX && f.kz == KZ && f.ky == KY &&
           f.kx == KX && x_extent_ok(f, 16 / int(sizeof(XT)), int(sizeof(XT)));
  }
  static int fits(FastGeom g) {
    dim3 grid;
    return tile_grid(g, 64, 4, &grid) ? 1 : 0;
  }
  static int64_t tiles(FastGeom g) {
    dim3 grid;
    return tile_grid(g, 64, 4, &grid) ? g.gz * int64_t(g.tiles_yx) : 0;
  }
  template <bool kRagged, bool kStats, bool kTailX>
  static void launch(const FastGeom& g, dim3 grid, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    hipLaunchKernelGGL((k_compress_lane<TF, T, XT, IT, NT, BZ, BY, BX, KZ, KY, KX, kRagged, kStats, kTailX>), grid,
                       dim3(256), 0, s, g, static_cast<const XT*>(x), N, static_cast<IT*>(F), tile_sums);
  }
  template <bool kRagged, bool kTailX>
  static void launch_inverse(const FastGeom& g, dim3 grid, const void* N, const void* F, void* y, hipStream_t s) {
    hipLaunchKernelGGL((k_decompress_lane<TF, T, XT, IT, NT, BZ, BY, BX, KZ, KY, KX, kRagged, kTailX>), grid, dim3(256), 0,
                       s, g, N, static_cast<const IT*>(F), static_cast<XT*>(y));
  }
  // tile_sums != nullptr: also the per-wave statistic sums (two doubles per tile)
  static int compress(FastGeom g, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, 64, 4, &grid)) return 0;
    const bool ragged = g.Z % BZ || g.Y % BY;
    if (g.X % BX) tile_sums ? launch<true, true, true>(g, grid, x, N, F, tile_sums, s) : launch<true, false, true>(g, grid, x, N, F, nullptr, s);
    else if (tile_sums) ragged ? launch<true, true, false>(g, grid, x, N, F, tile_sums, s) : launch<false, true, false>(g, grid, x, N, F, tile_sums, s);
    else ragged ? launch<true, false, false>(g, grid, x, N, F, nullptr, s) : launch<false, false, false>(g, grid, x, N, F, nullptr, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, 64, 4, &grid)) return 0;
    if (g.X % BX) launch_inverse<true, true>(g, grid, N, F, y, s);
    else if (g.Z % BZ || g.Y % BY) launch_inverse<true, false>(g, grid, N, F, y, s);
    else launch_inverse<false, false>(g, grid, N, F, y, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

// 2-D 8x8, FP32 arrays: int8 (FP32 arithmetic), int16 (FP64 arithmetic) with all 64 or the 4x4 low-frequency box kept
template <int TF> using Lane_f32_8x8_i8 = LaneKernel<TF, float, float, int8_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_bf16_8x8_i8 = LaneKernel<TF, float, bf16_t, int8_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f16_8x8_i8 = LaneKernel<TF, float, f16_t, int8_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f32_8x8_i16_box4 = LaneKernel<TF, double, float, int16_t, float, 1, 8, 8, 1, 4, 4>;
template <int TF> using Lane_f32_8x8_i16 = LaneKernel<TF, double, float, int16_t, float, 1, 8, 8, 1, 8, 8>;
// 3-D 4x4x4, FP64 arrays, int16
template <int TF> using Lane_f64_4x4x4_i16 = LaneKernel<TF, double, double, int16_t, double, 4, 4, 4, 4, 4, 4>;
// the settings of the paper's own timing experiments that the workloads above do not cover (Sec. V-A: square 2-D
// FP64 arrays in 8x8 blocks with int8 indices; hypercubic 2-D / 3-D arrays with int8 and int16 indices; cubic
// arrays in blocks of 4)
template <int TF> using Lane_f64_4x4x4_i8 = LaneKernel<TF, double, double, int8_t, double, 4, 4, 4, 4, 4, 4>;
template <int TF> using Lane_f32_4x4x4_i8 = LaneKernel<TF, float, float, int8_t, float, 4, 4, 4, 4, 4, 4>;
template <int TF> using Lane_f32_4x4x4_i16 = LaneKernel<TF, double, float, int16_t, float, 4, 4, 4, 4, 4, 4>;
template <int TF> using Lane_f64_8x8_i8 = LaneKernel<TF, double, double, int8_t, double, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f64_8x8_i16 = LaneKernel<TF, double, double, int16_t, double, 1, 8, 8, 1, 8, 8>;

// 16x16 (2-D) and 4x16x16 blocks, FP32 / bfloat16 / FP16 arrays, int8, nothing pruned
template <int TF, typename XT, int BZ>
struct Quad16Kernel {
  static constexpr int kBlocksPerWave = BZ == 1 ? 16 : 4;
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->transform == TF && !c->compute_f64 && xtype == xtype_code<XT>() && c->itype == PBZ_I8 &&
           c->ftype != PBZ_F64 && f.bz == BZ && f.by == 16 && f.bx == 16 && f.kz == BZ && f.ky == 16 && f.kx == 16 &&
           x_extent_ok(f, 4, int(sizeof(XT)));
  }
  static int fits(FastGeom g) {
    dim3 grid;
    return tile_grid(g, kBlocksPerWave, 2, &grid) ? 1 : 0;
  }
  static int64_t tiles(FastGeom g) {
    dim3 grid;
    return tile_grid(g, kBlocksPerWave, 2, &grid) ? g.gz * int64_t(g.tiles_yx) : 0;
  }
  template <bool kRagged, bool kStats, bool kTailX>
  static void launch(const FastGeom& g, dim3 grid, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    hipLaunchKernelGGL((k_compress_quad16<TF, XT, BZ, kRagged, kStats, kTailX>), grid, dim3(128), 0, s, g,
                       static_cast<const XT*>(x), N, static_cast<int8_t*>(F), tile_sums);
  }
  static int compress(FastGeom g, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, kBlocksPerWave, 2, &grid)) return 0;
    const bool ragged = g.Y % 16 || g.Z % BZ;
    if (g.X % 16) tile_sums ? launch<true, true, true>(g, grid, x, N, F, tile_sums, s) : launch<true, false, true>(g, grid, x, N, F, nullptr, s);
    else if (tile_sums) ragged ? launch<true, true, false>(g, grid, x, N, F, tile_sums, s) : launch<false, true, false>(g, grid, x, N, F, tile_sums, s);
    else ragged ? launch<true, false, false>(g, grid, x, N, F, nullptr, s) : launch<false, false, false>(g, grid, x, N, F, nullptr, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, kBlocksPerWave, 2, &grid)) return 0;
    if (g.X % 16)
      hipLaunchKernelGGL((k_decompress_quad16<TF, XT, BZ, true>), grid, dim3(128), 0, s, g, N,
                         static_cast<const int8_t*>(F), static_cast<XT*>(y));
    else
      hipLaunchKernelGGL((k_decompress_quad16<TF, XT, BZ, false>), grid, dim3(128), 0, s, g, N,
                         static_cast<const int8_t*>(F), static_cast<XT*>(y));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

// 3-D 8x8x8 bfloat16 or FP32 arrays, FP32 arithmetic and N, int8, box KZ x KY x KX kept
template <int TF, typename XT, int KZ, int KY, int KX>
struct Oct8Kernel {
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->transform == TF && !c->compute_f64 && xtype == xtype_code<XT>() && c->itype == PBZ_I8 &&
           c->ftype != PBZ_F64 && f.bz == 8 && f.by == 8 && f.bx == 8 && f.kz == KZ && f.ky == KY && f.kx == KX &&
           x_extent_ok(f, 16 / int(sizeof(XT)), int(sizeof(XT)));
  }
  static int fits(FastGeom g) {
    dim3 grid;
    return tile_grid(g, 8, kOctWaves, &grid) ? 1 : 0;
  }
  static int64_t tiles(FastGeom g) {
    dim3 grid;
    return tile_grid(g, 8, kOctWaves, &grid) ? g.gz * int64_t(g.tiles_yx) : 0;
  }
  template <bool kRagged, bool kStats, bool kTailX>
  static void launch(const FastGeom& g, dim3 grid, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    hipLaunchKernelGGL((k_compress_oct8<TF, XT, KZ, KY, KX, kRagged, kStats, kTailX>), grid, dim3(kOctWaves * 64), 0, s, g,
                       static_cast<const XT*>(x), N, static_cast<int8_t*>(F), tile_sums);
  }
  static int compress(FastGeom g, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, 8, kOctWaves, &grid)) return 0;
    const bool ragged = g.Z % 8 || g.Y % 8;
    if (g.X % 8) tile_sums ? launch<true, true, true>(g, grid, x, N, F, tile_sums, s) : launch<true, false, true>(g, grid, x, N, F, nullptr, s);
    else if (tile_sums) ragged ? launch<true, true, false>(g, grid, x, N, F, tile_sums, s) : launch<false, true, false>(g, grid, x, N, F, tile_sums, s);
    else ragged ? launch<true, false, false>(g, grid, x, N, F, nullptr, s) : launch<false, false, false>(g, grid, x, N, F, nullptr, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    dim3 grid;
    const void* n = N;
    const int8_t* f = static_cast<const int8_t*>(F);
    XT* out = static_cast<XT*>(y);
    const bool tail = g.X % 8 != 0;
    if (g.gx >= 48) {        // at least three quarters of the lanes of a 64-block tile busy
      if (!tile_grid(g, 64, 1, &grid)) return 0;
      if (tail) hipLaunchKernelGGL((k_decompress_oct8_rows<TF, XT, KZ, KY, KX, true>), grid, dim3(512), 0, s, g, n, f, out);
      else hipLaunchKernelGGL((k_decompress_oct8_rows<TF, XT, KZ, KY, KX, false>), grid, dim3(512), 0, s, g, n, f, out);
    } else {
      if (!tile_grid(g, 8, 4, &grid)) return 0;
      if (tail) hipLaunchKernelGGL((k_decompress_oct8<TF, XT, KZ, KY, KX, true>), grid, dim3(256), 0, s, g, n, f, out);
      else hipLaunchKernelGGL((k_decompress_oct8<TF, XT, KZ, KY, KX, false>), grid, dim3(256), 0, s, g, n, f, out);
    }
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};
template <int TF> using Oct8_box4 = Oct8Kernel<TF, bf16_t, 4, 4, 4>;
template <int TF> using Oct8_full = Oct8Kernel<TF, bf16_t, 8, 8, 8>;
template <int TF> using Oct8_f32_box4 = Oct8Kernel<TF, float, 4, 4, 4>;
template <int TF> using Oct8_f32_full = Oct8Kernel<TF, float, 8, 8, 8>;
template <int TF> using Oct8_f16_box4 = Oct8Kernel<TF, f16_t, 4, 4, 4>;
template <int TF> using Oct8_f16_full = Oct8Kernel<TF, f16_t, 8, 8, 8>;

#define COMMA ,
#define PBZ_FOR_EACH_SHAPE(X, TF, SUFFIX)                             \
  X(Lane_f32_8x8_i8<TF>, "lane_f32_8x8_i8" SUFFIX)                     \
  X(Lane_bf16_8x8_i8<TF>, "lane_bf16_8x8_i8" SUFFIX)                   \
  X(Lane_f16_8x8_i8<TF>, "lane_f16_8x8_i8" SUFFIX)                     \
  X(Lane_f32_8x8_i16_box4<TF>, "lane_f32_8x8_i16_box4x4" SUFFIX)       \
  X(Lane_f32_8x8_i16<TF>, "lane_f32_8x8_i16" SUFFIX)                   \
  X(Lane_f64_4x4x4_i16<TF>, "lane_f64_4x4x4_i16" SUFFIX)               \
  X(Lane_f64_4x4x4_i8<TF>, "lane_f64_4x4x4_i8" SUFFIX)                 \
  X(Lane_f32_4x4x4_i8<TF>, "lane_f32_4x4x4_i8" SUFFIX)                 \
  X(Lane_f32_4x4x4_i16<TF>, "lane_f32_4x4x4_i16" SUFFIX)               \
  X(Lane_f64_8x8_i8<TF>, "lane_f64_8x8_i8" SUFFIX)                     \
  X(Lane_f64_8x8_i16<TF>, "lane_f64_8x8_i16" SUFFIX)                   \
  X(Quad16Kernel<TF COMMA float COMMA 1>, "quad16_f32_16x16_i8" SUFFIX)            \
  X(Quad16Kernel<TF COMMA float COMMA 4>, "quad16_f32_4x16x16_i8" SUFFIX)          \
  X(Quad16Kernel<TF COMMA f16_t COMMA 1>, "quad16_f16_16x16_i8" SUFFIX)            \
  X(Quad16Kernel<TF COMMA bf16_t COMMA 1>, "quad16_bf16_16x16_i8" SUFFIX)          \
  X(Quad16Kernel<TF COMMA f16_t COMMA 4>, "quad16_f16_4x16x16_i8" SUFFIX)          \
  X(Oct8_box4<TF>, "oct8_bf16_8x8x8_i8_box4x4x4" SUFFIX)               \
  X(Oct8_full<TF>, "oct8_bf16_8x8x8_i8" SUFFIX)                        \
  X(Oct8_f32_box4<TF>, "oct8_f32_8x8x8_i8_box4x4x4" SUFFIX)            \
  X(Oct8_f32_full<TF>, "oct8_f32_8x8x8_i8" SUFFIX)                     \
  X(Oct8_f16_box4<TF>, "oct8_f16_8x8x8_i8_box4x4x4" SUFFIX)            \
  X(Oct8_f16_full<TF>, "oct8_f16_8x8x8_i8" SUFFIX)
// every shape for the DCT (plain names) and for the Haar transform (names ending in _haar)
#define PBZ_FOR_EACH_LANE_KERNEL(X)    \
  PBZ_FOR_EACH_SHAPE(X, kTfDct, "")    \
  PBZ_FOR_EACH_SHAPE(X, kTfHaar, "_haar")

}  // namespace

int try_compress_fast(const pbz_codec* c, const Geom& geo, const void* x, int xtype, void* N, void* F, hipStream_t s,
                      bool dry_run, const char** name, double* tile_sums) {
  if (!aligned16(x) || !aligned16(F)) return 0;
  const Folded f = fold(c, geo);
  if (!f.ok) return 0;
#define X(K, NAME)                                          \
  if (K::matches(c, f, xtype)) {                            \
    *name = NAME;                                           \
    return dry_run ? K::fits(f.g) : K::compress(f.g, x, N, F, tile_sums, s); \
  }
  PBZ_FOR_EACH_LANE_KERNEL(X)
#undef X
  return 0;
}

int64_t fast_compress_tiles(const pbz_codec* c, const Geom& geo, int xtype) {
  const Folded f = fold(c, geo);
  if (!f.ok) return 0;
#define X(K, NAME) \
  if (K::matches(c, f, xtype)) return K::tiles(f.g);
  PBZ_FOR_EACH_LANE_KERNEL(X)
#undef X
  return 0;
}

int try_decompress_fast(const pbz_codec* c, const Geom& geo, const void* N, const void* F, void* y, int ytype,
                        hipStream_t s, bool dry_run, const char** name) {
  if (!aligned16(y) || !aligned16(F)) return 0;
  const Folded f = fold(c, geo);
  if (!f.ok) return 0;
#define X(K, NAME)                                            \
  if (K::matches(c, f, ytype)) {                              \
    *name = NAME;                                             \
    return dry_run ? K::fits(f.g) : K::decompress(f.g, N, F, y, s); \
  }
  PBZ_FOR_EACH_LANE_KERNEL(X)
#undef X
  return 0;
}

}  // namespace pbz
