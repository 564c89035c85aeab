// Specialised codec kernels for the block shapes that matter for throughput.
//
// Every kernel here is "wave autonomous": a 64-lane wave owns a run of consecutive blocks along the
// contiguous (last) array dimension, reads whole block rows straight from HBM with 16-byte loads (the
// lanes of a wave cover a contiguous span of every row, which measures at the same bandwidth as a
// linear copy on MI355X), transforms in registers with the even/odd-split DCT of pbz_dct.h, and writes
// N and F.  There is no workgroup barrier anywhere; LDS, where used, is private to a wave.
//
// Family "lane": one lane owns one whole block (blocks of at most 64 elements: 8x8, 4x4x4).
//
// Preconditions checked on the host (otherwise the call falls back to the general kernels): the array
// reduces to at most three dimensions (leading dimensions with block extent 1 fold into the slowest one),
// the block shape / types / mask box match an instantiation, the last array extent is a multiple of the
// block's last extent, and rows start 16-byte aligned.  The other dimensions may be ragged.
#include "pbz_dct.h"
#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace {

struct FastGeom {
  int64_t Z, Y, X;        // array extents after folding
  int64_t gz, gy, gx;     // block grid
  int64_t tiles_x;        // waves needed to cover gx blocks
  int64_t n_tiles;
  double r;
};

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

// ---- index packing ---------------------------------------------------------------------------------
template <typename IT>
struct IdxPack;   // kPer indices per dword
template <>
struct IdxPack<int8_t> {
  static constexpr int per = 4;
  static __device__ __forceinline__ uint32_t pack(const int* q) {
    return (uint32_t(q[0]) & 0xffu) | ((uint32_t(q[1]) & 0xffu) << 8) | ((uint32_t(q[2]) & 0xffu) << 16) |
           (uint32_t(q[3]) << 24);
  }
  static __device__ __forceinline__ int get(uint32_t w, int i) { return int(int8_t((w >> (8 * i)) & 0xffu)); }
};
template <>
struct IdxPack<int16_t> {
  static constexpr int per = 2;
  static __device__ __forceinline__ uint32_t pack(const int* q) {
    return (uint32_t(q[0]) & 0xffffu) | (uint32_t(q[1]) << 16);
  }
  static __device__ __forceinline__ int get(uint32_t w, int i) { return int(int16_t((w >> (16 * i)) & 0xffffu)); }
};

template <typename T>
__device__ __forceinline__ T abs_t(T v) { return v < T(0) ? -v : v; }
template <>
__device__ __forceinline__ float abs_t<float>(float v) { return fabsf(v); }
template <>
__device__ __forceinline__ double abs_t<double>(double v) { return fabs(v); }

// forward transform of a register-resident [BZ][BY][BX] block, one dimension after the other
template <typename T, int BZ, int BY, int BX>
__device__ __forceinline__ void forward_block(T* v) {
  if constexpr (BX > 1) {
#pragma unroll
    for (int row = 0; row < BZ * BY; ++row) dct::forward<T, BX, 1>(v + row * BX);
  }
  if constexpr (BY > 1) {
#pragma unroll
    for (int z = 0; z < BZ; ++z)
#pragma unroll
      for (int xx = 0; xx < BX; ++xx) dct::forward<T, BY, BX>(v + z * BY * BX + xx);
  }
  if constexpr (BZ > 1) {
#pragma unroll
    for (int yx = 0; yx < BY * BX; ++yx) dct::forward<T, BZ, BY * BX>(v + yx);
  }
}

// inverse transform; only the low-frequency box [KZ][KY][KX] of the input is non-zero
template <typename T, int BZ, int BY, int BX, int KZ, int KY, int KX>
__device__ __forceinline__ void inverse_block(T* v) {
  if constexpr (BZ > 1) {
#pragma unroll
    for (int y = 0; y < KY; ++y)
#pragma unroll
      for (int xx = 0; xx < KX; ++xx) dct::inverse<T, BZ, BY * BX, KZ>(v + y * BX + xx);
  }
  if constexpr (BY > 1) {
#pragma unroll
    for (int z = 0; z < BZ; ++z)
#pragma unroll
      for (int xx = 0; xx < KX; ++xx) dct::inverse<T, BY, BX, KY>(v + z * BY * BX + xx);
  }
  if constexpr (BX > 1) {
#pragma unroll
    for (int row = 0; row < BZ * BY; ++row) dct::inverse<T, BX, 1, KX>(v + row * BX);
  }
}

// =====================================================================================================
// Family "lane": one lane = one block
// =====================================================================================================
template <typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX>
__global__ __launch_bounds__(256) void k_compress_lane(FastGeom g, const XT* __restrict__ x, NT* __restrict__ N,
                                                       IT* __restrict__ F) {
  constexpr int VOL = BZ * BY * BX, ROWS = BZ * BY;
  constexpr int RV = BX * int(sizeof(XT)) / 16;       // 16-byte loads per block row
  constexpr int PER16 = Unpack<T, XT>::n;
  constexpr int KEPT = KZ * KY * KX;
  constexpr int KW = KEPT * int(sizeof(IT)) / 4;      // dwords of F per block
  static_assert(BX * sizeof(XT) % 16 == 0 && (KEPT * sizeof(IT)) % 16 == 0, "rows and F blocks are whole 16-byte vectors");

  const int lane = threadIdx.x & 63;
  const int64_t wave = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (wave >= g.n_tiles) return;
  const int64_t tx = wave % g.tiles_x;
  const int64_t rest = wave / g.tiles_x;
  const int64_t by = rest % g.gy, bz = rest / g.gy;
  const int64_t bx = tx * 64 + lane;
  const bool active = bx < g.gx;
  const int64_t bxc = active ? bx : g.gx - 1;   // lanes past the end re-read the last block and store nothing

  uint4 raw[ROWS * RV];
#pragma unroll
  for (int z = 0; z < BZ; ++z)
#pragma unroll
    for (int y = 0; y < BY; ++y) {
      const int64_t zz = bz * BZ + z, yy = by * BY + y;
      if (zz < g.Z && yy < g.Y) {   // uniform over the wave
        const uint4* p = reinterpret_cast<const uint4*>(x + (zz * g.Y + yy) * g.X + bxc * BX);
#pragma unroll
        for (int k = 0; k < RV; ++k) raw[(z * BY + y) * RV + k] = p[k];
      } else {
#pragma unroll
        for (int k = 0; k < RV; ++k) raw[(z * BY + y) * RV + k] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
  T v[VOL];
#pragma unroll
  for (int i = 0; i < ROWS * RV; ++i) Unpack<T, XT>::run(raw[i], v + i * PER16);

  forward_block<T, BZ, BY, BX>(v);

  T m = T(0);
#pragma unroll
  for (int i = 0; i < VOL; ++i) m = fmax(m, abs_t(v[i]));
  const T inv = m > T(0) ? T(g.r) / m : T(0);

  uint32_t w[KW];
  constexpr int PER = IdxPack<IT>::per;
#pragma unroll
  for (int kw = 0; kw < KW; ++kw) {
    int q[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = kw * PER + e;                         // position in F
      const int kx = j % KX, ky = (j / KX) % KY, kz = j / (KX * KY);
      q[e] = int(rint(v[(kz * BY + ky) * BX + kx] * inv));
    }
    w[kw] = IdxPack<IT>::pack(q);
  }
  if (active) {
    const int64_t block = (bz * g.gy + by) * g.gx + bx;
    N[block] = NT(m);
    uint4* dst = reinterpret_cast<uint4*>(F + block * KEPT);
#pragma unroll
    for (int k = 0; k < KW / 4; ++k) dst[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
  }
}

template <typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX>
__global__ __launch_bounds__(256) void k_decompress_lane(FastGeom g, const NT* __restrict__ N, const IT* __restrict__ F,
                                                         XT* __restrict__ y) {
  constexpr int VOL = BZ * BY * BX, ROWS = BZ * BY;
  constexpr int RV = BX * int(sizeof(XT)) / 16;
  constexpr int PER16 = Unpack<T, XT>::n;
  constexpr int KEPT = KZ * KY * KX;
  constexpr int KW = KEPT * int(sizeof(IT)) / 4;
  constexpr int PER = IdxPack<IT>::per;

  const int lane = threadIdx.x & 63;
  const int64_t wave = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (wave >= g.n_tiles) return;
  const int64_t tx = wave % g.tiles_x;
  const int64_t rest = wave / g.tiles_x;
  const int64_t by = rest % g.gy, bz = rest / g.gy;
  const int64_t bx = tx * 64 + lane;
  if (bx >= g.gx) return;
  const int64_t block = (bz * g.gy + by) * g.gx + bx;

  uint32_t w[KW];
  const uint4* src = reinterpret_cast<const uint4*>(F + block * KEPT);
#pragma unroll
  for (int k = 0; k < KW / 4; ++k) {
    const uint4 u = src[k];
    w[4 * k] = u.x; w[4 * k + 1] = u.y; w[4 * k + 2] = u.z; w[4 * k + 3] = u.w;
  }
  const T scale = T(N[block]) / T(g.r);          // Algorithm 3: N F / r, the division hoisted per block

  T v[VOL];
#pragma unroll
  for (int i = 0; i < VOL; ++i) v[i] = T(0);
#pragma unroll
  for (int j = 0; j < KEPT; ++j) {
    const int kx = j % KX, ky = (j / KX) % KY, kz = j / (KX * KY);
    v[(kz * BY + ky) * BX + kx] = scale * T(IdxPack<IT>::get(w[j / PER], j % PER));
  }

  inverse_block<T, BZ, BY, BX, KZ, KY, KX>(v);

#pragma unroll
  for (int z = 0; z < BZ; ++z)
#pragma unroll
    for (int yy0 = 0; yy0 < BY; ++yy0) {
      const int64_t zz = bz * BZ + z, yy = by * BY + yy0;
      if (zz < g.Z && yy < g.Y) {
        uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + bx * BX);
#pragma unroll
        for (int k = 0; k < RV; ++k) p[k] = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + k) * PER16);
      }
    }
}

// ---- host side --------------------------------------------------------------------------------------
struct Folded {
  bool ok;
  int bz, by, bx;     // block extents
  int kz, ky, kx;     // kept box (== block extents when nothing is pruned), 0 when the mask is not a box
  FastGeom g;
};

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
  if (g.X % blk[2] != 0) return f;
  f.ok = true;
  return f;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename XT>
constexpr int xtype_code();
template <> constexpr int xtype_code<float>() { return PBZ_F32; }
template <> constexpr int xtype_code<double>() { return PBZ_F64; }
template <> constexpr int xtype_code<bf16_t>() { return PBZ_BF16; }
template <typename IT>
constexpr int itype_code();
template <> constexpr int itype_code<int8_t>() { return PBZ_I8; }
template <> constexpr int itype_code<int16_t>() { return PBZ_I16; }

// One table row per instantiation.
template <typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX>
struct LaneKernel {
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->compute_f64 == (sizeof(T) == 8) && xtype == xtype_code<XT>() && int(c->itype) == itype_code<IT>() &&
           int(c->ftype) == xtype_code<NT>() && f.bz == BZ && f.by == BY && f.bx == BX && f.kz == KZ && f.ky == KY &&
           f.kx == KX && (f.g.X * sizeof(XT)) % 16 == 0;
  }
  static void prepare(FastGeom& g) {
    g.tiles_x = (g.gx + 63) / 64;
    g.n_tiles = g.gz * g.gy * g.tiles_x;
  }
  static int compress(FastGeom g, const void* x, void* N, void* F, hipStream_t s) {
    prepare(g);
    const int64_t groups = (g.n_tiles + 3) / 4;
    if (groups > 0x7fffffff) return 0;
    hipLaunchKernelGGL((k_compress_lane<T, XT, IT, NT, BZ, BY, BX, KZ, KY, KX>), dim3(unsigned(groups)), dim3(256), 0, s,
                       g, static_cast<const XT*>(x), static_cast<NT*>(N), static_cast<IT*>(F));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    prepare(g);
    const int64_t groups = (g.n_tiles + 3) / 4;
    if (groups > 0x7fffffff) return 0;
    hipLaunchKernelGGL((k_decompress_lane<T, XT, IT, NT, BZ, BY, BX, KZ, KY, KX>), dim3(unsigned(groups)), dim3(256), 0,
                       s, g, static_cast<const NT*>(N), static_cast<const IT*>(F), static_cast<XT*>(y));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

// 2-D 8x8, FP32 arrays: int8 (FP32 arithmetic), int16 (FP64 arithmetic) with all 64 or the 4x4 low-frequency box kept
using Lane_f32_8x8_i8 = LaneKernel<float, float, int8_t, float, 1, 8, 8, 1, 8, 8>;
using Lane_f32_8x8_i16_box4 = LaneKernel<double, float, int16_t, float, 1, 8, 8, 1, 4, 4>;
using Lane_f32_8x8_i16 = LaneKernel<double, float, int16_t, float, 1, 8, 8, 1, 8, 8>;
// 3-D 4x4x4, FP64 arrays, int16
using Lane_f64_4x4x4_i16 = LaneKernel<double, double, int16_t, double, 4, 4, 4, 4, 4, 4>;

#define PBZ_FOR_EACH_LANE_KERNEL(X)                        \
  X(Lane_f32_8x8_i8, "lane_f32_8x8_i8")                    \
  X(Lane_f32_8x8_i16_box4, "lane_f32_8x8_i16_box4x4")      \
  X(Lane_f32_8x8_i16, "lane_f32_8x8_i16")                  \
  X(Lane_f64_4x4x4_i16, "lane_f64_4x4x4_i16")

}  // namespace

int try_compress_fast(const pbz_codec* c, const Geom& geo, const void* x, int xtype, void* N, void* F, hipStream_t s,
                      bool dry_run, const char** name) {
  if (!aligned16(x) || !aligned16(F)) return 0;
  const Folded f = fold(c, geo);
  if (!f.ok) return 0;
#define X(K, NAME)                                \
  if (K::matches(c, f, xtype)) {                  \
    *name = NAME;                                 \
    return dry_run ? 1 : K::compress(f.g, x, N, F, s); \
  }
  PBZ_FOR_EACH_LANE_KERNEL(X)
#undef X
  return 0;
}

int try_decompress_fast(const pbz_codec* c, const Geom& geo, const void* N, const void* F, void* y, int ytype,
                        hipStream_t s, bool dry_run, const char** name) {
  if (!aligned16(y) || !aligned16(F)) return 0;
  const Folded f = fold(c, geo);
  if (!f.ok) return 0;
#define X(K, NAME)                                  \
  if (K::matches(c, f, ytype)) {                    \
    *name = NAME;                                   \
    return dry_run ? 1 : K::decompress(f.g, N, F, y, s); \
  }
  PBZ_FOR_EACH_LANE_KERNEL(X)
#undef X
  return 0;
}

}  // namespace pbz
