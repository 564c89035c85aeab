// Specialised codec kernels, family "cube16" (see pbz_fast.hip for the overview).
#include "pbz_fast_common.h"

namespace pbz {
namespace fast {
namespace {

// =====================================================================================================
// Family "cube16": 16 x 16 x 16 blocks, nothing pruned.  FP32 arrays with int16 indices in FP64 arithmetic (the
// setting of the paper's fission-density experiment, Sec. V), with int32 likewise, or with int8 in FP32
// arithmetic; FP64 arrays with int8 to int32 in FP64 arithmetic (a lane's four columns are then two 16-byte pieces)
// =====================================================================================================
// A workgroup of two waves owns two blocks that are neighbours along x; wave w ends up with block w (4096 values,
// 64 per lane).  The values pass through three layouts, one per transformed dimension, with an LDS exchange
// between them:
//   A  wave w, lane = (zl, blk, q)  holds rows y = 0..15 of the four columns x = 4q..4q+3 of plane z = 8 w + zl of
//                                   block blk                                                 -> transform along y
//   C  wave = block, lane = (ky, q) holds planes z = 0..15 of the same four columns at coefficient row ky
//                                                                                             -> transform along z
//   B  wave = block, lane = (ky, zh) holds the whole rows x = 0..15 of planes kz = 4 zh .. 4 zh + 3
//                                                                                             -> transform along x
// Layout A is how the array is read and written: eight consecutive lanes cover the 128 contiguous bytes that the
// two blocks have in one array row, so that every memory line is touched by one instruction of one wave (with
// one block per wave and 64-byte pieces, two waves shared every line and the counters showed 1.46 bytes fetched
// per byte of input and 1.23 written per byte of output).  The exchange between A and C therefore crosses the two
// waves (workgroup barriers); the one between C and B is private to a wave.  Layout B is how F is written
// (whole rows of indices, consecutive in y).  An exchange moves 16 bytes per slot, i.e. four FP32 or two FP64
// values of a lane's column group, so FP64 takes two rounds per exchange through the same 16 KiB per block.  A
// 16-byte LDS access is served eight consecutive lanes at a time, and those eight must fall into different slots
// modulo 8; one side of either exchange is linear in the lane, the other side's slot index is swizzled so that
// it meets the rule as well (shader counters: 768 conflict cycles per wave with a plain transposed index, none
// with the swizzles).
constexpr int kCubeRow = 64;                       // uint4 slots per LDS row
constexpr int kCubeSlots = 16 * kCubeRow;          // per block

// exchange A <-> C: element (row y, plane z, column group q) of block blk, in the workgroup's LDS
__device__ __forceinline__ int cube_slot_zy(int blk, int y, int z, int q) {
  return blk * kCubeSlots + y * kCubeRow + ((z * 4 + q) ^ (((y & 1) ^ blk) << 2));
}
// exchange C <-> B: element (plane kz, column group q, row y), in the block's own LDS
__device__ __forceinline__ int cube_slot_zx(int kz, int q, int y) { return kz * kCubeRow + q * 16 + ((y + 2 * q) & 15); }

// Which pair of blocks does this workgroup own?  Uniform over the workgroup (both waves stay or leave together).
__device__ __forceinline__ bool decode_pair(const FastGeom& g, int64_t& pair_x, int64_t& by, int64_t& bz) {
  const uint32_t t = blockIdx.x;
  const uint32_t slab = blockIdx.y + blockIdx.z * gridDim.y;
  if (t >= g.tiles_yx || slab >= g.gz) return false;
  const uint32_t row = t / g.tiles_x;
  pair_x = t - row * g.tiles_x;
  by = row;
  bz = slab;
  return true;
}

// layout A <-> layout C across the two waves of the workgroup.  In A, wave w's lane (zl, blk, q) holds value
// [y * 4 + e] of plane 8 w + zl of block blk; in C, wave w's lane (ky, q) holds value [z * 4 + e] of block w.
// kToC: from A to C; otherwise from C to A.  Both waves must call it (barriers).
template <typename T, bool kToC>
__device__ __forceinline__ void cube_exchange_zy(uint4* lds, int wave, int lane, const T* from, T* to) {
  using Slot = ExchangeSlot<T>;
  const int z = 8 * wave + (lane >> 3), blk = (lane >> 2) & 1, q = lane & 3;     // as a lane of layout A
  const int cy = lane >> 2;                                                      // as a lane of layout C
#pragma unroll
  for (int e0 = 0; e0 < 4; e0 += Slot::n) {
    if (e0) __syncthreads();                       // the previous round's reads precede this round's writes
#pragma unroll
    for (int i = 0; i < 16; ++i)
      lds[kToC ? cube_slot_zy(blk, i, z, q) : cube_slot_zy(wave, cy, i, q)] = Slot::pack(from + i * 4 + e0);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i)
      Slot::unpack(lds[kToC ? cube_slot_zy(wave, cy, i, q) : cube_slot_zy(blk, i, z, q)], to + i * 4 + e0);
  }
}

// layout C <-> layout B.  In C the lane is (ky, q) and value [kz * 4 + e] is column 4 q + e of plane kz; in B the
// lane is (ky, zh) = (lane & 15, lane >> 4) and value [zl * 16 + x] is column x of plane 4 zh + zl.
template <typename T, bool kToB>
__device__ __forceinline__ void cube_exchange_zx(uint4* st, int lane, const T* from, T* to) {
  using Slot = ExchangeSlot<T>;
  const int cy = lane >> 2, q = lane & 3;          // as a lane of layout C
  const int ky = lane & 15, zh = lane >> 4;        // as a lane of layout B
#pragma unroll
  for (int e0 = 0; e0 < 4; e0 += Slot::n) {
    if (e0) wave_lds_sync();
    if constexpr (kToB) {
#pragma unroll
      for (int kz = 0; kz < 16; ++kz) st[cube_slot_zx(kz, q, cy)] = Slot::pack(from + kz * 4 + e0);
    } else {
#pragma unroll
      for (int zl = 0; zl < 4; ++zl)
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
          st[cube_slot_zx(4 * zh + zl, qq, ky)] = Slot::pack(from + zl * 16 + qq * 4 + e0);
    }
    wave_lds_sync();
    if constexpr (kToB) {
#pragma unroll
      for (int zl = 0; zl < 4; ++zl)
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
          Slot::unpack(st[cube_slot_zx(4 * zh + zl, qq, ky)], to + zl * 16 + qq * 4 + e0);
    } else {
#pragma unroll
      for (int kz = 0; kz < 16; ++kz) Slot::unpack(st[cube_slot_zx(kz, q, cy)], to + kz * 4 + e0);
    }
  }
}

template <int TF, typename T, typename IT, typename XT, bool kRagged, bool kStats, bool kTailX>
__global__ __launch_bounds__(128) void k_compress_cube16(FastGeom g, const XT* __restrict__ x, void* __restrict__ N,
                                                         IT* __restrict__ F, double* __restrict__ tile_sums) {
  using Q4 = Quad4<XT>;
  constexpr int PER = IdxPack<IT>::per;            // indices per dword
  constexpr int ROWW = 16 / PER;                   // dwords per row of 16 indices
  __shared__ uint4 lds[2 * kCubeSlots];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int64_t pair_x, by, bz;
  if (!decode_pair(g, pair_x, by, bz)) return;
  // The pair's second block may lie past the end of the row: its lanes then load the first block again, and the
  // wave that would own it works on those values and stores nothing (it still takes part in the barriers).
  const int64_t bx = pair_x * 2 + wave;            // this wave's block
  const bool block_in = bx < g.gx;

  T a[64], c[64];
  {  // layout A: plane z = 8 wave + (lane >> 3) of block (lane >> 2) & 1, columns 4 q .. 4 q + 3, all 16 rows
    const int pz = 8 * wave + (lane >> 3), blk = (lane >> 2) & 1, q = lane & 3;
    const int64_t bxl = pair_x * 2 + blk < g.gx ? pair_x * 2 + blk : g.gx - 1;
    int64_t zz = bz * 16 + pz;
    uint32_t keep_z = 0xffffffffu;
    if constexpr (kRagged) {
      keep_z = zz < g.Z ? 0xffffffffu : 0u;        // planes past the end: load a valid one, zero it below
      zz = zz < g.Z ? zz : g.Z - 1;
    }
    typename Q4::raw_t raw[16];
    const int64_t x_first = bxl * 16 + q * 4;
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      int64_t yy = by * 16 + yy0;
      if constexpr (kRagged) yy = yy < g.Y ? yy : g.Y - 1;
      int64_t x0 = x_first;
      if constexpr (kTailX) x0 = x0 + 4 <= g.X ? x0 : g.X - 4;
      raw[yy0] = Q4::template load<kTailX>(x + (zz * g.Y + yy) * g.X + x0);
    }
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      if constexpr (kRagged) Q4::keep(raw[yy0], by * 16 + yy0 < g.Y ? keep_z : 0u);
      quad4_unpack<T, XT>(raw[yy0], a + yy0 * 4);
    }
    if constexpr (kTailX) {
      if (x_first + 4 > g.X) {           // a piece of the row's last, partial block: element by element, zeros beyond
#pragma unroll
        for (int yy0 = 0; yy0 < 16; ++yy0) {
          const int64_t yy = by * 16 + yy0;
          const bool row_in = yy < g.Y && keep_z != 0u;
          const XT* row = x + (zz * g.Y + (yy < g.Y ? yy : g.Y - 1)) * g.X;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int64_t xi = x_first + e;
            const XT val = row[xi < g.X ? xi : g.X - 1];
            a[yy0 * 4 + e] = row_in && xi < g.X ? T(val) : T(0);
          }
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) tf_forward<TF, T, 16, 4>(a + e);
  }
  cube_exchange_zy<T, true>(lds, wave, lane, a, c);
#pragma unroll
  for (int e = 0; e < 4; ++e) tf_forward<TF, T, 16, 4>(c + e);
  uint4* st = lds + wave * kCubeSlots;             // from here on a wave stays inside its block's half
  wave_lds_sync();
  cube_exchange_zx<T, true>(st, lane, c, a);
#pragma unroll
  for (int zl = 0; zl < 4; ++zl) tf_forward<TF, T, 16, 1>(a + zl * 16);
  if (!block_in) return;

  // layout B: lane = (ky, zh) holds rows (kz = 4 zh + zl, ky) of the coefficients
  T m = T(0);
#pragma unroll
  for (int i = 0; i < 64; ++i) m = fmax(m, fabs(a[i]));
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) m = fmax(m, __shfl_xor(m, off, 64));
  const T inv = m > T(0) ? T(g.r) / m : T(0);
  const int ky = lane & 15, zh = lane >> 4;
  const int64_t block = (bz * g.gy + by) * g.gx + bx;
  uint32_t w[4 * ROWW];
#pragma unroll
  for (int zl = 0; zl < 4; ++zl)
#pragma unroll
    for (int k = 0; k < ROWW; ++k) {
      uint32_t q[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e) q[e] = bin_bits(a[zl * 16 + k * PER + e], inv);
      w[zl * ROWW + k] = IdxPack<IT>::pack(q);
    }
  uint4* dst = reinterpret_cast<uint4*>(F + block * 4096);
#pragma unroll
  for (int zl = 0; zl < 4; ++zl)
#pragma unroll
    for (int k = 0; k < ROWW / 4; ++k)
      dst[(((4 * zh + zl) * 16 + ky) * ROWW) / 4 + k] =
          make_uint4(w[zl * ROWW + 4 * k], w[zl * ROWW + 4 * k + 1], w[zl * ROWW + 4 * k + 2], w[zl * ROWW + 4 * k + 3]);
  if (lane == 0) store_float(N, g.ntype, block, m);
  if constexpr (kStats) {
    const double n = stored_N(m, g.ntype);
    const double f0 = lane == 0 ? double(IdxPack<IT>::get(w[0], 0)) : 0.0;
    const double rest = sum_of_squares_rest<IT, 4 * ROWW>(w, lane == 0) * (n * n);
    const double K = tile_pilot(n * f0);           // one record per block: its first coefficient is the pilot value
    FastGeom per_block = g;                        // records are indexed by block, not by pair
    per_block.tiles_x = uint32_t(g.gx);
    per_block.tiles_yx = uint32_t(g.gx * g.gy);
    emit_tile_sums(tile_sums, per_block, bx, by, bz, rest, 0.0, 0.0, lane == 0 ? 1.0 : 0.0, K);
  }
}

template <int TF, typename T, typename IT, typename XT, bool kTailX>
__global__ __launch_bounds__(128) void k_decompress_cube16(FastGeom g, const void* __restrict__ N,
                                                           const IT* __restrict__ F, XT* __restrict__ y) {
  using Q4 = Quad4<XT>;
  constexpr int PER = IdxPack<IT>::per;
  constexpr int ROWW = 16 / PER;
  __shared__ uint4 lds[2 * kCubeSlots];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int64_t pair_x, by, bz;
  if (!decode_pair(g, pair_x, by, bz)) return;
  // a second block past the end of the row: that wave decodes the first block again, and nothing of it is stored
  const int64_t bx = pair_x * 2 + wave < g.gx ? pair_x * 2 + wave : g.gx - 1;
  const int64_t block = (bz * g.gy + by) * g.gx + bx;
  uint4* st = lds + wave * kCubeSlots;

  T a[64], c[64];
  {  // layout B: rows (kz = 4 zh + zl, ky) of the indices
    const int ky = lane & 15, zh = lane >> 4;
    const uint4* src = reinterpret_cast<const uint4*>(F + block * 4096);
    uint4 f[4 * (ROWW / 4)];
#pragma unroll
    for (int zl = 0; zl < 4; ++zl)
#pragma unroll
      for (int k = 0; k < ROWW / 4; ++k) f[zl * (ROWW / 4) + k] = src[(((4 * zh + zl) * 16 + ky) * ROWW) / 4 + k];
    const T scale = load_float<T>(N, g.ntype, block) / T(g.r);        // Algorithm 3: N F / r
#pragma unroll
    for (int zl = 0; zl < 4; ++zl)
#pragma unroll
      for (int k = 0; k < ROWW / 4; ++k) {
        const uint4 u = f[zl * (ROWW / 4) + k];
        const uint32_t uw[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int e = 0; e < PER; ++e)
            a[zl * 16 + (4 * k + d) * PER + e] = scale * T(IdxPack<IT>::get(uw[d], e));
      }
#pragma unroll
    for (int zl = 0; zl < 4; ++zl) tf_inverse<TF, T, 16, 1, 16>(a + zl * 16);
  }
  cube_exchange_zx<T, false>(st, lane, a, c);
#pragma unroll
  for (int e = 0; e < 4; ++e) tf_inverse<TF, T, 16, 4, 16>(c + e);
  wave_lds_sync();
  cube_exchange_zy<T, false>(lds, wave, lane, c, a);
#pragma unroll
  for (int e = 0; e < 4; ++e) tf_inverse<TF, T, 16, 4, 16>(a + e);

  // layout A: plane z = 8 wave + (lane >> 3) of block (lane >> 2) & 1, columns 4 q .. 4 q + 3
  const int pz = 8 * wave + (lane >> 3), blk = (lane >> 2) & 1, q = lane & 3;
  const int64_t zz = bz * 16 + pz;
  const int64_t bxl = pair_x * 2 + blk;
  if (zz < g.Z && bxl < g.gx) {
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      const int64_t yy = by * 16 + yy0;
      if (yy < g.Y) {
        XT* row = y + (zz * g.Y + yy) * g.X;
        const int64_t x0 = bxl * 16 + q * 4;
        if constexpr (kTailX) {
          if (x0 + 4 <= g.X) {
            Q4::template store<true>(row + x0, quad4_pack<T, XT>(a + yy0 * 4));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (x0 + e < g.X) row[x0 + e] = XT(a[yy0 * 4 + e]);
          }
        } else {
          Q4::template store<false>(row + x0, quad4_pack<T, XT>(a + yy0 * 4));
        }
      }
    }
  }
}

template <int TF, typename T, typename IT, typename XT>
struct Cube16Kernel {
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->transform == TF && c->compute_f64 == (sizeof(T) == 8) && xtype == xtype_code<XT>() &&
           int(c->itype) == itype_code<IT>() && f.bz == 16 && f.by == 16 && f.bx == 16 && f.kz == 16 && f.ky == 16 &&
           f.kx == 16 && x_extent_ok(f, 4, int(sizeof(XT)));
  }
  // one workgroup per pair of blocks; the statistics records are per block
  static bool grid_for(FastGeom& g, dim3* grid) {
    return g.gx * g.gy < (int64_t(1) << 31) && tile_grid(g, 2, 1, grid);
  }
  static int fits(FastGeom g) {
    dim3 grid;
    return grid_for(g, &grid) ? 1 : 0;
  }
  static int64_t tiles(FastGeom g) {
    dim3 grid;
    return grid_for(g, &grid) ? g.gz * g.gy * g.gx : 0;
  }
  template <bool kRagged, bool kStats, bool kTailX>
  static void launch(const FastGeom& g, dim3 grid, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    hipLaunchKernelGGL((k_compress_cube16<TF, T, IT, XT, kRagged, kStats, kTailX>), grid, dim3(128), 0, s, g,
                       static_cast<const XT*>(x), N, static_cast<IT*>(F), tile_sums);
  }
  static int compress(FastGeom g, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    dim3 grid;
    if (!grid_for(g, &grid)) return 0;
    const bool ragged = g.Y % 16 || g.Z % 16;
    if (g.X % 16) tile_sums ? launch<true, true, true>(g, grid, x, N, F, tile_sums, s) : launch<true, false, true>(g, grid, x, N, F, nullptr, s);
    else if (tile_sums) ragged ? launch<true, true, false>(g, grid, x, N, F, tile_sums, s) : launch<false, true, false>(g, grid, x, N, F, tile_sums, s);
    else ragged ? launch<true, false, false>(g, grid, x, N, F, nullptr, s) : launch<false, false, false>(g, grid, x, N, F, nullptr, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    dim3 grid;
    if (!grid_for(g, &grid)) return 0;
    if (g.X % 16)
      hipLaunchKernelGGL((k_decompress_cube16<TF, T, IT, XT, true>), grid, dim3(128), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    else
      hipLaunchKernelGGL((k_decompress_cube16<TF, T, IT, XT, false>), grid, dim3(128), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

#define PBZ_ROWS(X, TF, SUFFIX) \
  X(Cube16Kernel<TF COMMA double COMMA int16_t COMMA float>, "cube16_f32_16x16x16_i16" SUFFIX) \
  X(Cube16Kernel<TF COMMA float COMMA int8_t COMMA float>, "cube16_f32_16x16x16_i8" SUFFIX) \
  X(Cube16Kernel<TF COMMA double COMMA int32_t COMMA float>, "cube16_f32_16x16x16_i32" SUFFIX) \
  X(Cube16Kernel<TF COMMA double COMMA int8_t COMMA double>, "cube16_f64_16x16x16_i8" SUFFIX) \
  X(Cube16Kernel<TF COMMA double COMMA int16_t COMMA double>, "cube16_f64_16x16x16_i16" SUFFIX) \
  X(Cube16Kernel<TF COMMA double COMMA int32_t COMMA double>, "cube16_f64_16x16x16_i32" SUFFIX) \
  X(Cube16Kernel<TF COMMA float COMMA int8_t COMMA double>, "cube16_f64_w32_16x16x16_i8" SUFFIX)

}  // namespace

PBZ_DEFINE_FAST_FAMILY(cube16, PBZ_ROWS)

}  // namespace fast
}  // namespace pbz
