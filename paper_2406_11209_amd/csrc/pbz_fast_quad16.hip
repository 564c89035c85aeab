// Specialised codec kernels, family "quad16" (see pbz_fast.hip for the overview).
#include "pbz_fast_common.h"

namespace pbz {
namespace fast {
namespace {

// =====================================================================================================
// Family "quad16": BZ x 16 x 16 blocks with BZ = 1 (2-D) or 4, nothing pruned.  FP32 / FP16 / bfloat16 arrays with int8
// indices in FP32 arithmetic; FP32 arrays with int16 / int32 and FP64 arrays with int8 to int32 in FP64 arithmetic
// (T, IT, XT), whose exchange takes two rounds of two values per slot
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

template <int TF, typename T, typename IT, typename XT, int BZ, bool kRagged, bool kStats, bool kTailX = false>
__global__ __launch_bounds__(128) void k_compress_quad16(FastGeom g, const XT* __restrict__ x, void* __restrict__ N,
                                                         IT* __restrict__ F, double* __restrict__ tile_sums) {
  using Q4 = Quad4<XT>;
  using Slot = ExchangeSlot<T>;
  constexpr int PER = IdxPack<IT>::per;            // indices per dword
  constexpr int ROWW = 16 / PER;                   // dwords per row of 16 indices
  static_assert(BZ == 1 || BZ == 4, "one plane or four");
  using Map = QuadMap<BZ>;
  constexpr int BPW = Map::kBlocksPerWave;
  __shared__ uint4 lds[2][16 * kQuadRow];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<2>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];

  T v[64];
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
      quad4_unpack<T, XT>(raw[yy0], v + yy0 * 4);
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
            const T val = Elem<T, XT>::load(row + (xi < g.X ? xi : g.X - 1));
            v[yy0 * 4 + e] = row_in && xi < g.X ? val : T(0);
          }
        }
      }
    }
#pragma unroll
    for (int xl = 0; xl < 4; ++xl) tf_forward<TF, T, 16, 4>(v + xl);
  }
  // exchange: lane (p, q) -> lane (row yrow, s), which takes four whole rows, row yrow of planes 4 j + s
  const int yrow = lane & 15, bsub = lane >> 4;
  T u[64];
#pragma unroll
  for (int e0 = 0; e0 < 4; e0 += Slot::n) {
    if (e0) wave_lds_sync();                       // the previous round's reads precede this round's writes
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) st[yy0 * kQuadRow + lane] = Slot::pack(v + yy0 * 4 + e0);
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int xq = 0; xq < 4; ++xq)
        Slot::unpack(st[yrow * kQuadRow + (4 * j + bsub) * 4 + xq], u + j * 16 + xq * 4 + e0);
  }
  // phase B: transform along x (and z)
#pragma unroll
  for (int j = 0; j < 4; ++j) tf_forward<TF, T, 16, 1>(u + j * 16);
  if constexpr (BZ == 4) {
#pragma unroll
    for (int i = 0; i < 16; ++i) tf_forward<TF, T, 4, 16>(u + i);
  }

  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * BPW;
  double rest = 0.0;                                   // statistics: N^2 sum F^2 without the first coefficients,
  double firsts[4] = {0.0, 0.0, 0.0, 0.0};             // the first coefficients N F_0 this lane holds (yrow == 0),
  bool has_first[4] = {false, false, false, false};    // of blocks inside the array
  T m4 = T(0);                                         // BZ = 4: the block's maximum over its four planes
  if constexpr (BZ == 4) {
#pragma unroll
    for (int i = 0; i < 64; ++i) m4 = fmax(m4, fabs(u[i]));
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) m4 = fmax(m4, __shfl_xor(m4, off, 64));
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    T m = m4;
    if constexpr (BZ == 1) {
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmax(m, fabs(u[j * 16 + i]));
#pragma unroll
      for (int off = 1; off < 16; off <<= 1) m = fmax(m, __shfl_xor(m, off, 64));   // the 16 rows of the block
    }
    const T inv = m > T(0) ? T(g.r) / m : T(0);
    uint32_t w[ROWW];
#pragma unroll
    for (int k = 0; k < ROWW; ++k) {
      uint32_t qs[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e) qs[e] = bin_bits(u[j * 16 + k * PER + e], inv);
      w[k] = IdxPack<IT>::pack(qs);
    }
    const int blk = Map::block_of(4 * j + bsub);
    if (tx * BPW + blk < g.gx) {
      // the wave's pieces of F are linear in the lane: 16 consecutive pieces per (plane, block)
      const int piece = BZ == 1 ? yrow : j * 16 + yrow;       // row of 16 indices within the block
      uint4* dst = reinterpret_cast<uint4*>(F + (block0 + blk) * (BZ * 256)) + piece * (ROWW / 4);
#pragma unroll
      for (int k = 0; k < ROWW / 4; ++k) dst[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
      const bool first = yrow == 0 && (BZ == 1 || j == 0);
      if (first) store_float(N, g.ntype, block0 + blk, m);
      if constexpr (kStats) {
        const double n = stored_N(m, g.ntype);
        const double f0 = first ? double(IdxPack<IT>::get(w[0], 0)) : 0.0;
        rest += sum_of_squares_rest<IT, ROWW>(w, first) * (n * n);
        firsts[j] = n * f0;
        has_first[j] = first;
      }
    }
  }
  if constexpr (kStats) {
    const double K = tile_pilot(firsts[0]);            // lane 0, j = 0: the tile's first block, always inside the array
    double sq = 0.0, d = 0.0, count = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double dj = has_first[j] ? firsts[j] - K : 0.0;
      sq += dj * dj;
      d += dj;
      count += has_first[j] ? 1.0 : 0.0;
    }
    emit_tile_sums(tile_sums, g, tx, by, bz, rest, sq, d, count, K);
  }
}

template <int TF, typename T, typename IT, typename XT, int BZ, bool kTailX = false>
__global__ __launch_bounds__(128) void k_decompress_quad16(FastGeom g, const void* __restrict__ N,
                                                           const IT* __restrict__ F, XT* __restrict__ y) {
  using Q4 = Quad4<XT>;
  using Map = QuadMap<BZ>;
  using Slot = ExchangeSlot<T>;
  constexpr int BPW = Map::kBlocksPerWave;
  constexpr int PER = IdxPack<IT>::per;
  constexpr int ROWW = 16 / PER;
  __shared__ uint4 lds[2][16 * kQuadRow];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<2>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * BPW;
  const int yrow = lane & 15, bsub = lane >> 4;
  T u[64];
  {
    int64_t blocks[4];
    uint4 fs[4][ROWW / 4];
    T ns[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t blk = Map::block_of(4 * j + bsub);
      if (tx * BPW + blk >= g.gx) blk = g.gx - 1 - tx * BPW;   // past the end: decode the last block again, stored nowhere
      blocks[j] = block0 + blk;
      const int piece = BZ == 1 ? yrow : j * 16 + yrow;
      const uint4* src = reinterpret_cast<const uint4*>(F + blocks[j] * (BZ * 256)) + piece * (ROWW / 4);
#pragma unroll
      for (int k = 0; k < ROWW / 4; ++k) fs[j][k] = src[k];
    }
    load_N_many<4, T>(N, g.ntype, blocks, ns);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const T scale = ns[j] / T(g.r);
#pragma unroll
      for (int k = 0; k < ROWW / 4; ++k) {
        const uint4 f = fs[j][k];
        const uint32_t w[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int e = 0; e < PER; ++e)
            u[j * 16 + (4 * k + d) * PER + e] = scale * T(IdxPack<IT>::get(w[d], e));
      }
    }
    if constexpr (BZ == 4) {
#pragma unroll
      for (int i = 0; i < 16; ++i) tf_inverse<TF, T, 4, 16, 4>(u + i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) tf_inverse<TF, T, 16, 1, 16>(u + j * 16);
  }
  // exchange: lane (row yrow, s) -> lane (plane p, column quarter q)
  T v[64];
#pragma unroll
  for (int e0 = 0; e0 < 4; e0 += Slot::n) {
    if (e0) wave_lds_sync();
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int xq = 0; xq < 4; ++xq)
        st[yrow * kQuadRow + (4 * j + bsub) * 4 + xq] = Slot::pack(u + j * 16 + xq * 4 + e0);
    wave_lds_sync();
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) Slot::unpack(st[yy0 * kQuadRow + lane], v + yy0 * 4 + e0);
  }
  const int p = lane >> 2, q = lane & 3;
  const int64_t bx = tx * BPW + Map::block_of(p);
  const int64_t zz = bz * BZ + Map::plane_of(p);
#pragma unroll
  for (int xl = 0; xl < 4; ++xl) tf_inverse<TF, T, 16, 4, 16>(v + xl);
  if (bx < g.gx && zz < g.Z) {
#pragma unroll
    for (int yy0 = 0; yy0 < 16; ++yy0) {
      const int64_t yy = by * 16 + yy0;
      if (yy < g.Y) {
        if constexpr (kTailX) {
          XT* row = y + (zz * g.Y + yy) * g.X;
          const int64_t x0 = bx * 16 + q * 4;
          if (x0 + 4 <= g.X) {
            Q4::template store<true>(row + x0, quad4_pack<T, XT>(v + yy0 * 4));
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (x0 + e < g.X) Elem<T, XT>::store(row + x0 + e, v[yy0 * 4 + e]);
          }
        } else {
          Q4::template store<false>(y + (zz * g.Y + yy) * g.X + bx * 16 + q * 4, quad4_pack<T, XT>(v + yy0 * 4));
        }
      }
    }
  }
}


// 16x16 (2-D) and 4x16x16 blocks, nothing pruned; T = float with int8 (FP32 / bfloat16 / FP16 arrays), double otherwise
template <int TF, typename T, typename IT, typename XT, int BZ>
struct Quad16Kernel {
  static constexpr int kBlocksPerWave = BZ == 1 ? 16 : 4;
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    return f.ok && c->transform == TF && c->compute_f64 == (sizeof(T) == 8) && xtype == xtype_code<XT>() &&
           int(c->itype) == itype_code<IT>() &&
           (sizeof(T) == 8 || c->ftype != PBZ_F64) && f.bz == BZ && f.by == 16 && f.bx == 16 && f.kz == BZ && f.ky == 16 && f.kx == 16 &&
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
    hipLaunchKernelGGL((k_compress_quad16<TF, T, IT, XT, BZ, kRagged, kStats, kTailX>), grid, dim3(128), 0, s, g,
                       static_cast<const XT*>(x), N, static_cast<IT*>(F), tile_sums);
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
      hipLaunchKernelGGL((k_decompress_quad16<TF, T, IT, XT, BZ, true>), grid, dim3(128), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    else
      hipLaunchKernelGGL((k_decompress_quad16<TF, T, IT, XT, BZ, false>), grid, dim3(128), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

#define PBZ_ROWS(X, TF, SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA float COMMA 1>, "quad16_f32_16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA float COMMA 4>, "quad16_f32_4x16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA f16_t COMMA 1>, "quad16_f16_16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA bf16_t COMMA 1>, "quad16_bf16_16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA f16_t COMMA 4>, "quad16_f16_4x16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int16_t COMMA float COMMA 1>, "quad16_f32_16x16_i16" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int16_t COMMA float COMMA 4>, "quad16_f32_4x16x16_i16" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int32_t COMMA float COMMA 1>, "quad16_f32_16x16_i32" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int32_t COMMA float COMMA 4>, "quad16_f32_4x16x16_i32" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int8_t COMMA double COMMA 1>, "quad16_f64_16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int16_t COMMA double COMMA 1>, "quad16_f64_16x16_i16" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int32_t COMMA double COMMA 1>, "quad16_f64_16x16_i32" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int16_t COMMA double COMMA 4>, "quad16_f64_4x16x16_i16" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int8_t COMMA double COMMA 4>, "quad16_f64_4x16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA double COMMA int32_t COMMA double COMMA 4>, "quad16_f64_4x16x16_i32" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA double COMMA 1>, "quad16_f64_w32_16x16_i8" SUFFIX) \
  X(Quad16Kernel<TF COMMA float COMMA int8_t COMMA double COMMA 4>, "quad16_f64_w32_4x16x16_i8" SUFFIX)

}  // namespace

PBZ_DEFINE_FAST_FAMILY(quad16, PBZ_ROWS)

}  // namespace fast
}  // namespace pbz
