// Specialised codec kernels, family "lane" (see pbz_fast.hip for the overview).
#include <type_traits>

#include "pbz_fast_common.h"

namespace pbz {
namespace fast {
namespace {

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
    const double f0 = double(IdxPack<IT>::get(w[0], 0));
    const double K = tile_pilot(n * f0);                      // lane 0 always holds a block of the array
    const double d = active ? n * f0 - K : 0.0;
    emit_tile_sums(tile_sums, g, tx, by, bz, sum_of_squares_rest<IT, KW>(w, true) * (n * n), d * d, d,
                   active ? 1.0 : 0.0, K);
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

// Two workgroups per compute unit, i.e. two waves per SIMD, are asked for explicitly: the FP64-array 4x4x4 variants
// otherwise come out at 256 vector registers plus a few accumulation registers, which is one wave per SIMD (the
// register file holds 512 per lane).  Held to 256 they run 6 % faster (workload 4 decompress: 0.264 -> 0.248 ms on
// random data); three waves (168 registers, 95 values spilled) take 0.44 ms, and a scheduling fence after each
// row's stores changes neither the register count nor the time.  With the choice between the whole-wave stores
// and those of a partly filled wave made once, outside the loops over the rows, the bound costs no spill (with
// the choice inside the loops: nine values per lane, 4.5 % more bytes written than the array has).
template <int TF, typename T, typename XT, typename IT, typename NT, int BZ, int BY, int BX, int KZ, int KY, int KX,
          bool kRagged, bool kTailX = false>
__global__ __launch_bounds__(256, 2) void k_decompress_lane(FastGeom g, const void* __restrict__ N, const IT* __restrict__ F,
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

  // whole waves and partly filled ones store differently; the choice is made once, outside the loops over the rows
  auto store_rows = [&](auto whole_tag) {
    constexpr bool kWhole = decltype(whole_tag)::value;
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
          } else if constexpr (RV == 2 && kWhole) {
            // A block row is two 16-byte pieces, so a plain store instruction would write every other piece of a
            // 2 KiB span.  The two half-waves trade pieces instead (lanes 32-63 hand the first piece of their row
            // to lanes 0-31 and take those lanes' second piece): the first store then writes the rows of blocks
            // 0-31 as one contiguous KiB, the second those of blocks 32-63 (workload 4: 0.251 -> 0.240 ms).  Whole
            // KiB per instruction is also what the non-temporal hint needs (back-to-back repeats of workload 4:
            // 0.248 -> 0.238 ms; inside the benchmark step the kernel now waits for its own writes and still
            // shows 0.249 ms, the negate after it 0.090 instead of 0.111 ms).
            // The compiler hoists every row's trade above the first store
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
            store16_stream(p, h0);
            store16_stream(p + 64, h1);
          } else if constexpr (RV == 4 && kWhole) {
            // four pieces per block row: after the quarter transpose store j writes the rows of blocks
            // 16j .. 16j+15 as one contiguous KiB (8192^2 FP64 in 8x8 blocks, non-temporal: 0.129 -> 0.104 ms)
            uint4 h[4];
  #pragma unroll
            for (int k = 0; k < 4; ++k) h[k] = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + k) * PER16);
            transpose_quarter_waves(h[0], h[1], h[2], h[3]);
            uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + tx * 64 * BX) + 4 * (lane & 15) + (lane >> 4);
  #pragma unroll
            for (int k = 0; k < 4; ++k) store16_stream(p + 64 * k, h[k]);
          } else {
            uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + bx * BX);
            if constexpr (RV == 1) {     // one piece per block row: the lanes' pieces are contiguous as they are
              store16_stream(p, Pack<T, XT>::run(v + (z * BY + yy0) * PER16));
            } else {
              // a partly filled wave.  Plain stores: a lane's pieces alternate with its neighbours' within a line,
              // which the L2 merges into whole lines; with the non-temporal hint these 16-byte pieces reach memory
              // singly (measured: twice as slow)
  #pragma unroll
              for (int k = 0; k < RV; ++k) p[k] = Pack<T, XT>::run(v + ((z * BY + yy0) * RV + k) * PER16);
            }
          }
        }
      }
  };
  if constexpr (kTailX || RV == 1 || (RV != 2 && RV != 4)) {
    store_rows(std::false_type{});
  } else {
    if (whole_wave) store_rows(std::true_type{});
    else store_rows(std::false_type{});
  }
}

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
  // tile_sums != nullptr: also the per-wave statistic sums (four doubles per tile)
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
// FP64 arrays with a narrower working type (N stored as FP32 or a 16-bit type): FP32 arithmetic with int8 indices,
// FP64 arithmetic with int16
template <int TF> using Lane_f64_w32_8x8_i8 = LaneKernel<TF, float, double, int8_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f64_w32_8x8_i16 = LaneKernel<TF, double, double, int16_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f64_w32_4x4x4_i8 = LaneKernel<TF, float, double, int8_t, float, 4, 4, 4, 4, 4, 4>;
template <int TF> using Lane_f64_w32_4x4x4_i16 = LaneKernel<TF, double, double, int16_t, float, 4, 4, 4, 4, 4, 4>;

// int32 indices (FP64 arithmetic whatever the array's type): a block's F is 256 bytes, 16 pieces per lane
template <int TF> using Lane_f32_8x8_i32 = LaneKernel<TF, double, float, int32_t, float, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f64_8x8_i32 = LaneKernel<TF, double, double, int32_t, double, 1, 8, 8, 1, 8, 8>;
template <int TF> using Lane_f32_4x4x4_i32 = LaneKernel<TF, double, float, int32_t, float, 4, 4, 4, 4, 4, 4>;
template <int TF> using Lane_f64_4x4x4_i32 = LaneKernel<TF, double, double, int32_t, double, 4, 4, 4, 4, 4, 4>;

#define PBZ_ROWS(X, TF, SUFFIX) \
  X(Lane_f32_8x8_i8<TF>, "lane_f32_8x8_i8" SUFFIX) \
  X(Lane_bf16_8x8_i8<TF>, "lane_bf16_8x8_i8" SUFFIX) \
  X(Lane_f16_8x8_i8<TF>, "lane_f16_8x8_i8" SUFFIX) \
  X(Lane_f32_8x8_i16_box4<TF>, "lane_f32_8x8_i16_box4x4" SUFFIX) \
  X(Lane_f32_8x8_i16<TF>, "lane_f32_8x8_i16" SUFFIX) \
  X(Lane_f64_4x4x4_i16<TF>, "lane_f64_4x4x4_i16" SUFFIX) \
  X(Lane_f64_4x4x4_i8<TF>, "lane_f64_4x4x4_i8" SUFFIX) \
  X(Lane_f32_4x4x4_i8<TF>, "lane_f32_4x4x4_i8" SUFFIX) \
  X(Lane_f32_4x4x4_i16<TF>, "lane_f32_4x4x4_i16" SUFFIX) \
  X(Lane_f64_8x8_i8<TF>, "lane_f64_8x8_i8" SUFFIX) \
  X(Lane_f64_8x8_i16<TF>, "lane_f64_8x8_i16" SUFFIX) \
  X(Lane_f64_w32_8x8_i8<TF>, "lane_f64_w32_8x8_i8" SUFFIX) \
  X(Lane_f64_w32_8x8_i16<TF>, "lane_f64_w32_8x8_i16" SUFFIX) \
  X(Lane_f64_w32_4x4x4_i8<TF>, "lane_f64_w32_4x4x4_i8" SUFFIX) \
  X(Lane_f64_w32_4x4x4_i16<TF>, "lane_f64_w32_4x4x4_i16" SUFFIX) \
  X(Lane_f32_8x8_i32<TF>, "lane_f32_8x8_i32" SUFFIX) \
  X(Lane_f64_8x8_i32<TF>, "lane_f64_8x8_i32" SUFFIX) \
  X(Lane_f32_4x4x4_i32<TF>, "lane_f32_4x4x4_i32" SUFFIX) \
  X(Lane_f64_4x4x4_i32<TF>, "lane_f64_4x4x4_i32" SUFFIX)

}  // namespace

PBZ_DEFINE_FAST_FAMILY(lane, PBZ_ROWS)

}  // namespace fast
}  // namespace pbz
