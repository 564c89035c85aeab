// Specialised codec kernels, family "oct8" (see pbz_fast.hip for the overview).
#include "pbz_fast_common.h"

namespace pbz {
namespace fast {
namespace {

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

// =====================================================================================================
// Family "oct8": 3-D 8x8x8 blocks, bfloat16, FP16 or FP32 arrays, FP32 arithmetic, int8 indices, low-frequency box kept
// =====================================================================================================
// LDS exchange, done in two rounds (left and right half of every 8-element row) so that a wave needs 8 KiB
// instead of 16 KiB and twice as many waves fit a CU (the kernel is latency-bound: halving its occupancy
// cost 40 %).  Per round block b occupies 64 sixteen-byte slots ordered [y][z].  A 16-byte LDS access is served
// eight consecutive lanes at a time, and those eight must fall into different slots modulo 8: the plane-wise
// writes come from lanes that differ in b, the row-wise reads from lanes that differ in y, so the low three bits
// of the slot are z ^ y ^ b (shader counters: 200 -> 8 bank-conflict cycles per wave against the earlier swizzle,
// which spread sixteen lanes over sixteen slots but put pairs of the eight into one).
__device__ __forceinline__ int oct_slot(int b, int yy, int z) { return b * 64 + yy * 8 + ((z ^ yy ^ b) & 7); }

constexpr int kOctWaves = 4;   // waves per workgroup: neighbouring tiles, so that a workgroup reads 512-byte row pieces

// Rows of 32-bit or 64-bit elements.  A row of a block is two (FP32) or four (FP64) 16-byte pieces, 32 or 64 bytes
// apart from the next lane's: stored as they are, an instruction would write every second or fourth piece of the
// run that the eight blocks of a plane have in a row (measured, 512 x 512 x 256 FP64: 3.0 TB/s moved).  Here the
// finished planes v (lane = (plane z, block b), 64 values of type T each) go through the wave's 8 KiB of LDS
// instead, 512 pieces per round: lane (z, b) writes pieces P = RV b + k of its rows, and on the way out 8 RV
// consecutive lanes take one row's pieces in order, so that an instruction stores two or four whole 256- or
// 512-byte rows, with the non-temporal hint (6.7 TB/s).  Slot P ^ (P / 8) keeps every eight consecutive lanes in
// distinct 16-byte slots modulo 8 in both directions.  Whole rows only (X a multiple of 8); blocks, rows and
// planes past the array's end are left out.
template <typename T, typename XT>
__device__ __forceinline__ void oct_store_rows_through_lds(const FastGeom& g, uint4* st, XT* __restrict__ y, int64_t tx,
                                                           int64_t by, int64_t bz, int lane, const T* v) {
  constexpr int PER16 = 16 / int(sizeof(XT)), RV = 8 / PER16;      // elements per piece, pieces per block row
  static_assert(RV == 2 || RV == 4, "16-bit rows are one piece per block and contiguous as they are");
  constexpr int kRowsPerRound = 512 / (64 * RV);
  constexpr int kLanesPerRow = 8 * RV, kRowsPerInst = 64 / kLanesPerRow;
  const int z = lane >> 3, b = lane & 7;
#pragma unroll
  for (int round = 0; round < 8 / kRowsPerRound; ++round) {
#pragma unroll
    for (int h = 0; h < kRowsPerRound; ++h)
#pragma unroll
      for (int k = 0; k < RV; ++k) {
        const int P = b * RV + k;
        st[(h * 8 + z) * kLanesPerRow + (P ^ (P >> 3))] = Pack<T, XT>::run(v + (round * kRowsPerRound + h) * 8 + PER16 * k);
      }
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < kRowsPerRound * 8 / kRowsPerInst; ++i) {
      const int rr = i * kRowsPerInst + lane / kLanesPerRow, P = lane % kLanesPerRow;      // row (h, z) of the round
      const int64_t yy = by * 8 + round * kRowsPerRound + rr / 8, zr = bz * 8 + rr % 8;
      const uint4 piece = st[rr * kLanesPerRow + (P ^ (P >> 3))];
      if (tx * 8 + P / RV < g.gx && zr < g.Z && yy < g.Y)
        store16_stream(y + (zr * g.Y + yy) * g.X + tx * 64 + P * PER16, piece);
    }
    wave_lds_sync();
  }
}

// The same regrouping for the way in: 8 RV consecutive lanes load one whole 256- or 512-byte row of the eight
// blocks, all 8 RV pieces of a lane are requested before the first is used, and the lanes (plane z, block b) then
// read their own rows' pieces back from LDS.  Pieces of blocks, rows and planes past the array's end are zeros.
template <typename T, typename XT>
__device__ __forceinline__ void oct_load_rows_through_lds(const FastGeom& g, uint4* st, const XT* __restrict__ x, int64_t tx,
                                                          int64_t by, int64_t bz, int lane, T* v) {
  constexpr int PER16 = 16 / int(sizeof(XT)), RV = 8 / PER16;
  constexpr int kRowsPerRound = 512 / (64 * RV), kRounds = 8 / kRowsPerRound;
  constexpr int kLanesPerRow = 8 * RV, kRowsPerInst = 64 / kLanesPerRow, kInstPerRound = kRowsPerRound * 8 / kRowsPerInst;
  const int z = lane >> 3, b = lane & 7;
  const int P = lane % kLanesPerRow;
  uint4 raw[kRounds * kInstPerRound];
#pragma unroll
  for (int round = 0; round < kRounds; ++round)
#pragma unroll
    for (int i = 0; i < kInstPerRound; ++i) {
      const int rr = i * kRowsPerInst + lane / kLanesPerRow;                               // row (h, z) of the round
      const int64_t yy = by * 8 + round * kRowsPerRound + rr / 8, zr = bz * 8 + rr % 8;
      raw[round * kInstPerRound + i] = make_uint4(0u, 0u, 0u, 0u);
      if (tx * 8 + P / RV < g.gx && zr < g.Z && yy < g.Y)
        raw[round * kInstPerRound + i] = load16_stream(x + (zr * g.Y + yy) * g.X + tx * 64 + P * PER16);
    }
#pragma unroll
  for (int round = 0; round < kRounds; ++round) {
    if (round) wave_lds_sync();
#pragma unroll
    for (int i = 0; i < kInstPerRound; ++i) {
      const int rr = i * kRowsPerInst + lane / kLanesPerRow;
      st[rr * kLanesPerRow + (P ^ (P >> 3))] = raw[round * kInstPerRound + i];
    }
    wave_lds_sync();
#pragma unroll
    for (int h = 0; h < kRowsPerRound; ++h)
#pragma unroll
      for (int k = 0; k < RV; ++k) {
        const int Q = b * RV + k;
        Unpack<T, XT>::run(st[(h * 8 + z) * kLanesPerRow + (Q ^ (Q >> 3))], v + (round * kRowsPerRound + h) * 8 + PER16 * k);
      }
  }
}

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
  if constexpr (sizeof(XT) == 8 && !kTailX) {
    // FP64 arrays: four pieces per lane and row, 64 bytes apart; whole rows in piece order, regrouped through LDS
    oct_load_rows_through_lds<float, XT>(g, st, x, tx, by, bz, lane, v);
    __builtin_amdgcn_s_setprio(0);
    wave_lds_sync();                   // the exchange below writes the same LDS
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) tf_forward<TF, float, 8, 1>(v + yy0 * 8);
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) tf_forward<TF, float, 8, 8>(v + xx);
  } else {
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
    const bool inside = tx * 8 + bb < g.gx;
    const double n = inside ? stored_N(m, g.ntype) : 0.0;
    const double f0 = j == 0 ? double(IdxPack<int8_t>::get(first, 0)) : 0.0;
    const double K = tile_pilot(n * f0);                      // lane 0: row 0 of the tile's first block
    const bool has_first = j == 0 && inside;
    const double d = has_first ? n * f0 - K : 0.0;
    emit_tile_sums(tile_sums, g, tx, by, bz, (double(squares) - f0 * f0) * (n * n), d * d, d, has_first ? 1.0 : 0.0, K);
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

// Nothing pruned: rebuilding a plane per lane as above would have every lane read and convert the block's whole
// 512 indices, eight times the work.  This variant mirrors the compress kernel instead: lane = (block bb, row j)
// takes row j of all eight coefficient planes (eight 8-byte pieces of F), transforms back along z, the wave
// exchanges through LDS (the same slots and two half rounds as compress), then lane = (plane z, block b)
// transforms back along y and x and stores its plane.  512 x 512 x 1024: FP32 0.458 -> 0.338 ms, bfloat16 0.395 -> 0.144 ms;
// FP32 rows regrouped through LDS before they are stored: 0.338 -> 0.214 ms.
template <int TF, typename XT, bool kTailX>
__global__ __launch_bounds__(kOctWaves * 64) void k_decompress_oct8_full(FastGeom g, const void* __restrict__ N,
                                                                         const int8_t* __restrict__ F,
                                                                         XT* __restrict__ y) {
  __shared__ uint4 lds[kOctWaves][8 * 64];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<kOctWaves>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * 8;

  float u[64];
  {
    const int bb = lane >> 3, j = lane & 7;
    // a block past the end of the row: decode the row's last block again; nothing of it is stored
    const int64_t blk = tx * 8 + bb < g.gx ? bb : g.gx - 1 - tx * 8;
    const uint2* rows = reinterpret_cast<const uint2*>(F + (block0 + blk) * 512) + j;     // row (kz, j) at rows[kz * 8]
    uint2 f[8];
#pragma unroll
    for (int kz = 0; kz < 8; ++kz) f[kz] = rows[kz * 8];
    const float scale = load_float<float>(N, g.ntype, block0 + blk) / float(g.r);         // Algorithm 3: N F / r
#pragma unroll
    for (int kz = 0; kz < 8; ++kz) {
      const uint32_t w[2] = {f[kz].x, f[kz].y};
#pragma unroll
      for (int e = 0; e < 8; ++e) u[kz * 8 + e] = scale * float(IdxPack<int8_t>::get(w[e >> 2], e & 3));
    }
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) tf_inverse<TF, float, 8, 8, 8>(u + xx);
  }
  float v[64];
  {
    const int bb = lane >> 3, j = lane & 7;
    const int z = lane >> 3, b = lane & 7;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int zz0 = 0; zz0 < 8; ++zz0) st[oct_slot(bb, j, zz0)] = f4_bits(u + zz0 * 8 + h * 4);
      wave_lds_sync();
#pragma unroll
      for (int yy0 = 0; yy0 < 8; ++yy0) bits_f4(st[oct_slot(b, yy0, z)], v + yy0 * 8 + h * 4);
      wave_lds_sync();
    }
  }
#pragma unroll
  for (int xx = 0; xx < 8; ++xx) tf_inverse<TF, float, 8, 8, 8>(v + xx);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) tf_inverse<TF, float, 8, 1, 8>(v + yy0 * 8);
  if constexpr (sizeof(XT) >= 4 && !kTailX) {
    oct_store_rows_through_lds<float, XT>(g, st, y, tx, by, bz, lane, v);
    return;
  }
  const int z = lane >> 3, b = lane & 7;
  const int64_t bx = tx * 8 + b;
  const int64_t zz = bz * 8 + z;
  if (bx < g.gx && zz < g.Z) {
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) {
      const int64_t yy = by * 8 + yy0;
      if (yy < g.Y) oct_store_row<XT, kTailX>(g, y + (zz * g.Y + yy) * g.X, bx, v + yy0 * 8);
    }
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
    if constexpr (sizeof(XT) == 8 && !kTailX) {
      if (whole_wave) {
        // FP64 rows are four pieces per block: the quarter-waves trade them so that store k writes the rows of
        // blocks 16 k .. 16 k + 15 as one contiguous KiB (512^3, FP32 working type: 0.354 -> 0.2 ms)
        uint4 h[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) h[k] = oct_pack<XT>(v + yy0 * 8 + 2 * k);
        transpose_quarter_waves(h[0], h[1], h[2], h[3]);
        uint4* p = reinterpret_cast<uint4*>(y + (zz * g.Y + yy) * g.X + tx * 64 * 8) + 4 * (lane & 15) + (lane >> 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) store16_stream(p + 64 * k, h[k]);
        continue;
      }
    }
    oct_store_row<XT, kTailX>(g, y + (zz * g.Y + yy) * g.X, bx, v + yy0 * 8);
  }
}


// 3-D 8x8x8 bfloat16, FP16, FP32 or FP64 arrays, FP32 arithmetic, N in FP32 or a 16-bit type, int8, box KZ x KY x KX kept
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
    if constexpr (KZ == 8 && KY == 8 && KX == 8) {
      if (!tile_grid(g, 8, kOctWaves, &grid)) return 0;
      if (tail) hipLaunchKernelGGL((k_decompress_oct8_full<TF, XT, true>), grid, dim3(kOctWaves * 64), 0, s, g, n, f, out);
      else hipLaunchKernelGGL((k_decompress_oct8_full<TF, XT, false>), grid, dim3(kOctWaves * 64), 0, s, g, n, f, out);
    } else if (g.gx >= 48) {        // at least three quarters of the lanes of a 64-block tile busy
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
// =====================================================================================================
// 8x8x8 blocks in FP64 arithmetic, nothing pruned: FP32 arrays with int16 or int32 indices, FP64 arrays with int8,
// int16 or int32.  The same two layouts and the same LDS slots as above; a slot holds two FP64 values, so the
// exchange takes four rounds (a quarter of every 8-element row each) through the same 8 KiB per wave.  A row of
// eight indices is 8, 16 or 32 bytes of F and the eight lanes of a block write consecutive rows, so F needs no
// staging.  A row of the array is two (FP32) or four (FP64) 16-byte pieces of a lane.
// =====================================================================================================
template <int kWords>
__device__ __forceinline__ void store_words(void* dst, const uint32_t* w) {      // 2, 4 or 8 dwords, naturally aligned
  if constexpr (kWords == 2) {
    *static_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
  } else {
#pragma unroll
    for (int k = 0; k < kWords / 4; ++k)
      static_cast<uint4*>(dst)[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
  }
}
template <int kWords>
__device__ __forceinline__ void load_words(const void* src, uint32_t* w) {
  if constexpr (kWords == 2) {
    const uint2 u = *static_cast<const uint2*>(src);
    w[0] = u.x; w[1] = u.y;
  } else {
#pragma unroll
    for (int k = 0; k < kWords / 4; ++k) {
      const uint4 u = static_cast<const uint4*>(src)[k];
      w[4 * k] = u.x; w[4 * k + 1] = u.y; w[4 * k + 2] = u.z; w[4 * k + 3] = u.w;
    }
  }
}

template <int TF, typename XT, typename IT, bool kRagged, bool kStats, bool kTailX>
__global__ __launch_bounds__(kOctWaves * 64) void k_compress_oct8_wide(FastGeom g, const XT* __restrict__ x,
                                                                       void* __restrict__ N, IT* __restrict__ F,
                                                                       double* __restrict__ tile_sums) {
  using Slot = ExchangeSlot<double>;
  constexpr int PER16 = Unpack<double, XT>::n;     // elements per 16-byte piece: 4 (FP32) or 2 (FP64)
  constexpr int RV = 8 / PER16;                    // pieces per block row
  constexpr int PER = IdxPack<IT>::per, RW = 8 / PER;       // indices per dword, dwords per row of eight indices
  __shared__ uint4 lds[kOctWaves][8 * 64];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<kOctWaves>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int z = lane >> 3, b = lane & 7;      // phase A: lane = (plane z, block b)
  const int bb = lane >> 3, j = lane & 7;     // phase B: lane = (block bb, row j)

  double v[64];
  {
    if constexpr (!kTailX && sizeof(XT) == 8) {
      // four pieces per lane and row, 64 bytes apart (512 x 512 x 256, int16: 0.167 -> 0.112 ms; the two pieces of
      // an FP32 row gain nothing from the detour: 0.145 -> 0.148 ms)
      oct_load_rows_through_lds<double, XT>(g, st, x, tx, by, bz, lane, v);
      wave_lds_sync();                 // the exchange below writes the same LDS
    } else {
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
#pragma unroll
      for (int yy0 = 0; yy0 < 8; ++yy0) {
#pragma unroll
        for (int k = 0; k < RV; ++k) {
          uint4& piece = raw[yy0 * RV + k];
          if constexpr (kRagged) {
            const uint32_t keep = by * 8 + yy0 < g.Y ? keep_z : 0u;
            piece.x &= keep; piece.y &= keep; piece.z &= keep; piece.w &= keep;
          }
          Unpack<double, XT>::run(piece, v + yy0 * 8 + k * PER16);
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
              const XT val = row[xi < g.X ? xi : g.X - 1];
              v[yy0 * 8 + e] = row_in && xi < g.X ? double(val) : 0.0;
            }
          }
        }
      }
    }
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) tf_forward<TF, double, 8, 1>(v + yy0 * 8);
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) tf_forward<TF, double, 8, 8>(v + xx);
  }
  // exchange: afterwards the lane holds the row y = j of all eight planes of block bb; transform along z
  double u[64];
#pragma unroll
  for (int h = 0; h < 8; h += Slot::n) {
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) st[oct_slot(b, yy0, z)] = Slot::pack(v + yy0 * 8 + h);
    wave_lds_sync();
#pragma unroll
    for (int zz0 = 0; zz0 < 8; ++zz0) Slot::unpack(st[oct_slot(bb, j, zz0)], u + zz0 * 8 + h);
    wave_lds_sync();
  }
#pragma unroll
  for (int xx = 0; xx < 8; ++xx) tf_forward<TF, double, 8, 8>(u + xx);

  double m = 0.0;
#pragma unroll
  for (int i = 0; i < 64; ++i) m = fmax(m, fabs(u[i]));
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) m = fmax(m, __shfl_xor(m, off, 64));     // the 8 rows of the block
  const double inv = m > 0.0 ? g.r / m : 0.0;
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * 8;
  const bool inside = tx * 8 + bb < g.gx;
  uint32_t w[8 * RW];
#pragma unroll
  for (int zq = 0; zq < 8; ++zq)
#pragma unroll
    for (int k = 0; k < RW; ++k) {
      uint32_t q[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e) q[e] = bin_bits(u[zq * 8 + k * PER + e], inv);
      w[zq * RW + k] = IdxPack<IT>::pack(q);
    }
  if (inside) {
    IT* dst = F + (block0 + bb) * 512 + j * 8;                                     // row (kz, j) at dst + kz * 64
#pragma unroll
    for (int zq = 0; zq < 8; ++zq) store_words<RW>(dst + zq * 64, w + zq * RW);
    if (j == 0) store_float(N, g.ntype, block0 + bb, m);
  }
  if constexpr (kStats) {
    const double n = inside ? stored_N(m, g.ntype) : 0.0;
    const double f0 = j == 0 ? double(IdxPack<IT>::get(w[0], 0)) : 0.0;
    const double K = tile_pilot(n * f0);                      // lane 0: row 0 of the tile's first block
    const bool has_first = j == 0 && inside;
    const double d = has_first ? n * f0 - K : 0.0;
    emit_tile_sums(tile_sums, g, tx, by, bz, sum_of_squares_rest<IT, 8 * RW>(w, j == 0) * (n * n), d * d, d,
                   has_first ? 1.0 : 0.0, K);
  }
}

// the eight FP64 values r8 of block bx's row at `row`, as the array's type
template <typename XT, bool kTailX>
__device__ __forceinline__ void oct_store_row_wide(const FastGeom& g, XT* row, int64_t bx, const double* r8) {
  if constexpr (sizeof(XT) == 4) {
    float f8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f8[e] = float(r8[e]);
    oct_store_row<float, kTailX>(g, row, bx, f8);
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t x0 = bx * 8 + k * 2;
      if constexpr (kTailX) {
        if (x0 + 2 <= g.X) {
          store16_a4(row + x0, Pack<double, double>::run(r8 + 2 * k));
        } else if (x0 < g.X) {
          row[x0] = r8[2 * k];
        }
      } else {
        // four pieces per lane, 64 bytes apart: plain stores, which the L2 merges into whole lines
        *reinterpret_cast<uint4*>(row + x0) = Pack<double, double>::run(r8 + 2 * k);
      }
    }
  }
}

template <int TF, typename XT, typename IT, bool kTailX>
__global__ __launch_bounds__(kOctWaves * 64) void k_decompress_oct8_wide(FastGeom g, const void* __restrict__ N,
                                                                         const IT* __restrict__ F,
                                                                         XT* __restrict__ y) {
  using Slot = ExchangeSlot<double>;
  constexpr int PER = IdxPack<IT>::per, RW = 8 / PER;
  __shared__ uint4 lds[kOctWaves][8 * 64];
  const int lane = threadIdx.x & 63;
  int64_t tx, by, bz;
  if (!decode_tile<kOctWaves>(g, tx, by, bz)) return;
  uint4* st = lds[threadIdx.x >> 6];
  const int64_t block0 = (bz * g.gy + by) * g.gx + tx * 8;
  const int z = lane >> 3, b = lane & 7;
  const int bb = lane >> 3, j = lane & 7;

  double u[64];
  {
    // a block past the end of the row: decode the row's last block again; nothing of it is stored
    const int64_t blk = tx * 8 + bb < g.gx ? bb : g.gx - 1 - tx * 8;
    const IT* rows = F + (block0 + blk) * 512 + j * 8;
    uint32_t fw[8][RW];
#pragma unroll
    for (int kz = 0; kz < 8; ++kz) load_words<RW>(rows + kz * 64, fw[kz]);
    const double scale = load_float<double>(N, g.ntype, block0 + blk) / g.r;          // Algorithm 3: N F / r
#pragma unroll
    for (int kz = 0; kz < 8; ++kz) {
#pragma unroll
      for (int e = 0; e < 8; ++e) u[kz * 8 + e] = scale * double(IdxPack<IT>::get(fw[kz][e / PER], e % PER));
    }
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) tf_inverse<TF, double, 8, 8, 8>(u + xx);
  }
  double v[64];
#pragma unroll
  for (int h = 0; h < 8; h += Slot::n) {
#pragma unroll
    for (int zz0 = 0; zz0 < 8; ++zz0) st[oct_slot(bb, j, zz0)] = Slot::pack(u + zz0 * 8 + h);
    wave_lds_sync();
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) Slot::unpack(st[oct_slot(b, yy0, z)], v + yy0 * 8 + h);
    wave_lds_sync();
  }
#pragma unroll
  for (int xx = 0; xx < 8; ++xx) tf_inverse<TF, double, 8, 8, 8>(v + xx);
#pragma unroll
  for (int yy0 = 0; yy0 < 8; ++yy0) tf_inverse<TF, double, 8, 1, 8>(v + yy0 * 8);
  const int64_t bx = tx * 8 + b;
  const int64_t zz = bz * 8 + z;
  if constexpr (!kTailX) {
    oct_store_rows_through_lds<double, XT>(g, st, y, tx, by, bz, lane, v);
  } else if (bx < g.gx && zz < g.Z) {
#pragma unroll
    for (int yy0 = 0; yy0 < 8; ++yy0) {
      const int64_t yy = by * 8 + yy0;
      if (yy < g.Y) oct_store_row_wide<XT, kTailX>(g, y + (zz * g.Y + yy) * g.X, bx, v + yy0 * 8);
    }
  }
}

template <int TF, typename XT, typename IT>
struct Oct8WideKernel {
  static bool matches(const pbz_codec* c, const Folded& f, int xtype) {
    // N of any type.  int8 with an FP32 array and FP32 / 16-bit N computes in FP32 and belongs to the kernels above.
    return f.ok && c->transform == TF && c->compute_f64 && xtype == xtype_code<XT>() &&
           int(c->itype) == itype_code<IT>() && f.bz == 8 && f.by == 8 &&
           f.bx == 8 && f.kz == 8 && f.ky == 8 && f.kx == 8 && x_extent_ok(f, 16 / int(sizeof(XT)), int(sizeof(XT)));
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
    hipLaunchKernelGGL((k_compress_oct8_wide<TF, XT, IT, kRagged, kStats, kTailX>), grid, dim3(kOctWaves * 64), 0, s, g,
                       static_cast<const XT*>(x), N, static_cast<IT*>(F), tile_sums);
  }
  static int compress(FastGeom g, const void* x, void* N, void* F, double* tile_sums, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, 8, kOctWaves, &grid)) return 0;
    const bool ragged = g.Y % 8 || g.Z % 8;
    if (g.X % 8) tile_sums ? launch<true, true, true>(g, grid, x, N, F, tile_sums, s) : launch<true, false, true>(g, grid, x, N, F, nullptr, s);
    else if (tile_sums) ragged ? launch<true, true, false>(g, grid, x, N, F, tile_sums, s) : launch<false, true, false>(g, grid, x, N, F, tile_sums, s);
    else ragged ? launch<true, false, false>(g, grid, x, N, F, nullptr, s) : launch<false, false, false>(g, grid, x, N, F, nullptr, s);
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
  static int decompress(FastGeom g, const void* N, const void* F, void* y, hipStream_t s) {
    dim3 grid;
    if (!tile_grid(g, 8, kOctWaves, &grid)) return 0;
    if (g.X % 8)
      hipLaunchKernelGGL((k_decompress_oct8_wide<TF, XT, IT, true>), grid, dim3(kOctWaves * 64), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    else
      hipLaunchKernelGGL((k_decompress_oct8_wide<TF, XT, IT, false>), grid, dim3(kOctWaves * 64), 0, s, g, N,
                         static_cast<const IT*>(F), static_cast<XT*>(y));
    return hipGetLastError() == hipSuccess ? 1 : PBZ_ERR_HIP;
  }
};

template <int TF> using Oct8_box4 = Oct8Kernel<TF, bf16_t, 4, 4, 4>;
template <int TF> using Oct8_full = Oct8Kernel<TF, bf16_t, 8, 8, 8>;
template <int TF> using Oct8_f32_box4 = Oct8Kernel<TF, float, 4, 4, 4>;
template <int TF> using Oct8_f32_full = Oct8Kernel<TF, float, 8, 8, 8>;
template <int TF> using Oct8_f16_box4 = Oct8Kernel<TF, f16_t, 4, 4, 4>;
template <int TF> using Oct8_f16_full = Oct8Kernel<TF, f16_t, 8, 8, 8>;
template <int TF> using Oct8_f64w32_box4 = Oct8Kernel<TF, double, 4, 4, 4>;
template <int TF> using Oct8_f64w32_full = Oct8Kernel<TF, double, 8, 8, 8>;
template <int TF> using Oct8_f32_i16 = Oct8WideKernel<TF, float, int16_t>;
template <int TF> using Oct8_f32_i32 = Oct8WideKernel<TF, float, int32_t>;
template <int TF> using Oct8_f64_i8 = Oct8WideKernel<TF, double, int8_t>;
template <int TF> using Oct8_f64_i16 = Oct8WideKernel<TF, double, int16_t>;
template <int TF> using Oct8_f64_i32 = Oct8WideKernel<TF, double, int32_t>;

#define PBZ_ROWS(X, TF, SUFFIX) \
  X(Oct8_box4<TF>, "oct8_bf16_8x8x8_i8_box4x4x4" SUFFIX) \
  X(Oct8_full<TF>, "oct8_bf16_8x8x8_i8" SUFFIX) \
  X(Oct8_f32_box4<TF>, "oct8_f32_8x8x8_i8_box4x4x4" SUFFIX) \
  X(Oct8_f32_full<TF>, "oct8_f32_8x8x8_i8" SUFFIX) \
  X(Oct8_f16_box4<TF>, "oct8_f16_8x8x8_i8_box4x4x4" SUFFIX) \
  X(Oct8_f16_full<TF>, "oct8_f16_8x8x8_i8" SUFFIX) \
  X(Oct8_f64w32_box4<TF>, "oct8_f64_w32_8x8x8_i8_box4x4x4" SUFFIX) \
  X(Oct8_f64w32_full<TF>, "oct8_f64_w32_8x8x8_i8" SUFFIX) \
  X(Oct8_f32_i16<TF>, "oct8_f32_8x8x8_i16" SUFFIX) \
  X(Oct8_f32_i32<TF>, "oct8_f32_8x8x8_i32" SUFFIX) \
  X(Oct8_f64_i8<TF>, "oct8_f64_8x8x8_i8" SUFFIX) \
  X(Oct8_f64_i16<TF>, "oct8_f64_8x8x8_i16" SUFFIX) \
  X(Oct8_f64_i32<TF>, "oct8_f64_8x8x8_i32" SUFFIX)

}  // namespace

PBZ_DEFINE_FAST_FAMILY(oct8, PBZ_ROWS)

}  // namespace fast
}  // namespace pbz
