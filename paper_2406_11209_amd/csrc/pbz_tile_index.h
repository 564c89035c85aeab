// Index arithmetic of the general tiled codec kernels (pbz_tiled.hip), free of anything that needs a GPU: the
// kernels include it, and a host program compiles the same functions and checks them against the plain definition
// (tests/host/tile_index_check.hip).
#pragma once
#include <cstdint>

#include "pbz.h"

#if defined(__HIPCC__)
#define PBZ_HD __host__ __device__ __forceinline__
#else
#define PBZ_HD inline
#endif

namespace pbz {
namespace tile {

constexpr int kTileElems = 4096;              // elements of a tile at most
constexpr int kMaxTileBlocks = 256;           // blocks of a tile at most
constexpr int kMaxRows = 256;                 // rows (runs along the last dimension) of a block whose place is tabulated

// The array's geometry right-aligned into a fixed number of dimensions (kDims = 4 or 8 in the kernels; unused
// leading dimensions have extent, block extent and grid extent 1 and stride 0), so that every loop over the
// dimensions unrolls and its operands stay in scalar registers instead of being fetched by a run-time index.
struct TileGeom {
  int G, g_shift;                 // blocks per tile
  int vol_shift;                  // log2(prod(block))
  int bx_shift;                   // log2 of the last block extent
  int dims;                       // 4 or 8
  int kept;
  int vec_x;                      // the array may be moved in 16-byte pieces
  int vec_f;                      // F may be moved in runs of four entries
  int64_t n_blocks;
  int bshift[PBZ_MAX_NDIM];       // log2 of every block extent
  int64_t shape[PBZ_MAX_NDIM], stride[PBZ_MAX_NDIM], grid[PBZ_MAX_NDIM];
};

inline int ilog2_ceil(int64_t v) {
  int s = 0;
  while ((int64_t(1) << s) < v) ++s;
  return s;
}

// host side: the geometry of an array of `shape` in blocks of `block` (powers of two, at most 32 each here and 4096
// elements together), `kept` entries per block
inline TileGeom make_tile_geom(int ndim, const int64_t* block, const int64_t* shape, int kept) {
  TileGeom tg{};
  int64_t vol = 1;
  for (int d = 0; d < ndim; ++d) vol *= block[d];
  int G = int(kTileElems / vol);
  if (G < 1) G = 1;
  if (G > kMaxTileBlocks) G = kMaxTileBlocks;
  tg.G = G;
  tg.g_shift = ilog2_ceil(G);
  tg.vol_shift = ilog2_ceil(vol);
  tg.bx_shift = ilog2_ceil(block[ndim - 1]);
  tg.dims = ndim <= 4 ? 4 : 8;
  tg.kept = kept;
  tg.vec_x = tg.vec_f = 0;
  tg.n_blocks = 1;
  int64_t stride = 1;
  for (int d = PBZ_MAX_NDIM - 1; d >= 0; --d) {        // right-aligned; leading dimensions of extent 1
    const int src = d - (PBZ_MAX_NDIM - ndim);
    tg.bshift[d] = src >= 0 ? ilog2_ceil(block[src]) : 0;
    tg.shape[d] = src >= 0 ? shape[src] : 1;
    tg.stride[d] = src >= 0 ? stride : 0;
    tg.grid[d] = src >= 0 ? (shape[src] + block[src] - 1) / block[src] : 1;
    if (src >= 0) stride *= shape[src];
    tg.n_blocks *= tg.grid[d];
  }
  return tg;
}

// Element i of the tile lives at slot pad(i) of the LDS buffer: one spare slot per 32 keeps strided line accesses
// from piling onto one bank (one per 16 for FP64 values, whose 32 fill the banks twice over, changed nothing
// measurable).  For a line of n elements `inner` apart that starts at a multiple of n * inner plus less than inner
// (all powers of two), pad(base + a * inner) = pad(base) + pad(a * inner).
PBZ_HD int pad(int i) { return i + (i >> 5); }

// first element of line l in a pass over lines of 2^n_shift elements that are 2^inner_shift apart
PBZ_HD int line_base(int l, int n_shift, int inner_shift) {
  return ((l >> inner_shift) << (n_shift + inner_shift)) + (l & ((1 << inner_shift) - 1));
}

// One byte per dimension (right-aligned: byte kDims - 1 belongs to the last one).  A block's `lim` holds how many
// entries (0 .. 32) along each dimension lie inside the array; a position's `coord` holds 0x80 | coordinate
// (0 .. 31).  Byte by byte, coord - lim = 128 + c - l lies in [96, 159], so nothing is borrowed across bytes, and
// bit 7 of a byte is clear exactly when c < l: one subtraction tests all dimensions at once.
template <int kDims> struct Packed;
template <> struct Packed<4> { typedef uint32_t type; static constexpr uint32_t kHigh = 0x80808080u; };
template <> struct Packed<8> { typedef uint64_t type; static constexpr uint64_t kHigh = 0x8080808080808080ull; };

struct BlockInfo {                            // 16 bytes: one LDS read
  int64_t origin;                             // element offset of the block's first element
  uint64_t lim;                               // all zero: no such block (past the end of the array's blocks)
};
struct RowInfo {                              // 16 bytes: one LDS read
  int64_t off;                                // offset of the row's first element from the block's first element
  uint64_t coord;                             // the last dimension's byte holds 0x80: the caller adds the position in the row
};

template <int kDims>
PBZ_HD bool inside(uint64_t lim, uint64_t coord) {
  typedef typename Packed<kDims>::type packed_t;
  return ((packed_t(coord) - packed_t(lim)) & Packed<kDims>::kHigh) == 0;
}

// block k of the array (block-major order)
template <int kDims>
PBZ_HD BlockInfo block_info(const TileGeom& tg, int64_t k) {
  BlockInfo info;
  info.origin = 0;
  info.lim = 0;
  if (k < tg.n_blocks) {
#pragma unroll
    for (int d = PBZ_MAX_NDIM - 1; d >= PBZ_MAX_NDIM - kDims; --d) {
      int64_t kb = 0;
      if (tg.grid[d] > 1) {             // uniform: no division for the padded dimensions
        kb = k % tg.grid[d];
        k /= tg.grid[d];
      }
      const int64_t c0 = kb << tg.bshift[d];
      const int64_t left = tg.shape[d] - c0;
      const int64_t extent = int64_t(1) << tg.bshift[d];
      info.lim |= uint64_t(left < extent ? left : extent) << (8 * (d - (PBZ_MAX_NDIM - kDims)));
      info.origin += c0 * tg.stride[d];
    }
  }
  return info;
}

// row i of a block (rows are numbered in the block's own row-major order)
template <int kDims>
PBZ_HD RowInfo row_info(const TileGeom& tg, int i) {
  RowInfo r;
  r.off = 0;
  r.coord = Packed<kDims>::kHigh;
#pragma unroll
  for (int d = PBZ_MAX_NDIM - 2; d >= PBZ_MAX_NDIM - kDims; --d) {
    const int jd = i & ((1 << tg.bshift[d]) - 1);
    i >>= tg.bshift[d];
    r.off += jd * tg.stride[d];
    r.coord += uint64_t(jd) << (8 * (d - (PBZ_MAX_NDIM - kDims)));
  }
  return r;
}

// position xin of a row of a block -> element offset; false when the element is padding
template <int kDims>
PBZ_HD bool locate_in(const BlockInfo& k, const RowInfo& r, int xin, int64_t* offset) {
  *offset = k.origin + r.off + xin;                                            // the last dimension has stride 1
  return inside<kDims>(k.lim, r.coord + (uint64_t(xin) << (8 * (kDims - 1))));
}

// The workgroup's LDS: G block records, the row records, 16 bytes per block for the kernels' own per-block
// values (maxima and reciprocals, or N / r), then the padded tile.
PBZ_HD int tabulated_rows(int vol_shift, int bx_shift) {
  const int rows = 1 << (vol_shift - bx_shift);
  return rows <= kMaxRows ? rows : 0;
}
PBZ_HD size_t per_block_offset(int G, int vol_shift, int bx_shift) {
  return 16 * size_t(G + tabulated_rows(vol_shift, bx_shift));
}
PBZ_HD size_t tile_offset(int G, int vol_shift, int bx_shift) {
  return per_block_offset(G, vol_shift, bx_shift) + 16 * size_t(G);
}

// enumeration of the tile that is friendly to memory: consecutive e walk along a row across the tile's blocks
PBZ_HD void row_major_across_blocks(const TileGeom& tg, int e, int* b, int* j) {
  const int bx = 1 << tg.bx_shift;
  const int xin = e & (bx - 1);
  *b = (e >> tg.bx_shift) & (tg.G - 1);
  *j = ((e >> (tg.bx_shift + tg.g_shift)) << tg.bx_shift) + xin;
}

// the same for 16-byte pieces of P elements (P = 2, 4 or 8, at most the last block extent): piece p -> block and
// intra-block index of its first element
template <int P>
PBZ_HD void piece_across_blocks(const TileGeom& tg, int p, int* b, int* j) {
  constexpr int pshift = P == 2 ? 1 : (P == 4 ? 2 : 3);
  const int ppr_shift = tg.bx_shift - pshift;                 // pieces per block row
  *b = (p >> ppr_shift) & (tg.G - 1);
  *j = ((p >> (ppr_shift + tg.g_shift)) << tg.bx_shift) + ((p & ((1 << ppr_shift) - 1)) << pshift);
}

}  // namespace tile
}  // namespace pbz
