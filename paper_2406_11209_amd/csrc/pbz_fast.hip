// Specialised codec kernels for the block shapes that matter for throughput.
//
// Every kernel here is "wave autonomous": a 64-lane wave owns a run of consecutive blocks along the
// contiguous (last) array dimension, reads whole block rows straight from HBM with 16-byte loads (the
// lanes of a wave cover a contiguous span of every row, which measures at the same bandwidth as a
// linear copy on MI355X), transforms in registers with the even/odd-split DCT of pbz_dct.h or the Haar
// cascade of pbz_haar.h (template switch TF), and writes N and F.  There is no workgroup barrier in the
// compress kernels and LDS, where used, is private to a wave (one exception: the first exchange of "cube16").
//
// Family "lane":   one lane owns one whole block (blocks of at most 64 elements: 8x8, 4x4x4).  Where a block
//                   row is two (four) 16-byte pieces the half-waves (quarter-waves) trade pieces, so that every
//                   load / store instruction of the array covers one contiguous KiB.  Indices leave through a wave-private
//                   LDS transpose when a block's F is 64 bytes or more, for the same reason.
// Family "quad16":  16x16 and 4x16x16 blocks of FP32, 16-bit or FP64 input (int8 in FP32 arithmetic; in FP64 arithmetic FP32 input
//                   with int16 / int32 and FP64 input with int8 to int32), 16 planes of 16x16 per wave.  Each lane first holds a 16-row x
//                   4-column strip (the column transform runs in registers), the wave exchanges through LDS,
//                   then each lane holds four whole rows (row transform, and for 4x16x16 the transform across
//                   the four planes); rows leave as 16-byte pieces in linear order.
// Family "oct8":    8x8x8 blocks of bfloat16, FP16, FP32 or FP64 input (int8 in FP32 arithmetic; in FP64 arithmetic FP32 input
//                   with int16 / int32 and FP64 input with int8 to int32), 8 blocks per wave.  Each lane first holds one z-plane of
//                   a block (x and y transforms), the wave exchanges through LDS, then each lane holds one
//                   y-row of all eight z-planes (z transform).  Decompression needs no exchange: every
//                   lane rebuilds its own z-plane from the block's few kept coefficients; wide arrays use a
//                   variant in which a wave owns one plane of 64 blocks and stores whole 1 KiB row pieces.
// Family "cube16":  16x16x16 blocks of FP32 input (int16 / int32 indices in FP64 arithmetic, int8 in FP32) or FP64 input (int8 in
//                   FP32 arithmetic, int8 to int32 in FP64), two neighbouring blocks
//                   per workgroup of two waves.  Three layouts, one per transformed dimension, with an LDS exchange
//                   between them; the first is how rows are read (eight lanes cover the 128 bytes the two blocks have
//                   in a row), the last how F is written (whole rows of indices).
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
// The families live in pbz_fast_lane.hip, pbz_fast_quad16.hip, pbz_fast_oct8.hip and pbz_fast_cube16.hip; this file folds the array
// and asks each family in turn.
#include "pbz_fast_common.h"

namespace pbz {

int try_compress_fast(const pbz_codec* c, const Geom& geo, const void* x, int xtype, void* N, void* F, hipStream_t s,
                      bool dry_run, const char** name, double* tile_sums) {
  if (!fast::aligned16(x) || !fast::aligned16(F)) return 0;
  const fast::Folded f = fast::fold(c, geo);
  if (!f.ok) return 0;
  *name = nullptr;
  int r = fast::lane_compress(c, f, xtype, x, N, F, s, dry_run, name, tile_sums);
  if (!*name) r = fast::quad16_compress(c, f, xtype, x, N, F, s, dry_run, name, tile_sums);
  if (!*name) r = fast::oct8_compress(c, f, xtype, x, N, F, s, dry_run, name, tile_sums);
  if (!*name) r = fast::cube16_compress(c, f, xtype, x, N, F, s, dry_run, name, tile_sums);
  return r;
}

int64_t fast_compress_tiles(const pbz_codec* c, const Geom& geo, int xtype) {
  const fast::Folded f = fast::fold(c, geo);
  if (!f.ok) return 0;
  int64_t t = fast::lane_tiles(c, f, xtype);
  if (t < 0) t = fast::quad16_tiles(c, f, xtype);
  if (t < 0) t = fast::oct8_tiles(c, f, xtype);
  if (t < 0) t = fast::cube16_tiles(c, f, xtype);
  return t < 0 ? 0 : t;
}

int try_decompress_fast(const pbz_codec* c, const Geom& geo, const void* N, const void* F, void* y, int ytype,
                        hipStream_t s, bool dry_run, const char** name) {
  if (!fast::aligned16(y) || !fast::aligned16(F)) return 0;
  const fast::Folded f = fast::fold(c, geo);
  if (!f.ok) return 0;
  *name = nullptr;
  int r = fast::lane_decompress(c, f, ytype, N, F, y, s, dry_run, name);
  if (!*name) r = fast::quad16_decompress(c, f, ytype, N, F, y, s, dry_run, name);
  if (!*name) r = fast::oct8_decompress(c, f, ytype, N, F, y, s, dry_run, name);
  if (!*name) r = fast::cube16_decompress(c, f, ytype, N, F, y, s, dry_run, name);
  return r;
}

}  // namespace pbz
