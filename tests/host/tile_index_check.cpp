// Host check of the general tiled kernels' index arithmetic (csrc/pbz_tile_index.h): reads geometries from standard
// input, one per line as "ndim block... shape...", and compares every function against the plain definition by
// enumerating all elements.  Prints one "ok" or "FAIL <what>" line per geometry.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pbz_tile_index.h"

using namespace pbz::tile;

namespace {

struct Plain {                 // block k, intra-block index j -> offset and whether inside, by the definition
  int ndim;
  int64_t block[PBZ_MAX_NDIM], shape[PBZ_MAX_NDIM], grid[PBZ_MAX_NDIM], stride[PBZ_MAX_NDIM];
  int64_t n_blocks;
  bool locate(int64_t k, int64_t j, int64_t* off) const {
    if (k >= n_blocks) return false;
    int64_t kb[PBZ_MAX_NDIM], jd[PBZ_MAX_NDIM];
    for (int d = ndim - 1; d >= 0; --d) {
      kb[d] = k % grid[d];
      k /= grid[d];
      jd[d] = j % block[d];
      j /= block[d];
    }
    bool in = true;
    *off = 0;
    for (int d = 0; d < ndim; ++d) {
      const int64_t c = kb[d] * block[d] + jd[d];
      in = in && c < shape[d];
      *off += c * stride[d];
    }
    return in;
  }
};

template <int kDims>
const char* check(const TileGeom& tg, const Plain& pl) {
  const int total = tg.G << tg.vol_shift;
  const int vol = 1 << tg.vol_shift;
  int64_t elements = 1;
  for (int d = 0; d < pl.ndim; ++d) elements *= pl.shape[d];
  std::vector<int> seen(size_t(elements), 0);
  const int64_t n_tiles = (tg.n_blocks + tg.G - 1) / tg.G;
  for (int64_t tile = 0; tile < n_tiles; ++tile) {
    const int64_t k0 = tile * tg.G;
    std::vector<char> slot(size_t(total), 0);
    for (int e = 0; e < total; ++e) {
      int b, j;
      row_major_across_blocks(tg, e, &b, &j);
      if (b < 0 || b >= tg.G || j < 0 || j >= vol) return "enumeration out of range";
      if (slot[size_t(b) * vol + j]++) return "enumeration hits an element twice";
      const BlockInfo bi = block_info<kDims>(tg, k0 + b);
      const RowInfo ri = row_info<kDims>(tg, j >> tg.bx_shift);
      int64_t off = -1, want = -1;
      const bool in = locate_in<kDims>(bi, ri, j & ((1 << tg.bx_shift) - 1), &off);
      const bool in_want = pl.locate(k0 + b, j, &want);
      if (in != in_want) return "inside / outside differs from the definition";
      if (in && off != want) return "offset differs from the definition";
      if (in) {
        if (off < 0 || off >= elements) return "offset outside the array";
        ++seen[size_t(off)];
      }
    }
  }
  for (int64_t i = 0; i < elements; ++i)
    if (seen[size_t(i)] != 1) return "an element of the array is not visited exactly once";
  return nullptr;
}

template <int P>
const char* check_pieces(const TileGeom& tg) {
  if ((1 << tg.bx_shift) < P) return nullptr;
  const int total = tg.G << tg.vol_shift, vol = 1 << tg.vol_shift;
  std::vector<char> slot(size_t(total), 0);
  for (int p = 0; p < total / P; ++p) {
    int b, j;
    piece_across_blocks<P>(tg, p, &b, &j);
    if (b < 0 || b >= tg.G || j < 0 || j + P > vol) return "piece out of range";
    if ((j >> tg.bx_shift) != ((j + P - 1) >> tg.bx_shift)) return "piece leaves its row";
    if (pad(b * vol + j + P - 1) != pad(b * vol + j) + P - 1) return "piece is not contiguous in the padded tile";
    for (int i = 0; i < P; ++i)
      if (slot[size_t(b) * vol + j + i]++) return "pieces overlap";
    // consecutive pieces are consecutive in memory across the tile's blocks
    int b2, j2;
    row_major_across_blocks(tg, p * P, &b2, &j2);
    if (b2 != b || j2 != j) return "piece order differs from element order";
  }
  for (int i = 0; i < total; ++i)
    if (slot[size_t(i)] != 1) return "pieces do not cover the tile";
  return nullptr;
}

const char* check_passes(const TileGeom& tg) {
  const int total = tg.G << tg.vol_shift;
  int inner_shift = tg.vol_shift;
  for (int d = 0; d < PBZ_MAX_NDIM; ++d) {
    const int ns = tg.bshift[d];
    inner_shift -= ns;
    if (ns == 0) continue;
    std::vector<char> hit(size_t(total), 0);
    const int lines = total >> ns;
    for (int l = 0; l < lines; ++l) {
      const int base = line_base(l, ns, inner_shift);
      for (int a = 0; a < (1 << ns); ++a) {
        const int e = base + (a << inner_shift);
        if (e < 0 || e >= total) return "line element out of range";
        if (hit[size_t(e)]++) return "lines overlap";
        if (pad(e) != pad(base) + pad(a << inner_shift)) return "padded address of a line element is not base + offset";
        if ((e >> tg.vol_shift) != (l >> (tg.vol_shift - ns))) return "a line's block is not l >> (vol_shift - n_shift)";
      }
    }
    for (int e = 0; e < total; ++e)
      if (hit[size_t(e)] != 1) return "lines do not cover the tile";
  }
  if (inner_shift != 0) return "inner stride does not end at one";
  // four consecutive elements from a multiple of four are contiguous in the padded tile (F in runs of four)
  for (int e = 0; e + 3 < total; e += 4)
    if (pad(e + 3) != pad(e) + 3) return "a run of four is not contiguous in the padded tile";
  return nullptr;
}

}  // namespace

int main() {
  int ndim;
  while (std::scanf("%d", &ndim) == 1) {
    Plain pl{};
    pl.ndim = ndim;
    for (int d = 0; d < ndim; ++d) { long long v; if (std::scanf("%lld", &v) != 1) return 2; pl.block[d] = v; }
    for (int d = 0; d < ndim; ++d) { long long v; if (std::scanf("%lld", &v) != 1) return 2; pl.shape[d] = v; }
    int64_t st = 1;
    pl.n_blocks = 1;
    for (int d = ndim - 1; d >= 0; --d) {
      pl.stride[d] = st;
      st *= pl.shape[d];
      pl.grid[d] = (pl.shape[d] + pl.block[d] - 1) / pl.block[d];
      pl.n_blocks *= pl.grid[d];
    }
    const TileGeom tg = make_tile_geom(ndim, pl.block, pl.shape, 1);
    const char* bad = tg.n_blocks != pl.n_blocks ? "block count" : nullptr;
    if (!bad) bad = tg.dims == 4 ? check<4>(tg, pl) : check<8>(tg, pl);
    if (!bad && ndim <= 4) bad = check<8>(tg, pl);          // the wider packing must agree on the same geometry
    if (!bad) bad = check_pieces<2>(tg);
    if (!bad) bad = check_pieces<4>(tg);
    if (!bad) bad = check_pieces<8>(tg);
    if (!bad) bad = check_passes(tg);
    if (!bad && tile_offset(tg.G, tg.vol_shift, tg.bx_shift) % 16 != 0) bad = "tile offset not 16-byte aligned";
    if (bad) std::printf("FAIL %s\n", bad);
    else std::printf("ok\n");
  }
  return 0;
}
