// Host side of the C ABI: argument validation, layout arithmetic, kernel dispatch.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "pbz_internal.h"

using namespace pbz;

namespace {

bool valid_ftype(int t) { return t == PBZ_F64 || t == PBZ_F32 || t == PBZ_BF16 || t == PBZ_F16; }

bool is_pow2(int64_t v) { return v >= 1 && (v & (v - 1)) == 0; }

// orthonormal DCT-II matrix, H[m][q] = a_q cos(pi (2m+1) q / (2n))  (Sec. III-A, Appendix A)
void fill_dct(double* H, int n) {
  const double pi = 3.14159265358979323846264338327950288;
  for (int m = 0; m < n; ++m)
    for (int q = 0; q < n; ++q) {
      double a = q == 0 ? std::sqrt(1.0 / n) : std::sqrt(2.0 / n);
      H[m * n + q] = a * std::cos(pi * (2.0 * m + 1.0) * q / (2.0 * n));
    }
}

// orthonormal Haar matrix in sequency order, same index convention (Sec. III-A names the transform only)
void fill_haar(double* H, int n) {
  for (int i = 0; i < n * n; ++i) H[i] = 0.0;
  for (int m = 0; m < n; ++m) H[m * n] = std::sqrt(1.0 / n);
  int q = 1;
  for (int count = 1; count < n; count *= 2) {
    const int width = n / count;
    const double amp = std::sqrt(double(count) / n);
    for (int j = 0; j < count; ++j, ++q)
      for (int m = 0; m < width; ++m) H[(j * width + m) * n + q] = m < width / 2 ? amp : -amp;
  }
}

int make_geom(const pbz_codec* c, const int64_t* shape, Geom* g) {
  if (!c || !shape) return PBZ_ERR_NULL;
  std::memset(g, 0, sizeof(*g));
  g->ndim = c->ndim;
  g->vol = c->vol;
  g->kept = c->kept;
  int64_t nb = 1, elems = 1;
  const int64_t lim = int64_t(1) << 40;   // elements; keeps every launch grid below 2^31 workgroups
  for (int d = 0; d < c->ndim; ++d) {
    if (shape[d] < 1) return PBZ_ERR_SHAPE;
    g->shape[d] = shape[d];
    g->block[d] = int32_t(c->block[d]);
    g->grid[d] = (shape[d] + c->block[d] - 1) / c->block[d];
    g->h_offset[d] = c->h_offset[d];
    if (shape[d] > lim || elems > lim / shape[d]) return PBZ_ERR_SHAPE;
    elems *= shape[d];
    if (nb > lim / g->grid[d]) return PBZ_ERR_SHAPE;
    nb *= g->grid[d];
  }
  if (nb > lim / c->vol) return PBZ_ERR_SHAPE;
  int64_t st = 1;
  for (int d = c->ndim - 1; d >= 0; --d) {
    g->stride[d] = st;
    st *= shape[d];
  }
  g->n_blocks = nb;
  return PBZ_OK;
}

int check_blocks(const pbz_codec* c, int64_t n_blocks) {
  if (!c) return PBZ_ERR_NULL;
  if (n_blocks < 1 || n_blocks > (int64_t(1) << 40) / c->vol) return PBZ_ERR_SHAPE;   // keeps every grid below 2^31
  return PBZ_OK;
}

}  // namespace

int pbz::ensure_tables(const pbz_codec* c, const DeviceTables** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return PBZ_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return PBZ_ERR_HIP;
  std::lock_guard<std::mutex> lock(c->mu);
  DeviceTables& t = c->dev[dev];
  if (!t.ready) {
    bool ok = hipMalloc(&t.H, sizeof(double) * c->h_total) == hipSuccess &&
              hipMalloc(&t.kept_pos, sizeof(int32_t) * c->vol) == hipSuccess &&
              hipMalloc(&t.kept_list, sizeof(int32_t) * c->kept) == hipSuccess &&
              hipMemcpy(t.kept_list, c->kept_list, sizeof(int32_t) * c->kept, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(t.H, c->H_host, sizeof(double) * c->h_total, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(t.kept_pos, c->kept_pos, sizeof(int32_t) * c->vol, hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {   // leave nothing half-made behind
      if (t.H) (void)hipFree(t.H);
      if (t.kept_pos) (void)hipFree(t.kept_pos);
      if (t.kept_list) (void)hipFree(t.kept_list);
      t.kept_list = nullptr;
      t.H = nullptr;
      t.kept_pos = nullptr;
      return PBZ_ERR_HIP;
    }
    t.ready = true;
  }
  *out = &t;
  return PBZ_OK;
}

extern "C" {

int pbz_codec_create(pbz_codec** out, int ndim, const int64_t* block_shape, pbz_ftype work_type,
                     pbz_itype index_type, const uint8_t* mask) {
  if (!out || !block_shape) return PBZ_ERR_NULL;
  *out = nullptr;
  if (ndim < 1 || ndim > PBZ_MAX_NDIM) return PBZ_ERR_NDIM;
  int64_t vol = 1;
  for (int d = 0; d < ndim; ++d) {
    if (!is_pow2(block_shape[d]) || block_shape[d] > PBZ_MAX_BLOCK_EXTENT) return PBZ_ERR_BLOCK_SHAPE;
    vol *= block_shape[d];
    if (vol > PBZ_MAX_BLOCK_VOLUME) return PBZ_ERR_BLOCK_SHAPE;
  }
  if (!valid_ftype(work_type)) return PBZ_ERR_TYPE;
  if (index_type != PBZ_I8 && index_type != PBZ_I16 && index_type != PBZ_I32) return PBZ_ERR_TYPE;

  int kept = 0;
  if (mask) {
    for (int64_t j = 0; j < vol; ++j) kept += mask[j] ? 1 : 0;
    if (kept == 0) return PBZ_ERR_MASK_EMPTY;
  } else {
    kept = int(vol);
  }

  pbz_codec* c = new (std::nothrow) pbz_codec();
  if (!c) return PBZ_ERR_ALLOC;
  c->ndim = ndim;
  c->vol = int(vol);
  c->ftype = work_type;
  c->itype = index_type;
  c->index_bits = 8 << int(index_type);
  c->r = std::ldexp(1.0, c->index_bits - 1) - 1.0;
  c->compute_f64 = (work_type == PBZ_F64) || (c->index_bits > 8);
  c->kept = kept;
  c->path = PBZ_PATH_AUTO;
  c->transform = PBZ_TRANSFORM_DCT;
  c->mask = static_cast<uint8_t*>(std::malloc(size_t(vol)));
  c->kept_pos = static_cast<int32_t*>(std::malloc(sizeof(int32_t) * size_t(vol)));
  c->kept_list = static_cast<int32_t*>(std::malloc(sizeof(int32_t) * size_t(kept)));
  int h_total = 0;
  for (int d = 0; d < ndim; ++d) {
    c->block[d] = block_shape[d];
    c->h_offset[d] = h_total;
    h_total += int(block_shape[d] * block_shape[d]);
  }
  c->h_total = h_total;
  c->H_host = static_cast<double*>(std::malloc(sizeof(double) * size_t(h_total)));
  if (!c->mask || !c->kept_pos || !c->kept_list || !c->H_host) {
    pbz_codec_destroy(c);
    return PBZ_ERR_ALLOC;
  }
  int pos = 0;
  for (int64_t j = 0; j < vol; ++j) {
    c->mask[j] = mask ? (mask[j] ? 1 : 0) : 1;
    if (c->mask[j]) c->kept_list[pos] = int32_t(j);
    c->kept_pos[j] = c->mask[j] ? pos++ : -1;
  }
  c->dc_kept = c->mask[0] != 0;
  for (int d = 0; d < ndim; ++d) fill_dct(c->H_host + c->h_offset[d], int(block_shape[d]));

  // is the mask a low-frequency corner box?  extent along d = run of kept entries along axis d from the origin
  int64_t stride = 1;
  int64_t strides[PBZ_MAX_NDIM];
  for (int d = ndim - 1; d >= 0; --d) {
    strides[d] = stride;
    stride *= block_shape[d];
  }
  bool is_box = c->dc_kept;
  if (is_box) {
    for (int d = 0; d < ndim; ++d) {
      int e = 0;
      while (e < block_shape[d] && c->mask[e * strides[d]]) ++e;
      c->box[d] = e;
    }
    for (int64_t j = 0; j < vol && is_box; ++j) {
      bool inside = true;
      for (int d = 0; d < ndim; ++d) inside = inside && ((j / strides[d]) % block_shape[d] < c->box[d]);
      is_box = (inside == (c->mask[j] != 0));
    }
  }
  if (!is_box)
    for (int d = 0; d < ndim; ++d) c->box[d] = 0;
  *out = c;
  return PBZ_OK;
}

void pbz_codec_destroy(pbz_codec* c) {
  if (!c) return;
  for (int d = 0; d < kMaxDevices; ++d) {
    if (c->dev[d].H || c->dev[d].kept_pos) {
      int cur = 0;
      bool have = hipGetDevice(&cur) == hipSuccess;
      if (have && hipSetDevice(d) == hipSuccess) {
        if (c->dev[d].H) (void)hipFree(c->dev[d].H);
        if (c->dev[d].kept_pos) (void)hipFree(c->dev[d].kept_pos);
        if (c->dev[d].kept_list) (void)hipFree(c->dev[d].kept_list);
        (void)hipSetDevice(cur);
      }
    }
  }
  std::free(c->mask);
  std::free(c->kept_pos);
  std::free(c->kept_list);
  std::free(c->H_host);
  delete c;
}

int pbz_codec_set_transform(pbz_codec* c, pbz_transform transform) {
  if (!c) return PBZ_ERR_NULL;
  if (transform != PBZ_TRANSFORM_DCT && transform != PBZ_TRANSFORM_HAAR) return PBZ_ERR_TYPE;
  std::lock_guard<std::mutex> lock(c->mu);
  if (c->used.load()) return PBZ_ERR_STATE;          // arrays compressed so far would no longer decompress
  c->transform = int(transform);
  for (int d = 0; d < c->ndim; ++d) {
    double* H = c->H_host + c->h_offset[d];
    if (transform == PBZ_TRANSFORM_HAAR) fill_haar(H, int(c->block[d]));
    else fill_dct(H, int(c->block[d]));
  }
  return PBZ_OK;
}

int pbz_codec_set_kernel_path(pbz_codec* c, pbz_kernel_path path) {
  if (!c) return PBZ_ERR_NULL;
  if (path != PBZ_PATH_AUTO && path != PBZ_PATH_GENERIC) return PBZ_ERR_TYPE;
  c->path = path;
  return PBZ_OK;
}

int pbz_layout(const pbz_codec* c, const int64_t* shape, int64_t* n_blocks, int64_t* kept_per_block,
               size_t* n_bytes, size_t* f_bytes, size_t* workspace_bytes) {
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  if (n_blocks) *n_blocks = g.n_blocks;
  if (kept_per_block) *kept_per_block = c->kept;
  if (n_bytes) *n_bytes = size_t(g.n_blocks) * size_t(ftype_bytes(c->ftype));
  if (f_bytes) *f_bytes = size_t(g.n_blocks) * size_t(c->kept) * size_t(itype_bytes(c->itype));
  if (workspace_bytes) *workspace_bytes = kWorkspaceBytes;
  return PBZ_OK;
}

int pbz_compressed_bits(const pbz_codec* c, const int64_t* shape, uint64_t* bits) {
  if (!bits) return PBZ_ERR_NULL;
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  uint64_t d = uint64_t(c->ndim);
  uint64_t nb = uint64_t(g.n_blocks);
  *bits = 4 + 64 * d + 64 + 64 * d + uint64_t(c->vol) + uint64_t(8 * ftype_bytes(c->ftype)) * nb +
          uint64_t(c->index_bits) * uint64_t(c->kept) * nb;
  return PBZ_OK;
}

int pbz_compress(const pbz_codec* c, const void* x, pbz_ftype x_type, const int64_t* shape, void* N, void* F,
                 void* stream) {
  if (!c || !x || !shape || !N || !F) return PBZ_ERR_NULL;
  if (!valid_ftype(x_type)) return PBZ_ERR_TYPE;
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  c->used.store(true);
  if (c->path == PBZ_PATH_AUTO) {
    const char* name = nullptr;
    int r = try_compress_fast(c, g, x, x_type, N, F, s, false, &name);
    if (r != 0) return r < 0 ? r : PBZ_OK;
  }
  const DeviceTables* t = nullptr;
  st = ensure_tables(c, &t);
  if (st != PBZ_OK) return st;
  if (tiled_kernels_cover(c)) return launch_compress_tiled(c, g, t, x, x_type, N, F, s);
  return launch_compress_generic(c, g, t, x, x_type, N, F, s);
}

int pbz_compress_statistics_workspace(const pbz_codec* c, const int64_t* shape, pbz_ftype x_type, size_t* bytes) {
  if (!c || !shape || !bytes) return PBZ_ERR_NULL;
  if (!valid_ftype(x_type)) return PBZ_ERR_TYPE;
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  const int64_t tiles = c->path == PBZ_PATH_AUTO ? fast_compress_tiles(c, g, x_type) : 0;
  *bytes = kWorkspaceBytes + size_t(tiles) * 4 * sizeof(double);
  return PBZ_OK;
}

int pbz_compress_statistics(const pbz_codec* c, const void* x, pbz_ftype x_type, const int64_t* shape, void* N, void* F,
                            int per_step, double* statistics, void* ws, size_t ws_bytes, void* stream) {
  if (!c || !x || !shape || !N || !F || !statistics || !ws) return PBZ_ERR_NULL;
  if (!valid_ftype(x_type)) return PBZ_ERR_TYPE;
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  if (!c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (ws_bytes < kWorkspaceBytes || (reinterpret_cast<uintptr_t>(ws) & 15u)) return PBZ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t segments = per_step ? g.grid[0] : 1;       // one triple per block index along dimension 0
  c->used.store(true);
  if (c->path == PBZ_PATH_AUTO) {
    // the compress kernel leaves a record of four doubles per tile behind the reduction scratch; adding them costs two small launches
    const int64_t tiles = fast_compress_tiles(c, g, x_type);
    if (tiles > 0 && ws_bytes >= kWorkspaceBytes + size_t(tiles) * 4 * sizeof(double)) {
      double* tile_sums = reinterpret_cast<double*>(static_cast<char*>(ws) + kWorkspaceBytes);
      const char* name = nullptr;
      int r = try_compress_fast(c, g, x, x_type, N, F, s, false, &name, tile_sums);
      if (r < 0) return r;
      // tiles follow the block grid's order, so the tiles of one index along dimension 0 are consecutive
      if (r > 0) return launch_statistics_from_tiles(c, g.n_blocks / segments, tile_sums, tiles / segments, segments,
                                                     statistics, ws, s);
    } else if (tiles > 0) {
      return PBZ_ERR_WORKSPACE;
    }
  }
  // no specialised kernel: compress, then one pass over {N, F} for the two sums
  st = pbz_compress(c, x, x_type, shape, N, F, stream);
  if (st != PBZ_OK) return st;
  return launch_reduce(c, kStatistics, g.n_blocks / segments, N, F, nullptr, nullptr, statistics, ws, s, nullptr,
                       segments);
}

int pbz_decompress(const pbz_codec* c, const void* N, const void* F, const int64_t* shape, void* y,
                   pbz_ftype y_type, void* stream) {
  if (!c || !N || !F || !shape || !y) return PBZ_ERR_NULL;
  if (!valid_ftype(y_type)) return PBZ_ERR_TYPE;
  Geom g;
  int st = make_geom(c, shape, &g);
  if (st != PBZ_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  c->used.store(true);
  if (c->path == PBZ_PATH_AUTO) {
    const char* name = nullptr;
    int r = try_decompress_fast(c, g, N, F, y, y_type, s, false, &name);
    if (r != 0) return r < 0 ? r : PBZ_OK;
  }
  const DeviceTables* t = nullptr;
  st = ensure_tables(c, &t);
  if (st != PBZ_OK) return st;
  if (tiled_kernels_cover(c)) return launch_decompress_tiled(c, g, t, N, F, y, y_type, s);
  return launch_decompress_generic(c, g, t, N, F, y, y_type, s);
}

const char* pbz_kernel_name(const pbz_codec* c, const char* op, const int64_t* shape, pbz_ftype array_type) {
  if (!c || !op || !shape || !valid_ftype(array_type)) return nullptr;
  Geom g;
  if (make_geom(c, shape, &g) != PBZ_OK) return nullptr;
  const char* name = "generic";
  if (c->path == PBZ_PATH_AUTO) {
    // dry runs only inspect the geometry; a non-null dummy pointer stands in for the 16-byte-aligned buffers
    void* aligned = reinterpret_cast<void*>(uintptr_t(256));
    const char* fast = nullptr;
    int r = 0;
    if (std::strcmp(op, "compress") == 0)
      r = try_compress_fast(c, g, aligned, array_type, aligned, aligned, nullptr, true, &fast);
    else if (std::strcmp(op, "decompress") == 0)
      r = try_decompress_fast(c, g, aligned, aligned, aligned, array_type, nullptr, true, &fast);
    else
      return nullptr;
    if (r == 1 && fast) name = fast;
  } else if (std::strcmp(op, "compress") != 0 && std::strcmp(op, "decompress") != 0) {
    return nullptr;
  }
  return name;
}

int pbz_negate(const pbz_codec* c, int64_t n_blocks, const void* F_in, void* F_out, void* stream) {
  if (!c || !F_in || !F_out) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  return launch_negate(c, n_blocks, F_in, F_out, static_cast<hipStream_t>(stream));
}

int pbz_mul_scalar(const pbz_codec* c, int64_t n_blocks, const void* N_in, const void* F_in, double x,
                   void* N_out, void* F_out, void* stream) {
  if (!c || !N_in || !F_in || !N_out || !F_out) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (!std::isfinite(x)) return PBZ_ERR_SCALAR;
  return launch_mul_scalar(c, n_blocks, N_in, F_in, x, N_out, F_out, static_cast<hipStream_t>(stream));
}

int pbz_add(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
            void* N_out, void* F_out, void* stream) {
  if (!c || !N1 || !F1 || !N2 || !F2 || !N_out || !F_out) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  return launch_add(c, n_blocks, N1, F1, N2, F2, N_out, F_out, static_cast<hipStream_t>(stream));
}

int pbz_subtract(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
                 void* N_out, void* F_out, void* stream) {
  if (!c || !N1 || !F1 || !N2 || !F2 || !N_out || !F_out) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  return launch_add(c, n_blocks, N1, F1, N2, F2, N_out, F_out, static_cast<hipStream_t>(stream), -1.0);
}

static int reduce2(const pbz_codec* c, ReduceOp op, int64_t n_blocks, const void* N1, const void* F1,
                   const void* N2, const void* F2, double* out, void* ws, size_t ws_bytes, void* stream,
                   bool two, bool needs_dc) {
  if (!c || !N1 || !F1 || !out || !ws) return PBZ_ERR_NULL;
  if (two && (!N2 || !F2)) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (needs_dc && !c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (ws_bytes < kWorkspaceBytes || (reinterpret_cast<uintptr_t>(ws) & 15u)) return PBZ_ERR_WORKSPACE;
  return launch_reduce(c, op, n_blocks, N1, F1, two ? N2 : nullptr, two ? F2 : nullptr, out, ws,
                       static_cast<hipStream_t>(stream));
}

int pbz_dot(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
            double* out, void* ws, size_t ws_bytes, void* stream) {
  return reduce2(c, kDot, n_blocks, N1, F1, N2, F2, out, ws, ws_bytes, stream, true, false);
}
int pbz_covariance(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                   const void* F2, double* out, void* ws, size_t ws_bytes, void* stream) {
  return reduce2(c, kCovariance, n_blocks, N1, F1, N2, F2, out, ws, ws_bytes, stream, true, true);
}
int pbz_cosine_similarity(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                          const void* F2, double* out, void* ws, size_t ws_bytes, void* stream) {
  return reduce2(c, kCosine, n_blocks, N1, F1, N2, F2, out, ws, ws_bytes, stream, true, false);
}
int pbz_norm2(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out, void* ws,
              size_t ws_bytes, void* stream) {
  return reduce2(c, kNorm2, n_blocks, N, F, nullptr, nullptr, out, ws, ws_bytes, stream, false, false);
}
int pbz_difference_norm2(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                         const void* F2, double* out, void* ws, size_t ws_bytes, void* stream) {
  return reduce2(c, kDiffNorm2, n_blocks, N1, F1, N2, F2, out, ws, ws_bytes, stream, true, false);
}
int pbz_mean(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out, void* ws,
             size_t ws_bytes, void* stream) {
  return reduce2(c, kMean, n_blocks, N, F, nullptr, nullptr, out, ws, ws_bytes, stream, false, true);
}
int pbz_statistics(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* statistics, void* ws,
                   size_t ws_bytes, void* stream) {
  return reduce2(c, kStatistics, n_blocks, N, F, nullptr, nullptr, statistics, ws, ws_bytes, stream, false, true);
}

int pbz_pair_statistics(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                        const void* F2, double* statistics, void* ws, size_t ws_bytes, void* stream) {
  return reduce2(c, kPairStatistics, n_blocks, N1, F1, N2, F2, statistics, ws, ws_bytes, stream, true, true);
}

int pbz_variance(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out, void* ws,
                 size_t ws_bytes, void* stream) {
  return reduce2(c, kVariance, n_blocks, N, F, nullptr, nullptr, out, ws, ws_bytes, stream, false, true);
}

int pbz_segmented(const pbz_codec* c, pbz_statistic stat, int64_t n_segments, int64_t blocks_per_segment, const void* N1,
                  const void* F1, const void* N2, const void* F2, double* out, void* ws, size_t ws_bytes, void* stream) {
  if (!c || !N1 || !F1 || !out || !ws) return PBZ_ERR_NULL;
  if (int(stat) < 0 || int(stat) > int(PBZ_STAT_DIFFERENCE_NORM2)) return PBZ_ERR_TYPE;
  const bool two = stat == PBZ_STAT_DOT || stat == PBZ_STAT_COSINE_SIMILARITY || stat == PBZ_STAT_COVARIANCE ||
                   stat == PBZ_STAT_DIFFERENCE_NORM2;
  const bool needs_dc = stat == PBZ_STAT_MEAN || stat == PBZ_STAT_COVARIANCE || stat == PBZ_STAT_VARIANCE;
  if (two && (!N2 || !F2)) return PBZ_ERR_NULL;
  int st = check_blocks(c, blocks_per_segment);
  if (st != PBZ_OK) return st;
  if (n_segments < 1 || n_segments > (int64_t(1) << 40) / c->vol / blocks_per_segment) return PBZ_ERR_SHAPE;
  if (needs_dc && !c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (ws_bytes < kWorkspaceBytes || (reinterpret_cast<uintptr_t>(ws) & 15u)) return PBZ_ERR_WORKSPACE;
  const ReduceOp op = stat == PBZ_STAT_DIFFERENCE_NORM2 ? kDiffNorm2 : ReduceOp(int(stat));
  return launch_reduce(c, op, blocks_per_segment, N1, F1, two ? N2 : nullptr, two ? F2 : nullptr, out,
                       ws, static_cast<hipStream_t>(stream), nullptr, n_segments);
}

int pbz_approximate_wasserstein_workspace(const pbz_codec* c, int64_t n_blocks, size_t* bytes) {
  if (!bytes) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (n_blocks >= (int64_t(1) << 31)) return PBZ_ERR_SHAPE;      // the sort counts positions in 32 bits
  *bytes = wasserstein_workspace_bytes(n_blocks);
  return PBZ_OK;
}

int pbz_approximate_wasserstein(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                                const void* F2, double p, double* out, void* ws, size_t ws_bytes, void* stream) {
  if (!c || !N1 || !F1 || !N2 || !F2 || !out || !ws) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (n_blocks >= (int64_t(1) << 31)) return PBZ_ERR_SHAPE;
  if (!std::isfinite(p) || p < 1.0) return PBZ_ERR_SCALAR;
  if (!c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (ws_bytes < wasserstein_workspace_bytes(n_blocks) || (reinterpret_cast<uintptr_t>(ws) & 15u))
    return PBZ_ERR_WORKSPACE;
  return launch_approximate_wasserstein(c, n_blocks, N1, F1, N2, F2, p, out, ws, static_cast<hipStream_t>(stream));
}

int pbz_add_scalar(const pbz_codec* c, int64_t n_blocks, const void* N_in, const void* F_in, double x, void* N_out,
                   void* F_out, void* stream) {
  if (!c || !N_in || !F_in || !N_out || !F_out) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (!std::isfinite(x)) return PBZ_ERR_SCALAR;
  if (!c->dc_kept) return PBZ_ERR_DC_PRUNED;
  return launch_add_scalar(c, n_blocks, N_in, F_in, x, N_out, F_out, static_cast<hipStream_t>(stream));
}

int pbz_ssim(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2, const void* F2,
             double s_l, double s_c, double w_l, double w_c, double w_s, double* out, void* ws, size_t ws_bytes,
             void* stream) {
  if (!c || !N1 || !F1 || !N2 || !F2 || !out || !ws) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (!std::isfinite(s_l) || !std::isfinite(s_c) || !std::isfinite(w_l) || !std::isfinite(w_c) || !std::isfinite(w_s))
    return PBZ_ERR_SCALAR;
  if (!c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (ws_bytes < kWorkspaceBytes || (reinterpret_cast<uintptr_t>(ws) & 15u)) return PBZ_ERR_WORKSPACE;
  const double params[5] = {s_l, s_c, w_l, w_c, w_s};
  return launch_reduce(c, kSsim, n_blocks, N1, F1, N2, F2, out, ws, static_cast<hipStream_t>(stream), params);
}

static int blockwise(const pbz_codec* c, int mode, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                     const void* F2, double* out, void* stream) {
  if (!c || !N1 || !F1 || !out) return PBZ_ERR_NULL;
  if (mode == 2 && (!N2 || !F2)) return PBZ_ERR_NULL;
  int st = check_blocks(c, n_blocks);
  if (st != PBZ_OK) return st;
  if (!c->dc_kept) return PBZ_ERR_DC_PRUNED;
  if (mode < 0) return launch_blockwise_mean(c, n_blocks, N1, F1, out, static_cast<hipStream_t>(stream));
  return launch_blockwise(c, mode, n_blocks, N1, F1, N2, F2, out, static_cast<hipStream_t>(stream));
}

int pbz_blockwise_mean(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out, void* stream) {
  return blockwise(c, -1, n_blocks, N, F, nullptr, nullptr, out, stream);
}
int pbz_blockwise_variance(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out,
                           void* stream) {
  return blockwise(c, 0, n_blocks, N, F, nullptr, nullptr, out, stream);
}
int pbz_blockwise_std(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out, void* stream) {
  return blockwise(c, 1, n_blocks, N, F, nullptr, nullptr, out, stream);
}
int pbz_blockwise_covariance(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                             const void* F2, double* out, void* stream) {
  return blockwise(c, 2, n_blocks, N1, F1, N2, F2, out, stream);
}

const char* pbz_status_string(int status) {
  switch (status) {
    case PBZ_OK: return "ok";
    case PBZ_ERR_NULL: return "a required pointer is NULL";
    case PBZ_ERR_NDIM: return "ndim must be between 1 and 8";
    case PBZ_ERR_BLOCK_SHAPE:
      return "block extents must be powers of two, at most 256 each and 4096 elements per block";
    case PBZ_ERR_TYPE: return "unknown or unsupported float / index type";
    case PBZ_ERR_MASK_EMPTY: return "the pruning mask keeps no coefficient";
    case PBZ_ERR_DC_PRUNED: return "the first coefficient of each block is pruned; mean/variance/covariance need it";
    case PBZ_ERR_SHAPE: return "array extents and n_blocks must be >= 1 and sizes must not overflow";
    case PBZ_ERR_WORKSPACE: return "workspace is too small or not 16-byte aligned";
    case PBZ_ERR_SCALAR: return "scalar must be finite";
    case PBZ_ERR_HIP: return "HIP runtime error";
    case PBZ_ERR_ALLOC: return "host allocation failed";
    case PBZ_ERR_STATE: return "too late in the handle's life for this call";
    case PBZ_ERR_CAPACITY:
      return "input beyond the capacity of the library's fixed scratch array (at most 4096 segments and 2^40 elements)";
    default: return "unknown status";
  }
}

}  // extern "C"
