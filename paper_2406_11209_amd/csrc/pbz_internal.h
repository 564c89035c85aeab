// Internal declarations shared by the host API and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <atomic>
#include <mutex>

#include "pbz.h"

namespace pbz {

constexpr int kMaxDevices = 16;
constexpr int kReducePartialSlots = 8;      // doubles per workgroup partial
constexpr int kReduceMaxGroups = 4096;      // upper bound on reduction workgroups
constexpr size_t kWorkspaceBytes = size_t(kReduceMaxGroups) * kReducePartialSlots * sizeof(double);

// Per-device constant tables, created lazily at the first launch.
struct DeviceTables {
  bool ready = false;
  double* H = nullptr;          // concatenated forward matrices H_d[m][q], row-major, one per dimension
  int32_t* kept_pos = nullptr;  // [vol] position in F of intra-block entry j, or -1 when pruned
  int32_t* kept_list = nullptr; // [kept] intra-block entry stored at position pos of F (the inverse of kept_pos)
};

}  // namespace pbz

struct pbz_codec {
  int ndim;
  int64_t block[PBZ_MAX_NDIM];
  int vol;              // prod(block)
  pbz_ftype ftype;      // working type f: storage type of N
  pbz_itype itype;
  int index_bits;
  double r;             // index radius 2^(bits-1) - 1
  bool compute_f64;     // transform and binning precision
  uint8_t* mask;        // [vol] 0/1
  int32_t* kept_pos;    // [vol]
  int32_t* kept_list;   // [kept]
  int kept;             // sum(P)
  bool dc_kept;
  int box[PBZ_MAX_NDIM];  // mask == low-frequency corner box of these extents (box[0] = 0 when it is not)
  int h_offset[PBZ_MAX_NDIM];
  int h_total;
  double* H_host;       // concatenated matrices
  pbz_kernel_path path;
  int transform;        // pbz_transform
  mutable std::atomic<bool> used{false};   // a compress / decompress has been issued: the transform is fixed from then on
  mutable std::mutex mu;
  mutable pbz::DeviceTables dev[pbz::kMaxDevices];
};

namespace pbz {

inline int ftype_bytes(int t) { return t == PBZ_F64 ? 8 : t == PBZ_F32 ? 4 : 2; }
inline int itype_bytes(int t) { return 1 << t; }

// Geometry of one compress / decompress call, passed to kernels by value.
struct Geom {
  int ndim;
  int vol;
  int kept;
  int pad_;
  int64_t n_blocks;
  int64_t shape[PBZ_MAX_NDIM];
  int64_t stride[PBZ_MAX_NDIM];
  int64_t grid[PBZ_MAX_NDIM];
  int32_t block[PBZ_MAX_NDIM];
  int32_t h_offset[PBZ_MAX_NDIM];
};

int ensure_tables(const pbz_codec* c, const DeviceTables** out);

// generic kernels (any ndim, any power-of-two block shape within the limits, any types)
// general kernels for block extents up to 32 (in-register transforms on LDS tiles); the dense ones below take the rest
bool tiled_kernels_cover(const pbz_codec* c);
int launch_compress_tiled(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* x, int xtype, void* N,
                          void* F, hipStream_t s);
int launch_decompress_tiled(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* N, const void* F,
                            void* y, int ytype, hipStream_t s);
int launch_compress_generic(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* x, int xtype,
                            void* N, void* F, hipStream_t s);
int launch_decompress_generic(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* N,
                              const void* F, void* y, int ytype, hipStream_t s);

// specialised codec kernels; return 1 when they handled the call, 0 when the shape / types are not
// covered (caller falls back to the generic kernels), negative on a HIP error
// tile_sums != nullptr: the kernel also leaves two FP64 sums per tile (wave) there, fast_compress_tiles() pairs
// in all, from which launch_statistics_from_tiles() makes the mean, variance and L2 norm of the compressed array
int try_compress_fast(const pbz_codec* c, const Geom& g, const void* x, int xtype, void* N, void* F,
                      hipStream_t s, bool dry_run, const char** name, double* tile_sums = nullptr);
int64_t fast_compress_tiles(const pbz_codec* c, const Geom& g, int xtype);   // 0: no specialised kernel covers it
int try_decompress_fast(const pbz_codec* c, const Geom& g, const void* N, const void* F, void* y, int ytype,
                        hipStream_t s, bool dry_run, const char** name);

// element-wise compressed-space operations
int launch_negate(const pbz_codec* c, int64_t n_blocks, const void* Fin, void* Fout, hipStream_t s);
int launch_mul_scalar(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double x,
                      void* Nout, void* Fout, hipStream_t s);
int launch_add(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
               const void* F2, void* Nout, void* Fout, hipStream_t s, double sign2 = 1.0);   // sign2 = -1: A - B

enum ReduceOp { kDot = 0, kNorm2 = 1, kCosine = 2, kMean = 3, kCovariance = 4, kVariance = 5, kSsim = 6,
                kDiffNorm2 = 7, kStatistics = 8 /* out[0..3) = mean, variance, norm2 from one pass */,
                kPairStatistics = 9 /* out[0..9): see pbz_pair_statistics */ };
// ssim_params: {s_l, s_c, w_l, w_c, w_s} for kSsim, otherwise nullptr.  n_segments > 1: the operands are
// n_segments consecutive runs of n_blocks blocks, one result per run goes to out[0 .. n_segments).
int launch_reduce(const pbz_codec* c, ReduceOp op, int64_t n_blocks, const void* N1, const void* F1,
                  const void* N2, const void* F2, double* out, void* workspace, hipStream_t s,
                  const double* ssim_params = nullptr, int64_t n_segments = 1);
// n_segments runs of tiles_per_segment tiles (blocks_per_segment blocks) each: out[3 t .. 3 t + 3) for run t
int launch_statistics_from_tiles(const pbz_codec* c, int64_t blocks_per_segment, const double* tile_sums,
                                 int64_t tiles_per_segment, int64_t n_segments, double* out, void* workspace,
                                 hipStream_t s);
// Algorithm 13; workspace of wasserstein_workspace_bytes(n_blocks) bytes
size_t wasserstein_workspace_bytes(int64_t n_blocks);
int launch_approximate_wasserstein(const pbz_codec* c, int64_t n_blocks, const void* N1, const void* F1,
                                   const void* N2, const void* F2, double order, double* out, void* workspace,
                                   hipStream_t s);
int launch_add_scalar(const pbz_codec* c, int64_t n_blocks, const void* Nin, const void* Fin, double x, void* Nout,
                      void* Fout, hipStream_t s);
int launch_blockwise_mean(const pbz_codec* c, int64_t n_blocks, const void* N, const void* F, double* out,
                          hipStream_t s);
int launch_blockwise(const pbz_codec* c, int mode, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                     const void* F2, double* out, hipStream_t s);

inline int hip_status(hipError_t e) { return e == hipSuccess ? PBZ_OK : PBZ_ERR_HIP; }

}  // namespace pbz
