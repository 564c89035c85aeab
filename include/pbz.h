/*
 * pbz -- blockwise orthonormal-transform codec and compressed-space operations for
 * AMD Instinct MI355X (gfx950).  C ABI.
 *
 * The method is the one of arXiv 2406.11209 ("What Operations can be Performed Directly on
 * Compressed Arrays, and with What Error?"); citations below name that paper's sections,
 * algorithms and tables.
 *
 * A compressed array is the tuple {s, i, N, F} of Sec. III-B:
 *   s  original shape                      (host, passed to the calls that need it)
 *   i  block shape                         (fixed by the codec handle)
 *   N  biggest coefficient of every block  (device; one working-type float per block, row-major
 *                                           over the block grid b = ceil(s / i))
 *   F  kept bin indices                    (device; block-major [block][kept index], kept indices in
 *                                           row-major order of the intra-block coordinate)
 * plus the pruning mask P and the two type tags, which live in the codec handle.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device pointers on the current device; "host" pointers are ordinary
 *     host memory read during the call.  The library never takes ownership of caller memory.
 *   - Arrays are contiguous, row-major (last dimension fastest).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All device work is
 *     enqueued on it and the call returns without synchronising; scalar results are written to
 *     device memory by the enqueued work.
 *   - The return value is PBZ_OK or a negative pbz_status.  All argument checks happen on the host
 *     before anything is launched, so a failing call has touched no device memory.  Nothing throws
 *     or aborts across this boundary.
 *   - The only device memory the library allocates is a few small constant tables (transform
 *     matrices, kept-position table) owned by the codec handle, created at the first launch that
 *     needs them and released by pbz_codec_destroy.
 *   - Non-finite input values are a precondition violation: results are unspecified (no trap).
 *
 * Arithmetic precision.  The working float type f (Sec. III-A, "Data type conversion") is the storage
 * type of N.  The transform and the binning decision are carried out in FP32 only when f is FP32 (or a
 * 16-bit type) and the index type is int8; for every wider index type, and for f = FP64, they are
 * carried out in FP64, because an FP32 transform error of a few 1e-7 N shifts r*C/N by more than the
 * allowed index mismatch rate once r >= 32767.  Element-wise addition always rebins in FP64.
 * Reductions multiply integer block sums by N in FP64 and accumulate in FP64 in a fixed order (results
 * are bit-reproducible run to run).
 */
#ifndef PBZ_H
#define PBZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The enumerations below are plain ints at the ABI.  A C++ caller sees them with a fixed underlying type, so that a
 * value outside the list, which every entry point answers with an error status, is an ordinary int there too. */
#ifdef __cplusplus
#define PBZ_ENUM : int
#else
#define PBZ_ENUM
#endif

#define PBZ_MAX_NDIM 8
#define PBZ_MAX_BLOCK_EXTENT 256   /* per-dimension block extent limit */
#define PBZ_MAX_BLOCK_VOLUME 4096  /* elements per block limit */

/* Float types of Sec. III-A ("Data type conversion"): array element types and the working type f. */
typedef enum PBZ_ENUM { PBZ_F64 = 0, PBZ_F32 = 1, PBZ_BF16 = 2, PBZ_F16 = 3 } pbz_ftype;
/* Bin index types of Sec. III-A ("Binning"); the index radius is r = 2^(bits-1) - 1.
 * PBZ_I64 is declared because the paper lists it, but is rejected with PBZ_ERR_TYPE: its radius is not
 * representable in FP64. */
typedef enum PBZ_ENUM { PBZ_I8 = 0, PBZ_I16 = 1, PBZ_I32 = 2, PBZ_I64 = 3 } pbz_itype;

typedef enum PBZ_ENUM {
  PBZ_OK = 0,
  PBZ_ERR_NULL = -1,        /* a required pointer is NULL */
  PBZ_ERR_NDIM = -2,        /* ndim outside 1..PBZ_MAX_NDIM */
  PBZ_ERR_BLOCK_SHAPE = -3, /* a block extent is not a power of two, or exceeds the limits above */
  PBZ_ERR_TYPE = -4,        /* unknown or unsupported float / index type */
  PBZ_ERR_MASK_EMPTY = -5,  /* the pruning mask keeps nothing */
  PBZ_ERR_DC_PRUNED = -6,   /* mean / variance / covariance need the first coefficient of each block */
  PBZ_ERR_SHAPE = -7,       /* an array extent or n_blocks is < 1, or sizes overflow */
  PBZ_ERR_WORKSPACE = -8,   /* workspace smaller than pbz_layout reports */
  PBZ_ERR_SCALAR = -9,      /* non-finite scalar */
  PBZ_ERR_HIP = -10,        /* the HIP runtime reported an error (no device, launch failure, ...) */
  PBZ_ERR_ALLOC = -11,      /* host allocation failed */
  PBZ_ERR_STATE = -12,      /* the call comes too late in the handle's life (see pbz_codec_set_transform) */
  PBZ_ERR_CAPACITY = -13    /* the input exceeds what the library's fixed scratch array serves (pbz_segmented_static) */
} pbz_status;

/* Kernel families, for pbz_codec_set_kernel_path / pbz_kernel_name. */
typedef enum PBZ_ENUM { PBZ_PATH_AUTO = 0, PBZ_PATH_GENERIC = 1 } pbz_kernel_path;

typedef struct pbz_codec pbz_codec; /* opaque compression settings (Sec. III-A): i, f, index type, P */

/* Create the settings object: block shape i (each extent a power of two, possibly non-hypercubic;
 * Sec. III-A "Blocking"), working float type f, index type, pruning mask P (Sec. III-A "Pruning").
 *   block_shape  host, ndim entries.
 *   mask         host, prod(block_shape) bytes, row-major over the block, non-zero = keep; NULL keeps all.
 * Needs no GPU.  On success *out owns the handle; release it with pbz_codec_destroy. */
int pbz_codec_create(pbz_codec** out, int ndim, const int64_t* block_shape, pbz_ftype work_type,
                     pbz_itype index_type, const uint8_t* mask);
void pbz_codec_destroy(pbz_codec* codec);

/* The orthonormal transform of Sec. III-A step 3: the DCT-II (the default) or the Haar wavelet transform that
 * the same passage names as an alternative (orthonormal Haar basis in sequency order: coefficient 0 is the block
 * sum over sqrt(n); coefficient 2^p + j is +-sqrt(2^p / n) on the two halves of the j-th run of n / 2^p samples).
 * Both have a constant first basis function, so every operation of Sec. IV-A applies unchanged.  Arrays
 * compressed under different transforms must not be combined.  Must be called before the handle's first
 * compress / decompress (its per-device tables are built then): PBZ_ERR_STATE afterwards.  Needs no GPU. */
typedef enum PBZ_ENUM { PBZ_TRANSFORM_DCT = 0, PBZ_TRANSFORM_HAAR = 1 } pbz_transform;
int pbz_codec_set_transform(pbz_codec* codec, pbz_transform transform);

/* Force the general kernels (PBZ_PATH_GENERIC) instead of the ones specialised to a block shape; for testing. */
int pbz_codec_set_kernel_path(pbz_codec* codec, pbz_kernel_path path);

/* Sizes of the compressed form of an array of shape `shape` (host, ndim entries): number of blocks
 * prod(ceil(s / i)), kept indices per block sum(P), bytes of N and of F, and the bytes of scratch the
 * reduction entry points need (independent of shape).  Any output pointer may be NULL.  Needs no GPU. */
int pbz_layout(const pbz_codec* codec, const int64_t* shape, int64_t* n_blocks, int64_t* kept_per_block,
               size_t* n_bytes, size_t* f_bytes, size_t* workspace_bytes);

/* Storage of the serialised compressed form in bits, following the component list of Sec. IV-C:
 * 4 (type tags) + 64 d (s) + 64 (end marker) + 64 d (i) + prod(i) (P) + f prod(b) (N) + bits sum(P) prod(b) (F).
 * Needs no GPU. */
int pbz_compressed_bits(const pbz_codec* codec, const int64_t* shape, uint64_t* bits);

/* Sec. III-A, all five steps fused: convert x to the compute type, tile into blocks (zero padding at the
 * high end of each dimension), orthonormal DCT-II along every block dimension, N_k = max |C_k| over the
 * whole block, I = rint(r C / N_k) (ties to even; an all-zero block gives N = 0, I = 0), F = I[P].
 *   x       device, prod(shape) elements of x_type.
 *   N, F    device, sizes from pbz_layout; written. */
int pbz_compress(const pbz_codec* codec, const void* x, pbz_ftype x_type, const int64_t* shape, void* N,
                 void* F, void* stream);

/* Compression as pbz_compress plus, from the same pass over x, the statistics of the compressed array that a
 * time-series analysis takes of every step (Sec. V): statistics (device, FP64, written) receives the triple
 * {mean (Algorithm 7), variance (Algorithm 9), L2 norm (Algorithm 10)}, the values pbz_mean, pbz_variance and
 * pbz_norm2 return for the {N, F} produced, up to FP64 summation order, without reading {N, F} back.
 *   per_step    0: one triple for the whole array (3 values).  Non-zero: one triple per block index along
 *               dimension 0, i.e. per run of prod(b[1:]) consecutive blocks, 3 * ceil(shape[0] / block[0]) values,
 *               triple t at statistics[3 t]; with block extent 1 along time these are the statistics of every time
 *               step (what pbz_segmented returns for the runs of {N, F}).
 * Requires the mask to keep each block's first coefficient (PBZ_ERR_DC_PRUNED otherwise).
 *   workspace   device, 16-byte aligned, at least the bytes pbz_compress_statistics_workspace reports for this
 *               shape and x_type (the reduction scratch plus four FP64 values per wave of the compress kernel);
 *               contents on entry do not matter; PBZ_ERR_WORKSPACE when too small or misaligned. */
int pbz_compress_statistics_workspace(const pbz_codec* codec, const int64_t* shape, pbz_ftype x_type,
                                      size_t* bytes);
int pbz_compress_statistics(const pbz_codec* codec, const void* x, pbz_ftype x_type, const int64_t* shape, void* N,
                            void* F, int per_step, double* statistics, void* workspace, size_t workspace_bytes,
                            void* stream);

/* Sec. III-B: C = N F / r at the mask positions and zero elsewhere, inverse transform, merge blocks,
 * crop to `shape`, convert to y_type (round to nearest even).
 *   y       device, prod(shape) elements of y_type; written. */
int pbz_decompress(const pbz_codec* codec, const void* N, const void* F, const int64_t* shape, void* y,
                   pbz_ftype y_type, void* stream);

/* Algorithm 1: F_out = -F_in (N is unchanged and not touched).  F_out may alias F_in. */
int pbz_negate(const pbz_codec* codec, int64_t n_blocks, const void* F_in, void* F_out, void* stream);

/* Algorithm 5: N_out = N_in |x| (rounded to f), F_out = F_in sign(x) with sign(0) = 0.
 * Outputs may alias the corresponding inputs. */
int pbz_mul_scalar(const pbz_codec* codec, int64_t n_blocks, const void* N_in, const void* F_in, double x,
                   void* N_out, void* F_out, void* stream);

/* Algorithm 2: per block C = F1 N1 + F2 N2, N = max|C| / r, F = rint(C / N) (N = 0 gives F = 0).
 * Both operands must come from this codec and the same array shape.  Outputs may alias an operand. */
int pbz_add(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
            const void* F2, void* N_out, void* F_out, void* stream);

/* A - B, the compressed-space difference of Sec. V (shallow-water experiment: "negation and element-wise
 * addition"), in one pass: Algorithm 2 applied to A and Algorithm 1's negation of B without writing the
 * negated array; bit for bit the result of pbz_negate followed by pbz_add.  Arguments as for pbz_add. */
int pbz_subtract(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                 const void* F2, void* N_out, void* F_out, void* stream);

/* Reductions.  Each writes one FP64 scalar to out (device).  `workspace` is device scratch of at least the
 * size pbz_layout reports, 16-byte aligned; its contents on entry do not matter.  Calls that may run
 * concurrently must use distinct workspaces.
 *   pbz_dot                Algorithm 6   sum(C1 . C2)
 *   pbz_norm2              Algorithm 10  ||C||_2
 *   pbz_cosine_similarity  Algorithm 11  dot / (||A|| ||B||)
 *   pbz_mean               Algorithm 7   mean of the first coefficients / prod(sqrt(i))
 *   pbz_covariance         Algorithm 8   first coefficients centred by their mean over blocks, then
 *                                        sum(C1 . C2) / (n_blocks prod(i))
 *   pbz_variance           Algorithm 9   covariance(A, A)
 * mean, covariance and variance return PBZ_ERR_DC_PRUNED when P drops the first coefficient (Sec. IV-A).
 * n_blocks may be a sub-range of an array's blocks (e.g. one time step of a series). */
int pbz_dot(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
            const void* F2, double* out, void* workspace, size_t workspace_bytes, void* stream);
int pbz_covariance(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                   const void* F2, double* out, void* workspace, size_t workspace_bytes, void* stream);
int pbz_cosine_similarity(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1,
                          const void* N2, const void* F2, double* out, void* workspace,
                          size_t workspace_bytes, void* stream);
int pbz_norm2(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
              void* workspace, size_t workspace_bytes, void* stream);
/* {mean, variance, L2 norm} (Algorithms 7, 9, 10) of one compressed array from a single pass over {N, F}:
 * statistics (device) receives 3 FP64 values.  Other arguments as for pbz_variance. */
int pbz_statistics(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* statistics,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Every statistic of Algorithms 6-11 of a pair of compressed arrays from a single pass over both: the five sums
 * that pass takes (sum C1.C2, sum C1.C1, sum C2.C2 and the two sums of first coefficients) determine them all, so
 * a caller that wants several (as Algorithm 12 does internally) pays for one.  statistics (device) receives 9 FP64
 * values: {dot, cosine similarity, covariance, mean_A, mean_B, variance_A, variance_B, norm_A, norm_B}, each the
 * value its own entry point returns up to FP64 summation order.  Needs the first coefficient of every block
 * (PBZ_ERR_DC_PRUNED otherwise).  Other arguments as for pbz_dot. */
int pbz_pair_statistics(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                        const void* F2, double* statistics, void* workspace, size_t workspace_bytes, void* stream);

/* ||A - B||_2 of two compressed arrays (the quantity compared between adjacent time steps in Sec. V, fission
 * experiment), taken on the specified coefficients of Algorithm 3: sqrt(sum_kj (N1_k F1_kj - N2_k F2_kj)^2) / r,
 * each difference formed in FP64 before squaring.  The transform being orthonormal, this is the L2 norm of the
 * difference of the two decompressed (uncropped) arrays; no intermediate compressed array and no second binning,
 * unlike negate + add + norm2.  Arguments as for pbz_dot. */
int pbz_difference_norm2(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
                         const void* F2, double* out, void* workspace, size_t workspace_bytes, void* stream);
int pbz_mean(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
             void* workspace, size_t workspace_bytes, void* stream);
int pbz_variance(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Segmented reductions: the operands are n_segments consecutive runs of blocks_per_segment blocks each (e.g. the
 * time steps of a series compressed with block extent 1 along time); out (device) receives n_segments FP64
 * values, out[t] being the statistic of run t of operand 1 (and run t of operand 2).  Two launches for any
 * number of segments instead of two per segment.  The covariance of consecutive steps of one series (or the
 * norm of their difference) is obtained by passing N2 / F2 = N1 / F1 advanced by one run and n_segments reduced
 * by one.  N2 / F2 are ignored (may be NULL) for norm2, mean and variance.  Workspace as for the plain reductions. */
typedef enum PBZ_ENUM {
  PBZ_STAT_DOT = 0, PBZ_STAT_NORM2 = 1, PBZ_STAT_COSINE_SIMILARITY = 2, PBZ_STAT_MEAN = 3, PBZ_STAT_COVARIANCE = 4,
  PBZ_STAT_VARIANCE = 5, PBZ_STAT_DIFFERENCE_NORM2 = 6
} pbz_statistic;
int pbz_segmented(const pbz_codec* codec, pbz_statistic statistic, int64_t n_segments, int64_t blocks_per_segment,
                  const void* N1, const void* F1, const void* N2, const void* F2, double* out, void* workspace,
                  size_t workspace_bytes, void* stream);

/* pbz_segmented for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same statistics, arguments and results (bit for bit) as pbz_segmented, without
 * the workspace: the partial sums go to a 256 KiB array inside the library's device image, of which every GPU the
 * library runs on holds one copy until the process ends.  The call itself allocates and frees nothing on the host
 * or the device and enqueues kernels only (no memset or copy nodes).  The array's device address is looked up at
 * the first call on each device, so make that call outside graph capture.
 *   n_segments   at most PBZ_STATIC_MAX_SEGMENTS, and n_segments * blocks_per_segment * prod(i) at most
 *                PBZ_STATIC_MAX_ELEMENTS: PBZ_ERR_CAPACITY beyond either (use pbz_segmented with a workspace).
 *   n_segments = 1 gives the plain reductions (pbz_dot, pbz_norm2, ...).
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different streams,
 * or graphs replayed concurrently) race on it and return garbage; calls ordered by a stream or by graph
 * dependencies are safe.  Nothing has to be cleared between calls: every record read has been written by the
 * same call. */
#define PBZ_STATIC_MAX_SEGMENTS 4096
#define PBZ_STATIC_MAX_ELEMENTS (INT64_C(1) << 40)
int pbz_segmented_static(const pbz_codec* codec, pbz_statistic statistic, int64_t n_segments,
                         int64_t blocks_per_segment, const void* N1, const void* F1, const void* N2, const void* F2,
                         double* out, void* stream);

/* Algorithm 4 (addition of a scalar): C = N F / r, x prod(sqrt(i)) is added to the first coefficient of every
 * block, then N = max|C| and F = rint(C r / N).  N is taken after the shift (the printed listing takes it
 * before, which lets the first index exceed r).  Needs the first coefficient (PBZ_ERR_DC_PRUNED otherwise).
 * Outputs may alias the inputs. */
int pbz_add_scalar(const pbz_codec* codec, int64_t n_blocks, const void* N_in, const void* F_in, double x,
                   void* N_out, void* F_out, void* stream);

/* Algorithm 12 (structural similarity): l^w_l c^w_c s^w_s with
 *   l = (2 mu_A mu_B + s_l) / (mu_A^2 + mu_B^2 + s_l),  c = (2 sd_A sd_B + s_c) / (var_A + var_B + s_c),
 *   s = (cov_AB + s_c / 2) / (sd_A sd_B + s_c / 2)
 * from the compressed-space mean, variance and covariance (Algorithms 7-9), all taken in one pass over both
 * operands.  One FP64 scalar to out (device); workspace as for the reductions above. */
int pbz_ssim(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1, const void* N2,
             const void* F2, double s_l, double s_c, double w_l, double w_c, double w_s, double* out,
             void* workspace, size_t workspace_bytes, void* stream);

/* Block-wise statistics (Sec. IV-A, the block-wise variants of mean, variance, standard deviation and
 * covariance): out (device) receives n_blocks FP64 values, one per block, in block order.
 *   mean_k       = C_k0 / prod(sqrt(i))
 *   covariance_k = (sum_j C1_kj C2_kj - C1_k0 C2_k0) / prod(i)   (a block centred by its own mean has no first
 *                  coefficient);  variance_k = covariance_k(A, A);  std_k = sqrt(variance_k)
 * All need the first coefficient (PBZ_ERR_DC_PRUNED otherwise). */
int pbz_blockwise_mean(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
                       void* stream);
int pbz_blockwise_variance(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
                           void* stream);
int pbz_blockwise_std(const pbz_codec* codec, int64_t n_blocks, const void* N, const void* F, double* out,
                      void* stream);
int pbz_blockwise_covariance(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1,
                             const void* N2, const void* F2, double* out, void* stream);

/* Algorithm 13 (Sec. IV-A, "Approximate Wasserstein distance"): the block-wise means of both arrays, each passed
 * through softmax unless it already sums to one (taken as |sum - 1| <= 1e-9), are sorted, and
 * (sum |P_A - P_B|^p / n_blocks)^(1/p) goes to out (device, one FP64).  The power sum is scaled by its largest
 * term, which changes nothing in exact arithmetic and keeps the orders the paper uses (p = 68 .. 80) from
 * underflowing.  All work (means, reductions, an 8-bit-digit radix sort of both sequences, power mean) is enqueued
 * on `stream`; nothing is read back to the host.
 *   p           order, finite and >= 1 (PBZ_ERR_SCALAR otherwise).
 *   workspace   device, 16-byte aligned, at least the bytes pbz_approximate_wasserstein_workspace reports for
 *               n_blocks (about 32 bytes per block); contents on entry do not matter.
 * n_blocks must be below 2^31 (PBZ_ERR_SHAPE).  Requires the mask to keep each block's first coefficient. */
int pbz_approximate_wasserstein_workspace(const pbz_codec* codec, int64_t n_blocks, size_t* bytes);
int pbz_approximate_wasserstein(const pbz_codec* codec, int64_t n_blocks, const void* N1, const void* F1,
                                const void* N2, const void* F2, double p, double* out, void* workspace,
                                size_t workspace_bytes, void* stream);

/* A plain copy kernel of known traffic: dst[0 .. bytes) = src[0 .. bytes), both device, 16-byte aligned
 * (PBZ_ERR_WORKSPACE otherwise), not overlapping; bytes between 1 and 2^43 (PBZ_ERR_SHAPE otherwise).  It moves
 * `bytes` in and `bytes` out and nothing else, which makes it the yardstick of the measurements (Sec. IV-E times
 * the method's operations against array size; here they are set against the memory system's own rate): the box's
 * practical streaming bandwidth, and the reference dispatch that hardware-counter readings are scaled by. */
int pbz_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Name of the kernel family pbz_compress ("compress") or pbz_decompress ("decompress") would run for
 * this shape and array type: "generic" or the name of a specialised kernel.  Host only; returns a static
 * string, or NULL on invalid arguments. */
const char* pbz_kernel_name(const pbz_codec* codec, const char* op, const int64_t* shape, pbz_ftype array_type);

/* Human-readable text for a status code (static string, never NULL). */
const char* pbz_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PBZ_H */
