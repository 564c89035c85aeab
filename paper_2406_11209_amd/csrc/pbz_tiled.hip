// General codec kernels for every setting without a specialised kernel whose block extents are at most 32:
// any dimensionality up to 8, any such block shape, any mask, every array / working / index type, any shape.
//
// A workgroup owns a tile of G consecutive blocks (block-major order, so usually neighbours along the last
// dimension), 4096 elements or fewer, in one LDS buffer laid out [block][intra-block index]:
//   load     elements are enumerated (row within the block, block, position in the row), so that consecutive
//            threads read consecutive memory across the blocks of the tile; padding is filled with zeros;
//   passes   one per block dimension, in place: a thread takes whole 1-D lines into registers and applies the
//            in-register transform of that length (Sec. III-A, "Orthonormal transform"; the same even/odd-split DCT
//            or Haar cascade as the specialised kernels), a workgroup barrier between passes;
//   binning  N_k = max |C_k| by LDS atomics on the bit patterns (non-negative floats order like integers),
//            I = rint(r C / N_k) for the kept entries only, enumerated in F order: the tile's part of F is one
//            contiguous run.
// Wherever the layout allows it the array and F are moved in wider units than one element, so that the index
// arithmetic is done once per unit: 16-byte pieces of the array when a block row holds at least one, rows start on
// 16-byte boundaries and the last extent is a multiple of the piece (a piece then lies wholly inside one block row
// and wholly inside or outside the array), and runs of four kept entries of F when the kept count is a multiple of
// four.  Finding an element costs two 16-byte LDS reads (the block's record, the row's record) and one packed
// comparison that tests all dimensions' bounds at once; no branch.  A workgroup takes exactly one tile, so what
// the block decode needs of the geometry is dead before the loops start (with a loop over tiles the compiler kept
// all of it live and spilled scalar registers into vector lanes inside the hottest loops), the loop over the
// dimensions is a real loop (one copy of each pass), and the kernels are built per longest line (8, 16, 32), because
// the pass for a line of 32 FP64 values alone needs 150 registers, the others 42-77.
// 512 x 512 x 256 FP64 in 8 x 8 x 8 blocks, int16: 168 vector instructions per element and 1.1 TB/s moved with
// element-wise accesses, 119 and 2.0-2.2 TB/s with pieces, 58 and 3.2 TB/s as described here.  Taking out
// one part at a time (compress, that case, 0.208 ms): without the passes 0.131 ms, without the array loads
// 0.166 ms, without binning and stores 0.178 ms, with none of them 0.037 ms (launch, block decode, N).
// Decompression mirrors this.  The block -> coordinates decode (divisions by the grid extents) happens once per
// block per tile; the per-element decode is shifts and masks because block extents are powers of two.
#include <type_traits>

#include "pbz_dct.h"
#include "pbz_device.h"
#include "pbz_haar.h"
#include "pbz_internal.h"
#include "pbz_tile_index.h"

namespace pbz {
namespace {

using namespace tile;

constexpr int kThreads = 256;

template <typename T> struct Bits;
template <> struct Bits<float> {
  typedef unsigned int type;
  static __device__ __forceinline__ type of(float v) { return __float_as_uint(v); }
  static __device__ __forceinline__ float from(type b) { return __uint_as_float(b); }
};
template <> struct Bits<double> {
  typedef unsigned long long type;
  static __device__ __forceinline__ type of(double v) { return (unsigned long long)__double_as_longlong(v); }
  static __device__ __forceinline__ double from(type b) { return __longlong_as_double((long long)b); }
};

struct TileBlocks {                           // both in LDS, sized by the tile: G blocks, the rows of one block
  BlockInfo* blk;
  RowInfo* row;                               // filled when a block has at most kMaxRows rows
};

constexpr int kBatch = 8;                     // global loads a thread keeps in flight while filling a tile

template <int kDims>
__device__ __forceinline__ void decode_blocks(const TileGeom& tg, int64_t k0, const TileBlocks& tb) {
  for (int b = threadIdx.x; b < tg.G; b += kThreads) tb.blk[b] = block_info<kDims>(tg, k0 + b);
}

// once per kernel
template <int kDims>
__device__ __forceinline__ void tabulate_rows(const TileGeom& tg, const TileBlocks& tb) {
  const int rows = 1 << (tg.vol_shift - tg.bx_shift);
  if (rows > kMaxRows) return;
  for (int i = threadIdx.x; i < rows; i += kThreads) tb.row[i] = row_info<kDims>(tg, i);
}

// intra-block index j of block b -> element offset; false when the element is padding.  No branch: two 16-byte
// LDS reads, one packed comparison.
template <int kDims>
__device__ __forceinline__ bool locate(const TileGeom& tg, const TileBlocks& tb, int b, int j, int64_t* offset) {
  const int i = j >> tg.bx_shift, xin = j & ((1 << tg.bx_shift) - 1);
  const bool tabulated = (1 << (tg.vol_shift - tg.bx_shift)) <= kMaxRows;     // uniform: the usual case
  const RowInfo r = tabulated ? tb.row[i] : row_info<kDims>(tg, i);
  return locate_in<kDims>(tb.blk[b], r, xin, offset);
}

template <typename T, typename XT>
__device__ __forceinline__ T widen(XT raw) { return T(raw); }
struct bf16_raw { uint16_t bits; };           // bfloat16 arrays are plain bit patterns
template <typename T>
__device__ __forceinline__ T widen_bf16(bf16_raw raw) { return T(bf16_bits_to_float(raw.bits)); }

// kBatch loads are issued before the first of them is used; padding gets zeros (the load then reads element 0:
// never a branch around a load)
template <int kDims, typename T, typename XT, bool kBf16>
__device__ __forceinline__ void load_tile(const TileGeom& tg, const TileBlocks& tb, const XT* x, T* buf,
                                          int total) {
  for (int e0 = threadIdx.x; e0 < total; e0 += kThreads * kBatch) {
    XT raw[kBatch];
    int slot[kBatch];
    bool in[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int e = e0 + u * kThreads;
      int b, j;
      row_major_across_blocks(tg, e < total ? e : 0, &b, &j);
      int64_t off;
      in[u] = locate<kDims>(tg, tb, b, j, &off) && e < total;
      slot[u] = e < total ? pad((b << tg.vol_shift) + j) : -1;
      raw[u] = x[in[u] ? off : 0];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (slot[u] < 0) continue;
      T v;
      if constexpr (kBf16) v = widen_bf16<T>(raw[u]);
      else v = widen<T, XT>(raw[u]);
      buf[slot[u]] = in[u] ? v : T(0);
    }
  }
}

template <int kDims, typename T, typename XT>
__device__ __forceinline__ void store_tile(const TileGeom& tg, const TileBlocks& tb, XT* y, const T* buf,
                                           int total) {
  for (int e = threadIdx.x; e < total; e += kThreads) {
    int b, j;
    row_major_across_blocks(tg, e, &b, &j);
    int64_t off;
    if (locate<kDims>(tg, tb, b, j, &off)) y[off] = XT(buf[pad((b << tg.vol_shift) + j)]);
  }
}

template <int kDims, typename T>
__device__ __forceinline__ void store_tile_bf16(const TileGeom& tg, const TileBlocks& tb, uint16_t* y,
                                                const T* buf, int total) {
  for (int e = threadIdx.x; e < total; e += kThreads) {
    int b, j;
    row_major_across_blocks(tg, e, &b, &j);
    int64_t off;
    if (locate<kDims>(tg, tb, b, j, &off)) {
      const T v = buf[pad((b << tg.vol_shift) + j)];
      y[off] = sizeof(T) == 8 ? double_to_bf16_bits(double(v)) : float_to_bf16_bits(float(v));
    }
  }
}
template <int kDims, typename T>
__device__ __forceinline__ void store_tile_f16(const TileGeom& tg, const TileBlocks& tb, _Float16* y,
                                               const T* buf, int total) {
  for (int e = threadIdx.x; e < total; e += kThreads) {
    int b, j;
    row_major_across_blocks(tg, e, &b, &j);
    int64_t off;
    if (locate<kDims>(tg, tb, b, j, &off)) {
      const T v = buf[pad((b << tg.vol_shift) + j)];
      y[off] = sizeof(T) == 8 ? double_to_f16(double(v)) : _Float16(float(v));
    }
  }
}

// ---- the array in 16-byte pieces ----------------------------------------------------------------------------
template <typename T, typename XT>
__device__ __forceinline__ void unpack_piece(const uint4& raw, T* out) {
  constexpr int P = 16 / int(sizeof(XT));
  XT e[P];
  __builtin_memcpy(e, &raw, 16);
#pragma unroll
  for (int i = 0; i < P; ++i) {
    if constexpr (std::is_same<XT, bf16_raw>::value) out[i] = widen_bf16<T>(e[i]);
    else out[i] = widen<T, XT>(e[i]);
  }
}

template <typename T, typename XT>
__device__ __forceinline__ uint4 pack_piece(const T* v) {
  constexpr int P = 16 / int(sizeof(XT));
  XT e[P];
#pragma unroll
  for (int i = 0; i < P; ++i) {
    if constexpr (std::is_same<XT, bf16_raw>::value)
      e[i].bits = sizeof(T) == 8 ? double_to_bf16_bits(double(v[i])) : float_to_bf16_bits(float(v[i]));
    else if constexpr (std::is_same<XT, _Float16>::value)
      e[i] = sizeof(T) == 8 ? double_to_f16(double(v[i])) : _Float16(float(v[i]));
    else
      e[i] = XT(v[i]);
  }
  uint4 raw;
  __builtin_memcpy(&raw, e, 16);
  return raw;
}

constexpr int kPieceBatch = 4;                // 16-byte loads a thread keeps in flight while filling a tile

template <int kDims, typename T, typename XT>
__device__ __forceinline__ void load_tile_pieces(const TileGeom& tg, const TileBlocks& tb, const XT* x, T* buf,
                                                 int total) {
  constexpr int P = 16 / int(sizeof(XT));
  // a thread's share of a 4096-element tile is 16 elements: all of its pieces are requested before the first is used
  constexpr int kInFlight = sizeof(XT) == 8 ? 8 : kPieceBatch;
  const int n_pieces = total / P;
  for (int p0 = threadIdx.x; p0 < n_pieces; p0 += kThreads * kInFlight) {
    uint4 raw[kInFlight];
    int slot[kInFlight];
    bool in[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int p = p0 + u * kThreads;
      int b, j;
      piece_across_blocks<P>(tg, p < n_pieces ? p : 0, &b, &j);
      int64_t off;
      in[u] = locate<kDims>(tg, tb, b, j, &off) && p < n_pieces;     // the piece's first element decides for all of it
      slot[u] = p < n_pieces ? pad((b << tg.vol_shift) + j) : -1;    // a piece never straddles a padding boundary
      raw[u] = *reinterpret_cast<const uint4*>(x + (in[u] ? off : 0));
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      if (slot[u] < 0) continue;
      T v[P];
      unpack_piece<T, XT>(raw[u], v);
#pragma unroll
      for (int i = 0; i < P; ++i) buf[slot[u] + i] = in[u] ? v[i] : T(0);
    }
  }
}

template <int kDims, typename T, typename XT>
__device__ __forceinline__ void store_tile_pieces(const TileGeom& tg, const TileBlocks& tb, XT* y, const T* buf,
                                                  int total) {
  constexpr int P = 16 / int(sizeof(XT));
  const int n_pieces = total / P;
  for (int p = threadIdx.x; p < n_pieces; p += kThreads) {
    int b, j;
    piece_across_blocks<P>(tg, p, &b, &j);
    int64_t off;
    if (locate<kDims>(tg, tb, b, j, &off)) {
      const int slot = pad((b << tg.vol_shift) + j);
      T v[P];
#pragma unroll
      for (int i = 0; i < P; ++i) v[i] = buf[slot + i];
      *reinterpret_cast<uint4*>(y + off) = pack_piece<T, XT>(v);
    }
  }
}

// ---- F in runs of four entries --------------------------------------------------------------------------------
// rint(t) as an integer for |t| below 2^22 (FP32) / 2^31 (FP64): adding 1.5 * 2^23 (2^52) rounds t to an integer in
// the current (nearest-even) mode and leaves it, in two's complement, in the low bits of the sum
__device__ __forceinline__ int round_to_int(float t) { return int(__float_as_uint(t + 12582912.0f)) - 0x4B400000; }
__device__ __forceinline__ int round_to_int(double t) {
  return int(uint32_t(__builtin_bit_cast(uint64_t, t + 6755399441055744.0)));
}

template <typename IT> struct Quad;           // four indices as one store / load
template <> struct Quad<int8_t> {
  typedef uint32_t type;
  static __device__ __forceinline__ type pack(const int* v) {
    return (uint32_t(v[0]) & 0xffu) | ((uint32_t(v[1]) & 0xffu) << 8) | ((uint32_t(v[2]) & 0xffu) << 16) | (uint32_t(v[3]) << 24);
  }
  static __device__ __forceinline__ void unpack(type w, int* v) {
    v[0] = int(int8_t(w & 0xffu)); v[1] = int(int8_t((w >> 8) & 0xffu)); v[2] = int(int8_t((w >> 16) & 0xffu)); v[3] = int(int8_t(w >> 24));
  }
};
template <> struct Quad<int16_t> {
  typedef uint2 type;
  static __device__ __forceinline__ type pack(const int* v) {
    return make_uint2((uint32_t(v[0]) & 0xffffu) | (uint32_t(v[1]) << 16), (uint32_t(v[2]) & 0xffffu) | (uint32_t(v[3]) << 16));
  }
  static __device__ __forceinline__ void unpack(type w, int* v) {
    v[0] = int(int16_t(w.x & 0xffffu)); v[1] = int(int16_t(w.x >> 16)); v[2] = int(int16_t(w.y & 0xffffu)); v[3] = int(int16_t(w.y >> 16));
  }
};
template <> struct Quad<int32_t> {
  typedef uint4 type;
  static __device__ __forceinline__ type pack(const int* v) {
    return make_uint4(uint32_t(v[0]), uint32_t(v[1]), uint32_t(v[2]), uint32_t(v[3]));
  }
  static __device__ __forceinline__ void unpack(type w, int* v) {
    v[0] = int(w.x); v[1] = int(w.y); v[2] = int(w.z); v[3] = int(w.w);
  }
};

// intra-block entries of the four kept positions pos .. pos + 3 (pos a multiple of four)
__device__ __forceinline__ void kept_entries(bool all_kept, const int32_t* kept_list, int pos, int* j) {
  if (all_kept) {
    j[0] = pos; j[1] = pos + 1; j[2] = pos + 2; j[3] = pos + 3;
  } else {
    const int4 q = *reinterpret_cast<const int4*>(kept_list + pos);
    j[0] = q.x; j[1] = q.y; j[2] = q.z; j[3] = q.w;
  }
}

// bin and prune, four kept entries per thread and step: one block look-up, one store.  |r C / N| <= r (1 + ulp)
// rounds to at most r, so no clamp is needed; an all-zero block has N = 1/N = 0 and every C = 0, which gives 0.
template <typename T, typename IT>
__device__ __forceinline__ void bin_quads(const TileGeom& tg, const T* buf, const typename Bits<T>::type* bmax,
                                          const T* binv, T r, IT* F, int64_t k0, const int32_t* kept_list) {
  typedef typename Quad<IT>::type quad_t;
  const bool all_kept = tg.kept == (1 << tg.vol_shift);
  const int n_quads = (tg.G * tg.kept) >> 2;
  quad_t* out = reinterpret_cast<quad_t*>(F + k0 * tg.kept);
  for (int q = threadIdx.x; q < n_quads; q += kThreads) {
    const int e = q << 2;
    const int b = all_kept ? e >> tg.vol_shift : e / tg.kept;
    if (k0 + b >= tg.n_blocks) continue;
    T c[4];
    if (all_kept) {                  // position e of the tile's F is element e of the tile; four in a row share a group of 32
      const T* src = buf + pad(e);
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = src[i];
    } else {
      int j[4];
      kept_entries(false, kept_list, e - b * tg.kept, j);
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = buf[pad((b << tg.vol_shift) + j[i])];
    }
    int idx[4];
    const T nk = Bits<T>::from(bmax[b]), inv = binv[b];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const T a = r * c[i];
      const T quo = a * inv;
      idx[i] = round_to_int(fma(fma(-quo, nk, a), inv, quo));
    }
    out[q] = Quad<IT>::pack(idx);
  }
}

// the tile's run of F -> specified coefficients at their intra-block positions, four entries per load
template <typename T, typename IT>
__device__ __forceinline__ void scatter_quads(const TileGeom& tg, const IT* F, int64_t k0, const T* bn,
                                              const int32_t* kept_list, T* buf) {
  typedef typename Quad<IT>::type quad_t;
  const bool all_kept = tg.kept == (1 << tg.vol_shift);
  const int n_quads = (tg.G * tg.kept) >> 2;
  const int64_t last = ((tg.n_blocks - k0) * int64_t(tg.kept) >> 2) - 1;      // last quad of the tile that exists
  const quad_t* in = reinterpret_cast<const quad_t*>(F + k0 * tg.kept);
  for (int q0 = threadIdx.x; q0 < n_quads; q0 += kThreads * kPieceBatch) {
    quad_t raw[kPieceBatch];
#pragma unroll
    for (int u = 0; u < kPieceBatch; ++u) {
      const int q = q0 + u * kThreads;
      raw[u] = in[q <= last ? q : last];
    }
#pragma unroll
    for (int u = 0; u < kPieceBatch; ++u) {
      const int q = q0 + u * kThreads;
      if (q >= n_quads || q > last) continue;
      const int e = q << 2;
      const int b = all_kept ? e >> tg.vol_shift : e / tg.kept;
      int f[4];
      Quad<IT>::unpack(raw[u], f);
      const T scale = bn[b];
      if (all_kept) {
        T* dst = buf + pad(e);
#pragma unroll
        for (int i = 0; i < 4; ++i) dst[i] = scale * T(f[i]);
      } else {
        int j[4];
        kept_entries(false, kept_list, e - b * tg.kept, j);
#pragma unroll
        for (int i = 0; i < 4; ++i) buf[pad((b << tg.vol_shift) + j[i])] = scale * T(f[i]);
      }
    }
  }
}

// one transform pass over the lines of length n with element stride 2^inner_shift, in place
// kMax: also fold max |.| of every transformed line into its block's entry of bmax (a line never leaves its block)
template <typename T, int kTf, int n, bool kForward, bool kMax = false>
__device__ __forceinline__ void pass_n(T* buf, int total, int n_shift, int inner_shift,
                                       typename Bits<T>::type* bmax = nullptr, int vol_shift = 0) {
  const int lines = total >> n_shift;
  for (int l = threadIdx.x; l < lines; l += kThreads) {
    const int base = line_base(l, n_shift, inner_shift);
    // pad(base + a * inner) = pad(base) + pad(a * inner): the line starts at a multiple of its span or, when that
    // span is below 32, stays inside one group of 32; the second term is the same for all threads (scalar unit)
    T* line = buf + pad(base);
    T v[n];
#pragma unroll
    for (int a = 0; a < n; ++a) v[a] = line[pad(a << inner_shift)];
    if (kForward) tf_forward<kTf, T, n, 1>(v);
    else tf_inverse<kTf, T, n, 1, n>(v);
#pragma unroll
    for (int a = 0; a < n; ++a) line[pad(a << inner_shift)] = v[a];
    if constexpr (kMax) {
      T m = fabs(v[0]);
#pragma unroll
      for (int a = 1; a < n; ++a) m = fmax(m, fabs(v[a]));
      // Consecutive lines belong to one block in runs of (lines per block), a power of two, so the lanes of a wave
      // that share a block are an aligned group: they combine by lane exchanges and one of them does the atomic
      // (64 lanes on one address would be served one after the other).  A group is active or idle as a whole:
      // the number of lines is a multiple of the run.
      const int run = 1 << (vol_shift - n_shift);
      const int group = run < 64 ? run : 64;
      for (int step = 1; step < group; step <<= 1) m = fmax(m, __shfl_xor(m, step));
      if ((threadIdx.x & (group - 1)) == 0) atomicMax(&bmax[base >> vol_shift], Bits<T>::of(m));
    }
  }
}

// forward: bmax != nullptr asks for the per-block maxima, taken in the last pass that has work to do.  The loop over
// the dimensions is kept a loop (one copy of each pass per kernel instead of one per dimension).  kMaxShift: log2 of
// the longest line the kernel is built for (the passes for longer lines set the kernel's register count: 64 values
// per thread for a line of 32 in FP64).
template <int kDims, typename T, int kTf, bool kForward, int kMaxShift>
__device__ __forceinline__ void transform_tile(const TileGeom& tg, T* buf, int total,
                                               typename Bits<T>::type* bmax = nullptr) {
  int last = -1;
#pragma unroll
  for (int d = PBZ_MAX_NDIM - kDims; d < PBZ_MAX_NDIM; ++d)
    if (tg.bshift[d] > 0) last = d;
  int inner_shift = tg.vol_shift;
#pragma nounroll
  for (int d = PBZ_MAX_NDIM - kDims; d < PBZ_MAX_NDIM; ++d) {
    const int ns = tg.bshift[d];
    inner_shift -= ns;
    if (ns == 0) continue;
    if (kForward && bmax != nullptr && d == last) {
      switch (ns) {
        case 1: pass_n<T, kTf, 2, kForward, true>(buf, total, 1, inner_shift, bmax, tg.vol_shift); break;
        case 2: pass_n<T, kTf, 4, kForward, true>(buf, total, 2, inner_shift, bmax, tg.vol_shift); break;
        case 3: pass_n<T, kTf, 8, kForward, true>(buf, total, 3, inner_shift, bmax, tg.vol_shift); break;
        case 4:
          if constexpr (kMaxShift >= 4) pass_n<T, kTf, 16, kForward, true>(buf, total, 4, inner_shift, bmax, tg.vol_shift);
          break;
        default:
          if constexpr (kMaxShift >= 5) pass_n<T, kTf, 32, kForward, true>(buf, total, 5, inner_shift, bmax, tg.vol_shift);
          break;
      }
    } else {
      switch (ns) {
        case 1: pass_n<T, kTf, 2, kForward>(buf, total, 1, inner_shift); break;
        case 2: pass_n<T, kTf, 4, kForward>(buf, total, 2, inner_shift); break;
        case 3: pass_n<T, kTf, 8, kForward>(buf, total, 3, inner_shift); break;
        case 4:
          if constexpr (kMaxShift >= 4) pass_n<T, kTf, 16, kForward>(buf, total, 4, inner_shift);
          break;
        default:
          if constexpr (kMaxShift >= 5) pass_n<T, kTf, 32, kForward>(buf, total, 5, inner_shift);
          break;
      }
    }
    __syncthreads();
  }
}

template <int kDims, typename T, int kTf, int kMaxShift>
__global__ __launch_bounds__(kThreads) void k_compress_tiled(TileGeom tg, const void* __restrict__ x, int xtype,
                                                             void* __restrict__ N, int ntype, void* __restrict__ F,
                                                             int itype, double r,
                                                             const int32_t* __restrict__ kept_list) {
  extern __shared__ __align__(16) unsigned char smem[];
  typedef typename Bits<T>::type bits_t;
  const int total = tg.G << tg.vol_shift;
  TileBlocks tb;
  tb.blk = reinterpret_cast<BlockInfo*>(smem);
  tb.row = reinterpret_cast<RowInfo*>(smem + 16 * tg.G);
  unsigned char* per_block = smem + per_block_offset(tg.G, tg.vol_shift, tg.bx_shift);
  bits_t* bmax = reinterpret_cast<bits_t*>(per_block);
  T* binv = reinterpret_cast<T*>(per_block + 8 * tg.G);
  T* buf = reinterpret_cast<T*>(smem + tile_offset(tg.G, tg.vol_shift, tg.bx_shift));
  const int vol = 1 << tg.vol_shift;
  // one tile per workgroup, so that what the decode below needs of the geometry is dead before the loops start
  const int64_t k0 = (int64_t(blockIdx.y) * gridDim.x + blockIdx.x) << tg.g_shift;
  if (k0 >= tg.n_blocks) return;               // uniform over the workgroup
  {
    tabulate_rows<kDims>(tg, tb);
    decode_blocks<kDims>(tg, k0, tb);
    for (int b = threadIdx.x; b < tg.G; b += kThreads) bmax[b] = 0;
    __syncthreads();
    if (tg.vec_x) {
      switch (xtype) {                     // one switch around the whole loop, not one per element
        case PBZ_F64: load_tile_pieces<kDims, T, double>(tg, tb, static_cast<const double*>(x), buf, total); break;
        case PBZ_F32: load_tile_pieces<kDims, T, float>(tg, tb, static_cast<const float*>(x), buf, total); break;
        case PBZ_BF16: load_tile_pieces<kDims, T, bf16_raw>(tg, tb, static_cast<const bf16_raw*>(x), buf, total); break;
        default: load_tile_pieces<kDims, T, _Float16>(tg, tb, static_cast<const _Float16*>(x), buf, total); break;
      }
    } else {
      switch (xtype) {
        case PBZ_F64: load_tile<kDims, T, double, false>(tg, tb, static_cast<const double*>(x), buf, total); break;
        case PBZ_F32: load_tile<kDims, T, float, false>(tg, tb, static_cast<const float*>(x), buf, total); break;
        case PBZ_BF16: load_tile<kDims, T, bf16_raw, true>(tg, tb, static_cast<const bf16_raw*>(x), buf, total); break;
        default: load_tile<kDims, T, _Float16, false>(tg, tb, static_cast<const _Float16*>(x), buf, total); break;
      }
    }
    __syncthreads();
    transform_tile<kDims, T, kTf, true, kMaxShift>(tg, buf, total, bmax);      // leaves N_k = max |C_k| in bmax
    if (vol == 1) {                        // single-element blocks: nothing was transformed
      for (int e = threadIdx.x; e < total; e += kThreads) bmax[e] = Bits<T>::of(fabs(buf[pad(e)]));
      __syncthreads();
    }
    for (int b = threadIdx.x; b < tg.G; b += kThreads) {
      const T nk = Bits<T>::from(bmax[b]);
      binv[b] = nk > T(0) ? T(1) / nk : T(0);
      if (k0 + b < tg.n_blocks) store_float(N, ntype, k0 + b, nk);
    }
    __syncthreads();
    // bin and prune: the kept entries of the tile in F order.  (r C) / N from the correctly rounded reciprocal
    // with one remainder correction: the correctly rounded quotient without a division per entry.
    const int n_kept = tg.vec_f ? 0 : tg.G * tg.kept;
    const bool all_kept = tg.kept == vol;            // then position pos of F holds intra-block entry pos
    if (tg.vec_f) {
      switch (itype) {
        case PBZ_I8: bin_quads<T, int8_t>(tg, buf, bmax, binv, T(r), static_cast<int8_t*>(F), k0, kept_list); break;
        case PBZ_I16: bin_quads<T, int16_t>(tg, buf, bmax, binv, T(r), static_cast<int16_t*>(F), k0, kept_list); break;
        default: bin_quads<T, int32_t>(tg, buf, bmax, binv, T(r), static_cast<int32_t*>(F), k0, kept_list); break;
      }
    }
    for (int e0 = threadIdx.x; e0 < n_kept; e0 += kThreads * kBatch) {
      int b[kBatch], j[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {            // the table look-ups of a batch are in flight together
        const int e = e0 + u * kThreads;
        const int ec = e < n_kept ? e : 0;
        b[u] = all_kept ? ec >> tg.vol_shift : ec / tg.kept;
        const int pos = ec - b[u] * tg.kept;
        j[u] = all_kept ? pos : kept_list[pos];
        if (e >= n_kept || k0 + b[u] >= tg.n_blocks) b[u] = -1;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (b[u] < 0) continue;
        const T nk = Bits<T>::from(bmax[b[u]]), inv = binv[b[u]];
        const T a = T(r) * buf[pad((b[u] << tg.vol_shift) + j[u])];
        const T q = a * inv;
        T t = fma(fma(-q, nk, a), inv, q);
        t = fmin(fmax(rint(t), T(-r)), T(r));
        store_index(F, itype, k0 * tg.kept + e0 + u * kThreads, int64_t(t));
      }
    }
  }
}

// the tile's run of F (contiguous) -> specified coefficients at their intra-block positions, kBatch loads in flight
template <typename T, typename IT>
__device__ __forceinline__ void scatter_coefficients(const TileGeom& tg, const IT* F, int64_t k0, const T* bn,
                                                     T r, const int32_t* kept_list, T* buf) {
  const int n_kept = tg.G * tg.kept;
  const int64_t last = tg.n_blocks * int64_t(tg.kept) - 1;
  for (int e0 = threadIdx.x; e0 < n_kept; e0 += kThreads * kBatch) {
    IT f[kBatch];
    int j[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int e = e0 + u * kThreads;
      const int64_t at = k0 * tg.kept + e;
      f[u] = F[at <= last ? at : last];
      const int ec = e < n_kept ? e : 0;
      const int b = ec / tg.kept;
      j[u] = e < n_kept ? pad((b << tg.vol_shift) + kept_list[ec - b * tg.kept]) : -1;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (j[u] < 0) continue;
      const int e = e0 + u * kThreads;
      buf[j[u]] = bn[e / tg.kept] * T(f[u]);
    }
  }
}

template <int kDims, typename T, int kTf, int kMaxShift>
__global__ __launch_bounds__(kThreads) void k_decompress_tiled(TileGeom tg, const void* __restrict__ N, int ntype,
                                                               const void* __restrict__ F, int itype, double r,
                                                               void* __restrict__ y, int ytype,
                                                               const int32_t* __restrict__ kept_list) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int total = tg.G << tg.vol_shift;
  TileBlocks tb;
  tb.blk = reinterpret_cast<BlockInfo*>(smem);
  tb.row = reinterpret_cast<RowInfo*>(smem + 16 * tg.G);
  T* bn = reinterpret_cast<T*>(smem + per_block_offset(tg.G, tg.vol_shift, tg.bx_shift));
  T* buf = reinterpret_cast<T*>(smem + tile_offset(tg.G, tg.vol_shift, tg.bx_shift));
  const int vol = 1 << tg.vol_shift;
  const int64_t k0 = (int64_t(blockIdx.y) * gridDim.x + blockIdx.x) << tg.g_shift;   // one tile per workgroup
  if (k0 >= tg.n_blocks) return;               // uniform over the workgroup
  {
    tabulate_rows<kDims>(tg, tb);
    decode_blocks<kDims>(tg, k0, tb);
    for (int b = threadIdx.x; b < tg.G; b += kThreads)      // blocks past the end: the last one again, never stored
      bn[b] = load_float<T>(N, ntype, k0 + b < tg.n_blocks ? k0 + b : tg.n_blocks - 1) / T(r);   // N / r once per block
    if (tg.kept != vol)
      for (int e = threadIdx.x; e < total; e += kThreads) buf[pad(e)] = T(0);
    __syncthreads();
    // Algorithm 3: N F / r at the kept positions
    if (tg.vec_f) {
      switch (itype) {
        case PBZ_I8: scatter_quads<T, int8_t>(tg, static_cast<const int8_t*>(F), k0, bn, kept_list, buf); break;
        case PBZ_I16: scatter_quads<T, int16_t>(tg, static_cast<const int16_t*>(F), k0, bn, kept_list, buf); break;
        default: scatter_quads<T, int32_t>(tg, static_cast<const int32_t*>(F), k0, bn, kept_list, buf); break;
      }
    } else {
      switch (itype) {
        case PBZ_I8: scatter_coefficients<T, int8_t>(tg, static_cast<const int8_t*>(F), k0, bn, T(r), kept_list, buf); break;
        case PBZ_I16: scatter_coefficients<T, int16_t>(tg, static_cast<const int16_t*>(F), k0, bn, T(r), kept_list, buf); break;
        default: scatter_coefficients<T, int32_t>(tg, static_cast<const int32_t*>(F), k0, bn, T(r), kept_list, buf); break;
      }
    }
    __syncthreads();
    transform_tile<kDims, T, kTf, false, kMaxShift>(tg, buf, total);
    if (tg.vec_x) {
      switch (ytype) {
        case PBZ_F64: store_tile_pieces<kDims, T, double>(tg, tb, static_cast<double*>(y), buf, total); break;
        case PBZ_F32: store_tile_pieces<kDims, T, float>(tg, tb, static_cast<float*>(y), buf, total); break;
        case PBZ_BF16: store_tile_pieces<kDims, T, bf16_raw>(tg, tb, static_cast<bf16_raw*>(y), buf, total); break;
        default: store_tile_pieces<kDims, T, _Float16>(tg, tb, static_cast<_Float16*>(y), buf, total); break;
      }
    } else {
      switch (ytype) {
        case PBZ_F64: store_tile<kDims, T, double>(tg, tb, static_cast<double*>(y), buf, total); break;
        case PBZ_F32: store_tile<kDims, T, float>(tg, tb, static_cast<float*>(y), buf, total); break;
        case PBZ_BF16: store_tile_bf16<kDims, T>(tg, tb, static_cast<uint16_t*>(y), buf, total); break;
        default: store_tile_f16<kDims, T>(tg, tb, static_cast<_Float16*>(y), buf, total); break;
      }
    }
  }
}

TileGeom make_tile(const pbz_codec* c, const Geom& g) {
  return make_tile_geom(c->ndim, c->block, g.shape, c->kept);
}

// may the array (elements of array_type at `array`) be moved in 16-byte pieces, and F in runs of four entries?
void choose_units(const pbz_codec* c, const Geom& g, const void* array, int array_type, const void* F, TileGeom* tg) {
  const int64_t piece = 16 / ftype_bytes(array_type);        // elements per piece
  const int64_t last = g.shape[c->ndim - 1];
  tg->vec_x = c->block[c->ndim - 1] >= piece && last % piece == 0 && (reinterpret_cast<uintptr_t>(array) & 15u) == 0;
  // every tile starts at a multiple of four entries (whole blocks of a kept count that is one); the kept-position
  // table is read four entries at a time as well (it comes from hipMalloc: aligned)
  tg->vec_f = c->kept % 4 == 0 && (reinterpret_cast<uintptr_t>(F) % size_t(4 * itype_bytes(c->itype))) == 0;
}

size_t tile_lds_bytes(const TileGeom& tg, size_t elem) {
  const int total = tg.G << tg.vol_shift;
  return tile_offset(tg.G, tg.vol_shift, tg.bx_shift) + elem * size_t(total + (total >> 5) + 1);
}

// one workgroup per tile: x up to 2^20, the rest in y (at most 2^40 elements in tiles of 256 or more: y <= 4096)
dim3 tile_grid(int64_t n_tiles) {
  const int64_t cap = int64_t(1) << 20;
  if (n_tiles <= cap) return dim3(unsigned(n_tiles));
  return dim3(unsigned(cap), unsigned((n_tiles + cap - 1) / cap));
}

}  // namespace

bool tiled_kernels_cover(const pbz_codec* c) {
  for (int d = 0; d < c->ndim; ++d)
    if (c->block[d] > 32) return false;
  return true;
}

int launch_compress_tiled(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* x, int xtype, void* N,
                          void* F, hipStream_t s) {
  TileGeom tg = make_tile(c, g);
  choose_units(c, g, x, xtype, F, &tg);
  const int64_t n_tiles = (tg.n_blocks + tg.G - 1) / tg.G;
  const dim3 grid = tile_grid(n_tiles), block(kThreads);
  int max_shift = 0;                               // log2 of the longest line
  for (int d = 0; d < PBZ_MAX_NDIM; ++d) max_shift = tg.bshift[d] > max_shift ? tg.bshift[d] : max_shift;
#define PBZ_TILED_M(T, TF, M)                                                                                         \
  do {                                                                                                                \
    if (tg.dims == 4)                                                                                                 \
      hipLaunchKernelGGL((k_compress_tiled<4, T, TF, M>), grid, block, tile_lds_bytes(tg, sizeof(T)), s, tg, x, xtype, \
                         N, int(c->ftype), F, int(c->itype), c->r, t->kept_list);                                     \
    else                                                                                                              \
      hipLaunchKernelGGL((k_compress_tiled<8, T, TF, M>), grid, block, tile_lds_bytes(tg, sizeof(T)), s, tg, x, xtype, \
                         N, int(c->ftype), F, int(c->itype), c->r, t->kept_list);                                     \
  } while (0)
#define PBZ_TILED(T, TF)                                                                                              \
  do {                                                                                                                \
    if (max_shift <= 3) PBZ_TILED_M(T, TF, 3);                                                                        \
    else if (max_shift == 4) PBZ_TILED_M(T, TF, 4);                                                                   \
    else PBZ_TILED_M(T, TF, 5);                                                                                       \
  } while (0)
  if (c->compute_f64) {
    if (c->transform == PBZ_TRANSFORM_HAAR) PBZ_TILED(double, kTfHaar);
    else PBZ_TILED(double, kTfDct);
  } else {
    if (c->transform == PBZ_TRANSFORM_HAAR) PBZ_TILED(float, kTfHaar);
    else PBZ_TILED(float, kTfDct);
  }
#undef PBZ_TILED
#undef PBZ_TILED_M
  return hip_status(hipGetLastError());
}

int launch_decompress_tiled(const pbz_codec* c, const Geom& g, const DeviceTables* t, const void* N, const void* F,
                            void* y, int ytype, hipStream_t s) {
  TileGeom tg = make_tile(c, g);
  choose_units(c, g, y, ytype, F, &tg);
  const int64_t n_tiles = (tg.n_blocks + tg.G - 1) / tg.G;
  const dim3 grid = tile_grid(n_tiles), block(kThreads);
  int max_shift = 0;                               // log2 of the longest line
  for (int d = 0; d < PBZ_MAX_NDIM; ++d) max_shift = tg.bshift[d] > max_shift ? tg.bshift[d] : max_shift;
#define PBZ_TILED_M(T, TF, M)                                                                                         \
  do {                                                                                                                \
    if (tg.dims == 4)                                                                                                 \
      hipLaunchKernelGGL((k_decompress_tiled<4, T, TF, M>), grid, block, tile_lds_bytes(tg, sizeof(T)), s, tg, N,      \
                         int(c->ftype), F, int(c->itype), c->r, y, ytype, t->kept_list);                              \
    else                                                                                                              \
      hipLaunchKernelGGL((k_decompress_tiled<8, T, TF, M>), grid, block, tile_lds_bytes(tg, sizeof(T)), s, tg, N,      \
                         int(c->ftype), F, int(c->itype), c->r, y, ytype, t->kept_list);                              \
  } while (0)
#define PBZ_TILED(T, TF)                                                                                              \
  do {                                                                                                                \
    if (max_shift <= 3) PBZ_TILED_M(T, TF, 3);                                                                        \
    else if (max_shift == 4) PBZ_TILED_M(T, TF, 4);                                                                   \
    else PBZ_TILED_M(T, TF, 5);                                                                                       \
  } while (0)
  if (c->compute_f64) {
    if (c->transform == PBZ_TRANSFORM_HAAR) PBZ_TILED(double, kTfHaar);
    else PBZ_TILED(double, kTfDct);
  } else {
    if (c->transform == PBZ_TRANSFORM_HAAR) PBZ_TILED(float, kTfHaar);
    else PBZ_TILED(float, kTfDct);
  }
#undef PBZ_TILED
#undef PBZ_TILED_M
  return hip_status(hipGetLastError());
}

}  // namespace pbz
