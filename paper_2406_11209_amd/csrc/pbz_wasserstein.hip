// Approximate Wasserstein distance of two compressed arrays (Sec. IV-A, "Approximate Wasserstein distance",
// Algorithm 13): block-wise means -> softmax unless they already sum to one -> sort -> p-th power mean of the
// differences of the two sorted sequences.
//
// Everything stays on the device and on the caller's stream:
//   1. block means of both operands (the block-wise mean kernel) into the workspace,
//   2. their sum and maximum, then sum of exp(x - max) (two-stage reductions; a one-workgroup kernel turns the
//      partial sums into the parameters of the softmax and the decision whether to apply it),
//   3. the raw means are sorted (softmax is increasing, so it commutes with sorting) by a least-significant-digit
//      radix sort on an order-preserving 64-bit image of the doubles, 8 bits per pass and three launches per pass,
//      both operands in the same launches (grid y),
//   4. m = max |P_A - P_B|, then sum (|P_A - P_B| / m)^p, then m (sum / n)^(1/p): the scaling by m changes
//      nothing in exact arithmetic and keeps orders such as p = 68 .. 80 from underflowing.
// All sums are two-stage with a fixed order, so the result is reproducible run to run.
#include <cmath>

#include "pbz_device.h"
#include "pbz_internal.h"

namespace pbz {
namespace {

constexpr int kThreads = 256;
constexpr int kRadixBits = 8;
constexpr int kBins = 1 << kRadixBits;
constexpr int kSortThreads = 256;                // threads of a sorting workgroup: four waves, one thread per digit
constexpr int kKeysPerLane = 16;
constexpr int kWaveKeys = 64 * kKeysPerLane;     // keys one wave ranks
constexpr int kTileKeys = kSortThreads * kKeysPerLane;   // keys of a tile (one workgroup)
// workgroups per operand in the small reductions, at most: 8 per compute unit (exp and pow are long dependent chains;
// with 256 the power sum over 2M keys took 36 us)
constexpr int kStatGroups = 2048;
constexpr double kSumTolerance = 1e-9;           // "the means sum to one" is taken as |sum - 1| <= this

// per operand: written by the one-workgroup kernels, read by everything after them
struct OperandParams {
  double sum, max, exp_sum, use_softmax;
};

struct Workspace {
  OperandParams* params;   // [2]
  double* partials;        // [2][kStatGroups][2]
  double* scalars;         // [2]: the largest difference, the result's power sum
  uint64_t* buf0;          // [2][n]: means, then keys; the sorted keys end up here
  uint64_t* buf1;          // [2][n]
  uint32_t* hist;          // [2][kBins][n_tiles]
  uint32_t* sums;          // [2][kBins]: the digits' totals
};

size_t align_up(size_t v) { return (v + 255) & ~size_t(255); }

size_t carve(void* base, int64_t n, Workspace* w) {
  const int64_t n_tiles = (n + kTileKeys - 1) / kTileKeys;
  size_t off = 0;
  char* p = static_cast<char*>(base);
  auto take = [&](size_t bytes) {
    char* q = p ? p + off : nullptr;
    off += align_up(bytes);
    return q;
  };
  char* a = take(sizeof(OperandParams) * 2);
  char* b = take(sizeof(double) * 2 * kStatGroups * 2);
  char* c = take(sizeof(double) * 2);
  char* d = take(sizeof(uint64_t) * 2 * size_t(n));
  char* e = take(sizeof(uint64_t) * 2 * size_t(n));
  char* f = take(sizeof(uint32_t) * 2 * kBins * size_t(n_tiles));
  char* g = take(sizeof(uint32_t) * 2 * kBins);
  if (w) {
    w->sums = reinterpret_cast<uint32_t*>(g);
    w->params = reinterpret_cast<OperandParams*>(a);
    w->partials = reinterpret_cast<double*>(b);
    w->scalars = reinterpret_cast<double*>(c);
    w->buf0 = reinterpret_cast<uint64_t*>(d);
    w->buf1 = reinterpret_cast<uint64_t*>(e);
    w->hist = reinterpret_cast<uint32_t*>(f);
  }
  return off;
}

__device__ __forceinline__ void wave_lds_sync() {   // orders one wave's LDS accesses; no workgroup barrier involved
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// doubles <-> unsigned keys with the same order (negative values: all bits flipped; others: sign bit set)
__device__ __forceinline__ uint64_t key_of(double v) {
  const uint64_t u = uint64_t(__double_as_longlong(v));
  return (u >> 63) ? ~u : (u | (uint64_t(1) << 63));
}
__device__ __forceinline__ double value_of(uint64_t k) {
  const uint64_t u = (k >> 63) ? (k & ~(uint64_t(1) << 63)) : ~k;
  return __longlong_as_double((long long)u);
}

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
  return v;
}

// workgroup totals of two values (sum, max) in thread 0
__device__ __forceinline__ void group_sum_max(double& s, double& m) {
  __shared__ double ls[kThreads / 64], lm[kThreads / 64];
  s = wave_sum(s);
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) {
    ls[threadIdx.x >> 6] = s;
    lm[threadIdx.x >> 6] = m;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    s = ls[0];
    m = lm[0];
    for (int w = 1; w < kThreads / 64; ++w) {
      s += ls[w];
      m = fmax(m, lm[w]);
    }
  }
}

// stage 0: sum and max of the means; stage 1: sum of exp(x - max).  grid (kStatGroups, 2)
template <int kStage>
__global__ __launch_bounds__(kThreads) void k_mean_stats(const double* __restrict__ means, int64_t n, int64_t chunk,
                                                         const OperandParams* __restrict__ params,
                                                         double* __restrict__ partials) {
  const double* x = means + int64_t(blockIdx.y) * n;
  const int64_t begin = int64_t(blockIdx.x) * chunk;
  const int64_t end = begin + chunk < n ? begin + chunk : n;
  double s = 0.0, m = -INFINITY;
  const double shift = kStage == 1 ? params[blockIdx.y].max : 0.0;
  for (int64_t i = begin + threadIdx.x; i < end; i += kThreads) {
    const double v = x[i];
    if (kStage == 0) {
      s += v;
      m = fmax(m, v);
    } else {
      s += exp(v - shift);
    }
  }
  group_sum_max(s, m);
  if (threadIdx.x == 0) {
    double* out = partials + (int64_t(blockIdx.y) * kStatGroups + blockIdx.x) * 2;
    out[0] = s;
    out[1] = m;
  }
}

// one workgroup per operand: partials -> parameters
template <int kStage>
__global__ __launch_bounds__(kThreads) void k_mean_params(const double* __restrict__ partials, int groups,
                                                          OperandParams* __restrict__ params) {
  const double* in = partials + int64_t(blockIdx.x) * kStatGroups * 2;
  double s = 0.0, m = -INFINITY;
  for (int g = threadIdx.x; g < groups; g += kThreads) {
    s += in[2 * g];
    m = fmax(m, in[2 * g + 1]);
  }
  group_sum_max(s, m);
  if (threadIdx.x == 0) {
    OperandParams& p = params[blockIdx.x];
    if (kStage == 0) {
      p.sum = s;
      p.max = m;
      p.use_softmax = fabs(s - 1.0) > kSumTolerance ? 1.0 : 0.0;
    } else {
      p.exp_sum = s;
    }
  }
}

__global__ __launch_bounds__(kThreads) void k_to_keys(uint64_t* __restrict__ buf, int64_t total) {
  const int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (i < total) buf[i] = key_of(__longlong_as_double((long long)buf[i]));
}

// ---- radix sort, one pass = histogram per tile, exclusive scan over (digit, tile), stable scatter --------------
// A tile is kTileKeys consecutive keys, ranked by one workgroup of four waves: wave w takes the tile's w-th quarter,
// and element j * 64 + lane of that quarter belongs to lane `lane` in round j, so waves, rounds and, within a
// round, lanes follow the input order.

// the lanes of this round that hold the same digit as this one (valid lanes only)
__device__ __forceinline__ uint64_t same_digit_lanes(uint32_t digit, bool valid) {
  uint64_t peers = __ballot(valid);
#pragma unroll
  for (int b = 0; b < kRadixBits; ++b) {
    const uint64_t set = __ballot(valid && ((digit >> b) & 1u));
    peers &= ((digit >> b) & 1u) ? set : ~set;
  }
  return peers;
}

// One count per digit and tile, one LDS atomic per key (measured against one atomic per group of lanes that share a
// digit, found with the ballots of the scatter kernel: 9.9 against 17.4 us for 2 x 2M keys).
__global__ __launch_bounds__(kSortThreads) void k_radix_hist(const uint64_t* __restrict__ keys, int64_t n,
                                                             int64_t n_tiles, int shift, uint32_t* __restrict__ hist) {
  __shared__ uint32_t count[kBins];
  static_assert(kBins == kSortThreads, "one thread per digit");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t* in = keys + int64_t(blockIdx.y) * n;
  uint32_t* h = hist + int64_t(blockIdx.y) * kBins * n_tiles;
  count[threadIdx.x] = 0;
  __syncthreads();
  // which lane counts which key does not matter here: two neighbouring keys per lane and load, all loads first
  const int64_t base = int64_t(blockIdx.x) * kTileKeys + wave * kWaveKeys;
  uint64_t key[kKeysPerLane];
  const bool whole = base + kWaveKeys <= n && (reinterpret_cast<uintptr_t>(in) & 15u) == 0;      // uniform over the wave
  if (whole) {
#pragma unroll
    for (int j = 0; j < kKeysPerLane / 2; ++j) {
      const uint4 two = *reinterpret_cast<const uint4*>(in + base + (j * 64 + lane) * 2);
      key[2 * j] = uint64_t(two.x) | (uint64_t(two.y) << 32);
      key[2 * j + 1] = uint64_t(two.z) | (uint64_t(two.w) << 32);
    }
  } else {
#pragma unroll
    for (int j = 0; j < kKeysPerLane; ++j) {
      const int64_t i = base + j * 64 + lane;
      key[j] = i < n ? in[i] : 0;
    }
  }
#pragma unroll
  for (int j = 0; j < kKeysPerLane; ++j) {
    const bool valid = whole || base + j * 64 + lane < n;
    if (valid) atomicAdd(&count[uint32_t(key[j] >> shift) & (kBins - 1)], 1u);
  }
  __syncthreads();
  h[int64_t(threadIdx.x) * n_tiles + blockIdx.x] = count[threadIdx.x];
}

__device__ __forceinline__ uint32_t group_exclusive_scan(uint32_t v, uint32_t* lds /* blockDim.x entries */,
                                                         uint32_t* total) {
  lds[threadIdx.x] = v;
  __syncthreads();
  for (int off = 1; off < int(blockDim.x); off <<= 1) {
    const uint32_t add = int(threadIdx.x) >= off ? lds[threadIdx.x - off] : 0u;
    __syncthreads();
    lds[threadIdx.x] += add;
    __syncthreads();
  }
  if (total) *total = lds[blockDim.x - 1];
  const uint32_t ex = lds[threadIdx.x] - v;
  __syncthreads();                                        // the buffer may be used again right away
  return ex;
}

// Per digit (grid x) and operand (grid y): the counts of the digit's tiles become their exclusive prefix sums, in
// place, and the digit's total goes to totals.  The scatter kernel adds the totals of the lower digits itself.
__global__ __launch_bounds__(kSortThreads) void k_scan_digit(uint32_t* __restrict__ hist, int64_t n_tiles,
                                                             uint32_t* __restrict__ totals) {
  __shared__ uint32_t lds[kSortThreads];
  uint32_t* row = hist + (int64_t(blockIdx.y) * kBins + blockIdx.x) * n_tiles;
  uint32_t carry = 0;
  for (int64_t t0 = 0; t0 < n_tiles; t0 += kSortThreads) {
    const int64_t t = t0 + threadIdx.x;
    const uint32_t v = t < n_tiles ? row[t] : 0u;
    uint32_t chunk_total;
    const uint32_t ex = group_exclusive_scan(v, lds, &chunk_total);
    if (t < n_tiles) row[t] = carry + ex;
    carry += chunk_total;
  }
  if (threadIdx.x == 0) totals[blockIdx.y * kBins + blockIdx.x] = carry;
}

// The keys of a tile are first put in digit order in LDS (ranks within a wave from lane ballots and a per-wave
// cursor per digit, then the waves' counts are chained), and then written out in that order, so that consecutive
// threads write consecutive keys of a digit's run.  A digit that all n keys share (the sign and exponent bytes of
// block means, typically) leaves the order as it is: the tile is copied.
__global__ __launch_bounds__(kSortThreads) void k_radix_scatter(const uint64_t* __restrict__ keys_in,
                                                                uint64_t* __restrict__ keys_out, int64_t n,
                                                                int64_t n_tiles, int shift,
                                                                const uint32_t* __restrict__ hist,
                                                                const uint32_t* __restrict__ totals) {
  __shared__ uint64_t sorted[kTileKeys];
  __shared__ uint32_t cursor[kSortThreads / 64][kBins];   // per wave: count so far, later the wave's offset in its digit
  __shared__ uint32_t tile_first[kBins];                  // position in the tile of the first key with that digit
  __shared__ uint32_t out_first[kBins];                   // position in the output of that key
  __shared__ uint32_t scan[kSortThreads];
  __shared__ uint32_t uniform;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t* in = keys_in + int64_t(blockIdx.y) * n;
  uint64_t* out = keys_out + int64_t(blockIdx.y) * n;
  const int64_t tile_base = int64_t(blockIdx.x) * kTileKeys;
  const int64_t base = tile_base + wave * kWaveKeys;
  uint64_t key[kKeysPerLane];
#pragma unroll
  for (int j = 0; j < kKeysPerLane; ++j) {
    const int64_t i = base + j * 64 + lane;
    key[j] = i < n ? in[i] : 0;
  }
  const uint32_t digit_total = totals[blockIdx.y * kBins + threadIdx.x];
  if (threadIdx.x == 0) uniform = 0;
#pragma unroll
  for (int w = 0; w < kSortThreads / 64; ++w) cursor[w][threadIdx.x] = 0;
  __syncthreads();
  if (int64_t(digit_total) == n) uniform = 1;
  const uint32_t digit_first = group_exclusive_scan(digit_total, scan, nullptr);   // (contains the barrier)
  if (uniform) {
#pragma unroll
    for (int j = 0; j < kKeysPerLane; ++j) {
      const int64_t i = base + j * 64 + lane;
      if (i < n) out[i] = key[j];
    }
    return;
  }
  const uint64_t below = (uint64_t(1) << lane) - 1;      // lanes before this one
  uint32_t local[kKeysPerLane];                          // rank among the wave's keys with the same digit
#pragma unroll
  for (int j = 0; j < kKeysPerLane; ++j) {
    const bool valid = base + j * 64 + lane < n;
    const uint32_t digit = uint32_t(key[j] >> shift) & (kBins - 1);
    const uint64_t peers = same_digit_lanes(digit, valid);
    const uint32_t start = valid ? cursor[wave][digit] : 0u;
    wave_lds_sync();                                       // every lane has read before any leader writes
    const uint32_t rank = uint32_t(__popcll(peers & below));
    if (valid && rank == 0) cursor[wave][digit] = start + uint32_t(__popcll(peers));
    local[j] = start + rank;
    wave_lds_sync();
  }
  __syncthreads();
  {  // thread d: the waves' counts of digit d become the waves' offsets; the tile's count of d is scanned over d
    uint32_t run = 0;
#pragma unroll
    for (int w = 0; w < kSortThreads / 64; ++w) {
      const uint32_t c = cursor[w][threadIdx.x];
      cursor[w][threadIdx.x] = run;
      run += c;
    }
    tile_first[threadIdx.x] = group_exclusive_scan(run, scan, nullptr);
    out_first[threadIdx.x] = digit_first + hist[int64_t(blockIdx.y) * kBins * n_tiles + int64_t(threadIdx.x) * n_tiles + blockIdx.x];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kKeysPerLane; ++j) {
    if (base + j * 64 + lane < n) {
      const uint32_t digit = uint32_t(key[j] >> shift) & (kBins - 1);
      sorted[tile_first[digit] + cursor[wave][digit] + local[j]] = key[j];
    }
  }
  __syncthreads();
  const int64_t left = n - tile_base;
  const int count = left < kTileKeys ? int(left) : kTileKeys;
#pragma unroll
  for (int k = 0; k < kKeysPerLane; ++k) {
    const int i = k * kSortThreads + threadIdx.x;
    if (i < count) {
      const uint64_t v = sorted[i];
      const uint32_t digit = uint32_t(v >> shift) & (kBins - 1);
      out[out_first[digit] + uint32_t(i) - tile_first[digit]] = v;
    }
  }
}

// ---- the distance ------------------------------------------------------------------------------------------
__device__ __forceinline__ double mapped(uint64_t key, const OperandParams& p) {
  const double v = value_of(key);
  return p.use_softmax != 0.0 ? exp(v - p.max) / p.exp_sum : v;
}

// stage 0: max |P_A - P_B|; stage 1: sum (|P_A - P_B| / m)^p.  grid (kStatGroups)
template <int kStage>
__global__ __launch_bounds__(kThreads) void k_distance(const uint64_t* __restrict__ sorted, int64_t n, int64_t chunk,
                                                       const OperandParams* __restrict__ params, double order,
                                                       const double* __restrict__ scalars,
                                                       double* __restrict__ partials) {
  const OperandParams pa = params[0], pb = params[1];
  const double m_all = kStage == 1 ? scalars[0] : 0.0;
  const int64_t begin = int64_t(blockIdx.x) * chunk;
  const int64_t end = begin + chunk < n ? begin + chunk : n;
  double s = 0.0, m = 0.0;
  for (int64_t i = begin + threadIdx.x; i < end; i += kThreads) {
    const double d = fabs(mapped(sorted[i], pa) - mapped(sorted[n + i], pb));
    if (kStage == 0) m = fmax(m, d);
    else if (m_all > 0.0) s += pow(d / m_all, order);
  }
  group_sum_max(s, m);
  if (threadIdx.x == 0) {
    partials[2 * blockIdx.x] = s;
    partials[2 * blockIdx.x + 1] = m;
  }
}

template <int kStage>
__global__ __launch_bounds__(kThreads) void k_distance_final(const double* __restrict__ partials, int groups,
                                                             double n, double order, double* __restrict__ scalars,
                                                             double* __restrict__ out) {
  double s = 0.0, m = 0.0;
  for (int g = threadIdx.x; g < groups; g += kThreads) {
    s += partials[2 * g];
    m = fmax(m, partials[2 * g + 1]);
  }
  group_sum_max(s, m);
  if (threadIdx.x == 0) {
    if (kStage == 0) {
      scalars[0] = m;
    } else {
      const double m_all = scalars[0];
      out[0] = m_all > 0.0 ? m_all * pow(s / n, 1.0 / order) : 0.0;
    }
  }
}

}  // namespace

size_t wasserstein_workspace_bytes(int64_t n_blocks) { return carve(nullptr, n_blocks, nullptr); }

int launch_approximate_wasserstein(const pbz_codec* c, int64_t n, const void* N1, const void* F1, const void* N2,
                                   const void* F2, double order, double* out, void* workspace, hipStream_t s) {
  Workspace w;
  carve(workspace, n, &w);
  double* means = reinterpret_cast<double*>(w.buf0);
  int st = launch_blockwise_mean(c, n, N1, F1, means, s);
  if (st != PBZ_OK) return st;
  st = launch_blockwise_mean(c, n, N2, F2, means + n, s);
  if (st != PBZ_OK) return st;

  int64_t chunk = ((n + kStatGroups - 1) / kStatGroups + kThreads - 1) / kThreads * kThreads;
  const int groups = int((n + chunk - 1) / chunk);
  hipLaunchKernelGGL(k_mean_stats<0>, dim3(groups, 2), dim3(kThreads), 0, s, means, n, chunk, w.params, w.partials);
  hipLaunchKernelGGL(k_mean_params<0>, dim3(2), dim3(kThreads), 0, s, w.partials, groups, w.params);
  hipLaunchKernelGGL(k_mean_stats<1>, dim3(groups, 2), dim3(kThreads), 0, s, means, n, chunk, w.params, w.partials);
  hipLaunchKernelGGL(k_mean_params<1>, dim3(2), dim3(kThreads), 0, s, w.partials, groups, w.params);
  st = hip_status(hipGetLastError());
  if (st != PBZ_OK) return st;

  const int64_t total = 2 * n;
  hipLaunchKernelGGL(k_to_keys, dim3(unsigned((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, w.buf0, total);
  const int64_t n_tiles = (n + kTileKeys - 1) / kTileKeys;
  uint64_t* src = w.buf0;
  uint64_t* dst = w.buf1;
  for (int pass = 0; pass < 64 / kRadixBits; ++pass) {
    const int shift = pass * kRadixBits;
    hipLaunchKernelGGL(k_radix_hist, dim3(unsigned(n_tiles), 2), dim3(kSortThreads), 0, s, src, n, n_tiles, shift, w.hist);
    hipLaunchKernelGGL(k_scan_digit, dim3(kBins, 2), dim3(kSortThreads), 0, s, w.hist, n_tiles, w.sums);
    hipLaunchKernelGGL(k_radix_scatter, dim3(unsigned(n_tiles), 2), dim3(kSortThreads), 0, s, src, dst, n, n_tiles, shift,
                       w.hist, w.sums);
    uint64_t* t = src;
    src = dst;
    dst = t;
  }
  st = hip_status(hipGetLastError());
  if (st != PBZ_OK) return st;
  // an even number of passes: the sorted keys are back in buf0 (== src)
  hipLaunchKernelGGL(k_distance<0>, dim3(groups), dim3(kThreads), 0, s, src, n, chunk, w.params, order, w.scalars,
                     w.partials);
  hipLaunchKernelGGL(k_distance_final<0>, dim3(1), dim3(kThreads), 0, s, w.partials, groups, double(n), order, w.scalars,
                     out);
  hipLaunchKernelGGL(k_distance<1>, dim3(groups), dim3(kThreads), 0, s, src, n, chunk, w.params, order, w.scalars,
                     w.partials);
  hipLaunchKernelGGL(k_distance_final<1>, dim3(1), dim3(kThreads), 0, s, w.partials, groups, double(n), order, w.scalars,
                     out);
  return hip_status(hipGetLastError());
}

}  // namespace pbz
