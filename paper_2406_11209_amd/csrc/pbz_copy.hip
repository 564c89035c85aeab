// pbz_stream_copy: a plain device-to-device copy kernel of known traffic (bytes read once, bytes written once).
// It is the yardstick of the measurements: its rate is the box's practical streaming bandwidth, quoted next to the
// datasheet peak, and hardware-counter runs scale FETCH_SIZE / WRITE_SIZE by what they read for it.
#include "pbz_internal.h"

namespace {

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;

// workgroup b copies the contiguous run of kCopyThreads * kCopyUnroll 16-byte vectors starting at b times that
__global__ __launch_bounds__(kCopyThreads) void k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                              int64_t nvec) {
  const int64_t base = int64_t(blockIdx.x) * (kCopyThreads * kCopyUnroll) + threadIdx.x;
  if (base + (kCopyUnroll - 1) * kCopyThreads < nvec) {
    uint4 v[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) v[u] = src[base + u * kCopyThreads];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) dst[base + u * kCopyThreads] = v[u];
  } else {
    for (int u = 0; u < kCopyUnroll; ++u) {
      const int64_t i = base + u * kCopyThreads;
      if (i < nvec) dst[i] = src[i];
    }
  }
}

__global__ __launch_bounds__(64) void k_copy_tail(const unsigned char* __restrict__ src,
                                                  unsigned char* __restrict__ dst, int n) {
  if (int(threadIdx.x) < n) dst[threadIdx.x] = src[threadIdx.x];
}

}  // namespace

extern "C" int pbz_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return PBZ_ERR_NULL;
  if (bytes == 0 || bytes > (size_t(1) << 43)) return PBZ_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) return PBZ_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t nvec = int64_t(bytes / 16);
  if (nvec > 0) {
    const int64_t per_group = int64_t(kCopyThreads) * kCopyUnroll;
    hipLaunchKernelGGL(k_stream_copy, dim3(unsigned((nvec + per_group - 1) / per_group)), dim3(kCopyThreads), 0, s,
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), nvec);
  }
  const int tail = int(bytes % 16);
  if (tail)
    hipLaunchKernelGGL(k_copy_tail, dim3(1), dim3(64), 0, s, static_cast<const unsigned char*>(src) + nvec * 16,
                       static_cast<unsigned char*>(dst) + nvec * 16, tail);
  return pbz::hip_status(hipGetLastError());
}
