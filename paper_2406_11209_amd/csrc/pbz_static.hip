// pbz_segmented_static: the segmented reductions for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  It is pbz_segmented with the workspace
// argument replaced by a fixed array in the library's own device image, so the call needs no buffer beyond its
// operands and result and never reaches hipMalloc / hipFree.
#include "pbz_internal.h"

// The reductions' scratch: one record of partial sums per workgroup (kWorkspaceBytes = 256 KiB).  Every GPU the
// library runs on holds its own copy of this array until the process ends.
static __device__ __align__(256) unsigned char scratch[pbz::kWorkspaceBytes];
static_assert(pbz::kReduceMaxGroups == PBZ_STATIC_MAX_SEGMENTS, "one record per segment must fit the array");

namespace {

// Device address of `scratch` on each GPU.  The array's name is only a host-side handle here: what kernels and
// copies need is the address hipGetSymbolAddress reports, which differs from GPU to GPU.
std::mutex g_mu;
void* g_scratch_ptr[pbz::kMaxDevices] = {};

// keeps the array in the device image even though no kernel names it (kernels receive its address as an argument)
__global__ void k_scratch_anchor(unsigned char* out) {
  if (out) out[0] = scratch[0];
}

int scratch_address(void** ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= pbz::kMaxDevices) return PBZ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PBZ_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return PBZ_OK;
}

}  // namespace

extern "C" int pbz_segmented_static(const pbz_codec* c, pbz_statistic stat, int64_t n_segments,
                                    int64_t blocks_per_segment, const void* N1, const void* F1, const void* N2,
                                    const void* F2, double* out, void* stream) {
  using namespace pbz;
  if (!c || !N1 || !F1 || !out) return PBZ_ERR_NULL;
  if (int(stat) < 0 || int(stat) > int(PBZ_STAT_DIFFERENCE_NORM2)) return PBZ_ERR_TYPE;
  const bool two = stat == PBZ_STAT_DOT || stat == PBZ_STAT_COSINE_SIMILARITY || stat == PBZ_STAT_COVARIANCE ||
                   stat == PBZ_STAT_DIFFERENCE_NORM2;
  const bool needs_dc = stat == PBZ_STAT_MEAN || stat == PBZ_STAT_COVARIANCE || stat == PBZ_STAT_VARIANCE;
  if (two && (!N2 || !F2)) return PBZ_ERR_NULL;
  if (blocks_per_segment < 1 || n_segments < 1) return PBZ_ERR_SHAPE;
  // the array holds one batch of partial records: at most PBZ_STATIC_MAX_SEGMENTS segments and
  // PBZ_STATIC_MAX_ELEMENTS coefficients (before pruning) per call
  if (n_segments > PBZ_STATIC_MAX_SEGMENTS) return PBZ_ERR_CAPACITY;
  if (blocks_per_segment > PBZ_STATIC_MAX_ELEMENTS / c->vol / n_segments) return PBZ_ERR_CAPACITY;
  if (needs_dc && !c->dc_kept) return PBZ_ERR_DC_PRUNED;
  void* ws = nullptr;
  const int st = scratch_address(&ws);
  if (st != PBZ_OK) return st;
  const ReduceOp op = stat == PBZ_STAT_DIFFERENCE_NORM2 ? kDiffNorm2 : ReduceOp(int(stat));
  // every record the final kernel reads is written by this call's streaming kernel first: nothing needs clearing
  return launch_reduce(c, op, blocks_per_segment, N1, F1, two ? N2 : nullptr, two ? F2 : nullptr, out, ws,
                       static_cast<hipStream_t>(stream), nullptr, n_segments);
}
