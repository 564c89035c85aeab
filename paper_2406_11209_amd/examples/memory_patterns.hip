// What the memory system of the GPU gives for the access patterns of the codec kernels, with no arithmetic at all:
// the yardsticks that the measured kernel times are set against.  Stand-alone (HIP runtime only; it does not use the
// library).  Every kernel reads or writes exactly the bytes of the pattern it stands for, once.
//
//   ./memory_patterns            all cases
//
// Cases (MI355X figures in the repository's profile summaries):
//   lane 4x4x4 FP64   the decompress of a 512^3 FP64 array in 4x4x4 blocks with int16 indices: a lane owns a block,
//                     a wave 64 blocks along x; per lane eight 16-byte loads of F and one of N, then 32 store
//                     instructions per wave that each cover one contiguous KiB (the half-waves have traded pieces).
//                     Loads alone, stores alone, both; stores with and without the non-temporal hint; the same
//                     bytes in other arrangements: every wave writing 16 rows of one plane and its workgroup 128
//                     contiguous KiB of that plane (not reachable with blocks that span four planes), and the two
//                     arrangements a workgroup can reach by trading planes between its waves (wave w on plane w).
//   oct 8x8x8 16-bit  a 1024 x 1024 x 512 array of 2-byte elements in 8x8x8 blocks, 8 blocks per wave: lane = (plane,
//                     block), one row per instruction, against a linear sweep; loads and stores.
//   small read        a 68 MiB buffer (the compressed operand of that array) read by nothing but loads, for several
//                     grids: the floor of any reduction over it.
//   vector ALU        sixteen independent chains of one instruction type per lane and no memory access, eight waves
//                     per SIMD: how often a SIMD issues a vector instruction of that type and operand form, the
//                     yardstick for kernels whose time is their arithmetic.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                     \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      std::exit(1);                                                                  \
    }                                                                                \
  } while (0)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kReps = 20;

template <typename Launch>
float time_ms(Launch launch, int reps = kReps) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  for (int it = 0; it < 3; ++it) launch();
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  for (int it = 0; it < reps; ++it) launch();
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms = 0.f;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  CHECK(hipGetLastError());
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return ms / reps;
}

// ---- lane 4x4x4 FP64 ----------------------------------------------------------------------------------------
constexpr int64_t LX = 512, LY = 512, LZ = 512, LGX = LX / 4, LGY = LY / 4, LGZ = LZ / 4;
constexpr int64_t kPlanePieces = LX * LY / 2;            // 16-byte pieces per z-plane

// kLoads / kStores: which half of the pattern runs; kHint: non-temporal stores; kArrange: who writes what (the same
// bytes over the whole launch): 0 the decompress kernel's (a wave: its blocks' 4 rows of 4 planes); 1 a wave: 16
// half rows of one plane, its workgroup: 32 whole rows of that plane; 2 workgroup: four block rows of one half row,
// wave w on plane w; 3 workgroup: two block rows by both half rows, wave w on plane w
template <bool kLoads, bool kStores, bool kHint, int kArrange>
__global__ __launch_bounds__(256) void k_lane(const u32x4* __restrict__ F, const double* __restrict__ N,
                                              u32x4* __restrict__ y, uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);      // 64 blocks along x, then y, then z
  constexpr int64_t tiles_x = LGX / 64;
  const int64_t tx = tile % tiles_x, by = (tile / tiles_x) % LGY, bz = tile / (tiles_x * LGY);
  const int64_t block = (bz * LGY + by) * LGX + tx * 64 + lane;
  u32x4 w[8];
  if (kLoads) {
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = F[block * 8 + k];
    w[0].x ^= uint32_t(__double_as_longlong(N[block]));
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      w[k].x = uint32_t(lane); w[k].y = uint32_t(k); w[k].z = 3u; w[k].w = 4u;
    }
  }
  if (!kStores) {
    uint32_t acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc ^= w[k].x ^ w[k].y ^ w[k].z ^ w[k].w;
    if (acc == 0x12345678u) sink[0] = acc;           // keeps the loads alive; practically never true
    return;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    u32x4* p;
    const int wave = threadIdx.x >> 6;
    if (kArrange == 1) {
      const int64_t half = tile & 1, group = (tile >> 1) % (LY / 16), plane = tile / (2 * (LY / 16));
      p = y + plane * kPlanePieces + ((group * 16 + r) * LX + half * 256) / 2 + lane;
    } else if (kArrange == 2) {
      const int64_t wg = blockIdx.x, half = wg % tiles_x, quad = (wg / tiles_x) % (LGY / 4), slab = wg / (tiles_x * (LGY / 4));
      p = y + (slab * 4 + wave) * kPlanePieces + ((quad * 16 + r) * LX + half * 256) / 2 + lane;
    } else if (kArrange == 3) {
      const int64_t wg = blockIdx.x, pair = wg % (LGY / 2), slab = wg / (LGY / 2);
      p = y + (slab * 4 + wave) * kPlanePieces + ((pair * 8 + (r >> 1)) * LX + (r & 1) * 256) / 2 + lane;
    } else {
      const int z = r >> 2, yy = r & 3;
      p = y + (bz * 4 + z) * kPlanePieces + ((by * 4 + yy) * LX + tx * 256) / 2 + 2 * (lane & 31) + (lane >> 5);
    }
    if (kHint) {
      __builtin_nontemporal_store(w[r & 7], p);
      __builtin_nontemporal_store(w[(r + 1) & 7], p + 64);
    } else {
      p[0] = w[r & 7];
      p[64] = w[(r + 1) & 7];
    }
  }
}

// the compress direction of the same array: 32 load instructions per wave that each cover one contiguous KiB of the
// array (non-temporal, as in the kernel), then F as eight contiguous KiB per wave and N
__global__ __launch_bounds__(256) void k_lane_compress(const u32x4* __restrict__ x, u32x4* __restrict__ F,
                                                       double* __restrict__ N) {
  const int lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  constexpr int64_t tiles_x = LGX / 64;
  const int64_t tx = tile % tiles_x, by = (tile / tiles_x) % LGY, bz = tile / (tiles_x * LGY);
  u32x4 w[32];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int z = r >> 2, yy = r & 3;
    const u32x4* p = x + (bz * 4 + z) * kPlanePieces + ((by * 4 + yy) * LX + tx * 256) / 2 + 2 * (lane & 31) + (lane >> 5);
    w[2 * r] = __builtin_nontemporal_load(p);
    w[2 * r + 1] = __builtin_nontemporal_load(p + 64);
  }
  u32x4 acc = w[0];
#pragma unroll
  for (int i = 1; i < 32; ++i) acc ^= w[i];
  const int64_t block0 = (bz * LGY + by) * LGX + tx * 64;
#pragma unroll
  for (int k = 0; k < 8; ++k) F[block0 * 8 + k * 64 + lane] = acc + uint32_t(k);
  N[block0 + lane] = double(acc.x);
}

template <bool kLoads, bool kStores, bool kHint, int kArrange>
void lane_case(const char* what, const u32x4* F, const double* N, u32x4* y, uint32_t* sink) {
  const unsigned grid = unsigned(LGX * LGY * LGZ / 64 / 4);
  const float ms = time_ms([&] {
    hipLaunchKernelGGL((k_lane<kLoads, kStores, kHint, kArrange>), dim3(grid), dim3(256), 0, 0, F, N, y, sink);
  });
  const double bytes = (kLoads ? double(LGX * LGY * LGZ) * 136.0 : 0.0) + (kStores ? double(LX * LY * LZ) * 8.0 : 0.0);
  std::printf("lane 4x4x4 FP64   %-68s %.3f ms  %5.0f GB/s\n", what, ms, bytes / ms / 1e6);
}

// ---- oct 8x8x8, 2-byte elements -------------------------------------------------------------------------------
constexpr int64_t OX = 512, OY = 1024, OZ = 1024, OGX = OX / 8, OGY = OY / 8, OGZ = OZ / 8;
constexpr int64_t kRowPieces = OX * 2 / 16;

template <bool kLinear, bool kStore>
__global__ __launch_bounds__(256) void k_oct(u32x4* __restrict__ a, uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  constexpr int64_t tiles_x = OGX / 8;
  const int64_t tx = tile % tiles_x, by = (tile / tiles_x) % OGY, bz = tile / (tiles_x * OGY);
  const int plane = lane >> 3, b = lane & 7;
  uint32_t acc = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int64_t at = kLinear ? tile * 512 + k * 64 + lane
                               : ((bz * 8 + plane) * OY + by * 8 + k) * kRowPieces + tx * 8 + b;
    if (kStore) {
      u32x4 v;
      v.x = uint32_t(lane); v.y = uint32_t(k); v.z = 1u; v.w = 2u;
      a[at] = v;
    } else {
      const u32x4 v = a[at];
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  if (!kStore && acc == 0x12345678u) sink[0] = acc;
}

template <bool kLinear, bool kStore>
void oct_case(const char* what, u32x4* a, uint32_t* sink) {
  const unsigned grid = unsigned(OGX * OGY * OGZ / 8 / 4);
  const float ms = time_ms([&] { hipLaunchKernelGGL((k_oct<kLinear, kStore>), dim3(grid), dim3(256), 0, 0, a, sink); });
  std::printf("oct 8x8x8 16-bit  %-68s %.3f ms  %5.0f GB/s\n", what, ms, double(OX * OY * OZ * 2) / ms / 1e6);
}

// ---- small read --------------------------------------------------------------------------------------------
template <int kInFlight>
__global__ __launch_bounds__(256) void k_read(const u32x4* __restrict__ a, int64_t nvec, int64_t chunk, uint32_t* sink) {
  const int64_t v0 = int64_t(blockIdx.x) * chunk, v1 = v0 + chunk < nvec ? v0 + chunk : nvec;
  uint32_t acc = 0;
  for (int64_t v = v0 + threadIdx.x; v < v1; v += 256 * kInFlight) {
    u32x4 w[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int64_t i = v + u * 256;
      w[u] = a[i < v1 ? i : v1 - 1];
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) acc += w[u].x ^ w[u].y ^ w[u].z ^ w[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;
}

template <int kInFlight>
void read_case(const u32x4* a, int64_t nvec, int groups, uint32_t* sink) {
  int64_t chunk = (nvec + groups - 1) / groups;
  chunk = (chunk + 256 * kInFlight - 1) / (256 * kInFlight) * (256 * kInFlight);
  const int g = int((nvec + chunk - 1) / chunk);
  const float ms = time_ms([&] { hipLaunchKernelGGL((k_read<kInFlight>), dim3(g), dim3(256), 0, 0, a, nvec, chunk, sink); }, 50);
  std::printf("small read        68 MiB, %4d workgroups, %d loads in flight per thread          %.2f us per launch  %5.0f GB/s\n",
              g, kInFlight, ms * 1e3, double(nvec) * 16.0 / ms / 1e6);
}

// ---- vector ALU issue rate -------------------------------------------------------------------------------------
struct OpFma { template <typename T> static __device__ __forceinline__ T run(T a, T b, T c) { return a * b + c; } };
struct OpAdd { template <typename T> static __device__ __forceinline__ T run(T a, T, T c) { return a + c; } };
struct OpMul { template <typename T> static __device__ __forceinline__ T run(T a, T b, T) { return a * b; } };
struct OpMax { static __device__ __forceinline__ float run(float a, float, float c) { return fmaxf(a, c); } };
struct OpRint { static __device__ __forceinline__ float run(float a, float, float) { return rintf(a); } };
struct OpXor { static __device__ __forceinline__ uint32_t run(uint32_t a, uint32_t, uint32_t c) { return a ^ c; } };
struct OpShl { static __device__ __forceinline__ uint32_t run(uint32_t a, uint32_t b, uint32_t) { return a << (b & 31); } };

// kScalarOperand: b and c stay what kernel arguments are, scalar registers; otherwise they are moved to vector registers
template <typename T, typename Op, bool kScalarOperand>
__global__ __launch_bounds__(256) void k_alu(T* out, T b, T c, int iters) {
  constexpr int kChains = 16;
  T a[kChains];
#pragma unroll
  for (int i = 0; i < kChains; ++i) a[i] = T(threadIdx.x + i);
  if constexpr (!kScalarOperand) {
    b += T(threadIdx.x >> 20);
    c += T(threadIdx.x >> 21);
    asm volatile("" : "+v"(b), "+v"(c));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kChains; ++i) a[i] = Op::run(a[i], b, c);
  }
  T s = 0;
#pragma unroll
  for (int i = 0; i < kChains; ++i) s += a[i];
  if (s == T(123456)) out[threadIdx.x] = s;      // never true for the operands used: keeps the chains alive
}

template <typename T, typename Op, bool kScalarOperand = false>
void alu_case(const char* what, void* out) {
  // 64 workgroups of four waves per compute unit (256 units), eight resident at a time
  const int iters = 512, groups = 256 * 64;
  const float ms = time_ms([&] {
    hipLaunchKernelGGL((k_alu<T, Op, kScalarOperand>), dim3(groups), dim3(256), 0, 0, static_cast<T*>(out), T(3), T(5), iters);
  }, 5);
  const double per_simd = double(iters) * 16 * (groups / 256);        // wave-instructions per SIMD: one wave of a workgroup each
  std::printf("vector ALU        %-68s %.3f ms  %.2f ns per wave-instruction per SIMD\n", what, ms, ms * 1e6 / per_simd);
}

}  // namespace

int main() {
  uint32_t* sink;
  CHECK(hipMalloc(&sink, 64));
  {
    const size_t n_blocks = size_t(LGX * LGY * LGZ);
    u32x4 *F, *y;
    double* N;
    CHECK(hipMalloc(&F, n_blocks * 128));
    CHECK(hipMalloc(&N, n_blocks * 8));
    CHECK(hipMalloc(&y, size_t(LX * LY * LZ) * 8));
    CHECK(hipMemset(F, 1, n_blocks * 128));
    CHECK(hipMemset(N, 0, n_blocks * 8));
    lane_case<true, false, false, 0>("loads only (F and N: 272 MiB)", F, N, y, sink);
    lane_case<false, true, false, 0>("stores only (1 GiB), 4 rows of 4 planes per wave", F, N, y, sink);
    lane_case<false, true, true, 0>("stores only, non-temporal", F, N, y, sink);
    lane_case<false, true, false, 1>("stores only, wave and workgroup on one plane", F, N, y, sink);
    lane_case<true, true, false, 0>("loads + stores", F, N, y, sink);
    lane_case<true, true, true, 0>("loads + stores, non-temporal stores", F, N, y, sink);
    lane_case<true, true, false, 1>("loads + stores, wave and workgroup on one plane", F, N, y, sink);
    lane_case<true, true, true, 1>("the same, non-temporal stores", F, N, y, sink);
    lane_case<true, true, true, 2>("non-temporal, workgroup: 4 block rows, wave w on plane w", F, N, y, sink);
    lane_case<true, true, true, 3>("non-temporal, workgroup: 2 block rows x 2 halves, wave w on plane w", F, N, y, sink);
    lane_case<true, true, true, 0>("loads + stores, non-temporal stores (again)", F, N, y, sink);
    {
      const unsigned grid = unsigned(LGX * LGY * LGZ / 64 / 4);
      const float ms = time_ms([&] { hipLaunchKernelGGL(k_lane_compress, dim3(grid), dim3(256), 0, 0, y, F, N); });
      std::printf("lane 4x4x4 FP64   %-68s %.3f ms  %5.0f GB/s\n", "compress direction: array loads (1 GiB), F and N stores (272 MiB)",
                  ms, (double(LGX * LGY * LGZ) * 136.0 + double(LX * LY * LZ) * 8.0) / ms / 1e6);
    }
    CHECK(hipFree(F));
    CHECK(hipFree(N));
    CHECK(hipFree(y));
  }
  {
    u32x4* a;
    CHECK(hipMalloc(&a, size_t(OX * OY * OZ) * 2));
    CHECK(hipMemset(a, 1, size_t(OX * OY * OZ) * 2));
    oct_case<false, false>("loads, lane = (plane, block), one row per instruction", a, sink);
    oct_case<true, false>("loads, linear", a, sink);
    oct_case<false, true>("stores, lane = (plane, block), one row per instruction", a, sink);
    oct_case<true, true>("stores, linear", a, sink);
    CHECK(hipFree(a));
  }
  {
    const int64_t bytes = 71303168;          // N (4 MiB) + F (64 MiB) of the 1024 x 1024 x 512 array, 4x4x4 kept of 8x8x8
    u32x4* a;
    CHECK(hipMalloc(&a, size_t(bytes)));
    CHECK(hipMemset(a, 1, size_t(bytes)));
    for (int groups : {256, 1024, 4096}) {
      read_case<4>(a, bytes / 16, groups, sink);
      read_case<8>(a, bytes / 16, groups, sink);
    }
    CHECK(hipFree(a));
  }
  alu_case<float, OpFma>("FP32 multiply-add, vector-register operands", sink);
  alu_case<float, OpAdd>("FP32 add", sink);
  alu_case<float, OpMul>("FP32 multiply", sink);
  alu_case<float, OpAdd, true>("FP32 add, one operand a scalar register", sink);
  alu_case<float, OpFma, true>("FP32 multiply-add, two operands scalar registers", sink);
  alu_case<float, OpMax>("FP32 maximum (two instructions: one operand is canonicalised first)", sink);
  alu_case<float, OpRint>("FP32 round to integer", sink);
  alu_case<uint32_t, OpXor>("32-bit xor", sink);
  alu_case<uint32_t, OpShl>("32-bit shift", sink);
  alu_case<double, OpFma>("FP64 multiply-add", sink);
  alu_case<double, OpAdd>("FP64 add", sink);
  CHECK(hipFree(sink));
  return 0;
}
