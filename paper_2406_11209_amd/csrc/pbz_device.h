// Device-side helpers: storage-type loads / stores and wave-level reductions (wave64, gfx950).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "pbz.h"

namespace pbz {

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(uint32_t(b) << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// double -> bf16 with a single rounding: round to odd into float first, so that the second rounding
// (float -> bf16, 16 fewer bits) cannot double-round.
__device__ __forceinline__ uint16_t double_to_bf16_bits(double d) {
  float f = __double2float_rz(d);
  if (double(f) != d && !(d != d)) {
    uint32_t u = __float_as_uint(f);
    u |= 1u;  // sticky bit: truncation toward zero then "or 1" is round-to-odd
    f = __uint_as_float(u);
  }
  return float_to_bf16_bits(f);
}

__device__ __forceinline__ _Float16 double_to_f16(double d) {
  float f = __double2float_rz(d);
  if (double(f) != d && !(d != d)) f = __uint_as_float(__float_as_uint(f) | 1u);
  return _Float16(f);
}

template <typename T>
__device__ __forceinline__ T load_float(const void* p, int ftype, int64_t i) {
  switch (ftype) {
    case PBZ_F64: return T(static_cast<const double*>(p)[i]);
    case PBZ_F32: return T(static_cast<const float*>(p)[i]);
    case PBZ_BF16: return T(bf16_bits_to_float(static_cast<const uint16_t*>(p)[i]));
    default: return T(float(static_cast<const _Float16*>(p)[i]));
  }
}

__device__ __forceinline__ void store_float(void* p, int ftype, int64_t i, float v) {
  switch (ftype) {
    case PBZ_F64: static_cast<double*>(p)[i] = double(v); break;
    case PBZ_F32: static_cast<float*>(p)[i] = v; break;
    case PBZ_BF16: static_cast<uint16_t*>(p)[i] = float_to_bf16_bits(v); break;
    default: static_cast<_Float16*>(p)[i] = _Float16(v); break;
  }
}

__device__ __forceinline__ void store_float(void* p, int ftype, int64_t i, double v) {
  switch (ftype) {
    case PBZ_F64: static_cast<double*>(p)[i] = v; break;
    case PBZ_F32: static_cast<float*>(p)[i] = float(v); break;
    case PBZ_BF16: static_cast<uint16_t*>(p)[i] = double_to_bf16_bits(v); break;
    default: static_cast<_Float16*>(p)[i] = double_to_f16(v); break;
  }
}

__device__ __forceinline__ int64_t load_index(const void* p, int itype, int64_t i) {
  switch (itype) {
    case PBZ_I8: return static_cast<const int8_t*>(p)[i];
    case PBZ_I16: return static_cast<const int16_t*>(p)[i];
    default: return static_cast<const int32_t*>(p)[i];
  }
}

__device__ __forceinline__ void store_index(void* p, int itype, int64_t i, int64_t v) {
  switch (itype) {
    case PBZ_I8: static_cast<int8_t*>(p)[i] = int8_t(v); break;
    case PBZ_I16: static_cast<int16_t*>(p)[i] = int16_t(v); break;
    default: static_cast<int32_t*>(p)[i] = int32_t(v); break;
  }
}

// sum over the 64 lanes of a wave; every lane gets the total.  Fixed butterfly order.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

}  // namespace pbz
