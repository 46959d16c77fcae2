// Small device helpers shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace la {

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest even; inputs here are finite
__device__ __forceinline__ uint16_t float_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_as_float(const T *p);
template <> __device__ __forceinline__ float load_as_float<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t *p) { return bf16_to_float(*p); }

template <> __device__ __forceinline__ float load_as_float<_Float16>(const _Float16 *p) { return (float)*p; }

template <typename T> __device__ __forceinline__ void store_from_float(T *p, float v);
template <> __device__ __forceinline__ void store_from_float<_Float16>(_Float16 *p, float v) { *p = (_Float16)v; }
template <> __device__ __forceinline__ void store_from_float<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_float<uint16_t>(uint16_t *p, float v) { *p = float_to_bf16(v); }

// Index of V[row][h][c] inside one layer of the cache.
// Row-major: [row][Hkv][dh].  Key-blocked (MFMA path): positions are grouped in blocks of
// 32; inside a block the 32 positions of one (head, channel) are contiguous and permuted so
// that the 8 values one MFMA lane needs (positions 4q..4q+3 and 16+4q..16+4q+3, q = 0..3)
// are 16 contiguous bytes: position p = 16*b + 4*q + i is stored at slot 8*q + 4*b + i.
__host__ __device__ __forceinline__ size_t v_index(bool blocked, int row, int h, int c, int Hkv, int dh) {
  if (!blocked) return ((size_t)row * Hkv + h) * dh + c;
  int blk = row >> 5, p = row & 31;
  int slot = 8 * ((p & 15) >> 2) + 4 * (p >> 4) + (p & 3);
  return (((size_t)blk * Hkv + h) * dh + c) * 32 + slot;
}

}  // namespace la
