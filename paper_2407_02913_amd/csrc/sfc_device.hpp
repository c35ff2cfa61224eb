// Small device-side helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

namespace sfc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v3i __attribute__((ext_vector_type(3)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kBufferFlags = 0x00020000;  // raw buffer descriptor word 3: 32-bit data format
constexpr int kStreamStore = 2;           // buffer cache policy "nt": written once, not re-read here

// Workgroups are dealt to the 8 XCDs round-robin by id.  Maps an id to a position
// such that ids congruent modulo 8 (same XCD, same L2) cover one contiguous range.
__device__ __forceinline__ int xcd_contiguous(int id, int n) {
  const int q = n >> 3, r = n & 7;
  const int xcd = id & 7, idx = id >> 3;
  return xcd * q + min(xcd, r) + idx;
}

// round-half-even(v * inv) clamped to [-qmax, qmax] (qmax = 2^(bits-1) - 1, at most 127),
// as the low byte of the result.  Adding 1.5 * 2^23 inside one fused multiply-add rounds
// the exact product once, to an integer, ties to even; the integer then sits in the low
// mantissa bits.
__device__ __forceinline__ unsigned quantize_byte(int v, float inv, float qmax) {
  constexpr float kMagic = 12582912.0f;
  float t = __fmaf_rn((float)v, inv, kMagic);
  t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
  return __float_as_uint(t);
}

}  // namespace sfc
