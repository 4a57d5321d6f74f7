// Shared device/host helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ll.h"

namespace ll {

// Records a failed HIP call for ll_last_hip_error() and returns LL_EHIP.
int hip_failed(hipError_t e);

#define LL_HIP_CHECK(expr)                         \
  do {                                             \
    hipError_t e__ = (expr);                       \
    if (e__ != hipSuccess) return ll::hip_failed(e__); \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kWave = 64;

// ---- bf16 <-> fp32 on the device ------------------------------------------------------
// A bf16 value is the upper half of an fp32 word, so widening is a shift.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Two fp32 -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

// Sum over the 64 lanes of a wavefront; every lane gets the total.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

// Adds the squares of the 8 bf16 values in q: low halves into acc0, high halves into acc1.  The
// RMS statistic of every kernel goes through this (and wave_sum) so that all of them get the
// same bits for the same row.
__device__ __forceinline__ void accum_sq(const uint4 q, float& acc0, float& acc1) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = bf16_lo(w[i]), hi = bf16_hi(w[i]);
    acc0 = fmaf(lo, lo, acc0);
    acc1 = fmaf(hi, hi, acc1);
  }
}

__device__ __forceinline__ float inv_rms_from_sumsq(float ss, int d, float eps) {
  return 1.0f / sqrtf(ss / (float)d + eps);
}

}  // namespace ll
