// Capture store: appends the newest activations of every wrapped layer and activation type to
// the trajectories (paper Sec. 3.1, Stage 2; Alg. 1, Phase 1).  A strided copy, HBM-bound:
// 4 d bytes per appended row (read + write).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ll.h"
#include "ll_common.h"

namespace ll {
namespace {

// One wavefront per group of rows; a row is d bf16 = d/8 chunks of 16 bytes.  Row (lc, i) of the
// slices goes to row lc * T + t0 + i of the store.
__global__ __launch_bounds__(256) void ll_capture_append_kernel(const uint4* __restrict__ slices, uint4* __restrict__ store,
                                                                int64_t n_rows, int64_t n_tok, int64_t T, int64_t t0, int n16) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  for (int64_t row = wave; row < n_rows; row += n_waves) {
    const int64_t lc = row / n_tok, i = row - lc * n_tok;
    const uint4* src = slices + row * n16;
    uint4* dst = store + (lc * T + t0 + i) * n16;
    int c = lane;
    for (; c + 192 < n16; c += 256) {   // four loads in flight per lane
      const uint4 q0 = src[c], q1 = src[c + 64], q2 = src[c + 128], q3 = src[c + 192];
      dst[c] = q0;
      dst[c + 64] = q1;
      dst[c + 128] = q2;
      dst[c + 192] = q3;
    }
    for (; c < n16; c += 64) dst[c] = src[c];
  }
}

}  // namespace
}  // namespace ll

extern "C" {

int ll_capture_append(const ll_capture_shape* shape, void* store, const void* slices, int64_t t0, int64_t n_tok,
                      void* stream_) {
  if (shape == nullptr || shape->L <= 0 || shape->C <= 0 || shape->T <= 0 || shape->d <= 0 || (shape->d & 7) != 0)
    return LL_EINVAL;
  if (t0 < 0 || n_tok < 0 || t0 > shape->T || n_tok > shape->T - t0) return LL_EINVAL;
  if ((int64_t)shape->L * shape->C > INT64_MAX / shape->T) return LL_EINVAL;   // the store's row count fits 64 bits
  if (n_tok == 0) return LL_OK;
  if (store == nullptr || slices == nullptr || (((uintptr_t)store | (uintptr_t)slices) & 15)) return LL_EINVAL;
  const int64_t n_rows = (int64_t)shape->L * shape->C * n_tok;
  const int n16 = shape->d >> 3;
  // enough wavefronts to cover the chip several times over, never more than one per row
  int64_t blocks = (n_rows + 3) / 4;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(ll::ll_capture_append_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream_),
                     static_cast<const uint4*>(slices), static_cast<uint4*>(store), n_rows, n_tok, shape->T, t0, n16);
  LL_HIP_CHECK(hipGetLastError());
  return LL_OK;
}

}  // extern "C"
