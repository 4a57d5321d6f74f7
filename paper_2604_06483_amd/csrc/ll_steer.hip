// Steering direction (paper Sec. 3.4, Eq. 2) and post-norm injection (Eq. 3) for gfx950.
// Both are bandwidth-bound: 16-byte loads, fp32 arithmetic, no atomics.
#include "ll_common.h"

#include <math.h>

namespace {

using namespace ll;

constexpr int STEER_SLICES = 64;     // row slices of the two-stage column sum
constexpr int COLS_PER_BLOCK = 512;  // one wavefront's 16-byte loads cover 512 bf16 columns

// ---------------------------------------------------------------------------------------
// Column sums.  Block (x, y): columns [512 x, 512 x + 512), row slice y; its 4 wavefronts take
// rows y*4 + w, stepping by 4 * slices.  DIRECT (one slice): writes mean(target) - mean(base)
// straight to `out`; otherwise writes the two partial sums to part[2][slices][d].
// ---------------------------------------------------------------------------------------
template <bool DIRECT>
__global__ __launch_bounds__(256) void ll_steer_colsum_kernel(const uint16_t* __restrict__ base, int64_t n_base,
                                                              const uint16_t* __restrict__ target, int64_t n_target,
                                                              int d, int slices, float* __restrict__ out) {
  __shared__ float red[2][4][COLS_PER_BLOCK];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int col0 = blockIdx.x * COLS_PER_BLOCK + lane * 8;
  const bool active = col0 < d;
  const int64_t first = (int64_t)blockIdx.y * 4 + wave;
  const int64_t step = (int64_t)slices * 4;

  float sum[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[s][i] = 0.f;

#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const uint16_t* src = s == 0 ? base : target;
    const int64_t n = s == 0 ? n_base : n_target;
    if (active) {
      for (int64_t r = first; r < n; r += step) {
        const uint4 q = *reinterpret_cast<const uint4*>(src + r * d + col0);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sum[s][2 * i] += bf16_lo(w[i]);
          sum[s][2 * i + 1] += bf16_hi(w[i]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[s][wave][lane * 8 + i] = sum[s][i];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < COLS_PER_BLOCK; c += 256) {
    const int col = blockIdx.x * COLS_PER_BLOCK + c;
    if (col >= d) continue;
    const float sb = (red[0][0][c] + red[0][1][c]) + (red[0][2][c] + red[0][3][c]);
    const float st = (red[1][0][c] + red[1][1][c]) + (red[1][2][c] + red[1][3][c]);
    if (DIRECT) {
      out[col] = st / (float)n_target - sb / (float)n_base;
    } else {
      out[(int64_t)blockIdx.y * d + col] = sb;
      out[((int64_t)slices + blockIdx.y) * d + col] = st;
    }
  }
}

// Many slices: one thread per column sums them (consecutive threads, consecutive columns) and
// writes the difference of means; the one-workgroup finish below then only normalises.
__global__ __launch_bounds__(256) void ll_steer_reduce_kernel(const float* __restrict__ part, int slices, int64_t n_base,
                                                              int64_t n_target, int d, float* __restrict__ out_v) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= d) return;
  float sb = 0.f, st = 0.f;
  for (int s = 0; s < slices; ++s) {
    sb += part[(int64_t)s * d + c];
    st += part[((int64_t)slices + s) * d + c];
  }
  out_v[c] = st / (float)n_target - sb / (float)n_base;
}

// Finish: (sum the slices,) form the difference of means, L2-normalise.  One workgroup.
template <bool DIRECT>
__global__ __launch_bounds__(1024) void ll_steer_finish_kernel(const float* __restrict__ part, int slices, int64_t n_base,
                                                               int64_t n_target, int d, int normalize,
                                                               float* __restrict__ out_v) {
  __shared__ float red[16];
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 1024) {
    float diff;
    if (DIRECT) {
      diff = out_v[c];
    } else {
      float sb = 0.f, st = 0.f;
      for (int s = 0; s < slices; ++s) {
        sb += part[(int64_t)s * d + c];
        st += part[((int64_t)slices + s) * d + c];
      }
      diff = st / (float)n_target - sb / (float)n_base;
      out_v[c] = diff;
    }
    ss = fmaf(diff, diff, ss);
  }
  if (!normalize) return;
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float inv = tot > 0.f ? 1.0f / sqrtf(tot) : 0.f;
  for (int c = threadIdx.x; c < d; c += 1024) out_v[c] *= inv;   // each thread rescales what it wrote
}

// ---------------------------------------------------------------------------------------
// Injection: out = bf16(gamma * h * inv_rms + alpha * v).  One wavefront per row; the row is
// kept in registers between the statistic and the write when it fits (NITER 16-byte loads per
// lane), otherwise it is read twice.
// ---------------------------------------------------------------------------------------
template <int NITER>
__global__ __launch_bounds__(256) void ll_steer_inject_kernel(const uint16_t* hidden, const uint16_t* __restrict__ gamma,
                                                              const float* __restrict__ v, uint16_t* out, int64_t n_rows,
                                                              int d, float eps, float alpha) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const uint4* src = reinterpret_cast<const uint4*>(hidden + row * (int64_t)d);
  uint4* dst = reinterpret_cast<uint4*>(out + row * (int64_t)d);
  const uint4* g4 = reinterpret_cast<const uint4*>(gamma);
  const float4* v4 = reinterpret_cast<const float4*>(v);
  const int n16 = d >> 3;

  float acc0 = 0.f, acc1 = 0.f;
  uint4 cache[NITER > 0 ? NITER : 1];
  if (NITER > 0) {
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
      const int c = lane + 64 * it;
      if (c < n16) {
        cache[it] = src[c];
        accum_sq(cache[it], acc0, acc1);
      }
    }
  } else {
    for (int c = lane; c < n16; c += 64) accum_sq(src[c], acc0, acc1);
  }
  const float inv = inv_rms_from_sumsq(wave_sum(acc0 + acc1), d, eps);

  auto emit = [&](int c, const uint4 q) {
    const uint4 g = g4[c];
    const float4 va = v4[2 * c], vb = v4[2 * c + 1];
    const uint32_t hw[4] = {q.x, q.y, q.z, q.w};
    const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
    const float vv[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
    uint32_t ow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lo = fmaf(alpha, vv[2 * i], bf16_lo(hw[i]) * inv * bf16_lo(gw[i]));
      const float hi = fmaf(alpha, vv[2 * i + 1], bf16_hi(hw[i]) * inv * bf16_hi(gw[i]));
      ow[i] = pack_bf16(lo, hi);
    }
    dst[c] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  };
  if (NITER > 0) {
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
      const int c = lane + 64 * it;
      if (c < n16) emit(c, cache[it]);
    }
  } else {
    for (int c = lane; c < n16; c += 64) emit(c, src[c]);
  }
}

// In-model injection with the two safeguards (Sec. 3.4, stability paragraph): out = bf16(h + beta v)
// with beta = s clipped in magnitude to clip_ratio times the row's L2 norm (s = alpha times the
// layer's scale; clip_ratio <= 0: no clipping).  Same shape as the kernel above, without the norm.
template <int NITER>
__global__ __launch_bounds__(256) void ll_steer_inject_raw_kernel(const uint16_t* hidden, const float* __restrict__ v,
                                                                  uint16_t* out, int64_t n_rows, int d, float s,
                                                                  float clip_ratio) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const uint4* src = reinterpret_cast<const uint4*>(hidden + row * (int64_t)d);
  uint4* dst = reinterpret_cast<uint4*>(out + row * (int64_t)d);
  const float4* v4 = reinterpret_cast<const float4*>(v);
  const int n16 = d >> 3;

  float acc0 = 0.f, acc1 = 0.f;
  uint4 cache[NITER > 0 ? NITER : 1];
  if (NITER > 0) {
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
      const int c = lane + 64 * it;
      if (c < n16) {
        cache[it] = src[c];
        accum_sq(cache[it], acc0, acc1);
      }
    }
  } else {
    for (int c = lane; c < n16; c += 64) accum_sq(src[c], acc0, acc1);
  }
  float beta = s;
  if (clip_ratio > 0.f) {
    const float cap = clip_ratio * sqrtf(wave_sum(acc0 + acc1));
    beta = copysignf(fminf(fabsf(s), cap), s);
  }

  auto emit = [&](int c, const uint4 q) {
    const float4 va = v4[2 * c], vb = v4[2 * c + 1];
    const uint32_t hw[4] = {q.x, q.y, q.z, q.w};
    const float vv[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
    uint32_t ow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      ow[i] = pack_bf16(fmaf(beta, vv[2 * i], bf16_lo(hw[i])), fmaf(beta, vv[2 * i + 1], bf16_hi(hw[i])));
    dst[c] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  };
  if (NITER > 0) {
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
      const int c = lane + 64 * it;
      if (c < n16) emit(c, cache[it]);
    }
  } else {
    for (int c = lane; c < n16; c += 64) emit(c, src[c]);
  }
}

// one wavefront per row, four rows per workgroup, and the grid's x extent is a 31-bit number
constexpr int64_t kMaxInjectRows = (int64_t)4 * 0x7fffffff;

}  // namespace

extern "C" {

int ll_steer_inject_raw(const ll_shape* shape, const void* hidden, const float* v, float alpha, float layer_scale,
                        float clip_ratio, void* out_hidden, void* stream_) {
  if (shape == nullptr || shape->N < 0 || shape->d <= 0 || (shape->d & 7) != 0) return LL_EINVAL;
  if (shape->N > kMaxInjectRows) return LL_EINVAL;
  if (shape->N == 0) return LL_OK;
  if (hidden == nullptr || v == nullptr || out_hidden == nullptr) return LL_EINVAL;
  const float s = alpha * layer_scale;
  if (s - s != 0.f || clip_ratio - clip_ratio != 0.f) return LL_EINVAL;   // NaN or infinite
  if (((uintptr_t)hidden | (uintptr_t)v | (uintptr_t)out_hidden) & 15) return LL_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const int64_t N = shape->N;
  const int d = shape->d;
  const unsigned blocks = (unsigned)((N + 3) / 4);
  const uint16_t* h = static_cast<const uint16_t*>(hidden);
  uint16_t* o = static_cast<uint16_t*>(out_hidden);
  const int n16 = d >> 3;
#define LL_INJECT_RAW(NITER) \
  hipLaunchKernelGGL(ll_steer_inject_raw_kernel<NITER>, dim3(blocks), dim3(256), 0, stream, h, v, o, N, d, s, clip_ratio)
  if (n16 <= 64 * 2) {
    LL_INJECT_RAW(2);
  } else if (n16 <= 64 * 8) {
    LL_INJECT_RAW(8);
  } else if (n16 <= 64 * 16) {
    LL_INJECT_RAW(16);
  } else {
    LL_INJECT_RAW(0);
  }
#undef LL_INJECT_RAW
  LL_HIP_CHECK(hipGetLastError());
  return LL_OK;
}

size_t ll_steer_workspace_bytes(int32_t d) {
  if (d <= 0 || (d & 7) != 0) return 0;
  return (size_t)2 * STEER_SLICES * (size_t)d * sizeof(float);
}

int ll_steer_vector(const void* base, int64_t n_base, const void* target, int64_t n_target, int32_t d, int normalize,
                    float* out_v, void* workspace, size_t workspace_bytes, void* stream_) {
  if (base == nullptr || target == nullptr || out_v == nullptr) return LL_EINVAL;
  if (n_base < 1 || n_target < 1 || d <= 0 || (d & 7) != 0) return LL_EINVAL;
  if (((uintptr_t)base | (uintptr_t)target | (uintptr_t)out_v) & 15) return LL_EINVAL;
  if (workspace != nullptr && (workspace_bytes < ll_steer_workspace_bytes(d) || ((uintptr_t)workspace & 15)))
    return LL_EWORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const unsigned col_blocks = (unsigned)((d + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK);
  const uint16_t* b = static_cast<const uint16_t*>(base);
  const uint16_t* t = static_cast<const uint16_t*>(target);
  const int64_t n_max = n_base > n_target ? n_base : n_target;
  if (workspace == nullptr || n_max <= 16) {
    hipLaunchKernelGGL(ll_steer_colsum_kernel<true>, dim3(col_blocks, 1), dim3(256), 0, stream, b, n_base, t, n_target, d, 1,
                       out_v);
    LL_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(ll_steer_finish_kernel<true>, dim3(1), dim3(1024), 0, stream, (const float*)nullptr, 1, n_base,
                       n_target, d, normalize, out_v);
    LL_HIP_CHECK(hipGetLastError());
  } else {
    int slices = (int)((n_max + 15) / 16);
    if (slices > STEER_SLICES) slices = STEER_SLICES;
    float* part = static_cast<float*>(workspace);
    hipLaunchKernelGGL(ll_steer_colsum_kernel<false>, dim3(col_blocks, slices), dim3(256), 0, stream, b, n_base, t, n_target,
                       d, slices, part);
    LL_HIP_CHECK(hipGetLastError());
    if (slices <= 8) {
      hipLaunchKernelGGL(ll_steer_finish_kernel<false>, dim3(1), dim3(1024), 0, stream, (const float*)part, slices, n_base,
                         n_target, d, normalize, out_v);
    } else {   // same sums in the same order, spread over the chip
      hipLaunchKernelGGL(ll_steer_reduce_kernel, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, stream, (const float*)part,
                         slices, n_base, n_target, d, out_v);
      LL_HIP_CHECK(hipGetLastError());
      hipLaunchKernelGGL(ll_steer_finish_kernel<true>, dim3(1), dim3(1024), 0, stream, (const float*)nullptr, 1, n_base,
                         n_target, d, normalize, out_v);
    }
    LL_HIP_CHECK(hipGetLastError());
  }
  return LL_OK;
}

int ll_steer_inject(const ll_shape* shape, const void* hidden, const void* gamma, float eps, const float* v, float alpha,
                    void* out_hidden, void* stream_) {
  if (shape == nullptr || shape->N < 0 || shape->d <= 0 || (shape->d & 7) != 0) return LL_EINVAL;
  if (shape->N > kMaxInjectRows) return LL_EINVAL;
  if (shape->N == 0) return LL_OK;
  if (hidden == nullptr || gamma == nullptr || v == nullptr || out_hidden == nullptr || !(eps >= 0.f)) return LL_EINVAL;
  if (((uintptr_t)hidden | (uintptr_t)gamma | (uintptr_t)v | (uintptr_t)out_hidden) & 15) return LL_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const int64_t N = shape->N;
  const int d = shape->d;
  const unsigned blocks = (unsigned)((N + 3) / 4);
  const uint16_t* h = static_cast<const uint16_t*>(hidden);
  const uint16_t* g = static_cast<const uint16_t*>(gamma);
  uint16_t* o = static_cast<uint16_t*>(out_hidden);
  const int n16 = d >> 3;
#define LL_INJECT(NITER) \
  hipLaunchKernelGGL(ll_steer_inject_kernel<NITER>, dim3(blocks), dim3(256), 0, stream, h, g, v, o, N, d, eps, alpha)
  if (n16 <= 64 * 2) {
    LL_INJECT(2);
  } else if (n16 <= 64 * 8) {
    LL_INJECT(8);
  } else if (n16 <= 64 * 16) {
    LL_INJECT(16);
  } else {
    LL_INJECT(0);
  }
#undef LL_INJECT
  LL_HIP_CHECK(hipGetLastError());
  return LL_OK;
}

}  // extern "C"
