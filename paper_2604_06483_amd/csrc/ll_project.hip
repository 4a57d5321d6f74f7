// Fused logit-lens projection for gfx950: RMS statistics / normalised panel, bf16 MFMA GEMM over
// the vocabulary with an online-softmax / top-k / target-gather epilogue, and the merge of the
// vocabulary splits.
//
// Follows the paper's Sec. 3.3 (Eq. 1 and "Top-k extraction") and Alg. 1 Phase 2; the logits of
// Eq. 1 live only in MFMA accumulators.
#include "ll_epilogue.h"
#include "ll_epilogue_sweep.h"
#include "ll_gemm_lds.h"
#include "ll_gemm_staged.h"

#include <atomic>
#include <climits>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------------
// a2: inv_rms[r] = 1 / sqrt(mean_j h[r,j]^2 + eps).  One wavefront per row, 16-byte loads.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ll_rms_stats_kernel(const uint16_t* __restrict__ hidden, int64_t n_rows,
                                                           int d, float eps, float* __restrict__ inv_rms) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const uint4* src = reinterpret_cast<const uint4*>(hidden + row * (int64_t)d);
  const int n16 = d >> 3;
  float acc0 = 0.f, acc1 = 0.f;
  for (int c = lane; c < n16; c += 64) {
    accum_sq(src[c], acc0, acc1);
  }
  const float ss = wave_sum(acc0 + acc1);
  if (lane == 0) inv_rms[row] = inv_rms_from_sumsq(ss, d, eps);
}

// ---------------------------------------------------------------------------------------
// a2 + a3 materialised: panel[r, :] = bf16((h[r, :] * inv_rms[r]) * gamma), zero padded to the
// panel's row stride; gamma == nullptr copies the rows unchanged.  One wavefront per row; the
// row stays in registers between the statistic and the write when it fits.
// ---------------------------------------------------------------------------------------
template <int NITER>
__global__ __launch_bounds__(256) void ll_norm_panel_kernel(const uint16_t* __restrict__ hidden,
                                                            const uint16_t* __restrict__ gamma, uint16_t* __restrict__ panel,
                                                            int rows, int d, int64_t lda, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint4* src = reinterpret_cast<const uint4*>(hidden + (int64_t)row * d);
  uint4* dst = reinterpret_cast<uint4*>(panel + (int64_t)row * lda);
  const uint4* g4 = reinterpret_cast<const uint4*>(gamma);
  const int n16 = d >> 3;
  const int n16_pad = (int)(lda >> 3);
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
    if (gamma == nullptr) {
      dst[c] = q;
      return;
    }
    const uint4 g = g4[c];
    const uint32_t hw[4] = {q.x, q.y, q.z, q.w};
    const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
    uint32_t ow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      ow[i] = pack_bf16(bf16_lo(hw[i]) * inv * bf16_lo(gw[i]), bf16_hi(hw[i]) * inv * bf16_hi(gw[i]));
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
  for (int c = n16 + lane; c < n16_pad; c += 64) dst[c] = make_uint4(0, 0, 0, 0);
}

// Copy of the bias of Eq. 1 padded with zeros to whole vocabulary tiles, so that the epilogue
// reads 32 entries per group without looking at V.
__global__ __launch_bounds__(256) void ll_pad_bias_kernel(const float* __restrict__ bias, int V, float* __restrict__ padded,
                                                          int n_padded) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_padded; i += gridDim.x * blockDim.x)
    padded[i] = i < V ? bias[i] : 0.f;
}

__global__ __launch_bounds__(256) void ll_zero_u32_kernel(unsigned* __restrict__ p, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0u;
}

__global__ __launch_bounds__(256) void ll_fill_f32_kernel(float* __restrict__ p, int n, float value) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = value;
}

// ---------------------------------------------------------------------------------------
// Steering sweep, step 1: u = W_U v (one pass over W_U, HBM-bound: 2 V d bytes), written as the
// table au[a, id] = alpha_a * u[id] that the sweep epilogue adds to the logits.  One wavefront
// takes eight vocabulary rows at a time: a chunk of v read from LDS serves eight products, and
// eight 16-byte loads per lane are in flight.
// ---------------------------------------------------------------------------------------
struct AlphaList {
  float a[SWEEP_MAX];
};

constexpr int UD_ROWS = 8;   // vocabulary rows a wavefront takes at a time

__global__ __launch_bounds__(256) void ll_unembed_direction_kernel(const uint16_t* __restrict__ W, const float* __restrict__ v,
                                                                   int V, int d, AlphaList alphas, int n_alpha,
                                                                   float* __restrict__ au, int au_stride) {
  extern __shared__ __align__(16) float sv[];
  for (int j = threadIdx.x; j < d; j += blockDim.x) sv[j] = v[j];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n16 = d >> 3;
  for (int r0 = (blockIdx.x * 4 + wave) * UD_ROWS; r0 < V; r0 += gridDim.x * 4 * UD_ROWS) {
    float acc[UD_ROWS];
    const uint4* rows[UD_ROWS];
#pragma unroll
    for (int i = 0; i < UD_ROWS; ++i) {
      acc[i] = 0.f;
      rows[i] = reinterpret_cast<const uint4*>(W + (int64_t)min(r0 + i, V - 1) * d);
    }
    for (int c = lane; c < n16; c += 64) {
      uint4 q[UD_ROWS];
#pragma unroll
      for (int i = 0; i < UD_ROWS; ++i) q[i] = rows[i][c];   // all loads of the step in flight before the first use
      const float4 v0 = *reinterpret_cast<const float4*>(sv + 8 * c);
      const float4 v1 = *reinterpret_cast<const float4*>(sv + 8 * c + 4);
#pragma unroll
      for (int i = 0; i < UD_ROWS; ++i) {
        float a = acc[i];
        a = fmaf(bf16_lo(q[i].x), v0.x, a);
        a = fmaf(bf16_hi(q[i].x), v0.y, a);
        a = fmaf(bf16_lo(q[i].y), v0.z, a);
        a = fmaf(bf16_hi(q[i].y), v0.w, a);
        a = fmaf(bf16_lo(q[i].z), v1.x, a);
        a = fmaf(bf16_hi(q[i].z), v1.y, a);
        a = fmaf(bf16_lo(q[i].w), v1.z, a);
        a = fmaf(bf16_hi(q[i].w), v1.w, a);
        acc[i] = a;
      }
    }
#pragma unroll
    for (int i = 0; i < UD_ROWS; ++i) {
      const float u = wave_sum(acc[i]);
      if (lane == 0 && r0 + i < V) {
#pragma unroll
        for (int a = 0; a < SWEEP_MAX; ++a)
          if (a < n_alpha) au[(int64_t)a * au_stride + r0 + i] = alphas.a[a] * u;
      }
    }
  }
}

// Steering sweep, step 3: merge the splits of each (row, alpha) and finalise.  One wavefront per
// row, lane s = split s.
__global__ __launch_bounds__(256) void ll_sweep_merge_kernel(const float4* __restrict__ stats, const float* __restrict__ ztgt,
                                                             const float* __restrict__ au, int au_stride, int rows, int splits,
                                                             int n_alpha, int V, const int32_t* __restrict__ target,
                                                             int64_t out_stride, int32_t* __restrict__ out_ids,
                                                             float* __restrict__ out_p, float* __restrict__ out_logp,
                                                             float* __restrict__ out_entropy);

// ---------------------------------------------------------------------------------------
// a8: merge the splits of each row and finalise.  One wavefront per row, one lane per split.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}
__device__ __forceinline__ int wave_min_int(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off, kWave));
  return x;
}
// The same over the first `width` lanes only (a power of two; every lane below it gets the result):
// the k steps of the merge are a chain of these exchanges, and with eight splits three rounds do.
__device__ __forceinline__ float group_max(float x, int width) {
  for (int off = width >> 1; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}
__device__ __forceinline__ int group_min_int(int x, int width) {
  for (int off = width >> 1; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off, kWave));
  return x;
}

// One wavefront per row; lane s holds the lists of splits [s LPL, s LPL + LPL) (LPL = 1 while the splits fit one
// lane each; 4 when a pass of few rows cuts the vocabulary finer than that so as to fill the chip).  The row's
// lists (splits x k pairs, contiguous in the workspace) are first copied into LDS with coalesced loads: the k steps
// of the merge are a chain, each needing the next entry of whichever list won the step before, and from LDS that
// costs a fraction of a trip to memory.  At LPL = 1 a block is four wavefronts with a row each; at LPL = 4 a block
// has ONE row, all four wavefronts copy its lists (up to 64 KB: one wavefront alone would spend its time waiting for
// its own loads) and the first one merges.
// Dynamic LDS: rows of the block x splits x k x 8 bytes (at most 64 KB).
constexpr int MERGE_LPL = 4;                              // lists per lane of the merge when splits > 64
constexpr int MAX_PROJECT_SPLITS = MAX_SPLITS * MERGE_LPL;   // vocabulary splits per row block of the projection

template <int LPL>
__global__ __launch_bounds__(256) void ll_merge_kernel(const float4* __restrict__ stats, const uint2* __restrict__ top,
                                                       int rows, int splits, int k, int V, int topk_softmax,
                                                       const int32_t* __restrict__ target, int32_t* __restrict__ out_ids,
                                                       float* __restrict__ out_p, float* __restrict__ out_logp,
                                                       float* __restrict__ out_entropy, unsigned* __restrict__ bound) {
  extern __shared__ __align__(8) uint2 lists[];
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int row = LPL == 1 ? blockIdx.x * (blockDim.x >> 6) + wave : blockIdx.x;
  const bool valid = row < rows;          // (no early return: every wavefront reaches the barrier)
  const int n_entries = splits * k;
  uint2* mine = LPL == 1 ? lists + wave * n_entries : lists;
  if (valid) {
    const uint2* src = top + (int64_t)row * n_entries;
    if (LPL == 1)
      for (int i = lane; i < n_entries; i += 64) mine[i] = src[i];
    else
      for (int i = threadIdx.x; i < n_entries; i += blockDim.x) mine[i] = src[i];
  }
  __syncthreads();
  if (!valid || (LPL != 1 && wave != 0)) return;
  bool live[LPL];
  float4 q[LPL];
  float m_lane = -INFINITY, zt_lane = -INFINITY;
#pragma unroll
  for (int i = 0; i < LPL; ++i) {
    live[i] = lane * LPL + i < splits;
    q[i] = make_float4(-INFINITY, 0.f, 0.f, -INFINITY);
    if (live[i]) q[i] = stats[(int64_t)row * splits + lane * LPL + i];
    m_lane = fmaxf(m_lane, q[i].x);
    zt_lane = fmaxf(zt_lane, q[i].w);
  }
  const float M = wave_max(m_lane);
  float s_lane = 0.f, t_lane = 0.f;
#pragma unroll
  for (int i = 0; i < LPL; ++i) {
    const float sc = live[i] ? __builtin_amdgcn_exp2f((q[i].x - M) * LOG2E) : 0.f;
    s_lane += sc * q[i].y;
    t_lane += sc * q[i].z;
  }
  const float S = wave_sum(s_lane);
  const float T = wave_sum(t_lane);
  const float zt = wave_max(zt_lane);
  const float logS = logf(S);
  if (lane == 0) {
    if (bound != nullptr) bound[row] = 0u;   // the projection kernel of this pass is done with it: clear it for the next pass
    out_entropy[row] = (M - T / S) + logS;
    if (target != nullptr) {
      const int t = target[row];
      out_logp[row] = (t >= 0 && t < V) ? (zt - M) - logS : __builtin_nanf("");
    }
  }
  // k-way merge of the per-split sorted lists (descending logit, ascending id): every lane holds the
  // heads of its lists; the wavefront's best head goes out and that list moves on.
  const uint2* tl = mine + lane * LPL * k;
  int head[LPL];
  float z[LPL];
  int id[LPL];
#pragma unroll
  for (int i = 0; i < LPL; ++i) {
    head[i] = 0;
    z[i] = -INFINITY;
    id[i] = INT_MAX;
    if (live[i]) {
      const uint2 e = tl[i * k];
      z[i] = __uint_as_float(e.x);
      id[i] = (int)e.y;
    }
  }
  float z0 = 0.f, sk = 0.f;   // top-k-only softmax: the largest selected logit and the sum over the selection
  float my_z = 0.f;           // lane j keeps the j-th selected logit and id, written out together at the end
  int my_id = 0;
  int width = 1;   // lanes that hold a list, rounded up to a power of two (lanes past them hold the neutral head)
  while (width * LPL < splits) width <<= 1;
  for (int j = 0; j < k; ++j) {
    float lz = z[0];   // this lane's best head: largest logit, smallest id among equals
    int li = id[0];
#pragma unroll
    for (int i = 1; i < LPL; ++i) {
      const bool better = z[i] > lz || (z[i] == lz && id[i] < li);
      lz = better ? z[i] : lz;
      li = better ? id[i] : li;
    }
    const float bz = group_max(lz, width);
    const int bi = group_min_int(lz == bz ? li : INT_MAX, width);
#pragma unroll
    for (int i = 0; i < LPL; ++i) {
      if (live[i] && z[i] == bz && id[i] == bi) {   // ids are distinct: exactly one list of one lane
        ++head[i];
        if (head[i] < k) {
          const uint2 e = tl[i * k + head[i]];
          z[i] = __uint_as_float(e.x);
          id[i] = (int)e.y;
        } else {
          z[i] = -INFINITY;
          id[i] = INT_MAX;
        }
      }
    }
    // (lanes past `width` did not take part: what they keep comes from lane 0)
    const float out_z = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(bz)));
    const int out_id = __builtin_amdgcn_readfirstlane(bi);
    if (j == 0) z0 = out_z;
    sk += __builtin_amdgcn_exp2f((out_z - z0) * LOG2E);
    if (lane == j) {
      my_z = out_z;
      my_id = out_id;
    }
  }
  if (lane < k) {
    out_ids[(int64_t)row * k + lane] = my_id;
    // full-vocabulary probability, or the paper's own (Sec. 3.3): a softmax over the k selected logits only
    out_p[(int64_t)row * k + lane] = topk_softmax ? __builtin_amdgcn_exp2f((my_z - z0) * LOG2E) * (1.0f / sk)
                                                  : __builtin_amdgcn_exp2f(((my_z - M) - logS) * LOG2E);
  }
}

__global__ __launch_bounds__(256) void ll_sweep_merge_kernel(const float4* __restrict__ stats, const float* __restrict__ ztgt,
                                                             const float* __restrict__ au, int au_stride, int rows, int splits,
                                                             int n_alpha, int V, const int32_t* __restrict__ target,
                                                             int64_t out_stride, int32_t* __restrict__ out_ids,
                                                             float* __restrict__ out_p, float* __restrict__ out_logp,
                                                             float* __restrict__ out_entropy) {
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const bool live = lane < splits;
  int t = -1;
  float zt0 = -INFINITY;
  if (target != nullptr) {
    t = target[row];
    zt0 = wave_max(live ? ztgt[(int64_t)row * splits + lane] : -INFINITY);
  }
  const bool t_ok = t >= 0 && t < V;
  for (int a = 0; a < n_alpha; ++a) {
    float4 q = make_float4(-INFINITY, 0.f, 0.f, __int_as_float(INT_MAX));
    if (live) q = stats[((int64_t)row * splits + lane) * n_alpha + a];
    const float M = wave_max(q.x);
    // splits hold increasing id ranges, and within one the smallest id of its maximum is kept
    const int best = wave_min_int(q.x == M ? __float_as_int(q.w) : INT_MAX);
    const float sc = live ? __builtin_amdgcn_exp2f((q.x - M) * LOG2E) : 0.f;
    const float S = wave_sum(sc * q.y);
    const float T = wave_sum(sc * q.z);
    if (lane == 0) {
      const float logS = logf(S);
      const int64_t o = (int64_t)a * out_stride + row;
      out_ids[o] = best;
      out_p[o] = 1.0f / S;                      // exp(M - (M + log S))
      out_entropy[o] = (M - T / S) + logS;
      if (target != nullptr)
        out_logp[o] = t_ok ? ((zt0 + au[(int64_t)a * au_stride + t]) - M) - logS : __builtin_nanf("");
    }
  }
}

// The sweep with top-k lists: per (row, alpha) the splits' statistics and sorted lists of SWEEP_KS
// entries are merged as in ll_merge_kernel (one wavefront per row, lane s = split s; the lists
// are short, so their heads are read from the workspace directly).  Outputs are [n_alpha, N, k].
__global__ __launch_bounds__(256) void ll_sweep_topk_merge_kernel(const float4* __restrict__ stats, const uint2* __restrict__ top,
                                                                  const float* __restrict__ ztgt, const float* __restrict__ au,
                                                                  int au_stride, int rows, int splits, int n_alpha, int k, int V,
                                                                  const int32_t* __restrict__ target, int64_t out_stride,
                                                                  int32_t* __restrict__ out_ids, float* __restrict__ out_p,
                                                                  float* __restrict__ out_logp, float* __restrict__ out_entropy) {
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const bool live = lane < splits;
  int t = -1;
  float zt0 = -INFINITY;
  if (target != nullptr) {
    t = target[row];
    zt0 = wave_max(live ? ztgt[(int64_t)row * splits + lane] : -INFINITY);
  }
  const bool t_ok = t >= 0 && t < V;
  int width = 1;
  while (width < splits) width <<= 1;
  for (int a = 0; a < n_alpha; ++a) {
    const int64_t part = ((int64_t)row * splits + (live ? lane : 0)) * n_alpha + a;
    float4 q = make_float4(-INFINITY, 0.f, 0.f, 0.f);
    if (live) q = stats[part];
    const float M = wave_max(q.x);
    const float sc = live ? __builtin_amdgcn_exp2f((q.x - M) * LOG2E) : 0.f;
    const float S = wave_sum(sc * q.y);
    const float T = wave_sum(sc * q.z);
    const float logS = logf(S);
    const int64_t o = (int64_t)a * out_stride + row;
    if (lane == 0) {
      out_entropy[o] = (M - T / S) + logS;
      if (target != nullptr)
        out_logp[o] = t_ok ? ((zt0 + au[(int64_t)a * au_stride + t]) - M) - logS : __builtin_nanf("");
    }
    const uint2* tl = top + part * SWEEP_KS;
    int head = 0;
    float z = -INFINITY;
    int id = INT_MAX;
    if (live) {
      const uint2 e = tl[0];
      z = __uint_as_float(e.x);
      id = (int)e.y;
    }
    for (int j = 0; j < k; ++j) {
      const float bz = group_max(z, width);
      const int bi = group_min_int(z == bz ? id : INT_MAX, width);
      if (live && z == bz && id == bi) {
        ++head;
        if (head < SWEEP_KS) {
          const uint2 e = tl[head];
          z = __uint_as_float(e.x);
          id = (int)e.y;
        } else {
          z = -INFINITY;
          id = INT_MAX;
        }
      }
      if (lane == 0) {
        out_ids[o * k + j] = bi;
        out_p[o * k + j] = __builtin_amdgcn_exp2f(((bz - M) - logS) * LOG2E);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
struct Plan {
  size_t off_inv_rms, off_bound, off_bias, off_stats, off_top, off_panel, total;
  int64_t lda;
};

bool shape_ok(const ll_shape* s, int k) {
  if (s == nullptr) return false;
  if (s->N < 0 || s->d <= 0 || s->V <= 0 || (s->d & 7) != 0) return false;
  // rounding up to whole tiles (V) and whole K stages (d) stays inside 32 bits
  if (s->V > INT32_MAX - BM || s->d > INT32_MAX - 2 * DK) return false;
  if (k < 1 || k > LL_KMAX || k > s->V) return false;
  return true;
}

Plan make_plan(const ll_shape* s, int k, int chunk_rows = CHUNK_ROWS) {
  Plan p;
  size_t off = 0;
  p.off_inv_rms = off;
  off = align_up(off + (size_t)s->N * sizeof(float), 256);
  p.off_bound = off;  // per-row top-k bounds shared between the splits of a pass
  off = align_up(off + (size_t)(s->N < chunk_rows ? s->N : chunk_rows) * sizeof(unsigned), 256);
  p.off_bias = off;   // the bias padded to whole tiles (ll_project_ex)
  off = align_up(off + (size_t)((s->V + BM - 1) / BM) * BM * sizeof(float), 256);
  const size_t rows = (size_t)(s->N < chunk_rows ? s->N : chunk_rows);
  p.off_stats = off;
  const size_t partials = rows * MAX_PROJECT_SPLITS < (size_t)MAX_PARTIALS ? rows * MAX_PROJECT_SPLITS : (size_t)MAX_PARTIALS;
  off = align_up(off + partials * sizeof(float4), 256);
  p.off_top = off;
  off = align_up(off + partials * (size_t)k * sizeof(uint2), 256);
  p.lda = (s->d + DK - 1) / DK * DK;
  p.off_panel = off;
  off = align_up(off + rows * (size_t)p.lda * sizeof(uint16_t), 256);
  p.total = off;
  return p;
}

// A kernel that uses more than 64 KB of dynamic LDS has to be told so once per device; remembered
// here so that the hot path makes no attribute call.
int allow_dynamic_lds(const void* kern, size_t lds) {
  static std::mutex mu;
  static std::vector<std::pair<int, const void*>> done;
  int dev = -1;
  LL_HIP_CHECK(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& e : done)
    if (e.first == dev && e.second == kern) return LL_OK;
  LL_HIP_CHECK(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  done.emplace_back(dev, kern);
  return LL_OK;
}

int project_impl(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                 const void* W_U, const float* bias, unsigned flags, float eps, int k, const int32_t* target_ids,
                 int32_t* out_topk_ids, float* out_topk_p,
                 float* out_target_logp, float* out_entropy, hipStream_t stream, float* phase_ms,
                 int chunk_rows = CHUNK_ROWS) {
  if (!shape_ok(shape, k)) return LL_EINVAL;
  if (shape->N == 0) {
    if (phase_ms) phase_ms[0] = phase_ms[1] = phase_ms[2] = 0.f;
    return LL_OK;
  }
  if (hidden == nullptr || W_U == nullptr || out_topk_ids == nullptr || out_topk_p == nullptr || out_entropy == nullptr)
    return LL_EINVAL;
  if (target_ids != nullptr && out_target_logp == nullptr) return LL_EINVAL;
  if (!(eps >= 0.f)) return LL_EINVAL;
  if ((flags & ~(unsigned)(LL_FLAG_TOPK_SOFTMAX | LL_FLAG_REGISTER_STAGED)) != 0 || ((uintptr_t)bias & 3)) return LL_EINVAL;
  const uintptr_t align_or = (uintptr_t)hidden | (uintptr_t)W_U | (uintptr_t)gamma;
  if (align_or & 15) return LL_EINVAL;
  const Plan plan = make_plan(shape, k, chunk_rows);
  if (workspace == nullptr || workspace_bytes < plan.total || ((uintptr_t)workspace & 255)) return LL_EWORKSPACE;

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  float* inv_rms = reinterpret_cast<float*>(ws + plan.off_inv_rms);
  float4* stats = reinterpret_cast<float4*>(ws + plan.off_stats);
  uint2* top = reinterpret_cast<uint2*>(ws + plan.off_top);
  uint16_t* panel = reinterpret_cast<uint16_t*>(ws + plan.off_panel);

  const int64_t N = shape->N;
  const int d = shape->d, V = shape->V;
  const bool has_gamma = gamma != nullptr;
  // The direct-to-LDS kernel addresses rows with 32-bit byte offsets from a per-tile base.
  const bool dma_ok = d % DK == 0 && (int64_t)BM * d * 2 < (int64_t)1 << 31 && (int64_t)CHUNK_ROWS * plan.lda * 2 < (int64_t)1 << 31;
  // A bias (rare: the paper's model families have none) selects a separate instantiation of the
  // kernel, so that calls without one carry no code or registers for it.
  const bool dma = dma_ok && !(flags & LL_FLAG_REGISTER_STAGED);
  const size_t lds = dma ? (size_t)SLOTS * SLOT_BYTES : (size_t)(BM + BN) * BK * 2;
  // The top-k lists live in registers: the kernels are built for a few list lengths KR >= k.
  void (*kern)(const GemmArgs);
#define LL_PICK(KR) \
  (dma ? (bias ? ll_lens_gemm_dma_kernel<TopKEpilogue<KR, true>> : ll_lens_gemm_dma_kernel<TopKEpilogue<KR, false>>) \
       : (bias ? ll_lens_gemm_kernel<TopKEpilogue<KR, true>> : ll_lens_gemm_kernel<TopKEpilogue<KR, false>>))
  if (k <= 4)
    kern = LL_PICK(4);
  else if (k <= 12)
    kern = LL_PICK(12);
  else if (k <= 20)
    kern = LL_PICK(20);
  else
    kern = LL_PICK(32);
#undef LL_PICK
  if (const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds); rc != LL_OK) return rc;
  // The direct-to-LDS kernel reads hidden in place when the rows need neither scaling nor padding.
  const bool need_panel = dma && (has_gamma || plan.lda != d);

  // Timing (ll_project_timed only): events are recorded in-stream around every kernel and read
  // after one synchronisation at the end, so the kernels run back to back as in ll_project.
  // (the events are created once per thread and kept: a timed call costs no event creation after the first)
  static thread_local std::vector<hipEvent_t> ev_pool;
  size_t n_ev = 0;
  auto mark = [&]() -> hipError_t {
    if (!phase_ms) return hipSuccess;
    if (n_ev == ev_pool.size()) {
      hipEvent_t e = nullptr;
      hipError_t rc = hipEventCreate(&e);
      if (rc != hipSuccess) return rc;
      ev_pool.push_back(e);
    }
    return hipEventRecord(ev_pool[n_ev++], stream);
  };
  auto finish = [&](int rc) { return rc; };
  const std::vector<hipEvent_t>& ev = ev_pool;
#define LL_CHECK_F(expr)                                   \
  do {                                                     \
    hipError_t e__ = (expr);                               \
    if (e__ != hipSuccess) return finish(hip_failed(e__)); \
  } while (0)

  const int tiles = (V + BM - 1) / BM;
  // Top-k bounds shared between the vocabulary splits of a row (direct-to-LDS kernel): zero at the start of a
  // pass; the merge kernel of a pass clears them again for the next one.
  unsigned* bound = nullptr;
  if (dma) {
    bound = reinterpret_cast<unsigned*>(ws + plan.off_bound);
    const int n_zero = (int)(N < chunk_rows ? N : chunk_rows);
    hipLaunchKernelGGL(ll_zero_u32_kernel, dim3((n_zero + 255) / 256), dim3(256), 0, stream, bound, n_zero);
    LL_CHECK_F(hipGetLastError());
  }
  float* bias_padded = nullptr;
  if (bias != nullptr) {
    bias_padded = reinterpret_cast<float*>(ws + plan.off_bias);
    hipLaunchKernelGGL(ll_pad_bias_kernel, dim3((tiles * BM + 1023) / 1024), dim3(256), 0, stream, bias, V, bias_padded, tiles * BM);
    LL_CHECK_F(hipGetLastError());
  }
  for (int64_t r0 = 0; r0 < N; r0 += chunk_rows) {
    const int rows = (int)((N - r0) < chunk_rows ? (N - r0) : chunk_rows);
    const uint16_t* h_rows = static_cast<const uint16_t*>(hidden) + r0 * d;
    // a2 (+ a3 when the panel is used)
    LL_CHECK_F(mark());
    if (need_panel) {
      const dim3 grid((unsigned)((rows + 3) / 4));
      const uint16_t* g = static_cast<const uint16_t*>(gamma);
      if (d <= 64 * 8 * 4)
        hipLaunchKernelGGL(ll_norm_panel_kernel<4>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else if (d <= 64 * 8 * 16)
        hipLaunchKernelGGL(ll_norm_panel_kernel<16>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else
        hipLaunchKernelGGL(ll_norm_panel_kernel<0>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      LL_CHECK_F(hipGetLastError());
    } else if (!dma && has_gamma) {
      hipLaunchKernelGGL(ll_rms_stats_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, h_rows, (int64_t)rows, d,
                         eps, inv_rms + r0);
      LL_CHECK_F(hipGetLastError());
    }
    const int row_blocks = (rows + BN - 1) / BN;
    // One workgroup per compute unit: a pass of few rows cuts the vocabulary finer (its cost is then the one read
    // of W_U, spread over every compute unit's share of the memory system).
    int splits = NUM_CU / row_blocks;
    if (splits > MAX_PROJECT_SPLITS) splits = MAX_PROJECT_SPLITS;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    GemmArgs a;
    a.A = need_panel ? panel : h_rows;
    a.lda = need_panel ? plan.lda : d;
    a.inv_rms = (!dma && has_gamma) ? inv_rms + r0 : nullptr;
    a.gamma = static_cast<const uint16_t*>(gamma);
    a.W = static_cast<const uint16_t*>(W_U);
    a.target = target_ids ? target_ids + r0 : nullptr;
    a.bias = bias_padded;
    a.stats = stats;
    a.top = top;
    a.rows = rows;
    a.d = d;
    a.V = V;
    a.k = k;
    a.splits = splits;
    a.tiles = tiles;
    a.row_blocks = row_blocks;
    a.bound = bound;
    const int grid = (row_blocks * splits + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    LL_CHECK_F(mark());
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHREADS), lds, stream, a);
    LL_CHECK_F(hipGetLastError());
    LL_CHECK_F(mark());
    if (splits <= MAX_SPLITS)
      hipLaunchKernelGGL(ll_merge_kernel<1>, dim3((rows + 3) / 4), dim3(256), (size_t)4 * splits * k * sizeof(uint2), stream,
                         (const float4*)stats, (const uint2*)top,
                         rows, splits, k, V, (flags & LL_FLAG_TOPK_SOFTMAX) ? 1 : 0, a.target, out_topk_ids + r0 * k,
                         out_topk_p + r0 * k,
                         out_target_logp ? out_target_logp + r0 : nullptr, out_entropy + r0, bound);
    else   // (only passes of at most three row blocks get here: one row per block keeps the lists within 64 KB of LDS)
      hipLaunchKernelGGL(ll_merge_kernel<MERGE_LPL>, dim3(rows), dim3(256), (size_t)splits * k * sizeof(uint2), stream,
                         (const float4*)stats, (const uint2*)top,
                         rows, splits, k, V, (flags & LL_FLAG_TOPK_SOFTMAX) ? 1 : 0, a.target, out_topk_ids + r0 * k,
                         out_topk_p + r0 * k,
                         out_target_logp ? out_target_logp + r0 : nullptr, out_entropy + r0, bound);
    LL_CHECK_F(hipGetLastError());
    LL_CHECK_F(mark());
  }
  if (phase_ms) {
    LL_CHECK_F(hipStreamSynchronize(stream));
    phase_ms[0] = phase_ms[1] = phase_ms[2] = 0.f;
    for (size_t i = 0; i + 3 < n_ev; i += 4) {
      float ms = 0.f;
      LL_CHECK_F(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
      phase_ms[0] += ms;
      LL_CHECK_F(hipEventElapsedTime(&ms, ev[i + 1], ev[i + 2]));
      phase_ms[1] += ms;
      LL_CHECK_F(hipEventElapsedTime(&ms, ev[i + 2], ev[i + 3]));
      phase_ms[2] += ms;
    }
  }
#undef LL_CHECK_F
  return finish(LL_OK);
}

struct SweepPlan {
  size_t off_au, off_stats, off_ztgt, off_top, off_inv_rms, off_panel, total;
  int64_t lda;
  int au_stride;
};

// k == 1: the arg max travels inside the statistics; k > 1: room for the sorted lists as well.
SweepPlan make_sweep_plan(const ll_shape* s, int n_alpha, int k = 1) {
  SweepPlan p;
  size_t off = 0;
  p.au_stride = (s->V + BM - 1) / BM * BM;
  p.off_au = off;
  off = align_up(off + (size_t)n_alpha * p.au_stride * sizeof(float), 256);
  const size_t rows = (size_t)(s->N < CHUNK_ROWS ? s->N : CHUNK_ROWS);
  p.off_stats = off;
  const size_t partials = rows * MAX_SPLITS < (size_t)MAX_PARTIALS ? rows * MAX_SPLITS : (size_t)MAX_PARTIALS;
  off = align_up(off + partials * (size_t)n_alpha * sizeof(float4), 256);
  p.off_ztgt = off;
  off = align_up(off + partials * sizeof(float), 256);
  p.off_top = off;
  if (k > 1) off = align_up(off + partials * (size_t)SWEEP_TOPK_ALPHAS * SWEEP_KS * sizeof(uint2), 256);
  p.off_inv_rms = off;   // d not a multiple of 64: the register-staged kernel normalises inside its A-tile load
  off = align_up(off + rows * sizeof(float), 256);
  p.lda = s->d;
  p.off_panel = off;     // d a multiple of 64: normalised rows for the direct-to-LDS kernel
  off = align_up(off + rows * (size_t)p.lda * sizeof(uint16_t), 256);
  p.total = off;
  return p;
}

// The direction kernel keeps v in LDS: 4 d bytes of the 160 KB.
constexpr int SWEEP_MAX_D = 40960;

bool sweep_shape_ok(const ll_shape* s, int n_alpha, int k = 1) {
  return shape_ok(s, k) && k <= SWEEP_KS && s->d <= SWEEP_MAX_D && n_alpha >= 1 && n_alpha <= SWEEP_MAX;
}

int sweep_impl(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
               const void* W_U, float eps, const float* v, const float* alphas, int n_alpha, int k, const int32_t* target_ids,
               int32_t* out_ids, float* out_p, float* out_logp, float* out_entropy, hipStream_t stream) {
  if (!sweep_shape_ok(shape, n_alpha, k)) return LL_EINVAL;
  if (shape->N == 0) return LL_OK;
  if (hidden == nullptr || W_U == nullptr || v == nullptr || alphas == nullptr || out_ids == nullptr || out_p == nullptr ||
      out_entropy == nullptr)
    return LL_EINVAL;
  if (target_ids != nullptr && out_logp == nullptr) return LL_EINVAL;
  if (!(eps >= 0.f)) return LL_EINVAL;
  if (((uintptr_t)hidden | (uintptr_t)W_U | (uintptr_t)gamma | (uintptr_t)v) & 15) return LL_EINVAL;
  AlphaList al;
  for (int a = 0; a < SWEEP_MAX; ++a) {
    al.a[a] = a < n_alpha ? alphas[a] : 0.f;
    if (!(al.a[a] == al.a[a]) || al.a[a] - al.a[a] != 0.f) return LL_EINVAL;   // NaN or infinite
  }
  const SweepPlan plan = make_sweep_plan(shape, n_alpha, k);
  if (workspace == nullptr || workspace_bytes < plan.total || ((uintptr_t)workspace & 255)) return LL_EWORKSPACE;

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  float* au = reinterpret_cast<float*>(ws + plan.off_au);
  float4* stats = reinterpret_cast<float4*>(ws + plan.off_stats);
  float* ztgt = reinterpret_cast<float*>(ws + plan.off_ztgt);
  uint2* top = reinterpret_cast<uint2*>(ws + plan.off_top);
  float* inv_rms = reinterpret_cast<float*>(ws + plan.off_inv_rms);
  uint16_t* panel = reinterpret_cast<uint16_t*>(ws + plan.off_panel);
  const int64_t N = shape->N;
  const int d = shape->d, V = shape->V;
  const int tiles = (V + BM - 1) / BM;
#define LL_CHECK_S(expr)                           \
  do {                                             \
    hipError_t e__ = (expr);                       \
    if (e__ != hipSuccess) return hip_failed(e__); \
  } while (0)

  // the padding of the table (ids V .. au_stride) is read by the last tile and masked afterwards:
  // any finite value will do, zero it once
  if (plan.au_stride > V) {
    for (int a = 0; a < n_alpha; ++a)
      hipLaunchKernelGGL(ll_fill_f32_kernel, dim3(1), dim3(256), 0, stream, au + (size_t)a * plan.au_stride + V,
                         plan.au_stride - V, 0.f);
    LL_CHECK_S(hipGetLastError());
  }
  if ((size_t)d * sizeof(float) > 64 * 1024)
    if (const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(ll_unembed_direction_kernel), (size_t)d * sizeof(float));
        rc != LL_OK)
      return rc;
  hipLaunchKernelGGL(ll_unembed_direction_kernel, dim3(NUM_CU * 4), dim3(256), (size_t)d * sizeof(float), stream,
                     static_cast<const uint16_t*>(W_U), v, V, d, al, n_alpha, au, plan.au_stride);
  LL_CHECK_S(hipGetLastError());
  // The direct-to-LDS kernel needs whole K stages of 64 and 32-bit row offsets; otherwise the register-staged
  // kernel, which normalises inside its A-tile load.
  const bool dma = d % DK == 0 && (int64_t)BM * d * 2 < (int64_t)1 << 31 && (int64_t)CHUNK_ROWS * d * 2 < (int64_t)1 << 31;
  void (*kern)(const GemmArgs);
  if (k == 1)
    kern = dma ? ll_lens_gemm_dma_kernel<SweepEpilogue> : ll_lens_gemm_kernel<SweepEpilogue>;
  else
    kern = dma ? ll_lens_gemm_dma_kernel<SweepTopKEpilogue> : ll_lens_gemm_kernel<SweepTopKEpilogue>;
  const size_t lds = dma ? (size_t)SLOTS * SLOT_BYTES : (size_t)(BM + BN) * BK * 2;
  if (const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds); rc != LL_OK) return rc;

  for (int64_t r0 = 0; r0 < N; r0 += CHUNK_ROWS) {
    const int rows = (int)((N - r0 < CHUNK_ROWS) ? (N - r0) : CHUNK_ROWS);
    const uint16_t* h_rows = static_cast<const uint16_t*>(hidden) + r0 * d;
    if (gamma != nullptr && dma) {
      const dim3 grid((unsigned)((rows + 3) / 4));
      const uint16_t* g = static_cast<const uint16_t*>(gamma);
      if (d <= 64 * 8 * 4)
        hipLaunchKernelGGL(ll_norm_panel_kernel<4>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else if (d <= 64 * 8 * 16)
        hipLaunchKernelGGL(ll_norm_panel_kernel<16>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else
        hipLaunchKernelGGL(ll_norm_panel_kernel<0>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      LL_CHECK_S(hipGetLastError());
    } else if (gamma != nullptr) {
      hipLaunchKernelGGL(ll_rms_stats_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, h_rows, (int64_t)rows, d,
                         eps, inv_rms);
      LL_CHECK_S(hipGetLastError());
    }
    const int row_blocks = (rows + BN - 1) / BN;
    int splits = NUM_CU / row_blocks;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    GemmArgs a = {};
    a.A = (gamma != nullptr && dma) ? panel : h_rows;
    a.lda = plan.lda;
    a.inv_rms = (gamma != nullptr && !dma) ? inv_rms : nullptr;
    a.gamma = static_cast<const uint16_t*>(gamma);
    a.sweep_top = top;
    a.W = static_cast<const uint16_t*>(W_U);
    a.target = target_ids ? target_ids + r0 : nullptr;
    a.rows = rows;
    a.d = d;
    a.V = V;
    a.k = 1;
    a.splits = splits;
    a.tiles = tiles;
    a.row_blocks = row_blocks;
    a.au_stride = plan.au_stride;
    a.sweep_stats = stats;
    a.sweep_ztgt = ztgt;
    const int grid = (row_blocks * splits + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    // k == 1: all alphas in one pass over W_U; with lists: SWEEP_TOPK_ALPHAS alphas per pass
    const int per_pass = k == 1 ? n_alpha : SWEEP_TOPK_ALPHAS;
    for (int a0 = 0; a0 < n_alpha; a0 += per_pass) {
      const int na = n_alpha - a0 < per_pass ? n_alpha - a0 : per_pass;
      a.au = au + (size_t)a0 * plan.au_stride;
      a.n_alpha = na;
      hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHREADS), lds, stream, a);
      LL_CHECK_S(hipGetLastError());
      const int64_t o0 = (int64_t)a0 * N + r0;   // first output of this pass: alpha a0, row r0
      if (k == 1)
        hipLaunchKernelGGL(ll_sweep_merge_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, (const float4*)stats,
                           (const float*)ztgt, (const float*)a.au, plan.au_stride, rows, splits, na, V, a.target, N,
                           out_ids + o0, out_p + o0, out_logp ? out_logp + o0 : nullptr, out_entropy + o0);
      else   // outputs [n_alpha, N, k]
        hipLaunchKernelGGL(ll_sweep_topk_merge_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, (const float4*)stats,
                           (const uint2*)top, (const float*)ztgt, (const float*)a.au, plan.au_stride, rows, splits, na, k, V,
                           a.target, N, out_ids + o0 * k, out_p + o0 * k, out_logp ? out_logp + o0 : nullptr,
                           out_entropy + o0);
      LL_CHECK_S(hipGetLastError());
    }
  }
#undef LL_CHECK_S
  return LL_OK;
}

// ---------------------------------------------------------------------------------------
// Allocation-free variant: the workspace of ll_project in a device array of this library, for
// callers that cannot allocate.  The array's name is a host-side handle, not a device address:
// its address on the current device is looked up once per device and only that pointer is used
// from then on.  inv_rms, the partials and the panel are each written in full before they are
// read; the shared top-k bounds, which have to start at zero, are cleared by a fill kernel at the
// start of every call (project_impl does that for any workspace): stale contents of an earlier
// call do not matter.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char ll_static_scratch[LL_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_static_scratch_ptr[MAX_DEVICES];

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  LL_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return LL_EINVAL;
  void* ptr = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    LL_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(ll_static_scratch)));
    if (ptr == nullptr || ((uintptr_t)ptr & 255)) return LL_EHIP;
    g_static_scratch_ptr[dev].store(ptr, std::memory_order_release);   // the same address whoever gets here first
  }
  *out = ptr;
  return LL_OK;
}

// Rows per pass for the static buffer: the usual 8192 when the plan fits, else the largest
// multiple of the row block that does; 0 when not even one row block fits.
int static_chunk_rows(const ll_shape* s, int k) {
  for (int rows = CHUNK_ROWS; rows >= BN; rows -= BN)
    if (make_plan(s, k, rows).total <= (size_t)LL_STATIC_SCRATCH_BYTES) return rows;
  return 0;
}

}  // namespace

extern "C" {

int ll_project_static(const ll_shape* shape, const void* hidden, const void* gamma, const void* W_U, float eps, int k,
                      const int32_t* target_ids, int32_t* out_topk_ids, float* out_topk_p, float* out_target_logp,
                      float* out_entropy, void* stream) {
  if (!shape_ok(shape, k)) return LL_EINVAL;
  if (shape->N == 0) return LL_OK;
  const int chunk = static_chunk_rows(shape, k);
  if (chunk == 0) return LL_ESCRATCH;
  void* ws = nullptr;
  if (const int rc = static_scratch_of_current_device(&ws); rc != LL_OK) return rc;
  return project_impl(shape, ws, (size_t)LL_STATIC_SCRATCH_BYTES, hidden, gamma, W_U, nullptr, 0u, eps, k, target_ids,
                      out_topk_ids, out_topk_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream), nullptr, chunk);
}

int64_t ll_project_static_pass_rows(const ll_shape* shape, int k) {
  if (!shape_ok(shape, k)) return 0;
  return static_chunk_rows(shape, k);
}

size_t ll_steer_sweep_workspace_bytes(const ll_shape* shape, int n_alpha) {
  if (!sweep_shape_ok(shape, n_alpha)) return 0;
  return make_sweep_plan(shape, n_alpha).total;
}

size_t ll_steer_sweep_topk_workspace_bytes(const ll_shape* shape, int n_alpha, int k) {
  if (!sweep_shape_ok(shape, n_alpha, k)) return 0;
  return make_sweep_plan(shape, n_alpha, k).total;
}

int ll_steer_sweep_topk(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                        const void* W_U, float eps, const float* v, const float* alphas, int n_alpha, int k,
                        const int32_t* target_ids, int32_t* out_topk_ids, float* out_topk_p, float* out_target_logp,
                        float* out_entropy, void* stream) {
  return sweep_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, eps, v, alphas, n_alpha, k, target_ids, out_topk_ids,
                    out_topk_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream));
}

int ll_steer_sweep(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                   const void* W_U, float eps, const float* v, const float* alphas, int n_alpha, const int32_t* target_ids,
                   int32_t* out_top1_ids, float* out_top1_p, float* out_target_logp, float* out_entropy, void* stream) {
  return sweep_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, eps, v, alphas, n_alpha, 1, target_ids, out_top1_ids,
                    out_top1_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream));
}

size_t ll_workspace_bytes(const ll_shape* shape, int k) {
  if (!shape_ok(shape, k)) return 0;
  if (shape->N == 0) return 256;
  return make_plan(shape, k).total;
}

int ll_project(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
               const void* W_U, float eps, int k, const int32_t* target_ids, int32_t* out_topk_ids, float* out_topk_p,
               float* out_target_logp, float* out_entropy, void* stream) {
  return project_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, nullptr, 0u, eps, k, target_ids, out_topk_ids,
                      out_topk_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream), nullptr);
}

int ll_project_ex(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                  const void* W_U, const float* bias, unsigned flags, float eps, int k, const int32_t* target_ids,
                  int32_t* out_topk_ids, float* out_topk_p, float* out_target_logp, float* out_entropy, void* stream) {
  return project_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, bias, flags, eps, k, target_ids, out_topk_ids,
                      out_topk_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream), nullptr);
}

int ll_project_timed(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                     const void* W_U, float eps, int k, const int32_t* target_ids, int32_t* out_topk_ids, float* out_topk_p,
                     float* out_target_logp, float* out_entropy, void* stream, float* phase_ms) {
  if (phase_ms == nullptr) return LL_EINVAL;
  return project_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, nullptr, 0u, eps, k, target_ids, out_topk_ids,
                      out_topk_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream), phase_ms);
}

}  // extern "C"
