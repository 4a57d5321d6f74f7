// Fused logit-lens projection for gfx950: RMS statistics / normalised panel, bf16 MFMA GEMM over
// the vocabulary with an online-softmax / top-k / target-gather epilogue, and the merge of the
// vocabulary splits.
//
// Follows the paper's Sec. 3.3 (Eq. 1 and "Top-k extraction") and Alg. 1 Phase 2; the logits of
// Eq. 1 live only in MFMA accumulators.
#include "ll_common.h"

#include <limits.h>
#include <math.h>

#include <type_traits>
#include <vector>

namespace {

using namespace ll;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int BM = 256;          // vocabulary rows per tile (MFMA M side)
constexpr int BN = 256;          // lens rows per workgroup (MFMA N side)
constexpr int BK = 64;           // K step of the register-staged kernel
constexpr int NTHREADS = 256;    // 4 wavefronts, one per SIMD
constexpr int CHUNK_ROWS = 8192; // lens rows per pass
constexpr int MAX_SPLITS = 64;   // vocabulary splits per row block: one lane of the merging wavefront each
constexpr int MAX_PARTIALS = 256 * 256;   // rows of a pass x splits never exceeds rows per workgroup x workgroups
constexpr int NUM_XCD = 8;
constexpr int NUM_CU = 256;
constexpr float NEG_BIG = -3.0e38f;   // stands for "no logit" without the NaNs that -inf would breed
constexpr float LOG2E = 1.4426950408889634f;

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

// ---------------------------------------------------------------------------------------
// a3..a7: the fused kernels.
//
// One workgroup owns BN = 256 lens rows and one vocabulary split; it sweeps the split's 256-wide
// vocabulary tiles.  Per tile the logits Z^T[vocab, row] = W_tile . A^T are accumulated with bf16
// MFMAs, vocabulary on the M side, lens rows on the N side: wavefront w owns lens rows
// [64w, 64w+64) against all 256 vocabulary rows (8 x 2 accumulator tiles of 32 x 32 in the
// register-staged kernel, 16 x 4 tiles of 16 x 16 in the direct-to-LDS kernel).  In the
// accumulator layouts a lane holds vocabulary entries of ONE lens row per tile; after exchanging
// the row tiles between lane blocks (v_permlane32_swap, v_permlane16_swap) lane l of wavefront w
// holds all 256 logits of lens row 64w + l, so the whole epilogue is lane-private.
// ---------------------------------------------------------------------------------------
#define LL_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

struct GemmArgs {
  const uint16_t* A;        // [rows, lda] bf16 (this pass's rows)
  const float* inv_rms;     // [rows] or nullptr (rows already normalised)
  const uint16_t* gamma;    // [d] or nullptr
  const uint16_t* W;        // [V, d] bf16
  const int32_t* target;    // [rows] or nullptr
  const float* bias;        // [V] fp32 or nullptr: the b of Eq. 1
  float4* stats;            // [rows, splits]     (m, S, T, z_target)
  uint2* top;               // [rows, splits, k]  (logit bits, id), sorted
  int64_t lda;              // row stride of A in elements
  int rows, d, V, k, splits, tiles, row_blocks;
  // steering sweep only (Sec. 3.4, Eq. 3 for several alpha in one pass):
  const float* au;          // [n_alpha, au_stride] fp32: alpha_a * (W_U v)[id], zero padded to whole tiles
  float4* sweep_stats;      // [rows, splits, n_alpha]  (m, S, T, bits of the arg max id)
  float* sweep_ztgt;        // [rows, splits]           logit of the target id at alpha = 0
  int au_stride, n_alpha;
};

// ---------------------------------------------------------------------------------------
// Epilogue shared by both GEMM kernels.  State of one lens row, private to the lane that owns it.
// With m the running maximum: S = sum exp(z - m), T = sum exp(z - m) z.  Then
// logsumexp = m + log S and entropy = m + log S - T / S.
// The row's best KR logits (KR >= k) sit in registers, sorted: descending logit, and among equal
// logits ascending id.  A workgroup meets its vocabulary ids in increasing order, so a new
// candidate never outranks an equal logit already listed and a strict comparison is exact.
// ---------------------------------------------------------------------------------------
template <int KR>
struct RowState {
  float m = -INFINITY;
  float s = 0.f;
  float t = 0.f;
  float z_tgt = -INFINITY;  // logit of the target id, once its tile has passed
  int tgt = -1;             // target id of the row (-1: none)
  float lv[KR];             // top logits
  int li[KR];               // their ids
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int j = 0; j < KR; ++j) {
      lv[j] = -INFINITY;
      li[j] = INT_MAX;
    }
  }
  __device__ __forceinline__ float tau() const { return lv[KR - 1]; }
  // Branch-free sorted insert: slot j takes its upper neighbour if the candidate goes above that
  // neighbour, the candidate if it goes exactly here, and keeps its entry otherwise.  For the
  // logits that is the median of (upper neighbour, own entry, candidate): one instruction.  Four
  // slots at a time, written as instructions: all comparisons of a block first, into four SGPR
  // pairs, then the medians, then the id selects.  Left to the compiler every comparison goes
  // through VCC with two wait states before the select that reads it (a VALU result in an SGPR
  // must not be read by the next two VALU instructions on this hardware).
  __device__ __forceinline__ void insert(float z, int id) {
    static_assert(KR % 4 == 0, "blocks of four");
    unsigned long long above;   // lanes whose candidate ranks above the entry of the block's top slot
    asm("v_cmp_gt_f32_e64 %0, %1, %2" : "=s"(above) : "v"(z), "v"(lv[KR - 1]));
#pragma unroll
    for (int j = KR - 1; j >= 3; j -= 4) {
      const float up_v = j >= 4 ? lv[j >= 4 ? j - 4 : 0] : INFINITY;   // nothing ranks above slot 0's upper neighbour
      const int up_i = li[j >= 4 ? j - 4 : 0];
      unsigned long long m1, m2, m3, m4;
      asm("v_cmp_gt_f32_e64 %9, %13, %2\n\t"     // above slot j-1
          "v_cmp_gt_f32_e64 %10, %13, %3\n\t"    // above slot j-2
          "v_cmp_gt_f32_e64 %11, %13, %4\n\t"    // above slot j-3
          "v_cmp_gt_f32_e64 %12, %13, %15\n\t"   // above slot j-4 (the next block's top slot)
          "v_med3_f32 %1, %2, %1, %13\n\t"       // new logits, top slot first: each reads its still old upper neighbour
          "v_med3_f32 %2, %3, %2, %13\n\t"
          "v_med3_f32 %3, %4, %3, %13\n\t"
          "v_med3_f32 %4, %15, %4, %13\n\t"
          "v_cndmask_b32_e64 %5, %5, %14, %0\n\t"    // id of slot j: the candidate's if it ranks above the old entry ...
          "v_cndmask_b32_e64 %5, %5, %6, %9\n\t"     // ... the upper neighbour's if it ranks above that one too
          "v_cndmask_b32_e64 %6, %6, %14, %9\n\t"
          "v_cndmask_b32_e64 %6, %6, %7, %10\n\t"
          "v_cndmask_b32_e64 %7, %7, %14, %10\n\t"
          "v_cndmask_b32_e64 %7, %7, %8, %11\n\t"
          "v_cndmask_b32_e64 %8, %8, %14, %11\n\t"
          "v_cndmask_b32_e64 %8, %8, %16, %12\n\t"
          "s_mov_b64 %0, %12"
          : "+s"(above), "+v"(lv[j]), "+v"(lv[j - 1]), "+v"(lv[j - 2]), "+v"(lv[j - 3]), "+v"(li[j]), "+v"(li[j - 1]),
            "+v"(li[j - 2]), "+v"(li[j - 3]), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4)
          : "v"(z), "v"(id), "v"(up_v), "v"(up_i));
    }
  }
};

// Reads one accumulator element where it lives (an AGPR) at the point of use, so that the
// register allocator does not copy the whole 256-register tile into VGPRs ahead of the epilogue.
__device__ __forceinline__ float acc_read(float a) {
  float v;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

// x[o] for a per-lane o in [0, 32): registers cannot be indexed by a lane-varying position, so
// pick through a binary tree of 31 selects.  The selects are written as instructions because the
// optimiser would otherwise fold the tree back into an indexed access and move the 32 values
// to scratch memory.
__device__ __forceinline__ float cndmask(float if_clear, float if_set, unsigned long long lanes) {
  float r;
  asm("v_cndmask_b32 %0, %1, %2, %3" : "=v"(r) : "v"(if_clear), "v"(if_set), "s"(lanes));
  return r;
}

__device__ __forceinline__ float select32(const float (&x)[32], int o) {
  const unsigned long long b0 = __builtin_amdgcn_ballot_w64((o & 1) != 0);
  const unsigned long long b1 = __builtin_amdgcn_ballot_w64((o & 2) != 0);
  const unsigned long long b2 = __builtin_amdgcn_ballot_w64((o & 4) != 0);
  const unsigned long long b3 = __builtin_amdgcn_ballot_w64((o & 8) != 0);
  const unsigned long long b4 = __builtin_amdgcn_ballot_w64((o & 16) != 0);
  // All five masks exist from here on, and two wait states have passed: on this hardware a VALU
  // result in an SGPR must not be read by a VALU instruction issued within the next two, and the
  // compiler, which would otherwise slide each comparison down to its first use, does not see
  // inside the select instructions below.
  unsigned long long m0_ = b0, m1_ = b1, m2_ = b2, m3_ = b3, m4_ = b4;
  asm volatile("s_nop 1" : "+s"(m0_), "+s"(m1_), "+s"(m2_), "+s"(m3_), "+s"(m4_));
  float a[16], b[8], c[4], e[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) a[i] = cndmask(x[2 * i], x[2 * i + 1], m0_);
#pragma unroll
  for (int i = 0; i < 8; ++i) b[i] = cndmask(a[2 * i], a[2 * i + 1], m1_);
#pragma unroll
  for (int i = 0; i < 4; ++i) c[i] = cndmask(b[2 * i], b[2 * i + 1], m2_);
#pragma unroll
  for (int i = 0; i < 2; ++i) e[i] = cndmask(c[2 * i], c[2 * i + 1], m3_);
  return cndmask(e[0], e[1], m4_);
}

// x[o]: logit of vocabulary entry v0 + 32 I + o of the finished tile for this lane's row.  The swap
// hands the lower lane half the row tile j = 0 and the upper half j = 1, so that lane l owns row
// 64 w + l.
template <int I>
__device__ __forceinline__ void load_group(const f32x16 (&acc)[8][2], float (&x)[32]) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc_read(acc[I][0][r])),
                                               __float_as_uint(acc_read(acc[I][1][r])), false, false);
    const int o = 8 * (r >> 2) + (r & 3);
    x[o] = __uint_as_float(sw[0]);
    x[o + 4] = __uint_as_float(sw[1]);
  }
}

// The same for the accumulators of v_mfma_f32_16x16x32_bf16: 16 x 4 tiles of 16 x 16, where lane l
// holds, of tile (i, j), vocabulary rows 4 (l/16) + r (r = 0..3) of lens row 16 j + l%16.  Seen as
// blocks of 16 lanes, register j of lane block g has to go to register g of lane block j: a 4 x 4
// transpose, done by one round of v_permlane32_swap (blocks 2,3 of one register against blocks
// 0,1 of another) and one of v_permlane16_swap (odd blocks against even blocks).  Afterwards lane
// l owns lens row 64 w + l again, and register g holds vocabulary row 16 i + 4 g + r.
template <int I>
__device__ __forceinline__ void load_group(const f32x4 (&acc)[16][4], float (&x)[32]) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      unsigned R0 = __float_as_uint(acc_read(acc[2 * I + t][0][r])), R1 = __float_as_uint(acc_read(acc[2 * I + t][1][r]));
      unsigned R2 = __float_as_uint(acc_read(acc[2 * I + t][2][r])), R3 = __float_as_uint(acc_read(acc[2 * I + t][3][r]));
      auto a = __builtin_amdgcn_permlane32_swap(R0, R2, false, false);
      auto b = __builtin_amdgcn_permlane32_swap(R1, R3, false, false);
      auto c = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
      auto d = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
      x[16 * t + r] = __uint_as_float(c[0]);
      x[16 * t + 4 + r] = __uint_as_float(c[1]);
      x[16 * t + 8 + r] = __uint_as_float(d[0]);
      x[16 * t + 12 + r] = __uint_as_float(d[1]);
    }
  }
}

// Processes vocabulary entries [v0 + 32 I, v0 + 32 I + 32) of the finished tile for the lane's row.
template <int I, int KR, bool BIAS, class ACC>
__device__ __forceinline__ void epilogue_group(const ACC& acc, RowState<KR>& st, int v0, int V, bool partial,
                                               const float* __restrict__ bias) {
  float x[32];
  load_group<I>(acc, x);
  const int g0 = v0 + 32 * I;
  if (BIAS) {   // one coalesced load of the group's 32 biases, then a broadcast per entry
    const unsigned b = __float_as_uint(bias[min(g0 + (int)(threadIdx.x & 31), V - 1)]);
#pragma unroll
    for (int o = 0; o < 32; ++o) x[o] += __uint_as_float(__builtin_amdgcn_readlane(b, o));
  }
  if (partial) {   // only the last tile of the vocabulary: a real branch (the empty asm keeps it one)
    asm volatile("");
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (g0 + o >= V) x[o] = NEG_BIG;
  }
  // a7: target gather
  const int tl = st.tgt - g0;
  if (__builtin_amdgcn_ballot_w64((unsigned)tl < 32u) != 0) {
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (tl == o) st.z_tgt = x[o];
  }
  // a5: online max / sum exp / sum exp * z
  float gmax = x[0];
#pragma unroll
  for (int o = 1; o < 32; ++o) gmax = fmaxf(gmax, x[o]);
  const float m_new = fmaxf(st.m, gmax);
  if (__builtin_amdgcn_ballot_w64(m_new > st.m) != 0) {
    const float sc = __builtin_amdgcn_exp2f((st.m - m_new) * LOG2E);   // first group: exp2(-inf) = 0
    st.s *= sc;
    st.t *= sc;
    st.m = m_new;
  }
  const float mb = st.m * LOG2E;
  float s4[4] = {0.f, 0.f, 0.f, 0.f}, t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int o = 0; o < 32; ++o) {
    const float e = __builtin_amdgcn_exp2f(fmaf(x[o], LOG2E, -mb));
    s4[o & 3] += e;
    t4[o & 3] = fmaf(e, x[o], t4[o & 3]);
  }
  st.s += (s4[0] + s4[1]) + (s4[2] + s4[3]);
  st.t += (t4[0] + t4[1]) + (t4[2] + t4[3]);

  // a6: streaming top-k.  Only when some lane of the wavefront has a logit above its current
  // KR-th best: mark the candidates against that threshold, then insert them in id order.
  if (__builtin_amdgcn_ballot_w64(gmax > st.tau()) != 0) {
    const float tau0 = st.tau();
    // bit o of mask: x[o] > tau0.  Two instructions per entry: the comparison, then the mask
    // doubled plus the comparison's result as carry-in (entries taken from 31 down to 0).  Four
    // entries at a time, comparisons first: a VALU result in an SGPR must not be read by the
    // next two VALU instructions on this hardware.
    unsigned mask = 0;
#pragma unroll
    for (int o = 28; o >= 0; o -= 4) {
      unsigned long long c0, c1, c2, c3;
      asm("v_cmp_gt_f32_e64 %1, %5, %9\n\t"
          "v_cmp_gt_f32_e64 %2, %6, %9\n\t"
          "v_cmp_gt_f32_e64 %3, %7, %9\n\t"
          "v_cmp_gt_f32_e64 %4, %8, %9\n\t"
          "v_addc_co_u32_e64 %0, %1, %0, %0, %1\n\t"
          "v_addc_co_u32_e64 %0, %2, %0, %0, %2\n\t"
          "v_addc_co_u32_e64 %0, %3, %0, %0, %3\n\t"
          "v_addc_co_u32_e64 %0, %4, %0, %0, %4"
          : "+v"(mask), "=&s"(c0), "=&s"(c1), "=&s"(c2), "=&s"(c3)
          : "v"(x[o + 3]), "v"(x[o + 2]), "v"(x[o + 1]), "v"(x[o]), "v"(tau0));
    }
    if (partial) mask &= (g0 + 32 <= V) ? 0xffffffffu : (g0 >= V ? 0u : (1u << (V - g0)) - 1u);
    while (mask != 0) {
      const int o = __builtin_ctz(mask);
      mask &= mask - 1;
      st.insert(select32(x, o), g0 + o);
    }
  }
}

template <int KR, bool BIAS, class ACC>
__device__ __forceinline__ void epilogue_tile(const ACC& acc, RowState<KR>& st, int v0, int V,
                                              const float* __restrict__ bias) {
  const bool partial = v0 + BM > V;
  // The accumulators are read below through inline asm, which the compiler's MFMA hazard
  // bookkeeping does not see: let the last MFMA of the tile drain first.
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  epilogue_group<0, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<1, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<2, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<3, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<4, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<5, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<6, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
  epilogue_group<7, KR, BIAS, ACC>(acc, st, v0, V, partial, bias);
}

// Per-(row, split) partial results: (m, S, T, z_target) and the k best (logit bits, id) pairs.
template <int KR>
__device__ __forceinline__ void epilogue_store(const GemmArgs& p, const RowState<KR>& st, int my_row, int split) {
  if (my_row >= p.rows) return;
  const int64_t o = (int64_t)my_row * p.splits + split;
  p.stats[o] = make_float4(st.m, st.s, st.t, st.z_tgt);
#pragma unroll
  for (int j = 0; j < KR; ++j)
    if (j < p.k) p.top[o * p.k + j] = make_uint2(__float_as_uint(st.lv[j]), (unsigned)st.li[j]);
}

// What a GEMM kernel does with a finished tile is a policy: the state of the lane's row, how a
// tile updates it, and what goes to the workspace at the end of the sweep.
template <int KR>
struct TopKEpilogue {   // a5..a7: softmax statistics, k best logits, target logit
  using State = RowState<KR>;
  static __device__ __forceinline__ void init(State& st, const GemmArgs& p, int my_row) {
    st.init();
    st.tgt = (p.target != nullptr && my_row < p.rows) ? p.target[my_row] : -1;
  }
  template <class ACC>
  static __device__ __forceinline__ void tile(const ACC& acc, State& st, int v0, const GemmArgs& p) {
    epilogue_tile<KR, false, ACC>(acc, st, v0, p.V, nullptr);
  }
  static __device__ __forceinline__ void store(const GemmArgs& p, const State& st, int my_row, int split) {
    epilogue_store(p, st, my_row, split);
  }
};

// ---------------------------------------------------------------------------------------
// Steering sweep (Sec. 3.4): the logits of h' = norm(h) + alpha v are z + alpha u with u = W_U v,
// so one pass over W_U serves every alpha: per alpha the lane keeps the softmax statistics and the
// arg max of z + alpha u.  alpha_a u comes as a table of fp32 per vocabulary id, read through the
// constant address space (wave-uniform addresses: scalar loads, one SGPR operand per add).
// ---------------------------------------------------------------------------------------
constexpr int SWEEP_MAX = LL_SWEEP_MAX;
typedef const float __attribute__((address_space(4)))* const_f32_ptr;

struct SweepState {
  float m[SWEEP_MAX], s[SWEEP_MAX], t[SWEEP_MAX];
  int id[SWEEP_MAX];
  float z_tgt = -INFINITY;
  int tgt = -1;
};

template <int I, class ACC>
__device__ __forceinline__ void sweep_group(const ACC& acc, SweepState& st, int v0, int V, bool partial,
                                            const GemmArgs& p) {
  const int g0 = v0 + 32 * I;
  const int tl = st.tgt - g0;
  if (__builtin_amdgcn_ballot_w64((unsigned)tl < 32u) != 0) {
    float x[32];
    load_group<I>(acc, x);
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (tl == o) st.z_tgt = x[o];
  }
#pragma unroll
  for (int a = 0; a < SWEEP_MAX; ++a) {
    if (a < p.n_alpha) {
      // The group's logits are fetched from the accumulators again for every alpha: keeping
      // them next to the shifted copy would not fit the register file.
      const_f32_ptr au = (const_f32_ptr)(uintptr_t)(p.au + (int64_t)a * p.au_stride + g0);
      float y[32];
      load_group<I>(acc, y);
#pragma unroll
      for (int o = 0; o < 32; ++o) y[o] += au[o];
      if (partial) {   // only the last tile of the vocabulary: a real branch (the empty asm keeps it one)
        asm volatile("");
#pragma unroll
        for (int o = 0; o < 32; ++o)
          if (g0 + o >= V) y[o] = NEG_BIG;
      }
      float gmax = y[0];
#pragma unroll
      for (int o = 1; o < 32; ++o) gmax = fmaxf(gmax, y[o]);
      if (__builtin_amdgcn_ballot_w64(gmax > st.m[a]) != 0) {
        // a new maximum for some lane: ids come in increasing order, so strictly greater is the
        // tie rule, and within the group the lowest position with that value wins
        const bool up = gmax > st.m[a];
        int pos = 0;
#pragma unroll
        for (int o = 31; o >= 0; --o) pos = (y[o] == gmax) ? o : pos;
        const float m_new = fmaxf(st.m[a], gmax);
        const float sc = __builtin_amdgcn_exp2f((st.m[a] - m_new) * LOG2E);   // first group: exp2(-inf) = 0
        st.s[a] *= sc;
        st.t[a] *= sc;
        st.m[a] = m_new;
        st.id[a] = up ? g0 + pos : st.id[a];
      }
      const float mb = st.m[a] * LOG2E;
      float s4[4] = {0.f, 0.f, 0.f, 0.f}, t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int o = 0; o < 32; ++o) {
        const float e = __builtin_amdgcn_exp2f(fmaf(y[o], LOG2E, -mb));
        s4[o & 3] += e;
        t4[o & 3] = fmaf(e, y[o], t4[o & 3]);
      }
      st.s[a] += (s4[0] + s4[1]) + (s4[2] + s4[3]);
      st.t[a] += (t4[0] + t4[1]) + (t4[2] + t4[3]);
      // One alpha at a time: without a use of the sums right here the compiler postpones the
      // exponentials of all nine past the last one's maximum and keeps nine shifted copies alive.
      asm volatile("" : "+v"(st.s[a]), "+v"(st.t[a]));
    }
  }
}

struct SweepEpilogue {
  using State = SweepState;
  static __device__ __forceinline__ void init(State& st, const GemmArgs& p, int my_row) {
#pragma unroll
    for (int a = 0; a < SWEEP_MAX; ++a) {
      st.m[a] = -INFINITY;
      st.s[a] = 0.f;
      st.t[a] = 0.f;
      st.id[a] = INT_MAX;
    }
    st.tgt = (p.target != nullptr && my_row < p.rows) ? p.target[my_row] : -1;
  }
  template <class ACC>
  static __device__ __forceinline__ void tile(const ACC& acc, State& st, int v0, const GemmArgs& p) {
    const bool partial = v0 + BM > p.V;
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // as in epilogue_tile: let the last MFMA drain
    sweep_group<0, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<1, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<2, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<3, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<4, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<5, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<6, ACC>(acc, st, v0, p.V, partial, p);
    sweep_group<7, ACC>(acc, st, v0, p.V, partial, p);
  }
  static __device__ __forceinline__ void store(const GemmArgs& p, const State& st, int my_row, int split) {
    if (my_row >= p.rows) return;
    const int64_t o = (int64_t)my_row * p.splits + split;
    p.sweep_ztgt[o] = st.z_tgt;
#pragma unroll
    for (int a = 0; a < SWEEP_MAX; ++a)
      if (a < p.n_alpha) p.sweep_stats[o * p.n_alpha + a] = make_float4(st.m[a], st.s[a], st.t[a], __int_as_float(st.id[a]));
  }
};

// Workgroup ids are dealt round-robin over the 8 XCDs; remap so that one XCD (one L2) gets a
// compact rectangle of (row blocks) x (all splits) and its CUs share A panels and W tiles.
__device__ __forceinline__ int xcd_logical_block() {
  const int per_xcd = gridDim.x / NUM_XCD;
  return (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
}

// ---------------------------------------------------------------------------------------
// Register-staged kernel: any d that is a multiple of 8; operands go global -> registers -> LDS,
// with the RMSNorm scaling (a3) applied between the global load and the LDS store of every A tile.
// LDS tile: [256 rows][8 chunks of 16 B]; chunk index XOR-swizzled with (row/2)%8 so that both the
// 16-byte row-major stores and the MFMA fragment reads (32 consecutive rows, one chunk) spread
// over all banks.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int lds_off(int row, int chunk) { return (row * 8 + (chunk ^ ((row >> 1) & 7))) * 16; }

template <int KR, bool BIAS>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ll_lens_gemm_kernel(const GemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sW = smem;
  unsigned char* sA = smem + BM * BK * 2;
  const bool FUSED_NORM = p.inv_rms != nullptr;

  const int logical = xcd_logical_block();
  if (logical >= p.row_blocks * p.splits) return;
  const int split = logical % p.splits;
  const int rb = logical / p.splits;
  const int tile0 = (int)((int64_t)split * p.tiles / p.splits);
  const int tile1 = (int)((int64_t)(split + 1) * p.tiles / p.splits);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int d = p.d, V = p.V;
  const int64_t lda = p.lda;

  // --- global -> LDS staging map: thread handles physical chunk (tid % 8) of rows tid/8 + 32 i.
  const int ld_row = tid >> 3;
  const int ld_chunk = (tid & 7) ^ ((ld_row >> 1) & 7);     // logical K chunk this thread fetches
  const int st_off = (ld_row * 8 + (tid & 7)) * 16;          // + i * 32 rows * 128 B

  const uint16_t* a_ptr[8];
  float a_scale[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int r = rb * BN + ld_row + 32 * i;
    r = r < p.rows ? r : p.rows - 1;
    a_ptr[i] = p.A + (int64_t)r * lda + ld_chunk * 8;
    a_scale[i] = FUSED_NORM ? p.inv_rms[r] : 1.0f;
  }

  // --- MFMA fragment map: lane reads row (lane % 32) of each 32-row group, K chunk 2*kk + lane/32.
  const int f_row = lane & 31;
  const int f_half = lane >> 5;

  // --- epilogue state: this lane owns lens row (rb*BN + tid).
  const int my_row = rb * BN + tid;
  RowState<KR> st;
  st.init();
  st.tgt = (p.target != nullptr && my_row < p.rows) ? p.target[my_row] : -1;

  const int KT = (d + BK - 1) / BK;

  for (int tile = tile0; tile < tile1; ++tile) {
    const int v0 = tile * BM;
    const uint16_t* w_ptr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int v = v0 + ld_row + 32 * i;
      v = v < V ? v : V - 1;
      w_ptr[i] = p.W + (int64_t)v * d + ld_chunk * 8;
    }

    f32x16 acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 wreg[8], areg[8], greg;
    auto fetch = [&](int kt) {
      const int koff = kt * BK;
      const bool in = koff + ld_chunk * 8 < d;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        wreg[i] = in ? *reinterpret_cast<const uint4*>(w_ptr[i] + koff) : make_uint4(0, 0, 0, 0);
        areg[i] = in ? *reinterpret_cast<const uint4*>(a_ptr[i] + koff) : make_uint4(0, 0, 0, 0);
      }
      if (FUSED_NORM) greg = in ? *reinterpret_cast<const uint4*>(p.gamma + koff + ld_chunk * 8) : make_uint4(0, 0, 0, 0);
    };

    fetch(0);
    for (int kt = 0; kt < KT; ++kt) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        *reinterpret_cast<uint4*>(sW + st_off + i * 32 * 128) = wreg[i];
        uint4 a = areg[i];
        if (FUSED_NORM) {
          // a3: a = bf16((h * inv_rms) * gamma), one rounding
          const float s = a_scale[i];
          const uint32_t gw[4] = {greg.x, greg.y, greg.z, greg.w};
          uint32_t aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
          for (int q = 0; q < 4; ++q)
            aw[q] = pack_bf16(bf16_lo(aw[q]) * s * bf16_lo(gw[q]), bf16_hi(aw[q]) * s * bf16_hi(gw[q]));
          a = make_uint4(aw[0], aw[1], aw[2], aw[3]);
        }
        *reinterpret_cast<uint4*>(sA + st_off + i * 32 * 128) = a;
      }
      __syncthreads();
      if (kt + 1 < KT) fetch(kt + 1);
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int chunk = 2 * kk + f_half;
        bf16x8 fa[2], fw[8];
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fa[j] = *reinterpret_cast<const bf16x8*>(sA + lds_off(wave * 64 + j * 32 + f_row, chunk));
#pragma unroll
        for (int i = 0; i < 8; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(sW + lds_off(i * 32 + f_row, chunk));
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
      }
    }
    epilogue_tile<KR, BIAS, f32x16[8][2]>(acc, st, v0, V, p.bias);
  }
  epilogue_store(p, st, my_row, split);
}

// ---------------------------------------------------------------------------------------
// Direct-to-LDS kernel: both operands go from global memory straight into LDS (global_load_lds,
// 16 bytes per lane) in stages of K = 64, so that every load instruction takes whole 128-byte
// lines (8 rows x 128 B).  A must be a panel of already normalised bf16 rows with row stride
// lda, a multiple of 64, zero padded beyond d (the norm kernel above writes it); W rows are read
// in place.
//
// LDS holds five 32 KB slots, each one operand tile [256 rows][128 B]: a ring of three for the
// W tiles (stage g in slot g % 3) and a ring of two for the A tiles (stage g in slot 3 + g % 2).
// The 16-byte chunk index is XOR-swizzled with (row/2)%8, which makes the 8 rows x 8 chunks that
// one load instruction writes (1 KB, lane-linear) and the 16 rows x 4 chunks that a fragment read
// touches both bank-conflict free.
//
// The matrix instruction here is v_mfma_f32_16x16x32_bf16 (vocabulary on the M side as in the
// other kernel: 16 x 4 accumulator tiles of 16 x 16 per wavefront).  At the same rate it moves
// half the accumulator bytes per flop of the 32x32x16 form, and on this power-limited chip that
// is worth 11 % on a bare MFMA loop and 4 % on this kernel.
//
// Wavefront w loads rows [64w, 64w+64) of every tile.  Of a W tile it reads all rows, so W slots
// change hands at a workgroup barrier; of an A tile it reads exactly the rows it loaded itself,
// so an A slot is the wavefront's own again as soon as its last fragment of the stage is in
// registers, with no barrier.  That is what the two rings are for: the A fragments of a whole
// stage are read early (32 registers), and both streams get about two stages between sending a
// load and needing its data, from the same 160 KB.
//
// Schedule of stage g, four slices of 32 MFMAs: (K half 0, vocabulary tiles 0-7), (0, 8-15),
// (1, 0-7), (1, 8-15); W fragments alternate between two register sets of eight:
//   slice 0    : reads the W fragments of slice 1 and the A fragments of K half 1 (the last of
//                the stage: the wavefront's rows of A(g)'s slot are free); sends the second half
//                of W(g+2);
//   slices 1, 2: read the W fragments of the next slice; send A(g+2), half each;
//   wait + barrier: all loads but the last 16 (W(g+2), A(g+2)) have landed, so stage g+1 is in
//                LDS for everyone, and everyone holds its last fragments of W(g): that slot is free;
//   slice 3    : reads the W fragments of slice 0 and the A fragments of K half 0 of stage g+1;
//                sends the first half of W(g+3) into the slot of W(g).
// Four loads per slice, one behind every eighth MFMA, keep the load pipe evenly fed and the
// wavefront's issue slots free for the matrix pipe.  The rings are fed unconditionally and run on
// across vocabulary tiles (the next tile's first stages load under the epilogue); past the last
// real stage they re-fetch the last tile, never consumed, which keeps the count of loads in
// flight, and with it the s_waitcnt, constant.
// ---------------------------------------------------------------------------------------
constexpr int DK = 64;
constexpr int W_SLOTS = 3, A_SLOTS = 2, SLOTS = W_SLOTS + A_SLOTS;
constexpr int SLOT_BYTES = 256 * DK * 2;
constexpr int LOADS_PER_TILE = 8;    // per wavefront: 8 segments of 1 KB of one operand tile
// s_waitcnt immediate (gfx9 layout): vmcnt in bits 3:0 and 15:14, expcnt 6:4 (7 = no wait), lgkmcnt 11:8.
constexpr int waitcnt_imm(int vmcnt, int lgkmcnt) { return (vmcnt & 0xF) | ((vmcnt >> 4) << 14) | 0x70 | (lgkmcnt << 8); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// One global_load_lds_dwordx4: every lane fetches 16 bytes from base + off + IMM and the
// wavefront's 1 KB lands lane-linear at LDS byte address M0 + IMM (the instruction's immediate
// offset moves both addresses).  Written as an instruction rather than through the builtin: the
// compiler cannot tell which LDS bytes a builtin load-to-LDS writes, so it makes every later LDS
// read wait for ALL loads in flight, which would serialise the ring; here all waits are the
// explicit s_waitcnt of the main loop.  One instruction per load, with the LDS base set once per
// tile, matters: a wavefront alone on its SIMD issues one instruction every four cycles or so, and
// whatever sits between two MFMAs beyond the 16 cycles the first one runs leaves the pipe idle.
template <int IMM>
__device__ __forceinline__ void load_to_lds_16(const unsigned char* base, unsigned off) {
  static_assert(IMM >= -4096 && IMM < 4096, "13-bit signed immediate");
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(off), "s"(base), "n"(IMM) : "memory");
}

// LDS base of the loads that follow.  M0 is the compiler's own scratch register: it sets it right
// before each of its own uses and keeps nothing in it, and it knows from the clobber that this
// statement writes it.  Nothing in the main loop below (MFMA, ds_read, s_waitcnt, s_barrier)
// makes the compiler use M0, so the value holds from here to the last load of the tile.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void set_lds_dma_base(unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
  return c;
}

template <class EPI>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ll_lens_gemm_dma_kernel(const GemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem[];

  const int logical = xcd_logical_block();
  if (logical >= p.row_blocks * p.splits) return;
  const int split = logical % p.splits;
  const int rb = logical / p.splits;
  const int tile0 = (int)((int64_t)split * p.tiles / p.splits);
  const int tile1 = (int)((int64_t)(split + 1) * p.tiles / p.splits);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.d, V = p.V;
  const int lda = (int)p.lda;
  const int KT = lda / DK;

  // --- DMA map.  One load instruction fills 8 rows x 128 B; lane l lands at row l/8, physical
  // chunk l%8.  Wavefront w fills rows [64w, 64w+64) of a tile in 8 segments; segment s holds
  // rows 64w + 8s + l/8, whose swizzle is (l/16 + 4s) % 8, so the lane fetches logical chunk
  // (l%8) ^ (l/16) ^ 4(s%2).  M0 points at the middle of the wavefront's 8 KB and segment s uses
  // the immediate (s-4) KB; since the immediate also moves the global address, the lane's byte
  // offset carries the opposite shift, plus 7 KB so that it cannot go below zero, and the
  // wave-uniform base (tile, K step) starts 3 KB early: base + off + imm is the chunk's address.
  const int seg_row = 64 * wave + (lane >> 3);                        // + 8 s
  const int seg_koff0 = ((lane & 7) ^ (lane >> 4)) * 8;               // element offset, even segments
  const int seg_koff1 = seg_koff0 ^ 32;                               // odd segments
  const int a_last = p.rows - 1 - rb * BN;                            // last valid row of this block
  constexpr int IMM_BIAS = 3072;                                      // largest immediate, segment 7

  // Per-lane byte offsets of the 8 segments, fixed for the whole sweep (W: per vocabulary tile,
  // because the last tile clamps its rows to V-1): one load is one instruction.
  unsigned a_off[8], w_off[8];
#pragma unroll
  for (int s = 0; s < 8; ++s)
    a_off[s] = (unsigned)(min(seg_row + 8 * s, a_last) * lda + ((s & 1) ? seg_koff1 : seg_koff0)) * 2u + (7168u - 1024u * s);
  auto set_w_rows = [&](int tile) {
    const int w_last = V - 1 - tile * BM;
#pragma unroll
    for (int s = 0; s < 8; ++s)
      w_off[s] = (unsigned)(min(seg_row + 8 * s, w_last) * d + ((s & 1) ? seg_koff1 : seg_koff0)) * 2u + (7168u - 1024u * s);
  };

  // Producer state of the two operand streams, all wave-uniform and moved on by a few scalar
  // instructions per stage.
  const unsigned lds_mid = (unsigned)(uintptr_t)(lptr_t)smem + wave * (64 * DK * 2) + 4096;
  const unsigned w_lds_wrap = lds_mid + W_SLOTS * SLOT_BYTES;
  const unsigned a_lds_flip = (2 * W_SLOTS + 1) * SLOT_BYTES + 2 * lds_mid;   // slot 3 <-> slot 4
  const unsigned char* const a_base0 = reinterpret_cast<const unsigned char*>(p.A + (int64_t)rb * BN * lda) - IMM_BIAS;
  auto w_tile_base = [&](int tile) {
    return reinterpret_cast<const unsigned char*>(p.W + (int64_t)tile * BM * d) - IMM_BIAS;
  };
  // (LL_PIN_S: the value is computed where the statement stands; without it the compiler gathers
  // the scalar updates of a whole stage into one lump, and the matrix pipe idles behind it.)
#define LL_PIN_S(x) asm volatile("" : "+s"(x))
  int w_tile = tile0, w_kt = 0, a_kt = 0;
  unsigned w_lds = lds_mid, a_lds = lds_mid + W_SLOTS * SLOT_BYTES;   // M0 value of the stream's next tile
  const unsigned char* w_base = w_tile_base(tile0);
  const unsigned char* a_base = a_base0;
  set_w_rows(tile0);
  auto advance_w = [&]() {
    w_lds += SLOT_BYTES;
    if (w_lds >= w_lds_wrap) w_lds -= W_SLOTS * SLOT_BYTES;
    w_base += DK * 2;
    if (++w_kt == KT) {   // next vocabulary tile; past the end of the sweep the ring refetches the last one
      w_kt = 0;
      ++w_tile;
      const int t = w_tile < tile1 ? w_tile : tile1 - 1;
      set_w_rows(t);
      w_base = w_tile_base(t);
    }
    LL_PIN_S(w_lds);
    LL_PIN_S(w_base);
  };
  auto advance_a = [&]() {
    a_lds = a_lds_flip - a_lds;
    a_base += DK * 2;
    if (++a_kt == KT) {
      a_kt = 0;
      a_base = a_base0;
    }
    LL_PIN_S(a_lds);
    LL_PIN_S(a_base);
  };
#define LL_DMA_W(S) load_to_lds_16<((S) - 4) * 1024>(w_base, w_off[S])
#define LL_DMA_A(S) load_to_lds_16<((S) - 4) * 1024>(a_base, a_off[S])
#define LL_DMA_TILE(DMA) DMA(0); DMA(1); DMA(2); DMA(3); DMA(4); DMA(5); DMA(6); DMA(7)

  // --- MFMA fragment map (v_mfma_f32_16x16x32_bf16): lane reads row (lane % 16) of each 16-row
  // group; of the two K = 32 halves of a stage, half hk is the logical 16-byte chunks
  // 4 hk + lane/16 of the row.
  const int f_row = lane & 15;
  const int f_grp = lane >> 4;
  const int f_swz = (f_row >> 1) & 7;
  int f_off[2];
#pragma unroll
  for (int hk = 0; hk < 2; ++hk) f_off[hk] = f_row * (DK * 2) + (((4 * hk + f_grp) ^ f_swz) * 16);
  const int a_wave_off = (wave * 64) * (DK * 2);

  const int my_row = rb * BN + tid;
  typename EPI::State st;
  EPI::init(st, p, my_row);

  // prologue: W0 A0 W1 A1 and the first half of W2 in flight; stage 0 landed
  set_lds_dma_base(w_lds);
  LL_DMA_TILE(LL_DMA_W);
  advance_w();
  set_lds_dma_base(a_lds);
  LL_DMA_TILE(LL_DMA_A);
  advance_a();
  set_lds_dma_base(w_lds);
  LL_DMA_TILE(LL_DMA_W);
  advance_w();
  set_lds_dma_base(a_lds);
  LL_DMA_TILE(LL_DMA_A);
  advance_a();
  set_lds_dma_base(w_lds);
  LL_DMA_W(0); LL_DMA_W(1); LL_DMA_W(2); LL_DMA_W(3);
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * LOADS_PER_TILE + 4, 15));   // W0 and A0 landed
  __syncthreads();
  // A: the four row tiles of both K halves of the stage; W: two sets of eight vocabulary tiles of one half
  bf16x8 fa[2][4], fw0[8], fw1[8];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    fa[0][j] = *reinterpret_cast<const bf16x8*>(smem + W_SLOTS * SLOT_BYTES + a_wave_off + j * 16 * (DK * 2) + f_off[0]);
#pragma unroll
  for (int i = 0; i < 8; ++i) fw0[i] = *reinterpret_cast<const bf16x8*>(smem + i * 16 * (DK * 2) + f_off[0]);

  // A stage is four slices of 32 MFMAs: (K half 0, vocabulary tiles 0-7), (0, 8-15), (1, 0-7),
  // (1, 8-15).  One slice: eight vocabulary tiles (fragments fw) against the four row tiles of a
  // K half (fah), accumulators MB .. MB+7.  An MFMA runs for 16 cycles, so a gap between two of
  // them holds at most two or three other instructions: behind the first MFMA of a row of four
  // goes the LDS read of one W fragment of the next slice (into nw, from LDS offset tW),
  // behind the second an A fragment read (RHOOK), behind the third a load-to-LDS or a piece of
  // the streams' bookkeeping (HOOK).  The fences pin that order.
#define LL_LDS_FRAG(ptr) (*reinterpret_cast<const bf16x8*>(ptr))
  // Written as an instruction so that the 64 accumulator tiles stay in AGPRs: given the builtin,
  // the register allocator keeps some of them in VGPRs and copies them in and out around the MFMA.
  // (Operands come from LDS reads, whose waits the compiler still places; nothing reads an
  // accumulator before the epilogue's own drain.)
#define LL_MFMA16(a, b, c) mfma16(a, b, c)
#define LL_ROW(I, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                        \
  acc[MB + I][0] = LL_MFMA16(fw[I], fah[0], acc[MB + I][0]);                                         \
  nw[I] = LL_LDS_FRAG(smem + tW + (NMB + I) * 16 * (DK * 2) + (off));                                \
  LL_SCHED_FENCE();                                                                                  \
  acc[MB + I][1] = LL_MFMA16(fw[I], fah[1], acc[MB + I][1]);                                         \
  RHOOK(I);                                                                                          \
  LL_SCHED_FENCE();                                                                                  \
  acc[MB + I][2] = LL_MFMA16(fw[I], fah[2], acc[MB + I][2]);                                         \
  HOOK(I);                                                                                           \
  LL_SCHED_FENCE();                                                                                  \
  acc[MB + I][3] = LL_MFMA16(fw[I], fah[3], acc[MB + I][3]);                                         \
  LL_SCHED_FENCE();
#define LL_SLICE(MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                         \
  LL_SCHED_FENCE();                                                                                  \
  LL_ROW(0, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(1, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(2, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(3, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(4, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(5, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(6, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)                                              \
  LL_ROW(7, MB, fw, fah, nw, tW, NMB, off, RHOOK, HOOK)

#define LL_RHOOK_NONE(I) (void)0
  // slice 0 fetches the A fragments of the stage's second K half (the last of A(g) this wavefront
  // needs), slice 3 those of the next stage's first half
#define LL_RHOOK_S0(I) \
  if (I < 4) fa[1][I & 3] = LL_LDS_FRAG(smem + cA + (I & 3) * 16 * (DK * 2) + f_off[1])
#define LL_RHOOK_S3(I) \
  if (I < 4) fa[0][I & 3] = LL_LDS_FRAG(smem + nA + (I & 3) * 16 * (DK * 2) + f_off[0])
#define LL_HOOK_S0(I)                                \
  if (I == 0) set_lds_dma_base(w_lds);               \
  if (I == 3) LL_DMA_W(4);                           \
  if (I == 4) LL_DMA_W(5);                           \
  if (I == 5) LL_DMA_W(6);                           \
  if (I == 6) LL_DMA_W(7);                           \
  if (I == 7) advance_w()
  // (the last A fragments of the stage were read early in slice 0, and LDS reads return in order:
  // once slice 1 has its first W fragment, A(g)'s slot is the wavefront's own)
#define LL_HOOK_S1(I)                                \
  if (I == 3) set_lds_dma_base(a_lds);               \
  if (I == 4) LL_DMA_A(0);                           \
  if (I == 5) LL_DMA_A(1);                           \
  if (I == 6) LL_DMA_A(2);                           \
  if (I == 7) LL_DMA_A(3)
#define LL_HOOK_S2(I)                                \
  if (I == 2) LL_DMA_A(4);                           \
  if (I == 3) LL_DMA_A(5);                           \
  if (I == 4) LL_DMA_A(6);                           \
  if (I == 5) LL_DMA_A(7);                           \
  if (I == 6) advance_a()
#define LL_HOOK_S3(I)                                \
  if (I == 3) set_lds_dma_base(w_lds);               \
  if (I == 4) LL_DMA_W(0);                           \
  if (I == 5) {                                      \
    LL_DMA_W(1);                                     \
    nnW = nW + SLOT_BYTES >= W_SLOTS * SLOT_BYTES ? 0 : nW + SLOT_BYTES;   \
    LL_PIN_S(nnW);                                   \
  }                                                  \
  if (I == 6) {                                      \
    LL_DMA_W(2);                                     \
    const int t_ = cA;                               \
    cA = nA;                                         \
    nA = t_;                                         \
  }                                                  \
  if (I == 7) {   /* every row of the slice reads a W fragment from nW: move on after the last */ \
    LL_DMA_W(3);                                     \
    cW = nW;                                         \
    nW = nnW;                                        \
  }

  // Consumer state: LDS byte offsets of the W and A tiles of this stage and of the next (the A
  // offsets include the wavefront's own 64 rows).
  int cW = 0, nW = SLOT_BYTES, nnW = 2 * SLOT_BYTES;
  int cA = W_SLOTS * SLOT_BYTES + a_wave_off, nA = (W_SLOTS + 1) * SLOT_BYTES + a_wave_off;
  for (int tile = tile0; tile < tile1; ++tile) {
    f32x4 acc[16][4];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < KT; ++kt) {
      LL_SLICE(0, fw0, fa[0], fw1, cW, 8, f_off[0], LL_RHOOK_S0, LL_HOOK_S0)
      LL_SLICE(8, fw1, fa[0], fw0, cW, 0, f_off[1], LL_RHOOK_NONE, LL_HOOK_S1)
      LL_SLICE(0, fw0, fa[1], fw1, cW, 8, f_off[1], LL_RHOOK_NONE, LL_HOOK_S2)
      // stage g+1 landed (W(g+2) and A(g+2) may still be out); all my reads of W(g) are done
      __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * LOADS_PER_TILE, 0));
      __syncthreads();
      LL_SLICE(8, fw1, fa[1], fw0, nW, 0, f_off[0], LL_RHOOK_S3, LL_HOOK_S3)
    }
    EPI::tile(acc, st, tile * BM, p);
  }
#undef LL_SLICE
#undef LL_ROW
#undef LL_MFMA16
#undef LL_LDS_FRAG
#undef LL_DMA_TILE
#undef LL_HOOK_S3
#undef LL_RHOOK_S3
#undef LL_RHOOK_S0
#undef LL_RHOOK_NONE
#undef LL_PIN_S
#undef LL_HOOK_S2
#undef LL_HOOK_S1
#undef LL_HOOK_S0
#undef LL_DMA_A
#undef LL_DMA_W
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));   // drain the ring before the LDS is given back
  EPI::store(p, st, my_row, split);
}


__global__ __launch_bounds__(256) void ll_fill_f32_kernel(float* __restrict__ p, int n, float value) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = value;
}

// ---------------------------------------------------------------------------------------
// Steering sweep, step 1: u = W_U v (one pass over W_U, HBM-bound: 2 V d bytes), written as the
// table au[a, id] = alpha_a * u[id] that the sweep epilogue adds to the logits.  One wavefront
// takes four vocabulary rows at a time so that a chunk of v read from LDS serves four products.
// ---------------------------------------------------------------------------------------
struct AlphaList {
  float a[SWEEP_MAX];
};

__global__ __launch_bounds__(256) void ll_unembed_direction_kernel(const uint16_t* __restrict__ W, const float* __restrict__ v,
                                                                   int V, int d, AlphaList alphas, int n_alpha,
                                                                   float* __restrict__ au, int au_stride) {
  extern __shared__ __align__(16) float sv[];
  for (int j = threadIdx.x; j < d; j += blockDim.x) sv[j] = v[j];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n16 = d >> 3;
  for (int r0 = (blockIdx.x * 4 + wave) * 4; r0 < V; r0 += gridDim.x * 16) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const uint4* rows[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rows[i] = reinterpret_cast<const uint4*>(W + (int64_t)min(r0 + i, V - 1) * d);
    for (int c = lane; c < n16; c += 64) {
      const float4 v0 = *reinterpret_cast<const float4*>(sv + 8 * c);
      const float4 v1 = *reinterpret_cast<const float4*>(sv + 8 * c + 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 q = rows[i][c];
        float a = acc[i];
        a = fmaf(bf16_lo(q.x), v0.x, a);
        a = fmaf(bf16_hi(q.x), v0.y, a);
        a = fmaf(bf16_lo(q.y), v0.z, a);
        a = fmaf(bf16_hi(q.y), v0.w, a);
        a = fmaf(bf16_lo(q.z), v1.x, a);
        a = fmaf(bf16_hi(q.z), v1.y, a);
        a = fmaf(bf16_lo(q.w), v1.z, a);
        a = fmaf(bf16_hi(q.w), v1.w, a);
        acc[i] = a;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
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
// a8: merge the splits of each row and finalise.  One thread per row.
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

// One wavefront per row, lane s = split s (splits <= 64).
__global__ __launch_bounds__(256) void ll_merge_kernel(const float4* __restrict__ stats, const uint2* __restrict__ top,
                                                       int rows, int splits, int k, int V, int topk_softmax,
                                                       const int32_t* __restrict__ target, int32_t* __restrict__ out_ids,
                                                       float* __restrict__ out_p, float* __restrict__ out_logp,
                                                       float* __restrict__ out_entropy) {
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const bool live = lane < splits;
  float4 q = make_float4(-INFINITY, 0.f, 0.f, -INFINITY);
  if (live) q = stats[(int64_t)row * splits + lane];
  const float M = wave_max(q.x);
  const float sc = live ? __builtin_amdgcn_exp2f((q.x - M) * LOG2E) : 0.f;
  const float S = wave_sum(sc * q.y);
  const float T = wave_sum(sc * q.z);
  const float zt = wave_max(q.w);
  const float logS = logf(S);
  if (lane == 0) {
    out_entropy[row] = (M - T / S) + logS;
    if (target != nullptr) {
      const int t = target[row];
      out_logp[row] = (t >= 0 && t < V) ? (zt - M) - logS : __builtin_nanf("");
    }
  }
  // k-way merge of the per-split sorted lists (descending logit, ascending id): every lane holds the
  // head of its list; the wavefront's best head goes out and that lane moves on.
  const uint2* tl = top + ((int64_t)row * splits + lane) * k;
  int head = 0;
  float z = -INFINITY;
  int id = INT_MAX;
  if (live) {
    const uint2 e = tl[0];
    z = __uint_as_float(e.x);
    id = (int)e.y;
  }
  float z0 = 0.f, sk = 0.f;   // top-k-only softmax: the largest selected logit and the sum over the selection
  float mine = 0.f;           // lane j keeps the j-th selected logit
  for (int j = 0; j < k; ++j) {
    const float bz = wave_max(z);
    const int bi = wave_min_int(z == bz ? id : INT_MAX);
    if (live && z == bz && id == bi) {   // ids are distinct: exactly one lane
      ++head;
      if (head < k) {
        const uint2 e = tl[head];
        z = __uint_as_float(e.x);
        id = (int)e.y;
      } else {
        z = -INFINITY;
        id = INT_MAX;
      }
    }
    if (j == 0) z0 = bz;
    sk += __builtin_amdgcn_exp2f((bz - z0) * LOG2E);
    if (lane == j) mine = bz;
    if (lane == 0) {
      out_ids[(int64_t)row * k + j] = bi;
      if (!topk_softmax) out_p[(int64_t)row * k + j] = __builtin_amdgcn_exp2f(((bz - M) - logS) * LOG2E);
    }
  }
  // The paper's own probabilities (Sec. 3.3): a softmax over the k selected logits only.
  if (topk_softmax && lane < k) out_p[(int64_t)row * k + lane] = __builtin_amdgcn_exp2f((mine - z0) * LOG2E) * (1.0f / sk);
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

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
struct Plan {
  size_t off_inv_rms, off_stats, off_top, off_panel, total;
  int64_t lda;
};

bool shape_ok(const ll_shape* s, int k) {
  if (s == nullptr) return false;
  if (s->N < 0 || s->d <= 0 || s->V <= 0 || (s->d & 7) != 0) return false;
  if (k < 1 || k > LL_KMAX || k > s->V) return false;
  return true;
}

Plan make_plan(const ll_shape* s, int k) {
  Plan p;
  size_t off = 0;
  p.off_inv_rms = off;
  off = align_up(off + (size_t)s->N * sizeof(float), 256);
  const size_t rows = (size_t)(s->N < CHUNK_ROWS ? s->N : CHUNK_ROWS);
  p.off_stats = off;
  const size_t partials = rows * MAX_SPLITS < (size_t)MAX_PARTIALS ? rows * MAX_SPLITS : (size_t)MAX_PARTIALS;
  off = align_up(off + partials * sizeof(float4), 256);
  p.off_top = off;
  off = align_up(off + partials * (size_t)k * sizeof(uint2), 256);
  p.lda = (s->d + DK - 1) / DK * DK;
  p.off_panel = off;
  off = align_up(off + rows * (size_t)p.lda * sizeof(uint16_t), 256);
  p.total = off;
  return p;
}

// 0: automatic; 1: register-staged kernel with the norm fused into the A-tile load; 2: direct-to-LDS
// kernel fed from a normalised panel.
int g_gemm_path = 0;

int project_impl(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                 const void* W_U, const float* bias, unsigned flags, float eps, int k, const int32_t* target_ids,
                 int32_t* out_topk_ids, float* out_topk_p,
                 float* out_target_logp, float* out_entropy, hipStream_t stream, float* phase_ms) {
  if (!shape_ok(shape, k)) return LL_EINVAL;
  if (shape->N == 0) {
    if (phase_ms) phase_ms[0] = phase_ms[1] = phase_ms[2] = 0.f;
    return LL_OK;
  }
  if (hidden == nullptr || W_U == nullptr || out_topk_ids == nullptr || out_topk_p == nullptr || out_entropy == nullptr)
    return LL_EINVAL;
  if (target_ids != nullptr && out_target_logp == nullptr) return LL_EINVAL;
  if (!(eps >= 0.f)) return LL_EINVAL;
  if ((flags & ~(unsigned)LL_FLAG_TOPK_SOFTMAX) != 0 || ((uintptr_t)bias & 3)) return LL_EINVAL;
  const uintptr_t align_or = (uintptr_t)hidden | (uintptr_t)W_U | (uintptr_t)gamma;
  if (align_or & 15) return LL_EINVAL;
  const Plan plan = make_plan(shape, k);
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
  // A bias (rare: the paper's model families have none) goes through the register-staged kernel,
  // so that the fast kernel carries no code or registers for it.
  const bool dma = g_gemm_path != 1 && dma_ok && bias == nullptr;
  const size_t lds = dma ? (size_t)SLOTS * SLOT_BYTES : (size_t)(BM + BN) * BK * 2;
  // The top-k lists live in registers: the kernels are built for a few list lengths KR >= k.
  void (*kern)(const GemmArgs);
#define LL_PICK(KR) \
  (dma ? ll_lens_gemm_dma_kernel<TopKEpilogue<KR>> : (bias ? ll_lens_gemm_kernel<KR, true> : ll_lens_gemm_kernel<KR, false>))
  if (k <= 4)
    kern = LL_PICK(4);
  else if (k <= 12)
    kern = LL_PICK(12);
  else if (k <= 20)
    kern = LL_PICK(20);
  else
    kern = LL_PICK(32);
#undef LL_PICK
  LL_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  // The direct-to-LDS kernel reads hidden in place when the rows need neither scaling nor padding.
  const bool need_panel = dma && (has_gamma || plan.lda != d);

  // Timing (ll_project_timed only): events are recorded in-stream around every kernel and read
  // after one synchronisation at the end, so the kernels run back to back as in ll_project.
  std::vector<hipEvent_t> ev;
  auto mark = [&]() -> hipError_t {
    if (!phase_ms) return hipSuccess;
    hipEvent_t e = nullptr;
    hipError_t rc = hipEventCreate(&e);
    if (rc != hipSuccess) return rc;
    ev.push_back(e);
    return hipEventRecord(e, stream);
  };
  auto finish = [&](int rc) {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    return rc;
  };
#define LL_CHECK_F(expr)                                   \
  do {                                                     \
    hipError_t e__ = (expr);                               \
    if (e__ != hipSuccess) return finish(hip_failed(e__)); \
  } while (0)

  const int tiles = (V + BM - 1) / BM;
  for (int64_t r0 = 0; r0 < N; r0 += CHUNK_ROWS) {
    const int rows = (int)((N - r0) < CHUNK_ROWS ? (N - r0) : CHUNK_ROWS);
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
    int splits = NUM_CU / row_blocks;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    GemmArgs a;
    a.A = need_panel ? panel : h_rows;
    a.lda = need_panel ? plan.lda : d;
    a.inv_rms = (!dma && has_gamma) ? inv_rms + r0 : nullptr;
    a.gamma = static_cast<const uint16_t*>(gamma);
    a.W = static_cast<const uint16_t*>(W_U);
    a.target = target_ids ? target_ids + r0 : nullptr;
    a.bias = bias;
    a.stats = stats;
    a.top = top;
    a.rows = rows;
    a.d = d;
    a.V = V;
    a.k = k;
    a.splits = splits;
    a.tiles = tiles;
    a.row_blocks = row_blocks;
    const int grid = (row_blocks * splits + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    LL_CHECK_F(mark());
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHREADS), lds, stream, a);
    LL_CHECK_F(hipGetLastError());
    LL_CHECK_F(mark());
    hipLaunchKernelGGL(ll_merge_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, (const float4*)stats, (const uint2*)top,
                       rows, splits, k, V, (flags & LL_FLAG_TOPK_SOFTMAX) ? 1 : 0, a.target, out_topk_ids + r0 * k,
                       out_topk_p + r0 * k,
                       out_target_logp ? out_target_logp + r0 : nullptr, out_entropy + r0);
    LL_CHECK_F(hipGetLastError());
    LL_CHECK_F(mark());
  }
  if (phase_ms) {
    LL_CHECK_F(hipStreamSynchronize(stream));
    phase_ms[0] = phase_ms[1] = phase_ms[2] = 0.f;
    for (size_t i = 0; i + 3 < ev.size(); i += 4) {
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
  size_t off_au, off_stats, off_ztgt, off_panel, total;
  int64_t lda;
  int au_stride;
};

SweepPlan make_sweep_plan(const ll_shape* s, int n_alpha) {
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
  p.lda = s->d;
  p.off_panel = off;
  off = align_up(off + rows * (size_t)p.lda * sizeof(uint16_t), 256);
  p.total = off;
  return p;
}

bool sweep_shape_ok(const ll_shape* s, int n_alpha) {
  return shape_ok(s, 1) && s->d % DK == 0 && n_alpha >= 1 && n_alpha <= SWEEP_MAX &&
         (int64_t)BM * s->d * 2 < (int64_t)1 << 31 && (int64_t)CHUNK_ROWS * s->d * 2 < (int64_t)1 << 31;
}

int sweep_impl(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
               const void* W_U, float eps, const float* v, const float* alphas, int n_alpha, const int32_t* target_ids,
               int32_t* out_ids, float* out_p, float* out_logp, float* out_entropy, hipStream_t stream) {
  if (!sweep_shape_ok(shape, n_alpha)) return LL_EINVAL;
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
  const SweepPlan plan = make_sweep_plan(shape, n_alpha);
  if (workspace == nullptr || workspace_bytes < plan.total || ((uintptr_t)workspace & 255)) return LL_EWORKSPACE;

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  float* au = reinterpret_cast<float*>(ws + plan.off_au);
  float4* stats = reinterpret_cast<float4*>(ws + plan.off_stats);
  float* ztgt = reinterpret_cast<float*>(ws + plan.off_ztgt);
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
  hipLaunchKernelGGL(ll_unembed_direction_kernel, dim3(NUM_CU * 4), dim3(256), (size_t)d * sizeof(float), stream,
                     static_cast<const uint16_t*>(W_U), v, V, d, al, n_alpha, au, plan.au_stride);
  LL_CHECK_S(hipGetLastError());
  auto kern = ll_lens_gemm_dma_kernel<SweepEpilogue>;
  const size_t lds = (size_t)SLOTS * SLOT_BYTES;
  LL_CHECK_S(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));

  for (int64_t r0 = 0; r0 < N; r0 += CHUNK_ROWS) {
    const int rows = (int)((N - r0 < CHUNK_ROWS) ? (N - r0) : CHUNK_ROWS);
    const uint16_t* h_rows = static_cast<const uint16_t*>(hidden) + r0 * d;
    if (gamma != nullptr) {
      const dim3 grid((unsigned)((rows + 3) / 4));
      const uint16_t* g = static_cast<const uint16_t*>(gamma);
      if (d <= 64 * 8 * 4)
        hipLaunchKernelGGL(ll_norm_panel_kernel<4>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else if (d <= 64 * 8 * 16)
        hipLaunchKernelGGL(ll_norm_panel_kernel<16>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      else
        hipLaunchKernelGGL(ll_norm_panel_kernel<0>, grid, dim3(256), 0, stream, h_rows, g, panel, rows, d, plan.lda, eps);
      LL_CHECK_S(hipGetLastError());
    }
    const int row_blocks = (rows + BN - 1) / BN;
    int splits = NUM_CU / row_blocks;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    GemmArgs a = {};
    a.A = gamma != nullptr ? panel : h_rows;
    a.lda = plan.lda;
    a.W = static_cast<const uint16_t*>(W_U);
    a.target = target_ids ? target_ids + r0 : nullptr;
    a.rows = rows;
    a.d = d;
    a.V = V;
    a.k = 1;
    a.splits = splits;
    a.tiles = tiles;
    a.row_blocks = row_blocks;
    a.au = au;
    a.au_stride = plan.au_stride;
    a.n_alpha = n_alpha;
    a.sweep_stats = stats;
    a.sweep_ztgt = ztgt;
    const int grid = (row_blocks * splits + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHREADS), lds, stream, a);
    LL_CHECK_S(hipGetLastError());
    hipLaunchKernelGGL(ll_sweep_merge_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, (const float4*)stats,
                       (const float*)ztgt, (const float*)au, plan.au_stride, rows, splits, n_alpha, V, a.target, N,
                       out_ids + r0, out_p + r0, out_logp ? out_logp + r0 : nullptr, out_entropy + r0);
    LL_CHECK_S(hipGetLastError());
  }
#undef LL_CHECK_S
  return LL_OK;
}

}  // namespace

extern "C" {

size_t ll_steer_sweep_workspace_bytes(const ll_shape* shape, int n_alpha) {
  if (!sweep_shape_ok(shape, n_alpha)) return 0;
  return make_sweep_plan(shape, n_alpha).total;
}

int ll_steer_sweep(const ll_shape* shape, void* workspace, size_t workspace_bytes, const void* hidden, const void* gamma,
                   const void* W_U, float eps, const float* v, const float* alphas, int n_alpha, const int32_t* target_ids,
                   int32_t* out_top1_ids, float* out_top1_p, float* out_target_logp, float* out_entropy, void* stream) {
  return sweep_impl(shape, workspace, workspace_bytes, hidden, gamma, W_U, eps, v, alphas, n_alpha, target_ids, out_top1_ids,
                    out_top1_p, out_target_logp, out_entropy, static_cast<hipStream_t>(stream));
}

int ll_set_gemm_path(int path) {
  if (path < 0 || path > 2) return LL_EINVAL;
  g_gemm_path = path;
  return LL_OK;
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
