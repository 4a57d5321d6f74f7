// What the projection kernels share: tile constants, the kernel argument block, and the epilogue
// that turns a finished 256 x 256 tile of logits (paper Sec. 3.3, Eq. 1) into the row's running
// softmax statistics, top-k list and target logit, or into the steering sweep's per-alpha
// statistics (Sec. 3.4).  The logits exist only in MFMA accumulators; everything here is private to
// the lane that owns the lens row.
#pragma once

#include "ll_common.h"

#include <limits.h>
#include <math.h>

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

typedef const float __attribute__((address_space(4)))* const_f32_ptr;   // read through scalar loads when the address is wave-uniform

struct GemmArgs {
  const uint16_t* A;        // [rows, lda] bf16 (this pass's rows)
  const float* inv_rms;     // [rows] or nullptr (rows already normalised)
  const uint16_t* gamma;    // [d] or nullptr
  const uint16_t* W;        // [V, d] bf16
  const int32_t* target;    // [rows] or nullptr
  const float* bias;        // [tiles * BM] fp32 (zero padded beyond V) or nullptr: the b of Eq. 1
  float4* stats;            // [rows, splits]     (m, S, T, z_target)
  uint2* top;               // [rows, splits, k]  (logit bits, id), sorted
  int64_t lda;              // row stride of A in elements
  int rows, d, V, k, splits, tiles, row_blocks;
  // steering sweep only (Sec. 3.4, Eq. 3 for several alpha in one pass):
  const float* au;          // [n_alpha, au_stride] fp32: alpha_a * (W_U v)[id], zero padded to whole tiles
  float4* sweep_stats;      // [rows, splits, n_alpha]  (m, S, T, bits of the arg max id)
  float* sweep_ztgt;        // [rows, splits]           logit of the target id at alpha = 0
  uint2* sweep_top;         // [rows, splits, n_alpha, SWEEP_KS] (logit bits, id), sorted: the sweep with top-k lists
  int au_stride, n_alpha;
  // sharing top-k thresholds between the vocabulary splits of a row (nullptr: off)
  unsigned* bound;          // [rows] lower bounds on each row's k-th best logit, as ordered keys; zero at launch
};

// ---------------------------------------------------------------------------------------
// Epilogue shared by both GEMM kernels.  State of one lens row, private to the lane that owns it.
// With m the running maximum: S = sum exp(z - m), T = sum exp(z - m) z.  Then
// logsumexp = m + log S and entropy = m + log S - T / S.
// The row's best KR logits (KR >= k) sit in registers, sorted: descending logit, and among equal
// logits ascending id.  A workgroup meets its vocabulary ids in increasing order, so a new
// candidate never outranks an equal logit already listed and a strict comparison is exact.
// ---------------------------------------------------------------------------------------
// Floats as unsigned keys of the same order, so that an integer atomic max is a float max.  Key 0
// is below every float's key: "nothing known yet".
__device__ __forceinline__ unsigned float_key(float f) {
  const unsigned b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(unsigned k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
constexpr unsigned KEY_NEG_INF = 0x007fffffu;   // float_key(-inf)

template <int KR>
struct RowState {
  float m = -INFINITY;
  float s = 0.f;
  float t = 0.f;
  float z_tgt = -INFINITY;  // logit of the target id, once its tile has passed
  int tgt = -1;             // target id of the row (-1: none)
  float shared_bound = -INFINITY;   // nothing at or below this can reach the row's final top k (see exchange_bound)
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
  // A candidate has to beat both the row's own KR-th best and what the other splits report.
  __device__ __forceinline__ float threshold() const { return fmaxf(lv[KR - 1], shared_bound); }
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

// Bit o of the result: x[o] > tau0.  Two instructions per entry: the comparison, then the mask
// doubled plus the comparison's result as carry-in (entries taken from 31 down to 0).  Four
// entries at a time, comparisons first: a VALU result in an SGPR must not be read by the next two
// VALU instructions on this hardware.
__device__ __forceinline__ unsigned candidate_mask(const float (&x)[32], float tau0) {
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
  return mask;
}

// Processes vocabulary entries [v0 + 32 I, v0 + 32 I + 32) of the finished tile for the lane's row.
template <int I, int KR, bool BIAS, class ACC>
__device__ __forceinline__ void epilogue_group(const ACC& acc, RowState<KR>& st, int v0, int V, bool partial,
                                               const float* __restrict__ bias) {
  float x[32];
  load_group<I>(acc, x);
  const int g0 = v0 + 32 * I;
  if (BIAS) {
    // The b of Eq. 1: the same 32 values for every lane, from a copy of the bias that is padded
    // to whole tiles.  Wave-uniform addresses through the constant address space: scalar loads,
    // which do not count against the vector-memory counter the operand rings are waited on.
    const_f32_ptr b = (const_f32_ptr)(uintptr_t)(bias + g0);
#pragma unroll
    for (int o = 0; o < 32; ++o) x[o] += b[o];
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

  // a6: streaming top-k.  Only the lanes with a logit above their current KR-th best take part
  // (a divergent branch: the other lanes are masked off and cost no energy, which is what counts
  // on a power-limited chip): mark the candidates against that threshold, then insert them in
  // id order.
  if (gmax > st.threshold()) {
    const float tau0 = st.threshold();
    unsigned mask = candidate_mask(x, tau0);
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

// The workgroups that sweep other parts of the vocabulary for the same rows tell each other how
// good a logit has to be.  A split's k-th best logit so far is a lower bound on the row's k-th best
// overall, and nothing below the largest such bound can be in the final top k; without it every
// split collects candidates against its own slowly rising threshold (k (1 + ln(n/k)) insertions per
// row for n vocabulary entries: eight short streams cost far more than one long one).  After each
// tile a lane picks up the row's shared bound and publishes its own (atomic max on the key).  A
// logit EQUAL to the bound may still belong in the top k (a smaller id wins a tie), so the
// threshold is the next float below it.  The final result does not depend on timing: a bound only
// removes entries that cannot be in the final top k; a split's own list may end up with fewer
// than k real entries, which the merge treats as absent.
// Placed at the END of the tile's epilogue: the operand loads in flight were sent before the
// epilogue began and have landed, so the wait for this one load costs one trip to the L2 and no
// more.  The publish needs no answer and is never waited for.
template <int KR>
__device__ __forceinline__ void exchange_bound(RowState<KR>& st, const GemmArgs& p, int my_row) {
  if (p.bound == nullptr) return;
  unsigned* const b = p.bound + min(my_row, p.rows - 1);
  asm volatile("" ::: "memory");
  const unsigned fresh = __hip_atomic_load(b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  st.shared_bound = fresh > KEY_NEG_INF ? key_float(fresh - 1u) : -INFINITY;
  // own bound: the k-th best of this split's list (k <= KR, KR - k < 12)
  // (each entry goes through an empty asm statement: a plain chain of selects on k the optimiser
  // folds into an indexed access and moves the whole list to scratch memory)
  float mine = st.lv[KR - 1];
#pragma unroll
  for (int j = KR - 2; j >= 0 && j >= KR - 12; --j) {
    float entry = st.lv[j];
    asm volatile("" : "+v"(entry));
    mine = (p.k - 1 == j) ? entry : mine;
  }
  if (my_row < p.rows && mine > st.shared_bound) __hip_atomic_fetch_max(b, float_key(mine), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("" ::: "memory");
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
template <int KR, bool BIAS = false>
struct TopKEpilogue {   // a5..a7: softmax statistics, k best logits, target logit (BIAS: Eq. 1's b added to every logit first)
  using State = RowState<KR>;
  static __device__ __forceinline__ void init(State& st, const GemmArgs& p, int my_row) {
    st.init();
    st.tgt = (p.target != nullptr && my_row < p.rows) ? p.target[my_row] : -1;
  }
  template <class ACC>
  static __device__ __forceinline__ void tile(const ACC& acc, State& st, int v0, const GemmArgs& p, int my_row) {
    epilogue_tile<KR, BIAS, ACC>(acc, st, v0, p.V, p.bias);
    // (the longest list together with a bias leaves no register for the exchange: that one kernel goes without)
    if (!(KR == 32 && BIAS)) exchange_bound(st, p, my_row);
  }
  static __device__ __forceinline__ void store(const GemmArgs& p, const State& st, int my_row, int split) {
    epilogue_store(p, st, my_row, split);
  }
};

// Workgroup ids are dealt round-robin over the 8 XCDs; remap so that one XCD (one L2) gets a
// compact rectangle of (row blocks) x (all splits) and its CUs share A panels and W tiles.
__device__ __forceinline__ int xcd_logical_block() {
  const int per_xcd = gridDim.x / NUM_XCD;
  return (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
}

}  // namespace
