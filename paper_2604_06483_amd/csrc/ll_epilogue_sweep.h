// Epilogue policies of the steering sweep (Sec. 3.4, Eq. 3 read out for several alpha in one pass
// over W_U): the same GEMM kernels as the projection, with per-alpha row state.
#pragma once

#include "ll_epilogue.h"

namespace {

// ---------------------------------------------------------------------------------------
// Steering sweep (Sec. 3.4): the logits of h' = norm(h) + alpha v are z + alpha u with u = W_U v,
// so one pass over W_U serves every alpha: per alpha the lane keeps the softmax statistics and the
// arg max of z + alpha u.  alpha_a u comes as a table of fp32 per vocabulary id, read through the
// constant address space (wave-uniform addresses: scalar loads, one SGPR operand per add).
// ---------------------------------------------------------------------------------------
constexpr int SWEEP_MAX = LL_SWEEP_MAX;

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
  // The group's unshifted logits, fetched from the accumulators once; every alpha adds its table
  // entries on the fly, twice (for the maximum, then for the sums): an add costs a quarter of the
  // accumulator read and lane transpose it replaces, and a second array of 32 would not fit.
  float x[32];
  load_group<I>(acc, x);
  if (__builtin_amdgcn_ballot_w64((unsigned)tl < 32u) != 0) {
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (tl == o) st.z_tgt = x[o];
  }
  if (partial) {   // only the last tile of the vocabulary: a real branch (the empty asm keeps it one)
    asm volatile("");
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (g0 + o >= V) x[o] = NEG_BIG;   // (the table is zero there, and no alpha u comes near this magnitude)
  }
#pragma unroll
  for (int a = 0; a < SWEEP_MAX; ++a) {
    if (a < p.n_alpha) {
      const_f32_ptr au = (const_f32_ptr)(uintptr_t)(p.au + (int64_t)a * p.au_stride + g0);
      float gmax = x[0] + au[0];
#pragma unroll
      for (int o = 1; o < 32; ++o) gmax = fmaxf(gmax, x[o] + au[o]);
      if (gmax > st.m[a]) {
        // a new maximum for this lane: ids come in increasing order, so strictly greater is the
        // tie rule, and within the group the lowest position with that value wins
        int pos = 0;
#pragma unroll
        for (int o = 31; o >= 0; --o) pos = (x[o] + au[o] == gmax) ? o : pos;
        const float sc = __builtin_amdgcn_exp2f((st.m[a] - gmax) * LOG2E);   // first group: exp2(-inf) = 0
        st.s[a] *= sc;
        st.t[a] *= sc;
        st.m[a] = gmax;
        st.id[a] = g0 + pos;
      }
      const float mb = st.m[a] * LOG2E;
      float s4[4] = {0.f, 0.f, 0.f, 0.f}, t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int o = 0; o < 32; ++o) {
        const float y = x[o] + au[o];
        const float e = __builtin_amdgcn_exp2f(fmaf(y, LOG2E, -mb));
        s4[o & 3] += e;
        t4[o & 3] = fmaf(e, y, t4[o & 3]);
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
  static __device__ __forceinline__ void tile(const ACC& acc, State& st, int v0, const GemmArgs& p, int /*my_row*/) {
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

// ---------------------------------------------------------------------------------------
// The sweep with short top-k lists (the paper's figures list k = 3 tokens per cell): per alpha the
// lane keeps, next to (m, S, T), its SWEEP_KS best shifted logits and their ids, sorted.  The list
// replaces the single arg max of SweepEpilogue; candidates are found and picked as in the plain
// projection's epilogue and inserted with a few selects (the list is short).  Lists of four for
// nine alphas do not fit the register file next to the accumulators (the compiler reports 239
// spilled registers; 492 spill instructions even with lists of three), so one pass of this kernel
// serves at most SWEEP_TOPK_ALPHAS alphas and the host runs ceil(n_alpha / SWEEP_TOPK_ALPHAS)
// passes.  Five is the most that leaves both GEMM kernels without spills (six: 8 spilled registers
// on the register-staged one).
// ---------------------------------------------------------------------------------------
constexpr int SWEEP_KS = LL_SWEEP_KMAX;
constexpr int SWEEP_TOPK_ALPHAS = 5;

struct SweepTopKState {
  float m[SWEEP_TOPK_ALPHAS], s[SWEEP_TOPK_ALPHAS], t[SWEEP_TOPK_ALPHAS];
  float lv[SWEEP_TOPK_ALPHAS][SWEEP_KS];
  int li[SWEEP_TOPK_ALPHAS][SWEEP_KS];
  float z_tgt = -INFINITY;
  int tgt = -1;
};

// Sorted insert into a short list (descending logit; ids arrive in increasing order, so a strict
// comparison keeps the smaller id first among equal logits).  Slots are visited from the bottom:
// each reads its still unchanged upper neighbour.
template <int KS>
__device__ __forceinline__ void short_insert(float (&lv)[KS], int (&li)[KS], float z, int id) {
#pragma unroll
  for (int j = KS - 1; j >= 1; --j) {
    const bool above_upper = z > lv[j - 1];
    const bool above_here = z > lv[j];
    li[j] = above_upper ? li[j - 1] : (above_here ? id : li[j]);
    lv[j] = above_upper ? lv[j - 1] : (above_here ? z : lv[j]);
  }
  if (z > lv[0]) {
    lv[0] = z;
    li[0] = id;
  }
}

template <int I, class ACC>
__device__ __forceinline__ void sweep_topk_group(const ACC& acc, SweepTopKState& st, int v0, int V, bool partial,
                                                 const GemmArgs& p) {
  const int g0 = v0 + 32 * I;
  const int tl = st.tgt - g0;
  float x[32];   // the group's unshifted logits, fetched once (see sweep_group)
  load_group<I>(acc, x);
  if (__builtin_amdgcn_ballot_w64((unsigned)tl < 32u) != 0) {
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (tl == o) st.z_tgt = x[o];
  }
  if (partial) {   // only the last tile of the vocabulary: a real branch (the empty asm keeps it one)
    asm volatile("");
#pragma unroll
    for (int o = 0; o < 32; ++o)
      if (g0 + o >= V) x[o] = NEG_BIG;
  }
#pragma unroll
  for (int a = 0; a < SWEEP_TOPK_ALPHAS; ++a) {
    if (a < p.n_alpha) {
      const_f32_ptr au = (const_f32_ptr)(uintptr_t)(p.au + (int64_t)a * p.au_stride + g0);
      float gmax = x[0] + au[0];
#pragma unroll
      for (int o = 1; o < 32; ++o) gmax = fmaxf(gmax, x[o] + au[o]);
      if (gmax > st.m[a]) {
        const float sc = __builtin_amdgcn_exp2f((st.m[a] - gmax) * LOG2E);   // first group: exp2(-inf) = 0
        st.s[a] *= sc;
        st.t[a] *= sc;
        st.m[a] = gmax;
      }
      const float mb = st.m[a] * LOG2E;
      float s4[4] = {0.f, 0.f, 0.f, 0.f}, t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int o = 0; o < 32; ++o) {
        const float y = x[o] + au[o];
        const float e = __builtin_amdgcn_exp2f(fmaf(y, LOG2E, -mb));
        s4[o & 3] += e;
        t4[o & 3] = fmaf(e, y, t4[o & 3]);
      }
      st.s[a] += (s4[0] + s4[1]) + (s4[2] + s4[3]);
      st.t[a] += (t4[0] + t4[1]) + (t4[2] + t4[3]);
      if (gmax > st.lv[a][SWEEP_KS - 1]) {
        float y[32];   // the shifted copy exists only here, for the lanes that have a candidate
#pragma unroll
        for (int o = 0; o < 32; ++o) y[o] = x[o] + au[o];
        unsigned mask = candidate_mask(y, st.lv[a][SWEEP_KS - 1]);
        if (partial) mask &= (g0 + 32 <= V) ? 0xffffffffu : (g0 >= V ? 0u : (1u << (V - g0)) - 1u);
        while (mask != 0) {
          const int o = __builtin_ctz(mask);
          mask &= mask - 1;
          short_insert<SWEEP_KS>(st.lv[a], st.li[a], select32(y, o), g0 + o);
        }
      }
      // one alpha at a time (see sweep_group)
      asm volatile("" : "+v"(st.s[a]), "+v"(st.t[a]));
    }
  }
}

struct SweepTopKEpilogue {
  using State = SweepTopKState;
  static __device__ __forceinline__ void init(State& st, const GemmArgs& p, int my_row) {
#pragma unroll
    for (int a = 0; a < SWEEP_TOPK_ALPHAS; ++a) {
      st.m[a] = -INFINITY;
      st.s[a] = 0.f;
      st.t[a] = 0.f;
#pragma unroll
      for (int j = 0; j < SWEEP_KS; ++j) {
        st.lv[a][j] = -INFINITY;
        st.li[a][j] = INT_MAX;
      }
    }
    st.tgt = (p.target != nullptr && my_row < p.rows) ? p.target[my_row] : -1;
  }
  template <class ACC>
  static __device__ __forceinline__ void tile(const ACC& acc, State& st, int v0, const GemmArgs& p, int /*my_row*/) {
    const bool partial = v0 + BM > p.V;
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // as in epilogue_tile: let the last MFMA drain
    sweep_topk_group<0, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<1, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<2, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<3, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<4, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<5, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<6, ACC>(acc, st, v0, p.V, partial, p);
    sweep_topk_group<7, ACC>(acc, st, v0, p.V, partial, p);
  }
  static __device__ __forceinline__ void store(const GemmArgs& p, const State& st, int my_row, int split) {
    if (my_row >= p.rows) return;
    const int64_t o = (int64_t)my_row * p.splits + split;
    p.sweep_ztgt[o] = st.z_tgt;
#pragma unroll
    for (int a = 0; a < SWEEP_TOPK_ALPHAS; ++a)
      if (a < p.n_alpha) {
        p.sweep_stats[o * p.n_alpha + a] = make_float4(st.m[a], st.s[a], st.t[a], 0.f);
#pragma unroll
        for (int j = 0; j < SWEEP_KS; ++j)
          p.sweep_top[(o * p.n_alpha + a) * SWEEP_KS + j] = make_uint2(__float_as_uint(st.lv[a][j]), (unsigned)st.li[a][j]);
      }
  }
};

}  // namespace
