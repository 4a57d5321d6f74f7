// Direct-to-LDS projection kernel (d a multiple of 64; operands by global_load_lds into LDS rings,
// v_mfma_f32_16x16x32_bf16): the kernel the benchmark times.
#pragma once

#include "ll_epilogue.h"

namespace {

// ---------------------------------------------------------------------------------------
// Direct-to-LDS kernel: both operands go from global memory straight into LDS (global_load_lds,
// 16 bytes per lane) in stages of K = 64, so that every load instruction takes whole 128-byte
// lines (8 rows x 128 B).  A must be a panel of already normalised bf16 rows with row stride
// lda, a multiple of 64, zero padded beyond d (ll_norm_panel_kernel writes it); W rows are read
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
// stage are read one stage early (32 registers), and both streams get about two stages between
// sending a load and needing its data, from the same 160 KB.
//
// Schedule of stage g, four slices of 32 MFMAs: slice S is vocabulary tiles 4 S .. 4 S + 3 in both
// K halves, the two MFMAs of an accumulator tile back to back (the second takes the first one's
// result as it leaves the pipe; 1 % on this kernel, 3.5 % on a bare MFMA loop); W fragments
// alternate between two register sets of eight (four tiles x two halves):
//   slice 0    : reads the W fragments of slice 1; sends the second half of W(g+2);
//   slices 1, 2: read the W fragments of the next slice (slice 2 has its last reads out five pairs
//                before the wait, so that they are back when slice 3 starts); send A(g+2), half each (into the slot of
//                A(g), whose fragments all went into registers during stage g-1);
//   wait + barrier: all loads but the last 16 (W(g+2), A(g+2)) have landed, so stage g+1 is in
//                LDS for everyone, and everyone holds its last fragments of W(g): that slot is free;
//   slice 3    : reads the W fragments of slice 0 of stage g+1 and, row tile by row tile as they
//                fall dead, all eight A fragments of stage g+1; sends the first half of W(g+3)
//                into the slot of W(g).
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
// The same with C = 0: the first K half of a vocabulary tile starts its accumulators this way, so
// that the 256 of them need no clearing between tiles.
__device__ __forceinline__ f32x4 mfma16_from_zero(bf16x8 a, bf16x8 b) {
  f32x4 c;
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(c) : "v"(a), "v"(b));
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
  int w_tile = tile0, w_kt = 0;
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
  const unsigned char* const a_end = a_base0 + (int64_t)KT * (DK * 2);   // one past the panel's last K stage
  auto advance_a = [&]() {   // (a handful of scalar instructions: a long run of them between two MFMAs idles the matrix pipe)
    a_lds = a_lds_flip - a_lds;
    a_base += DK * 2;
    if (a_base == a_end) a_base = a_base0;
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
  // A: the four row tiles of both K halves of the stage.  W: two sets of eight fragments, each the
  // four vocabulary tiles of a slice in both K halves (fragment 2 t + hk).
  bf16x8 fa[2][4], fw0[8], fw1[8];
#pragma unroll
  for (int hk = 0; hk < 2; ++hk)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      fa[hk][j] = *reinterpret_cast<const bf16x8*>(smem + W_SLOTS * SLOT_BYTES + a_wave_off + j * 16 * (DK * 2) + f_off[hk]);
#pragma unroll
  for (int q = 0; q < 8; ++q) fw0[q] = *reinterpret_cast<const bf16x8*>(smem + (q >> 1) * 16 * (DK * 2) + f_off[q & 1]);

  // A stage is four slices of 32 MFMAs; slice S is vocabulary tiles 4 S .. 4 S + 3 against the
  // four row tiles, BOTH K halves: the two MFMAs of an accumulator tile are issued back to back,
  // the second reading the first one's result.  On this power-limited chip that order is worth
  // 3.5 % on a bare MFMA loop over the same work with the halves apart (the accumulator goes from
  // one instruction to the next without a trip through the register file), and it does not stall.
  // A slice is 16 such pairs.  Slices 1 and 2 walk tile by tile (rows back and forth); slices 0
  // and 3 walk row tile by row tile, because slice 3 refills the A fragments for the next stage as
  // it goes: a row tile's two fragments are dead once its four pairs are done, and the next stage's
  // slice 0 needs them in the same order, 24 MFMAs later at the least.
  // An MFMA runs for 16 cycles, so a gap between two of them holds at most two or three other
  // instructions.  Behind a pair goes the LDS read of one W fragment of the next slice (into nw,
  // from the tile at LDS offset tW) where RD names one, and a load-to-LDS or a piece of the streams'
  // bookkeeping where HOOK names one; slice 3's A fragment reads go between the two MFMAs of a pair
  // (AIN).  The fences pin that order.
  // Which pairs read: slices 0, 1 and 3 spread their eight reads over the even pairs.  Slice 2
  // reads ahead (LL_RD_AHEAD: the last three reads pulled forward to pairs 9, 10, 11): its
  // fragments are the ones slice 3 needs ALL of within its first four pairs (it walks row tile by
  // row tile), right behind the wait and the barrier, and a read sent two pairs before the wait
  // has not come back by then; measured 0.4 to 1.9 % per launch over the spread placement.  (The
  // same move in slice 3, whose fragments the next stage's slice 0 needs as early, measured
  // nothing: that slice's gaps already hold the eight A fragment reads.)
#define LL_LDS_FRAG(ptr) (*reinterpret_cast<const bf16x8*>(ptr))
  // Written as an instruction so that the 64 accumulator tiles stay in AGPRs: given the builtin,
  // the register allocator keeps some of them in VGPRs and copies them in and out around the MFMA.
  // (Operands come from LDS reads, whose waits the compiler still places; nothing reads an
  // accumulator before the epilogue's own drain.)
#define LL_MFMA16(a, b, c) mfma16(a, b, c)
#define LL_MFMA16_Z(a, b, c) mfma16_from_zero(a, b)
  // pair P of a slice: vocabulary tile LL_T and row tile LL_J of the slice
#define LL_SNAKE(outer, inner) (((outer) & 1) ? 3 - (inner) : (inner))
#define LL_T(JO, P) ((JO) ? LL_SNAKE((P) / 4, (P) % 4) : (P) / 4)
#define LL_J(JO, P) ((JO) ? (P) / 4 : LL_SNAKE((P) / 4, (P) % 4))
#define LL_RD_SPREAD(P) ((P) % 2 == 0 ? (P) / 2 : -1)
#define LL_RD_AHEAD(P) ((P) <= 8 ? ((P) % 2 == 0 ? (P) / 2 : -1) : ((P) <= 11 ? (P) - 4 : -1))
#define LL_PAIR(MF0, P, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                 \
  acc[4 * S + LL_T(JO, P)][LL_J(JO, P)] =                                                                            \
      MF0(fw[2 * LL_T(JO, P)], fa[0][LL_J(JO, P)], acc[4 * S + LL_T(JO, P)][LL_J(JO, P)]);                           \
  AIN(P);                                                                                                            \
  LL_SCHED_FENCE();                                                                                                  \
  acc[4 * S + LL_T(JO, P)][LL_J(JO, P)] =                                                                            \
      LL_MFMA16(fw[2 * LL_T(JO, P) + 1], fa[1][LL_J(JO, P)], acc[4 * S + LL_T(JO, P)][LL_J(JO, P)]);                 \
  if (RD(P) >= 0) { /* fragment q = RD(P): vocabulary tile 4 NS + q / 2, K half q % 2 */                            \
    nw[RD(P) >= 0 ? RD(P) : 0] =                                                                                     \
        LL_LDS_FRAG(smem + tW + (4 * NS + (RD(P) >= 0 ? RD(P) : 0) / 2) * 16 * (DK * 2) + f_off[(RD(P) >= 0 ? RD(P) : 0) & 1]); \
  }                                                                                                                  \
  HOOK(P);                                                                                                           \
  AOUT(P);                                                                                                           \
  LL_SCHED_FENCE();
#define LL_SLICE(MF0, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                    \
  LL_SCHED_FENCE();                                                                                                  \
  LL_PAIR(MF0, 0, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 1, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 2, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 3, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 4, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 5, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 6, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 7, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 8, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 9, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                            \
  LL_PAIR(MF0, 10, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                           \
  LL_PAIR(MF0, 11, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                           \
  LL_PAIR(MF0, 12, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                           \
  LL_PAIR(MF0, 13, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                           \
  LL_PAIR(MF0, 14, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)                                                           \
  LL_PAIR(MF0, 15, S, JO, fw, nw, tW, NS, AIN, AOUT, HOOK, RD)

#define LL_A_NONE(P) (void)0
  // slice 3 (row tile P / 4 in pairs 4 j .. 4 j + 3): the K half 0 fragment of a row tile is dead
  // after the first MFMA of its last pair, the K half 1 fragment after the second; both are read
  // for the next stage from its A tile (the wavefront's own rows), at LDS offset nA
#define LL_AIN_S3(P)                                                                                   \
  if ((P) % 4 == 3) fa[0][(P) / 4] = LL_LDS_FRAG(smem + nA + ((P) / 4) * 16 * (DK * 2) + f_off[0]);    \
  if ((P) % 4 == 0 && (P) > 0) fa[1][((P) / 4 + 3) % 4] = LL_LDS_FRAG(smem + nA + (((P) / 4 + 3) % 4) * 16 * (DK * 2) + f_off[1])
#define LL_AOUT_S3(P)                                                                                  \
  if ((P) == 15) {                                                                                     \
    fa[1][3] = LL_LDS_FRAG(smem + nA + 3 * 16 * (DK * 2) + f_off[1]);                                  \
    nA = a_flip - nA;   /* LDS reads return in order: the tile read from just now is the wavefront's to refill */ \
  }
  // (hooks: what goes behind pair P of the slice, besides a fragment read)
#define LL_HOOK_S0(P)                                \
  if (P == 1) set_lds_dma_base(w_lds);               \
  if (P == 7) LL_DMA_W(4);                           \
  if (P == 9) LL_DMA_W(5);                           \
  if (P == 11) LL_DMA_W(6);                          \
  if (P == 13) LL_DMA_W(7);                          \
  if (P == 15) advance_w()
  // (the A fragments of this stage were all read in the previous stage's slice 3: the slot of A(g),
  // which A(g+2) goes into, has been the wavefront's own since then)
#define LL_HOOK_S1(P)                                \
  if (P == 7) set_lds_dma_base(a_lds);               \
  if (P == 9) LL_DMA_A(0);                           \
  if (P == 11) LL_DMA_A(1);                          \
  if (P == 13) LL_DMA_A(2);                          \
  if (P == 15) LL_DMA_A(3)
#define LL_HOOK_S2(P)   /* (pair 9 is left to the fragment reads that slice 2 pulls forward) */ \
  if (P == 5) LL_DMA_A(4);                           \
  if (P == 7) LL_DMA_A(5);                           \
  if (P == 11) LL_DMA_A(6);                          \
  if (P == 13) LL_DMA_A(7)
#define LL_HOOK_S3(P)   /* (the A stream moves on here, behind the barrier, not in the last gap before the wait) */ \
  if (P == 1) advance_a();                           \
  if (P == 7) set_lds_dma_base(w_lds);               \
  if (P == 9) LL_DMA_W(0);                           \
  if (P == 11) {                                     \
    LL_DMA_W(1);                                     \
    nnW = nW + SLOT_BYTES >= W_SLOTS * SLOT_BYTES ? 0 : nW + SLOT_BYTES;   \
    LL_PIN_S(nnW);                                   \
  }                                                  \
  if (P == 13) LL_DMA_W(2);                          \
  if (P == 15) {   /* every even pair of the slice reads a W fragment from nW: move on after the last */ \
    LL_DMA_W(3);                                     \
    cW = nW;                                         \
    nW = nnW;                                        \
  }

  // Consumer state: LDS byte offsets of the W tiles of this stage and of the next, and of the A
  // tile the next stage's fragments come from (it includes the wavefront's own 64 rows).
  int cW = 0, nW = SLOT_BYTES, nnW = 2 * SLOT_BYTES;
  int nA = (W_SLOTS + 1) * SLOT_BYTES + a_wave_off;
  const int a_flip = (2 * W_SLOTS + 1) * SLOT_BYTES + 2 * a_wave_off;   // slot 3 <-> slot 4
  for (int tile = tile0; tile < tile1; ++tile) {
    f32x4 acc[16][4];   // first written by the K half 0 MFMAs of stage 0, with C = 0
    // One stage; MF0 is the MFMA form of K half 0: from zero in a tile's first stage, accumulating after.
#define LL_STAGE(MF0)                                                                                  \
    LL_SLICE(MF0, 0, 1, fw0, fw1, cW, 1, LL_A_NONE, LL_A_NONE, LL_HOOK_S0, LL_RD_SPREAD)               \
    LL_SLICE(MF0, 1, 0, fw1, fw0, cW, 2, LL_A_NONE, LL_A_NONE, LL_HOOK_S1, LL_RD_SPREAD)               \
    LL_SLICE(MF0, 2, 0, fw0, fw1, cW, 3, LL_A_NONE, LL_A_NONE, LL_HOOK_S2, LL_RD_AHEAD)                \
    /* stage g+1 landed (W(g+2) and A(g+2) may still be out); all my reads of W(g) are done */         \
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * LOADS_PER_TILE, 0));                                    \
    __syncthreads();                                                                                   \
    LL_SLICE(MF0, 3, 1, fw1, fw0, nW, 0, LL_AIN_S3, LL_AOUT_S3, LL_HOOK_S3, LL_RD_SPREAD)
    LL_STAGE(LL_MFMA16_Z)
    for (int kt = 1; kt < KT; ++kt) {
      LL_STAGE(LL_MFMA16)
    }
#undef LL_STAGE
    EPI::tile(acc, st, tile * BM, p, my_row);
  }
#undef LL_PAIR
#undef LL_RD_SPREAD
#undef LL_RD_AHEAD
#undef LL_T
#undef LL_J
#undef LL_SNAKE
#undef LL_A_NONE
#undef LL_AIN_S3
#undef LL_AOUT_S3
#undef LL_SLICE
#undef LL_MFMA16_Z
#undef LL_MFMA16
#undef LL_LDS_FRAG
#undef LL_DMA_TILE
#undef LL_HOOK_S3
#undef LL_PIN_S
#undef LL_HOOK_S2
#undef LL_HOOK_S1
#undef LL_HOOK_S0
#undef LL_DMA_A
#undef LL_DMA_W
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));   // drain the ring before the LDS is given back
  EPI::store(p, st, my_row, split);
}

}  // namespace
