// Register-staged projection kernel (any d that is a multiple of 8; RMSNorm scaling fused into the
// A-tile load; the epilogue is a policy as in the direct-to-LDS kernel).
#pragma once

#include "ll_epilogue.h"

namespace {

// ---------------------------------------------------------------------------------------
// Register-staged kernel: any d that is a multiple of 8; operands go global -> registers -> LDS,
// with the RMSNorm scaling (a3) applied between the global load and the LDS store of every A tile.
// LDS tile: [256 rows][8 chunks of 16 B]; chunk index XOR-swizzled with (row/2)%8 so that both the
// 16-byte row-major stores and the MFMA fragment reads (32 consecutive rows, one chunk) spread
// over all banks.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int lds_off(int row, int chunk) { return (row * 8 + (chunk ^ ((row >> 1) & 7))) * 16; }

template <class EPI>
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
  typename EPI::State st;
  EPI::init(st, p, my_row);

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
    EPI::tile(acc, st, v0, p, my_row);
  }
  EPI::store(p, st, my_row, split);
}

}  // namespace
