// Cross-attention keys/values of the condition memory for every transformer block in one launch:
// K_mem = W_k c, V_mem = W_v c (the condition c enters every block through cross-attention, Sec. 3.1).
// This is the one dense, MFMA-bound contraction of the path (M = mem_len rows, N = 2 d_model, K = d_model
// per block), so it is a classic LDS-tiled GEMM: 256 x 256 output tile per workgroup, 128 x 128 per wave
// (16 accumulators of 32x32), K walked 64 at a time through a two-buffer LDS ring, global loads one stage ahead.
//
// Both operands are already in MFMA fragment order in global memory ([rows/16][K/32][64 lanes][8 halves]:
// the weights from load time, the memory from k_tile_weight), so a fragment is one contiguous 1 KiB burst
// from HBM to registers to LDS to registers.  The epilogue writes straight into the blocked cache layouts:
// the V tile is computed as c W_v^T (a lane owns one dim and four consecutive keys = one 8-byte store), the
// K tile as W_k c^T (a lane owns one key and four consecutive dims = one 8-byte store).
#pragma once
#include "fm_kernels_mfma.h"

struct PrefillLayer {
  const f16_t* W;   // [2d/16][d/32][64][8]: rows 0..d-1 = W_k, d..2d-1 = W_v
  f16_t* Km;        // blocked key cache of the condition memory (all sequences)
  f16_t* Vm;
};

typedef unsigned pf_u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_prefill_kv(const f16_t* __restrict__ Xt, const PrefillLayer* __restrict__ layers,
                                                    long seq_off, int KT, int d, int capb) {
  extern __shared__ pf_u32x4 pf_smem[];   // [2 buffers][2 K-steps][X: 16 fragments x 64 lanes | W: 16 fragments x 64 lanes]
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.x * 256, n0 = blockIdx.y * 256;
  const PrefillLayer L = layers[blockIdx.z];
  const bool is_v = n0 >= d;
  // Pointers read from the table are generic to the compiler; as FLAT accesses they would count against the LDS
  // counter and every wait for an LDS read would also wait for HBM.  Say that they are global.
  typedef const __attribute__((address_space(1))) pf_u32x4* gptr_t;
  gptr_t Xg = (gptr_t)(reinterpret_cast<const pf_u32x4*>(Xt) + (long)(m0 / 16) * KT * 64 + lane);
  gptr_t Wg = (gptr_t)(reinterpret_cast<const pf_u32x4*>(L.W) + (long)(n0 / 16) * KT * 64 + lane);

  // 4 x 4 tiles of 32 x 32 per wave (v_mfma_f32_32x32x16_f16: one wave per SIMD keeps the matrix pipe full with
  // this shape, which it does not with back-to-back 16x16x32 issues: measured 1.85 against 1.26 PFLOP/s)
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++)
#pragma unroll
      for (int j = 0; j < 16; j++) acc[a][b][j] = 0.f;

  // One pipeline stage = two K-steps of 32 (64 KiB of LDS: X and W fragments of both).  The registers `rx`, `rw`
  // carry the stage after the one in LDS: they are written to the other LDS buffer right after the barrier and
  // refilled from global memory at once, so a load has a whole compute phase (128 MFMAs per wave) to land.
  pf_u32x4 rx[8], rw[8];     // this thread's share: fragments wave, wave+4, wave+8, wave+12 of both K-steps
#define PF_GLOAD(S)                                                             \
  _Pragma("unroll") for (int j = 0; j < 8; j++) {                               \
    const long f = (long)(wave + 4 * (j & 3)) * KT + 2 * (S) + (j >> 2);        \
    rx[j] = Xg[f * 64];                                                         \
    rw[j] = Wg[f * 64];                                                         \
  }
#define PF_SWRITE(ST)                                                           \
  _Pragma("unroll") for (int j = 0; j < 8; j++) {                               \
    pf_smem[(ST) * 4096 + (j >> 2) * 2048 + (wave + 4 * (j & 3)) * 64 + lane] = rx[j];        \
    pf_smem[(ST) * 4096 + (j >> 2) * 2048 + 1024 + (wave + 4 * (j & 3)) * 64 + lane] = rw[j]; \
  }
  // P = the operand whose rows become the rows of the MFMA result, Q = the one whose rows become its columns
  const int pbase = is_v ? wm * 512 : 1024 + wn * 512;
  const int qbase = is_v ? 1024 + wn * 512 : wm * 512;
  // A 32-row x 16-k operand of the 32x32x16 MFMA (lane l: row l%32, k (l/32)*8..+8) is gathered from two of the
  // stored 16-row x 32-k fragments: half h of the K-step, row group (l%32)/16 -> stored lane (2h + l/32)*16 + l%16.
  const int lrow = ((lane & 31) >> 4) * 64 + (lane >> 5) * 16 + (lane & 15);
#define PF_COMPUTE(ST)                                                          \
  _Pragma("unroll") for (int ks = 0; ks < 2; ks++) {                            \
    _Pragma("unroll") for (int h = 0; h < 2; h++) {                             \
      f16x8 pf[4], qf[4];                                                       \
      _Pragma("unroll") for (int a = 0; a < 4; a++)                             \
        pf[a] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 4096 + ks * 2048 + pbase + a * 128 + h * 32 + lrow]); \
      _Pragma("unroll") for (int b = 0; b < 4; b++)                             \
        qf[b] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 4096 + ks * 2048 + qbase + b * 128 + h * 32 + lrow]); \
      _Pragma("unroll") for (int a = 0; a < 4; a++)                             \
        _Pragma("unroll") for (int b = 0; b < 4; b++)                           \
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(pf[a], qf[b], acc[a][b], 0, 0, 0); \
    }                                                                           \
  }

  const int NS = KT >> 1;      // KT is a multiple of 8
  PF_GLOAD(0);
  PF_SWRITE(0);
  PF_GLOAD(1);
  for (int s = 0; s < NS; s += 2) {
    __syncthreads();           // everyone is done with LDS buffer 1; buffer 0 (stage s) is complete
    PF_SWRITE(1);              // stage s+1 (NS is even)
    if (s + 2 < NS) { PF_GLOAD(s + 2); }
    PF_COMPUTE(0);
    __syncthreads();
    if (s + 2 < NS) {
      PF_SWRITE(0);
      if (s + 3 < NS) { PF_GLOAD(s + 3); }
    }
    PF_COMPUTE(1);
  }
#undef PF_GLOAD
#undef PF_SWRITE
#undef PF_COMPUTE

  // epilogue: halves into the blocked cache layouts.  Result tile (a, b): lane l owns column l%32 (a row of Q) and
  // the P rows (j/4)*8 + (l/32)*4 + j%4, j = 0..15, i.e. four runs of four consecutive rows.
  const int hl4 = (lane >> 5) * 4, c32 = lane & 31;
  typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
  typedef _Float16 f16x8o __attribute__((ext_vector_type(8)));
#pragma unroll
  for (int a = 0; a < 4; a++) {
#pragma unroll
    for (int b = 0; b < 4; b++) {
      if (is_v) {
        // keys r..r+3 and r+16..r+19 of a block sit next to each other in the V layout: runs j/4 = q and q+2
        const int e = n0 - d + wn * 128 + b * 32 + c32;               // dim within the V projection
        f16_t* base = L.Vm + seq_off + (long)(e >> 6) * capb * 2048;
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const int key0 = m0 + wm * 128 + a * 32 + q * 8 + hl4;
          f16x8o o;
#pragma unroll
          for (int i = 0; i < 4; i++) { o[i] = (f16_t)acc[a][b][q * 4 + i]; o[4 + i] = (f16_t)acc[a][b][(q + 2) * 4 + i]; }
          *(__attribute__((address_space(1))) f16x8o*)(base + vblk_off(key0, e & 63)) = o;
        }
      } else {
        const int key = m0 + wm * 128 + b * 32 + c32;
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int e0 = n0 + wn * 128 + a * 32 + q * 8 + hl4;        // dims e0 .. e0+3 of the K projection
          f16x4 o;
#pragma unroll
          for (int i = 0; i < 4; i++) o[i] = (f16_t)acc[a][b][q * 4 + i];
          *(__attribute__((address_space(1))) f16x4*)(L.Km + seq_off + (long)(e0 >> 6) * capb * 2048 + kblk_off(key, e0 & 63)) = o;
        }
      }
    }
  }
}
