// Cross-attention keys/values of the condition memory for every transformer block in one launch:
// K_mem = W_k c, V_mem = W_v c (the condition c enters every block through cross-attention, Sec. 3.1).
// This is the one dense, MFMA-bound contraction of the path (M = mem_len rows, N = 2 d_model, K = d_model
// per block), so it is a classic LDS-tiled GEMM: 256 x 256 output tile per workgroup, 128 x 128 per wave
// (64 accumulators of 16x16), K walked 32 at a time through a two-stage LDS ring, global loads two steps ahead.
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

__global__ __launch_bounds__(256) void k_prefill_kv(const f16_t* __restrict__ Xt, const PrefillLayer* __restrict__ layers,
                                                    long seq_off, int KT, int d, int capb) {
  extern __shared__ pf_u32x4 pf_smem[];   // [2 stages][X: 16 fragments x 64 lanes | W: 16 fragments x 64 lanes]
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.x * 256, n0 = blockIdx.y * 256;
  const PrefillLayer L = layers[blockIdx.z];
  const bool is_v = n0 >= d;
  const pf_u32x4* Xg = reinterpret_cast<const pf_u32x4*>(Xt) + (long)(m0 / 16) * KT * 64 + lane;
  const pf_u32x4* Wg = reinterpret_cast<const pf_u32x4*>(L.W) + (long)(n0 / 16) * KT * 64 + lane;

  f32x4 acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; a++)
#pragma unroll
    for (int b = 0; b < 8; b++) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // staging registers: two sets, each one K-step (this thread's share: fragments wave, wave+4, wave+8, wave+12)
  pf_u32x4 rx0[4], rw0[4], rx1[4], rw1[4];
#define PF_GLOAD(RX, RW, KTI)                                                   \
  _Pragma("unroll") for (int j = 0; j < 4; j++) {                               \
    const long f = (long)(wave + 4 * j) * KT + (KTI);                           \
    RX[j] = Xg[f * 64];                                                         \
    RW[j] = Wg[f * 64];                                                         \
  }
#define PF_SWRITE(RX, RW, ST)                                                   \
  _Pragma("unroll") for (int j = 0; j < 4; j++) {                               \
    pf_smem[(ST) * 2048 + (wave + 4 * j) * 64 + lane] = RX[j];                  \
    pf_smem[(ST) * 2048 + 1024 + (wave + 4 * j) * 64 + lane] = RW[j];           \
  }
  // P = the operand whose rows become the rows of the MFMA result, Q = the one whose rows become its columns
  const int pbase = is_v ? wm * 512 : 1024 + wn * 512;
  const int qbase = is_v ? 1024 + wn * 512 : wm * 512;
#define PF_COMPUTE(ST)                                                          \
  {                                                                             \
    f16x8 pf[8], qf[8];                                                         \
    _Pragma("unroll") for (int a = 0; a < 8; a++)                               \
      pf[a] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 2048 + pbase + a * 64 + lane]); \
    _Pragma("unroll") for (int b = 0; b < 8; b++)                               \
      qf[b] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 2048 + qbase + b * 64 + lane]); \
    _Pragma("unroll") for (int a = 0; a < 8; a++)                               \
      _Pragma("unroll") for (int b = 0; b < 8; b++)                             \
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pf[a], qf[b], acc[a][b], 0, 0, 0); \
  }

  // prologue: step 0 into LDS stage 0, steps 1 and 2 in flight (KT is a multiple of 8)
  PF_GLOAD(rx0, rw0, 0);
  PF_GLOAD(rx1, rw1, 1);
  PF_SWRITE(rx0, rw0, 0);
  PF_GLOAD(rx0, rw0, 2);
  for (int kt = 0; kt < KT; kt += 2) {
    // even step: LDS stage 0 holds step kt; rx1 holds kt+1, rx0 holds kt+2
    __syncthreads();
    PF_SWRITE(rx1, rw1, 1);
    if (kt + 3 < KT) { PF_GLOAD(rx1, rw1, kt + 3); }
    PF_COMPUTE(0);
    // odd step: LDS stage 1 holds step kt+1; rx0 holds kt+2, rx1 holds kt+3
    __syncthreads();
    if (kt + 2 < KT) {
      PF_SWRITE(rx0, rw0, 0);
      if (kt + 4 < KT) { PF_GLOAD(rx0, rw0, kt + 4); }
    }
    PF_COMPUTE(1);
  }
#undef PF_GLOAD
#undef PF_SWRITE
#undef PF_COMPUTE

  // epilogue: halves, four at a time, into the blocked cache layouts
  const int g4 = (lane >> 4) * 4, c16 = lane & 15;
  typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int a = 0; a < 8; a++) {
#pragma unroll
    for (int b = 0; b < 8; b++) {
      f16x4 o;
#pragma unroll
      for (int i = 0; i < 4; i++) o[i] = (f16_t)acc[a][b][i];
      if (is_v) {
        const int key0 = m0 + wm * 128 + a * 16 + g4;                 // keys key0 .. key0+3
        const int e = n0 - d + wn * 128 + b * 16 + c16;               // dim within the V projection
        f16_t* dst = L.Vm + seq_off + (long)(e >> 6) * capb * 2048 + vblk_off(key0, e & 63);
        *reinterpret_cast<f16x4*>(dst) = o;
      } else {
        const int e0 = n0 + wn * 128 + a * 16 + g4;                   // dims e0 .. e0+3 of the K projection
        const int key = m0 + wm * 128 + b * 16 + c16;
        f16_t* dst = L.Km + seq_off + (long)(e0 >> 6) * capb * 2048 + kblk_off(key, e0 & 63);
        *reinterpret_cast<f16x4*>(dst) = o;
      }
    }
  }
}
