// Cross-attention keys/values of the condition memory for every transformer block in one launch:
// K_mem = W_k c, V_mem = W_v c (the condition c enters every block through cross-attention, Sec. 3.1).
// This is the one dense, MFMA-bound contraction of the path (M = mem_len rows, N = 2 d_model, K = d_model
// per block), so it is a classic LDS-tiled GEMM: 256 x 128 output tile per workgroup, 128 x 64 per wave
// (8 accumulators of 32x32), K walked 32 at a time through a two-buffer LDS ring, global loads one step ahead,
// two workgroups per CU.
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

__global__ __launch_bounds__(256, 2) void k_prefill_kv(const f16_t* __restrict__ Xt, const PrefillLayer* __restrict__ layers,
                                                       long seq_off, int KT, int d, int M, int n_layers) {
  // [2 buffers][A: 16 fragments x 64 lanes | B: 8 fragments x 64 lanes], one K-step of 32 each (24 KiB)
  __shared__ pf_u32x4 pf_smem[2 * 1536];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_layer = (M >> 8) * (d >> 7) + (d >> 8) * (M >> 7);
  // lrow: see PF_COMPUTE below
  const int lrow = ((lane & 31) >> 4) * 64 + (lane >> 5) * 16 + (lane & 15);
  const int xbase = wm * 512 + lrow, wbase = 1024 + wn * 256 + lrow;
  // A workgroup walks over tiles (two workgroups per CU are launched): the result stores of one tile are only
  // issued, not waited for, so they drain while the next tile is multiplied.
  for (int tile = blockIdx.x; tile < tiles_layer * n_layers; tile += gridDim.x) {
  const PrefillLayer L = layers[tile / tiles_layer];
  const int tl = tile % tiles_layer;
  // The result tile of a workgroup is 256 rows of operand A by 128 rows of operand B.  V tiles are c W_v^T
  // (A = memory rows = keys, B = W_v rows = dims), K tiles are W_k c^T (A = W_k rows = dims, B = keys): the
  // two kinds differ only in where A and B come from and in the epilogue.
  const int tiles_v = (M >> 8) * (d >> 7);
  const bool is_v = tl < tiles_v;
  int a0, b0;                                   // first row of the A / B operand of this tile
  // Pointers read from the table are generic to the compiler; as FLAT accesses they would count against the LDS
  // counter and every wait for an LDS read would also wait for HBM.  Say that they are global.
  typedef const __attribute__((address_space(1))) pf_u32x4* gptr_t;
  gptr_t Ag, Bg;
  if (is_v) {
    const int t = tl;
    a0 = (t % (M >> 8)) * 256;
    b0 = (t / (M >> 8)) * 128;
    Ag = (gptr_t)(reinterpret_cast<const pf_u32x4*>(Xt) + (long)(a0 / 16) * KT * 64 + lane);
    Bg = (gptr_t)(reinterpret_cast<const pf_u32x4*>(L.W) + (long)((d + b0) / 16) * KT * 64 + lane);
  } else {
    const int t = tl - tiles_v;
    a0 = (t % (d >> 8)) * 256;
    b0 = (t / (d >> 8)) * 128;
    Ag = (gptr_t)(reinterpret_cast<const pf_u32x4*>(L.W) + (long)(a0 / 16) * KT * 64 + lane);
    Bg = (gptr_t)(reinterpret_cast<const pf_u32x4*>(Xt) + (long)(b0 / 16) * KT * 64 + lane);
  }
  const int capb = M >> 5;

  // Per wave 128 rows of A by 64 rows of B: 4 x 2 tiles of 32 x 32 (v_mfma_f32_32x32x16_f16), 128 accumulator
  // registers, so that two workgroups share a CU: one multiplies while the other waits at a barrier, for LDS or
  // for its result stores (with one workgroup per CU all of them store at the same time and the matrix pipes idle).
  f32x16 acc[4][2];
#pragma unroll
  for (int x = 0; x < 4; x++)
#pragma unroll
    for (int w = 0; w < 2; w++)
#pragma unroll
      for (int j = 0; j < 16; j++) acc[x][w][j] = 0.f;

  // The registers carry the K-step after the one in LDS: written to the other LDS buffer right after the
  // barrier and refilled from global memory at once.  This thread's share: X fragments wave, +4, +8, +12 and
  // W fragments wave, +4.
  pf_u32x4 rx[4], rw[2];
#define PF_GLOAD(KTI)                                                           \
  {                                                                             \
    _Pragma("unroll") for (int j = 0; j < 4; j++) rx[j] = Ag[((long)(wave + 4 * j) * KT + (KTI)) * 64]; \
    _Pragma("unroll") for (int j = 0; j < 2; j++) rw[j] = Bg[((long)(wave + 4 * j) * KT + (KTI)) * 64]; \
  }
#define PF_SWRITE(ST)                                                           \
  {                                                                             \
    _Pragma("unroll") for (int j = 0; j < 4; j++) pf_smem[(ST) * 1536 + (wave + 4 * j) * 64 + lane] = rx[j];        \
    _Pragma("unroll") for (int j = 0; j < 2; j++) pf_smem[(ST) * 1536 + 1024 + (wave + 4 * j) * 64 + lane] = rw[j]; \
  }
  // A 32-row x 16-k operand of the 32x32x16 MFMA (lane l: row l%32, k (l/32)*8..+8) is gathered from two of the
  // stored 16-row x 32-k fragments: half h of the K-step, row group (l%32)/16 -> stored lane (2h + l/32)*16 + l%16.
#define PF_COMPUTE(ST)                                                          \
  _Pragma("unroll") for (int h = 0; h < 2; h++) {                               \
    f16x8 xf[4], wf[2];                                                         \
    _Pragma("unroll") for (int x = 0; x < 4; x++)                               \
      xf[x] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 1536 + xbase + x * 128 + h * 32]); \
    _Pragma("unroll") for (int w = 0; w < 2; w++)                               \
      wf[w] = __builtin_bit_cast(f16x8, pf_smem[(ST) * 1536 + wbase + w * 128 + h * 32]); \
    _Pragma("unroll") for (int x = 0; x < 4; x++)                               \
      _Pragma("unroll") for (int w = 0; w < 2; w++)                             \
        acc[x][w] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf[x], wf[w], acc[x][w], 0, 0, 0); \
  }

  PF_GLOAD(0);
  PF_SWRITE(0);
  PF_GLOAD(1);
  for (int kt = 0; kt < KT; kt += 2) {     // KT is a multiple of 8
    __syncthreads();           // everyone is done with LDS buffer 1; buffer 0 (step kt) is complete
    PF_SWRITE(1);              // step kt+1
    if (kt + 2 < KT) { PF_GLOAD(kt + 2); }
    PF_COMPUTE(0);
    __syncthreads();
    if (kt + 2 < KT) {
      PF_SWRITE(0);
      if (kt + 3 < KT) { PF_GLOAD(kt + 3); }
    }
    PF_COMPUTE(1);
  }
#undef PF_GLOAD
#undef PF_SWRITE
#undef PF_COMPUTE

  // epilogue: halves into the blocked cache layouts.  In a result tile lane l owns column l%32 (a row of B) and
  // the A rows (j/4)*8 + (l/32)*4 + j%4, j = 0..15, i.e. four runs of four consecutive rows.
  const int hl4 = (lane >> 5) * 4, c32 = lane & 31;
  typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
  typedef _Float16 f16x8o __attribute__((ext_vector_type(8)));
#pragma unroll
  for (int x = 0; x < 4; x++) {
#pragma unroll
    for (int w = 0; w < 2; w++) {
      const int col = b0 + wn * 64 + w * 32 + c32;
      const int row0 = a0 + wm * 128 + x * 32 + hl4;
      if (is_v) {
        // rows = keys, column = dim.  Keys r..r+3 and r+16..r+19 of a block sit next to each other in the V
        // layout: runs j/4 = q and q+2 make one 16-byte store
        f16_t* base = L.Vm + seq_off + (long)(col >> 6) * capb * 2048;
#pragma unroll
        for (int q = 0; q < 2; q++) {
          f16x8o o;
#pragma unroll
          for (int i = 0; i < 4; i++) { o[i] = (f16_t)acc[x][w][q * 4 + i]; o[4 + i] = (f16_t)acc[x][w][(q + 2) * 4 + i]; }
          *(__attribute__((address_space(1))) f16x8o*)(base + vblk_off(row0 + q * 8, col & 63)) = o;
        }
      } else {
        // rows = dims (four consecutive ones = one 8-byte store), column = key
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int e0 = row0 + q * 8;
          f16x4 o;
#pragma unroll
          for (int i = 0; i < 4; i++) o[i] = (f16_t)acc[x][w][q * 4 + i];
          *(__attribute__((address_space(1))) f16x4*)(L.Km + seq_off + (long)(e0 >> 6) * capb * 2048 + kblk_off(col, e0 & 63)) = o;
        }
      }
    }
  }
  }   // tile loop
}

// ------------------------------------------------------------------------------------------
// Probes of what this chip sustains, to put next to the published peaks: a streaming read, a streaming copy and
// a register-only MFMA loop (32x32x16 f16, 8 independent accumulators per wave, 4 waves per workgroup).
// ------------------------------------------------------------------------------------------
__global__ void k_probe_read(const float4* __restrict__ src, float* __restrict__ sink, long n) {
  float s = 0.f;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const float4 v = src[i];
    s += v.x + v.y + v.z + v.w;
  }
  if (s == 1.2345e30f) sink[0] = s;    // keeps the loads alive; never true for the zero-filled buffer
}
__global__ void k_probe_copy(const float4* __restrict__ src, float4* __restrict__ dst, long n) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void k_probe_mfma(float* __restrict__ sink, int iters) {
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) acc[i][j] = 0.f;
  f16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; j++) { a[j] = (f16_t)(threadIdx.x * 0.001f + j); b[j] = (f16_t)(j * 0.5f - threadIdx.x * 0.002f); }
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 16; j++) s += acc[i][j];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// ------------------------------------------------------------------------------------------
// Probe of the hand-off that the single-launch verify kernel is made of: `nstage` dependent rounds in which every one
// of the resident workgroups publishes its slice of a vector of tagged 8-byte elements (agent-scope stores) and then
// reads the whole vector (16-byte agent-scope loads, repeated until every tag matches) - one all-to-all hand-off per
// round, with no arithmetic between the rounds.  mode 1: a ping-pong between workgroups 0 and 1 instead (one element
// each way per round).  Every wait is bounded; *abort_word != 0 afterwards means a wait expired.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_probe_exchange(unsigned long long* buf, unsigned* arrive, unsigned* abort_word,
                                                        unsigned long long* ticks, int vol, int nstage, int mode) {
  typedef unsigned long long u64;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const int nwg = gridDim.x;
  auto expired = [&](u64 t0) -> bool {
    if (__hip_atomic_load(abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return true;
    if (wall_clock64() - t0 > 20000000ull) { __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); return true; }
    return false;
  };
  // all workgroups resident before the clock starts
  if (threadIdx.x == 0) __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  {
    const u64 t0 = wall_clock64();
    while (true) {
      const unsigned n = __hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__syncthreads_and(n == (unsigned)nwg)) break;
      if (__syncthreads_or(expired(t0))) return;
    }
  }
  const u64 tstart = wall_clock64();
  const int per = vol / nwg, n16 = vol / 2;
  for (int t = 1; t <= nstage; t++) {
    u64* g = buf + (long)(t % 3) * vol;
    if (mode == 1) {
      if (blockIdx.x > 1) break;
      if (threadIdx.x == 0) {
        u64* mine = g + blockIdx.x * 64;
        u64* other = g + (1 - blockIdx.x) * 64;
        const u64 t0 = wall_clock64();
        if (blockIdx.x == 0) __hip_atomic_store(mine, (u64)t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while (__hip_atomic_load(other, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (u64)t) if (expired(t0)) return;
        if (blockIdx.x == 1) __hip_atomic_store(mine, (u64)t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      continue;
    }
    if ((int)threadIdx.x < per)
      __hip_atomic_store(g + blockIdx.x * per + threadIdx.x, ((u64)t << 32) | (unsigned)(blockIdx.x * per + threadIdx.x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const u64 t0 = wall_clock64();
    int it = 0;
    while (true) {
      u32x4 v[12];
#pragma unroll
      for (int j = 0; j < 12; j++)
        if (256 * j < n16) {        // uniform guard, clamped address (n16 <= 3072)
          const u64* p = g + 2 * (long)min((int)threadIdx.x + 256 * j, n16 - 1);
          asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v[j]) : "v"(p) : "memory");
        }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      bool ok = true;
#pragma unroll
      for (int j = 0; j < 12; j++)
        if (256 * j < n16) { asm volatile("" : "+v"(v[j])); ok = ok && v[j][1] == (unsigned)t && v[j][3] == (unsigned)t; }
      if (__syncthreads_and(ok)) break;
      if ((++it & 3) == 0 && __syncthreads_or(expired(t0))) return;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { ticks[0] = tstart; ticks[1] = wall_clock64(); }
}
