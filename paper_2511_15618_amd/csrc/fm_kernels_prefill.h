// Cross-attention keys/values of the condition memory for every transformer block in one launch:
// K_mem = W_k c, V_mem = W_v c (the condition c enters every block through cross-attention, Sec. 3.1).
// This is the one dense, MFMA-bound contraction of the path (M = mem_len rows, N = 2 d_model, K = d_model
// per block), so it is an LDS-tiled GEMM built for one workgroup of four waves per compute unit:
//   * 256 x 256 output tile per workgroup, 128 x 128 per wave (16 accumulators of 32x32 = all 256 accumulation
//     registers), so that an operand fragment read from LDS feeds four MFMAs;
//   * K walked 32 at a time through a ring of four 32 KiB LDS stages, filled by loads that go from global memory
//     straight into LDS (no trip through registers), two stages ahead of the one being multiplied;
//   * one barrier per stage; the LDS reads of the next half-stage are issued under the MFMAs of the current one;
//   * the stage stream runs on across tile boundaries, so the loads of the next tile are in flight while the results
//     of the last one are stored, and the stores are only issued, never waited for, until two stages later.
//
// Both operands are already in MFMA fragment order in global memory ([rows/16][K/32][64 lanes][8 halves]:
// the weights from load time, the memory from k_tile_weight), so a fragment is one contiguous 1 KiB burst
// from HBM to LDS.  The epilogue writes straight into the blocked cache layouts, 16 bytes per lane and store:
// the V tile is computed as c W_v^T (a lane owns one dim and 2 x 4 keys that are neighbours in the V layout), the
// K tile as W_k c^T (a lane owns one key and 4 consecutive dims; two lanes trade halves to own 8).
#pragma once
#include "fm_kernels_mfma.h"

struct PrefillLayer {
  const f16_t* W;   // [2d/16][d/32][64][8]: rows 0..d-1 = W_k, d..2d-1 = W_v
  f16_t* Km;        // blocked key cache of the condition memory (all sequences)
  f16_t* Vm;
};

typedef unsigned pf_u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define PF_STAGES 4
#define PF_STAGE_ELEMS 2048   // 16-byte elements per stage: 16 fragments of A, 16 of B
#define PF_LDS_BYTES (PF_STAGES * PF_STAGE_ELEMS * 16)
#define PF_STORES 32          // result stores per lane and tile
// s_waitcnt with only the vector-memory counter set (loads, direct-to-LDS loads and stores complete in issue order)
#define PF_WAIT_VM(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

// Launch: gridDim.x a multiple of 8 (one workgroup per compute unit), 256 threads, PF_LDS_BYTES of dynamic LDS.
// Needs M % 256 == 0, d % 256 == 0 (whole tiles), KT = d / 32 and HD (the head width, a multiple of 32) dividing d.
template <int HD>
__global__ __launch_bounds__(256, 1) void k_prefill_kv(const f16_t* __restrict__ Xt, const PrefillLayer* __restrict__ layers,
                                                       long seq_off, int KT, int d, int M, int n_layers) {
  extern __shared__ pf_u32x4 pf_smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int nx = M >> 8, nw = d >> 8;
  const int total = 2 * nx * nw * n_layers;
  // A 32-row x 16-k operand of the 32x32x16 MFMA (lane l: row l%32, k (l/32)*8..+8) is gathered from two of the
  // stored 16-row x 32-k fragments: half h of the K-step, row group (l%32)/16 -> stored lane (2h + l/32)*16 + l%16.
  const int lrow = ((lane & 31) >> 4) * 64 + (lane >> 5) * 16 + (lane & 15);
  const int xbase = wm * 512 + lrow, wbase = 1024 + wn * 512 + lrow;
  const int capb = M >> 5;

  // Tile sequence.  Workgroup b runs on die b % 8, and each die has its own L2: a die takes gridDim/8 consecutive
  // tiles of the sequence per round, and the sequence is ordered in groups of XT memory tiles x all 2 nw weight tiles
  // of a block (V tiles first), so that for the usual shapes a die keeps working on the same XT memory tiles, which
  // stay in its L2, while the weights of a block stream through once per die.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
  auto tile_of = [&](int r) { return (r * 8 + xcd) * per_xcd + slot; };
  int n_my = 0;
  while (tile_of(n_my) < total) n_my++;
  if (n_my == 0) return;
  const int XT = (nx & 3) == 0 ? 4 : 1;
  // The result tile of a workgroup is 256 rows of operand A by 256 rows of operand B.  V tiles are c W_v^T
  // (A = memory rows = keys, B = W_v rows = dims), K tiles are W_k c^T (A = W_k rows = dims, B = keys): the
  // two kinds differ only in where A and B come from and in the epilogue.
  auto desc = [&](int q, int& a0, int& b0, bool& is_v, int& layer) {
    const int per_group = 2 * nw * XT, group = q / per_group, i = q % per_group;
    const int xi = i % XT, wsel = i / XT, ng = nx / XT;
    layer = group / ng;
    const int xt = (group % ng) * XT + xi;
    is_v = wsel < nw;
    const int wt = is_v ? wsel : wsel - nw;
    if (is_v) { a0 = xt * 256; b0 = wt * 256; } else { a0 = wt * 256; b0 = xt * 256; }
  };

  // Load cursor: this wave's 8 fragments (A rows for waves 0-1, B rows for waves 2-3) of K column c_kt of tile c_r.
  // Pointers read from the table are generic to the compiler; say that they are global.
  typedef const __attribute__((address_space(1))) pf_u32x4* gptr_t;
  typedef const __attribute__((address_space(1))) void* gvoid_t;
  typedef __attribute__((address_space(3))) void* lvoid_t;
  int c_r = 0, c_kt = 0, c_slot = 0;
  gptr_t c_src;
  auto cursor_tile = [&](int r) {
    int a0, b0, layer; bool is_v;
    desc(tile_of(r), a0, b0, is_v, layer);
    const pf_u32x4* W = reinterpret_cast<const pf_u32x4*>(layers[layer].W);
    const pf_u32x4* X = reinterpret_cast<const pf_u32x4*>(Xt);
    const pf_u32x4* Ab = is_v ? X + (long)(a0 / 16) * KT * 64 : W + (long)(a0 / 16) * KT * 64;
    const pf_u32x4* Bb = is_v ? W + (long)((d + b0) / 16) * KT * 64 : X + (long)(b0 / 16) * KT * 64;
    c_src = (gptr_t)((wave < 2 ? Ab : Bb) + (long)((wave & 1) * 8) * KT * 64 + lane);
  };
  cursor_tile(0);
  const int fstride = KT * 64;
  // the loads of the next stage of the stream into the next ring slot: lane l of a load writes its 16 bytes at
  // (wave-uniform LDS address) + 16 l, which is the fragment order the operands are read in
  auto issue = [&]() {
    pf_u32x4* dst = pf_smem + c_slot * PF_STAGE_ELEMS + wave * 512;
    gptr_t src = c_src + c_kt * 64;
#pragma unroll
    for (int j = 0; j < 8; j++)
      __builtin_amdgcn_global_load_lds((gvoid_t)(src + j * fstride), (lvoid_t)(dst + j * 64), 16, 0, 0);
    c_slot = c_slot + 1 == PF_STAGES ? 0 : c_slot + 1;
    // past the end the cursor stays on the last stage: the extra loads land in a slot nobody reads any more
    if (c_kt + 1 < KT) c_kt++;
    else if (c_r + 1 < n_my) { c_r++; c_kt = 0; cursor_tile(c_r); }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int x = 0; x < 4; x++)
#pragma unroll
    for (int w = 0; w < 4; w++)
#pragma unroll
      for (int j = 0; j < 16; j++) acc[x][w][j] = 0.f;

#pragma unroll
  for (int p = 0; p < PF_STAGES - 1; p++) issue();

  // operands of one half K-step (16 of the 32 k of a stage): 4 A and 4 B operands of 32 rows, two sets
  f16x8 cx[4], cw[4], ox[4], ow[4];
#define PF_READ(XF, WF, ST, H)                                                                       \
  {                                                                                                  \
    _Pragma("unroll") for (int x = 0; x < 4; x++) XF[x] = __builtin_bit_cast(f16x8, (ST)[xbase + x * 128 + (H) * 32]); \
    _Pragma("unroll") for (int w = 0; w < 4; w++) WF[w] = __builtin_bit_cast(f16x8, (ST)[wbase + w * 128 + (H) * 32]); \
  }
#define PF_MFMA(XF, WF)                                                                              \
  _Pragma("unroll") for (int x = 0; x < 4; x++)                                                      \
    _Pragma("unroll") for (int w = 0; w < 4; w++)                                                    \
      acc[x][w] = __builtin_amdgcn_mfma_f32_32x32x16_f16(XF[x], WF[w], acc[x][w], 0, 0, 0);
  // One stage.  In flight when it starts: this wave's loads of the next PF_STAGES-2 stages and, in the first
  // PF_STAGES-2 stages after an epilogue, the result stores of the last tile, which are younger than those loads.
  // The wait lets everything but the loads of the next stage stay in flight; behind the barrier everyone's loads of
  // that stage have landed and everyone is done reading the slot that is refilled next.  The first half-stage is
  // multiplied while the second is read, the second while the first of the next stage is read.
#define PF_STAGE(PREFETCH, AFTER_STORES)                                                             \
  {                                                                                                  \
    const pf_u32x4* st = pf_smem + slot_c * PF_STAGE_ELEMS;                                          \
    slot_c = slot_c + 1 == PF_STAGES ? 0 : slot_c + 1;                                               \
    const pf_u32x4* st_next = pf_smem + slot_c * PF_STAGE_ELEMS;                                     \
    PF_READ(ox, ow, st, 1);                                                                          \
    PF_MFMA(cx, cw);                                                                                 \
    if (AFTER_STORES) { PF_WAIT_VM(8 * (PF_STAGES - 3) + PF_STORES); } else { PF_WAIT_VM(8 * (PF_STAGES - 3)); } \
    __builtin_amdgcn_s_barrier();                                                                    \
    issue();                                                                                         \
    if (PREFETCH) PF_READ(cx, cw, st_next, 0);                                                       \
    PF_MFMA(ox, ow);                                                                                 \
    if (PREFETCH) {                                                                                  \
      /* instruction order of this part: the reads early, two behind each of the first four MFMAs */ \
      _Pragma("unroll") for (int i = 0; i < 4; i++) {                                                \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                           \
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                           \
      }                                                                                              \
      __builtin_amdgcn_sched_group_barrier(0x008, 12, 0);                                            \
    }                                                                                                \
  }

  // stage 0 must have landed before its first operands are read
  PF_WAIT_VM(8 * (PF_STAGES - 2));
  __builtin_amdgcn_s_barrier();
  int slot_c = 0;
  PF_READ(cx, cw, pf_smem, 0);
  for (int r = 0; r < n_my; r++) {
    int kt0 = 0;
    if (r > 0)
      for (; kt0 < PF_STAGES - 2; kt0++) PF_STAGE(true, true);
    for (int kt = kt0; kt < KT - 1; kt++) PF_STAGE(true, false);
    PF_STAGE(false, false);
    {
      // epilogue of the tile that just finished: halves into the blocked cache layouts.  In a result tile lane l owns
      // column l%32 (a row of B) and the A rows (j/4)*8 + (l/32)*4 + j%4, j = 0..15, i.e. four runs of four rows.
      int a0, b0, layer; bool is_v;
      desc(tile_of(r), a0, b0, is_v, layer);
      const PrefillLayer L = layers[layer];
      const int hl4 = (lane >> 5) * 4, c32 = lane & 31;
      typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
      typedef _Float16 f16x8o __attribute__((ext_vector_type(8)));
      typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
      for (int x = 0; x < 4; x++) {
#pragma unroll
        for (int w = 0; w < 4; w++) {
          const int col = b0 + wn * 128 + w * 32 + c32;
          if (is_v) {
            // rows = keys, column = dim.  Keys r..r+3 and r+16..r+19 of a block sit next to each other in the V
            // layout: runs j/4 = q and q+2 make one 16-byte store
            const int row0 = a0 + wm * 128 + x * 32 + hl4;
            f16_t* base = L.Vm + seq_off + (long)(col / HD) * capb * (32 * HD);
#pragma unroll
            for (int q = 0; q < 2; q++) {
              f16x8o o;
#pragma unroll
              for (int i = 0; i < 4; i++) { o[i] = (f16_t)acc[x][w][q * 4 + i]; o[4 + i] = (f16_t)acc[x][w][(q + 2) * 4 + i]; }
              *(__attribute__((address_space(1))) f16x8o*)(base + vblk_off<HD>(row0 + q * 8, col % HD)) = o;
            }
          } else {
            // rows = dims, column = key.  Lanes l and l+32 hold dims 0-3 and 4-7 of the same 8-dim run of a key, which
            // is 16 contiguous bytes of the K layout: the lower lane collects runs 0 and 2, the upper lane runs 1 and 3
#pragma unroll
            for (int qp = 0; qp < 2; qp++) {
              f16x4 lo, hi;
#pragma unroll
              for (int i = 0; i < 4; i++) { lo[i] = (f16_t)acc[x][w][(2 * qp) * 4 + i]; hi[i] = (f16_t)acc[x][w][(2 * qp + 1) * 4 + i]; }
              const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
              // the swap trades the upper 32 lanes of its first operand for the lower 32 lanes of its second:
              // result 0 = {lo of lanes 0-31, hi of lanes 0-31}, result 1 = {lo of lanes 32-63, hi of lanes 32-63}
              const auto s0 = __builtin_amdgcn_permlane32_swap(l2[0], h2[0], false, false);
              const auto s1 = __builtin_amdgcn_permlane32_swap(l2[1], h2[1], false, false);
              const pf_u32x4 o = {s0[0], s1[0], s0[1], s1[1]};
              const int e0 = a0 + wm * 128 + x * 32 + (2 * qp + (lane >> 5)) * 8;   // first dim of the run this lane stores
              *(__attribute__((address_space(1))) pf_u32x4*)(L.Km + seq_off + (long)(e0 / HD) * capb * (32 * HD) + kblk_off<HD>(col, e0 % HD)) = o;
            }
          }
#pragma unroll
          for (int j = 0; j < 16; j++) acc[x][w][j] = 0.f;
          __builtin_amdgcn_sched_barrier(0);   // keeps the conversions of one accumulator together (register pressure)
        }
      }
    }
    // first operands of the next tile (its first stage was confirmed by the barrier of the last stage)
    PF_READ(cx, cw, pf_smem + slot_c * PF_STAGE_ELEMS, 0);
  }
  PF_WAIT_VM(0);   // the extra loads past the end
#undef PF_READ
#undef PF_MFMA
#undef PF_STAGE
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
