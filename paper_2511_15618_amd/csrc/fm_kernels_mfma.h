// Half-precision MFMA kernels for gfx950 (64-wide wavefronts, v_mfma_f32_16x16x32_f16).
//
//  * k_gemm_mfma : skinny weight-streaming GEMM.  Weights are pre-tiled at load time into MFMA
//                  B-operand order so that every wave load is one contiguous 1 KiB burst; the four
//                  waves of a workgroup split K and reduce through LDS in a fixed order.  K is not
//                  split across workgroups: publishing partial sums inside a launch needs an
//                  agent-scope release fence, which costs more than the parallelism gains here.
//  * k_attn_mfma : block attention over a K/V cache (flash-decoding): fixed key ranges split across
//                  workgroups and waves, online softmax in fp32, P kept in registers between the two
//                  MFMAs by storing V in a blocked, slot-permuted transposed layout; partial results
//                  merged in range order (in the launch, or by k_attn_merge when there are many).
//
// MFMA 16x16x32 operand layout (lane l of 64):
//   A[16 x 32]: row l%16, k = (l/16)*8 .. +8      B[32 x 16]: col l%16, k = (l/16)*8 .. +8
//   C[16 x 16]: col l%16, rows (l/16)*4 + i, i = 0..3
#pragma once
#include <type_traits>
#include "fm_device.h"
#include "fm_kernels_basic.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Cross-workgroup exchange inside one launch (split-KV partials): values are written and read with
// agent-scope atomics and published with an agent-scope RELEASE fence before the arrival counter is
// bumped.  A workgroup-scope fence is not enough on this chip: the write-through of an agent-scope store
// can still be in flight when the counter increment lands, and the last arriver then reads the previous
// launch's data (seen as run-to-run differences in one token per ~10^4 steps).  The consumer side needs
// no invalidate because it reads the partials with agent-scope loads.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_fence() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }

#define FM_ATTN_MAX_SPLIT 64

// ------------------------------------------------------------------------------------------
// Cache layouts of the half-precision path: one 32-key block of a head = 32 HD halves (4 KiB for the 64-wide heads
// of the benchmark configurations; HD = 96 and 128 are the paper's own model shapes)
// ------------------------------------------------------------------------------------------
// K: HD/16 A-fragments per block, fragment f = (key/16)*(HD/32) + dim/32, lane = key%16 + 16*((dim%32)/8)
template <int HD = 64>
__device__ __forceinline__ long kblk_off(int key, int dim) {
  const int r = key & 31;
  const int f = (r >> 4) * (HD / 32) + (dim >> 5);
  const int lane = (r & 15) + 16 * ((dim & 31) >> 3);
  return (long)(key >> 5) * (32 * HD) + (f * 64 + lane) * 8 + (dim & 7);
}
// V: transposed inside the block, [dim][slot]; slot order matches the C-layout of the score tile so
// that the probabilities never leave registers: key r -> g = (r%16)/4, slot = g*8 + (r/16)*4 + r%4
template <int HD = 64>
__device__ __forceinline__ long vblk_off(int key, int dim) {
  const int r = key & 31;
  const int slot = ((r & 15) >> 2) * 8 + (r >> 4) * 4 + (r & 3);
  return (long)(key >> 5) * (32 * HD) + dim * 32 + slot;
}

// rotary + append for the half-precision caches (same contract as k_rope_append)
template <int HD>
__global__ void k_rope_append_h(const float* __restrict__ qkv, long ldq, const float2* __restrict__ cs,
                                const int* __restrict__ pos, int RPS, f16_t* __restrict__ q, f16_t* __restrict__ Kc,
                                f16_t* __restrict__ Vc, int H, int capb, const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  constexpr int NP = HD / 2;                                  // rotary pairs per head: dims i and i + NP
  const int r = blockIdx.x;
  const int p = pos[r] >= 0 ? pos[r] % (capb * 32) : -1;     // the cache is a ring when a window is set
  const int d = H * HD;
  const int s = r / RPS;
  for (int idx = threadIdx.x; idx < H * NP; idx += blockDim.x) {
    const int hh = idx / NP, i = idx % NP;
    const float2 c = cs[(long)r * NP + i];
    const float* row = qkv + (long)r * ldq;
    const float qa = row[hh * HD + i], qb = row[hh * HD + NP + i];
    q[(long)r * d + hh * HD + i] = (f16_t)(qa * c.x - qb * c.y);
    q[(long)r * d + hh * HD + NP + i] = (f16_t)(qb * c.x + qa * c.y);
    if (Kc && p >= 0) {
      const float ka = row[d + hh * HD + i], kb = row[d + hh * HD + NP + i];
      const long base = ((long)s * H + hh) * capb * (32 * HD);
      Kc[base + kblk_off<HD>(p, i)] = (f16_t)(ka * c.x - kb * c.y);
      Kc[base + kblk_off<HD>(p, i + NP)] = (f16_t)(kb * c.x + ka * c.y);
      Vc[base + vblk_off<HD>(p, i)] = (f16_t)row[2 * d + hh * HD + i];
      Vc[base + vblk_off<HD>(p, i + NP)] = (f16_t)row[2 * d + hh * HD + NP + i];
    }
  }
}

template <int HD>
__global__ void k_mem_kv_store_h(const float* __restrict__ kv, f16_t* __restrict__ Kc, f16_t* __restrict__ Vc, int H,
                                 int M, int capb) {
  const int m = blockIdx.x;
  const int d = H * HD;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const int hh = i / HD, e = i % HD;
    const long base = (long)hh * capb * (32 * HD);
    Kc[base + kblk_off<HD>(m, e)] = (f16_t)kv[(long)m * 2 * d + i];
    Vc[base + vblk_off<HD>(m, e)] = (f16_t)kv[(long)m * 2 * d + d + i];
  }
}

// weights [N][K] fp32 (bf16-valued) -> half, tiled: fragment (nt, kt) holds W[nt*16 + l%16][kt*32 + (l/16)*8 + j]
// perm_d > 0 (fused q,k,v projection of width perm_d each): the q and k tiles are re-ordered so that tile
// (head, quarter) holds dims quarter*8..+8 and the same dims + 32, i.e. both halves of 8 rotary pairs.
__global__ void k_tile_weight(const float* __restrict__ src, f16_t* __restrict__ dst, int N, int K, int Npad, int perm_d) {
  const long total = (long)Npad * K / 8;
  for (long v = blockIdx.x * (long)blockDim.x + threadIdx.x; v < total; v += (long)gridDim.x * blockDim.x) {
    const int lane = (int)(v & 63);
    const long frag = v >> 6;
    const int KT = K / 32;
    const int kt = (int)(frag % KT), nt = (int)(frag / KT);
    int n = nt * 16 + (lane & 15);
    const int k = kt * 32 + (lane >> 4) * 8;
    if (perm_d > 0 && n < 2 * perm_d) {
      const int part = n / perm_d, cp = n % perm_d;
      const int hh = cp >> 6, qd = (cp & 63) >> 4, c = cp & 15;
      n = part * perm_d + hh * 64 + (c < 8 ? qd * 8 + c : 32 + qd * 8 + (c - 8));
    }
    f16x8 o;
#pragma unroll
    for (int j = 0; j < 8; j++) o[j] = n < N ? (f16_t)src[(long)n * K + k + j] : (f16_t)0.f;
    *reinterpret_cast<f16x8*>(dst + v * 8) = o;
  }
}

// ------------------------------------------------------------------------------------------
// GEMM
// ------------------------------------------------------------------------------------------
// The wave index is made provably wave-uniform (readfirstlane) in every MFMA kernel: MFMA ignores the EXEC mask,
// so an MFMA guarded by a condition the compiler takes for divergent would run on a false guard as well.
struct GemmSplit {
  int kt_per_wave;   // K fragments (of 32) each wave walks
};

// NORM: X is fp32 and each row is RMS-normalised on the fly: the MFMA runs on half(x * gain) and the per-row factor
// 1/rms is applied to the accumulated tile (every workgroup walks the whole K of its rows, so it has the row sums
// of squares itself; partial sums per wave meet in LDS next to the partial tiles, in a fixed order).
// (two workgroups per CU: launches of 257..512 workgroups, e.g. the 288 and 384 tiles of d = 1536, then take one
// round instead of two)
// NW waves per workgroup (4, 8 or 16) split K: launches with few column tiles (N = d gives 64 to 96 of them)
// take more waves per workgroup so that enough loads are in flight and each wave's K walk stays short.
// NC column tiles of 16 per workgroup (1 or 2): with two, an activation fragment loaded (and normalised) once feeds two
// MFMAs, which halves what the wide projections (N >= 2048) pull out of L2 for their activations.
template <int MT, int EPI, bool NORM, int NW, int NC = 1>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void k_gemm_mfma(GemmArgs a, GemmSplit sp) {
  if (a.run_flag && *a.run_flag == 0) return;
  static_assert(NW * MT * NC <= 60, "partial tiles of all waves must fit the static LDS limit");
  __shared__ f32x4 red[NW][MT * NC][64];
  __shared__ float sq[NORM ? NW : 1][MT][16];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int nt = blockIdx.x;
  const int nmb = (a.M + MT * 16 - 1) / (MT * 16);
  const int g = blockIdx.z / nmb, mb = blockIdx.z % nmb;
  const int KT = a.K / 32;
  typedef typename std::conditional<NORM, float, f16_t>::type XT;
  const XT* X = (const XT*)a.X + (long)g * a.gsx;
  const f16_t* W = (const f16_t*)a.W + (long)g * a.gsw + ((long)nt * NC * KT) * 512;   // column tile c of this workgroup: + c * KT * 512
  const int m0 = mb * MT * 16;
  // A-fragment row pointers (rows past M are clamped: computed, never stored)
  const XT* xrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; mt++) {
    int m = m0 + mt * 16 + (lane & 15);
    m = m < a.M ? m : a.M - 1;
    xrow[mt] = X + (long)m * a.ldx + (lane >> 4) * 8;
  }
  f32x4 acc[MT][NC];
  float ss[MT];
#pragma unroll
  for (int mt = 0; mt < MT; mt++) {
    ss[mt] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; c++) acc[mt][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const int kt0 = wave * sp.kt_per_wave;
  const int kt1 = min(kt0 + sp.kt_per_wave, KT);

  // K is walked in chunks of U fragments; the loads of the next chunk are in flight while this one is
  // multiplied (a workgroup is often alone on its CU, so nothing else would hide the latency)
  constexpr int U4 = NORM ? (MT <= 2 ? 4 : MT <= 5 ? 2 : 1) : (MT <= 2 ? 8 : MT <= 5 ? 4 : 2);
  constexpr int U = NW == 16 ? (U4 >= 4 ? U4 / 4 : 1) : NW == 8 ? (U4 >= 2 ? U4 / 2 : 1) : U4;
  struct AFrag { typename std::conditional<NORM, f32x4, f16x8>::type lo; f32x4 hi; };   // hi only used when NORM
  f16x8 bc[NC][U];
  AFrag ac[MT][U];
  f32x4 gc[NORM ? U : 1][2];
  const int nk = kt1 - kt0;
  auto kmap = [&](int i) { return kt0 + i; };
  auto load_chunk = [&](f16x8 (&b)[NC][U], AFrag (&af)[MT][U], f32x4 (&gg)[NORM ? U : 1][2], int i0) {
#pragma unroll
    for (int u = 0; u < U; u++) {
      if (i0 + u < nk) {
        const int kt = kmap(i0 + u);
#pragma unroll
        for (int c = 0; c < NC; c++) b[c][u] = *reinterpret_cast<const f16x8*>(W + ((long)(c * KT + kt) * 64 + lane) * 8);
        if constexpr (NORM) {
          const float* gp = a.gain + kt * 32 + (lane >> 4) * 8;
          gg[u][0] = *reinterpret_cast<const f32x4*>(gp);
          gg[u][1] = *reinterpret_cast<const f32x4*>(gp + 4);
        }
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
          if constexpr (NORM) {
            af[mt][u].lo = *reinterpret_cast<const f32x4*>(xrow[mt] + kt * 32);
            af[mt][u].hi = *reinterpret_cast<const f32x4*>(xrow[mt] + kt * 32 + 4);
          } else {
            af[mt][u].lo = *reinterpret_cast<const f16x8*>(xrow[mt] + kt * 32);
          }
        }
      }
    }
  };
  load_chunk(bc, ac, gc, 0);
  for (int i0 = 0; i0 < nk; i0 += U) {
    f16x8 bn[NC][U];
    AFrag an[MT][U];
    f32x4 gn[NORM ? U : 1][2];
    load_chunk(bn, an, gn, i0 + U);
#pragma unroll
    for (int u = 0; u < U; u++) {
      if (i0 + u < nk) {
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
          f16x8 av;
          if constexpr (NORM) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
              const float x0 = ac[mt][u].lo[j], x1 = ac[mt][u].hi[j];
              ss[mt] += x0 * x0 + x1 * x1;
              av[j] = (f16_t)(x0 * gc[u][0][j]);
              av[4 + j] = (f16_t)(x1 * gc[u][1][j]);
            }
          } else {
            av = ac[mt][u].lo;
          }
#pragma unroll
          for (int c = 0; c < NC; c++) acc[mt][c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bc[c][u], acc[mt][c], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
#pragma unroll
      for (int c = 0; c < NC; c++) bc[c][u] = bn[c][u];
      if constexpr (NORM) { gc[u][0] = gn[u][0]; gc[u][1] = gn[u][1]; }
#pragma unroll
      for (int mt = 0; mt < MT; mt++) ac[mt][u] = an[mt][u];
    }
  }
  // reduce the K-slices of the waves through LDS, in wave order
#pragma unroll
  for (int mt = 0; mt < MT; mt++) {
#pragma unroll
    for (int c = 0; c < NC; c++) red[wave][mt * NC + c][lane] = acc[mt][c];
    if constexpr (NORM) {
      float t = ss[mt];
      t += __shfl_xor(t, 16, 64);
      t += __shfl_xor(t, 32, 64);
      if ((lane >> 4) == 0) sq[wave][mt][lane & 15] = t;
    }
  }
  __syncthreads();
  for (int t = wave; t < MT * NC; t += NW) {
    const int mt = t / NC, ntc = nt * NC + t % NC;     // row tile and column tile of this result tile
    const int n = ntc * 16 + (lane & 15);
    f32x4 v = red[0][t][lane];
#pragma unroll
    for (int w = 1; w < NW; w++) v += red[w][t][lane];
    if constexpr (NORM) {
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int row = (lane >> 4) * 4 + i;
        float tot = sq[0][mt][row];
#pragma unroll
        for (int w = 1; w < NW; w++) tot += sq[w][mt][row];
        v[i] *= 1.0f / sqrtf(tot / (float)a.K + a.eps);
      }
    }
    if constexpr (EPI == EPI_QKV) {
      // tile nt of the fused projection: part 0/1/2 = q/k/v, head hh, and for q and k the rotary pairs
      // qd*8 .. +8 (columns 0..7 = first halves, 8..15 = second halves), for v the dims qd*16 .. +16
      const int d = a.H * FM_HD, col = lane & 15;
      const int part = (ntc * 16) / d, cp = (ntc * 16) % d;
      const int hh = cp >> 6, qd = (cp & 63) >> 4;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const long m = m0 + mt * 16 + (lane >> 4) * 4 + i;
        const long mc = m < a.M ? m : a.M - 1;
        float val = v[i];
        int dim;
        if (part < 2) {
          const int j = qd * 8 + (col & 7);
          const float2 t = a.cs[mc * 32 + j];
          const float o = __shfl_xor(val, 8, 64);
          val = col < 8 ? val * t.x - o * t.y : val * t.x + o * t.y;
          dim = col < 8 ? j : j + 32;
        } else {
          dim = qd * 16 + col;
        }
        if (m < a.M) {
          if (part == 0) {
            ((f16_t*)a.Y)[m * a.ldy + hh * FM_HD + dim] = (f16_t)val;
          } else {
            const int pa = a.pos[m];
            if (pa >= 0) {
              const int p = pa % (a.capb * 32);      // the cache is a ring when a window is set
              const long base = (m / a.RPS) * a.seq_stride + (long)hh * a.capb * 2048;
              if (part == 1) ((f16_t*)a.Kc)[base + kblk_off(p, dim)] = (f16_t)val;
              else ((f16_t*)a.Vc)[base + vblk_off(p, dim)] = (f16_t)val;
            }
          }
        }
      }
    } else if (n < a.N) {
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const long m = m0 + mt * 16 + (lane >> 4) * 4 + i;
        if (m < a.M) {
          float val = v[i];
          if (EPI == EPI_F32) {
            if (a.R) val += a.R[(long)g * a.gsr + m * a.ldr + n];
            ((float*)a.Y)[(long)g * a.gsy + m * a.ldy + n] = val;
          } else {
            ((f16_t*)a.Y)[(long)g * a.gsy + m * a.ldy + n] = (f16_t)(EPI == EPI_GELU_T ? gelu_tanh_f(val) : val);
          }
        }
      }
    }
  }
}

struct MfmaRes {      // per-context resources of the MFMA kernels
  float* attn_ws;
  unsigned* attn_counters;
  size_t attn_ws_floats;
  int gemm_waves;     // 0 = choose per launch; 4, 8, 16 = forced (measurement switch)
  int gemm_mt_cap;    // 0 = default (below); 2, 3, 5, 8 = one workgroup covers up to that many 16-row tiles (measurement switch)
  int attn_wgs;       // key ranges of a growing cache: as few as give about this many workgroups per launch (768 by default,
                      // as for the condition memory); 0 = ranges as short as 8 blocks whatever the batch (measurement switch)
  int attn_merge;     // 2 = the last workgroup of a (sequence, head) always merges, publication without an L2 write-back (measurement)
  int gemm_nc;        // 0 = two column tiles per workgroup for the wide projections; 1 = one everywhere, 2 = two everywhere (measurement switches)
};

template <int MT, bool NORM, int NW, int NC>
void gemm_mfma_dispatch3(const GemmArgs& a, const GemmSplit& sp, int epi, dim3 grid, hipStream_t st) {
  if (epi == EPI_QKV) {
    if constexpr (NORM) hipLaunchKernelGGL((k_gemm_mfma<MT, EPI_QKV, true, NW, NC>), grid, dim3(NW * 64), 0, st, a, sp);
    return;
  }
  if (epi == EPI_F32) hipLaunchKernelGGL((k_gemm_mfma<MT, EPI_F32, NORM, NW, NC>), grid, dim3(NW * 64), 0, st, a, sp);
  else if (epi == EPI_GELU_T) hipLaunchKernelGGL((k_gemm_mfma<MT, EPI_GELU_T, NORM, NW, NC>), grid, dim3(NW * 64), 0, st, a, sp);
  else hipLaunchKernelGGL((k_gemm_mfma<MT, EPI_T, NORM, NW, NC>), grid, dim3(NW * 64), 0, st, a, sp);
}
template <int MT, bool NORM, int NC>
void gemm_mfma_dispatch2(const GemmArgs& a, const GemmSplit& sp, int nw, int epi, dim3 grid, hipStream_t st) {
  if constexpr (MT <= 3) { if (nw == 16) { gemm_mfma_dispatch3<MT, NORM, 16, NC>(a, sp, epi, grid, st); return; } }
  if constexpr (MT <= 5) { if (nw >= 8) { gemm_mfma_dispatch3<MT, NORM, 8, NC>(a, sp, epi, grid, st); return; } }
  gemm_mfma_dispatch3<MT, NORM, 4, NC>(a, sp, epi, grid, st);
}
template <int MT>
void gemm_mfma_dispatch(const GemmArgs& a, const GemmSplit& sp, int nw, int epi, int nc, dim3 grid, hipStream_t st) {
  if constexpr (MT == 1) {
    if (nc == 2) {
      if (a.gain) gemm_mfma_dispatch2<1, true, 2>(a, sp, nw, epi, grid, st);
      else gemm_mfma_dispatch2<1, false, 2>(a, sp, nw, epi, grid, st);
      return;
    }
  }
  if (a.gain) gemm_mfma_dispatch2<MT, true, 1>(a, sp, nw, epi, grid, st);
  else gemm_mfma_dispatch2<MT, false, 1>(a, sp, nw, epi, grid, st);
}

template <typename T>
bool mfma_gemm_launch(const MfmaRes&, const GemmArgs&, int, int, hipStream_t) { return false; }

template <>
inline bool mfma_gemm_launch<f16_t>(const MfmaRes& res, const GemmArgs& a, int epi, int groups, hipStream_t st) {
  if (a.K % 32 != 0 || a.M < 1) return false;
  const int KT = a.K / 32, Npad = (a.N + 15) / 16 * 16, NT = Npad / 16;
  const int mtiles = (a.M + 15) / 16;
  // Row tiles per workgroup.  Up to 128 rows (every launch of a decode step) a workgroup takes one 16-row tile and the
  // row tiles of a column tile go to different workgroups: the weight tile is then fetched once from HBM and again from
  // L2, but each workgroup reads a fifth of the activations at 72 rows and five times as many workgroups pull on the
  // weights (measured: -5 % per verify pass on 8 sequences at d = 1024, -7 % on 4 sequences at d = 1536).  Taller
  // problems (the per-block prefill GEMM) keep 128 rows per workgroup.
  int MT = mtiles <= 8 ? 1 : 8;
  if (res.gemm_mt_cap > 1) {
    MT = mtiles <= 1 ? 1 : mtiles <= 2 ? 2 : mtiles <= 3 ? 3 : mtiles <= 5 ? 5 : 8;
    if (MT > res.gemm_mt_cap) MT = res.gemm_mt_cap >= 8 ? 8 : res.gemm_mt_cap >= 5 ? 5 : res.gemm_mt_cap;
  }
  const int nmb = (a.M + MT * 16 - 1) / (MT * 16);
  // waves per workgroup: enough for about 2048 waves in the launch, at least two K fragments per wave, and the
  // partial tiles of all waves within the static LDS limit
  // two column tiles per workgroup for the wide projections (q,k,v, FFN up, output head) when rows are split 16 per
  // workgroup: FM_GEMM_NC=1 switches it off (measurement)
  const int nc = (MT == 1 && NT >= (res.gemm_nc == 2 ? 2 : 128) && NT % 2 == 0 && res.gemm_nc != 1) ? 2 : 1;   // gemm_nc == 2: every even launch (measurement)
  const long wgs = (long)(NT / nc) * groups * nmb;
  const int nw_max = MT <= 3 ? 16 : MT <= 5 ? 8 : 4;
  int nw = 4;
  while (nw < nw_max && wgs * nw < 2048 && KT / (nw * 2) >= 2) nw *= 2;
  if (res.gemm_waves == 4 || res.gemm_waves == 8 || res.gemm_waves == 16) nw = res.gemm_waves < nw_max ? res.gemm_waves : nw_max;
  GemmSplit sp{(KT + nw - 1) / nw};   // the waves of a workgroup split K
  dim3 grid(NT / nc, 1, groups * nmb);
  switch (MT) {
    case 1: gemm_mfma_dispatch<1>(a, sp, nw, epi, nc, grid, st); break;
    case 2: gemm_mfma_dispatch<2>(a, sp, nw, epi, nc, grid, st); break;
    case 3: gemm_mfma_dispatch<3>(a, sp, nw, epi, nc, grid, st); break;
    case 5: gemm_mfma_dispatch<5>(a, sp, nw, epi, nc, grid, st); break;
    default: gemm_mfma_dispatch<8>(a, sp, nw, epi, nc, grid, st); break;
  }
  return true;
}

// ------------------------------------------------------------------------------------------
// Attention
// ------------------------------------------------------------------------------------------
// Merge of the split-KV partials of one (sequence, head) by one workgroup, splits in ascending order.
// AGENT: the partials were written by other workgroups of the SAME launch (agent-scope loads; the compiler
// keeps those in program order, so each batch is requested in full before its first value is used);
// otherwise they come from an earlier launch and plain loads do.
template <int QT>
struct AttnMergeShared {
  float cf[FM_ATTN_MAX_SPLIT][QT * 16], cl[FM_ATTN_MAX_SPLIT][QT * 16], cden[QT * 16];
};

template <int QT, bool AGENT, int HD = 64>
__device__ __forceinline__ void attn_merge(AttnMergeShared<QT>& ms, const float* base, int nsplit, int RPS, f16_t* orow0, int d) {
  constexpr int NQ = QT * 16;
  constexpr int PSZ = NQ * HD + 2 * NQ;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  for (int e0 = 0; e0 < nsplit * NQ; e0 += 256 * 4) {
    float tm[4], tl[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int e = e0 + j * 256 + threadIdx.x;
      tm[j] = tl[j] = 0.f;
      if (e < nsplit * NQ) {
        const float* pp = base + (long)(e / NQ) * PSZ + NQ * HD + (e % NQ);
        tm[j] = AGENT ? ld_agent(pp) : *pp;
        tl[j] = AGENT ? ld_agent(pp + NQ) : pp[NQ];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int e = e0 + j * 256 + threadIdx.x;
      if (e < nsplit * NQ) { ms.cf[e / NQ][e % NQ] = tm[j]; ms.cl[e / NQ][e % NQ] = tl[j]; }
    }
  }
  __syncthreads();
  if (threadIdx.x < NQ) {
    const int qi = threadIdx.x;
    float M = -INFINITY;
    for (int k2 = 0; k2 < nsplit; k2++) M = fmaxf(M, ms.cf[k2][qi]);
    const float Ms = M == -INFINITY ? 0.f : M;
    float den = 0.f;
    for (int k2 = 0; k2 < nsplit; k2++) {
      const float f = __builtin_amdgcn_exp2f(ms.cf[k2][qi] - Ms);
      ms.cf[k2][qi] = f;
      den += ms.cl[k2][qi] * f;
    }
    ms.cden[qi] = den;
  }
  __syncthreads();
  // numerators: 16-byte loads (four dims of one query row), eight splits in flight per thread
  for (int v4 = threadIdx.x; v4 < NQ * (HD / 4); v4 += 256) {
    const int e = v4 * 4, qi = e / HD, dim = e % HD;
    float num[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < nsplit; c0 += 8) {
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; j++) {
        v[j] = u32x4{0u, 0u, 0u, 0u};
        if (c0 + j < nsplit) {
          const float* pp = base + (long)(c0 + j) * PSZ + e;
          if (AGENT) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v[j]) : "v"(pp) : "memory");
          else v[j] = *reinterpret_cast<const u32x4*>(pp);
        }
      }
      if (AGENT) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < 8; j++) {
        if (AGENT) asm volatile("" : "+v"(v[j]));
        if (c0 + j < nsplit) {
          const float f = ms.cf[c0 + j][qi];
#pragma unroll
          for (int i = 0; i < 4; i++) num[i] += __uint_as_float(v[j][i]) * f;
        }
      }
    }
    if (qi < RPS) {
      const float den = ms.cden[qi];
      f16_t* op = orow0 + (long)qi * d + dim;
#pragma unroll
      for (int i = 0; i < 4; i++) op[i] = (f16_t)(den > 0.f ? num[i] / den : 0.f);
    }
  }
}

// Workspace per (sequence, head): [nsplit][QT*16*HD unnormalised O | QT*16 running max (log2 units) | QT*16 sums]
// (the body of the launch; `split`, `hh`, `s` = key range, head and sequence of this workgroup)
template <int QT, int HD = 64>
__device__ __forceinline__ void attn_mfma_core(const f16_t* __restrict__ q, const int* __restrict__ limit, int RPS, int RS,
                                               const f16_t* __restrict__ Kc, const f16_t* __restrict__ Vc,
                                               long seq_stride, int capb, f16_t* __restrict__ out, int H,
                                               float* __restrict__ ws, unsigned* __restrict__ counters,
                                               int nsplit_cfg, int defer_merge, int window, int split, int hh, int s) {
  constexpr int NQ = QT * 16;
  constexpr int PSZ = NQ * HD + 2 * NQ;
  constexpr int KC = HD / 32, DT = HD / 16;     // 32-dim chunks of a key row, 16-dim tiles of the output
  __shared__ float lo[4][NQ][HD + 1];
  __shared__ float lm[4][NQ], ll[4][NQ];
  __shared__ AttnMergeShared<QT> ms;
  __shared__ int s_last;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int d = H * HD;
  const int g = lane >> 4, ql = lane & 15;
  const float kScale = (HD == 64 ? 0.125f : 1.0f / sqrtf((float)HD)) * 1.4426950408889634f;   // 1/sqrt(HD) * log2(e)

  // this lane's query rows (one per q-tile), their visibility limits and B-operand fragments
  int lim[QT], first[QT];
  f16x8 qf[QT][KC];
  int maxlim = -1;
#pragma unroll
  for (int t = 0; t < QT; t++) {
    const int qi = t * 16 + ql;
    const bool on = qi < RPS;
    const long row = (long)s * RS + (on ? qi : 0);     // RS = rows per sequence in the buffers (>= RPS)
    lim[t] = on ? limit[row] : -1;
    first[t] = window > 0 ? max(lim[t] - window + 1, 0) : 0;     // sliding window: keys first .. lim
    maxlim = max(maxlim, lim[t]);
    const f16_t* qp = q + row * d + hh * HD + g * 8;
#pragma unroll
    for (int kc = 0; kc < KC; kc++) qf[t][kc] = *reinterpret_cast<const f16x8*>(qp + kc * 32);
  }
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) maxlim = max(maxlim, __shfl_xor(maxlim, o, 64));
  // With a window the cache is a ring of capb blocks: position p lives in slot p mod (32 capb), and a slot holds
  // the latest position written to it.  Seen from the newest visible position `maxlim`, slot j holds
  // lapbase + j if that is <= maxlim, else the position one lap earlier (anything newer in the ring is a stale
  // row of a rejected block: it maps below the window and is masked).  Without a window lapbase = 0.
  const int nblk = min((maxlim + 32) >> 5, capb);     // slot blocks that can hold a visible key (0 if none)
  const int ringn = capb * 32;
  const int lapbase = max(maxlim, 0) / ringn * ringn;
  // Fixed partition of the key axis: split k owns blocks [k*per, (k+1)*per) whatever the current length,
  // so the arithmetic for one query position never depends on what else is in the block or on how far
  // the sequence has grown (speculative and one-token decoding then agree bit for bit).  Splits with no
  // visible key leave at once; every workgroup of this (sequence, head) derives the same count.
  // (the launch may hold fewer than nsplit_cfg workgroups per head when the host knows the cache is short)
  const int per = (capb + nsplit_cfg - 1) / nsplit_cfg;
  const int nsplit = max(1, (nblk + per - 1) / per);
  if (split >= nsplit) return;
  const int b0 = split * per, b1 = min(b0 + per, nblk);

  float mrun[QT], lrun[QT];
  f32x4 o[QT][DT];
#pragma unroll
  for (int t = 0; t < QT; t++) {
    mrun[t] = -INFINITY;
    lrun[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  constexpr int BLK = 32 * HD;                 // halves per 32-key block of a head
  const f16_t* Kb = Kc + (long)s * seq_stride + (long)hh * capb * BLK;
  const f16_t* Vb = Vc + (long)s * seq_stride + (long)hh * capb * BLK;
  // the next block of this wave is requested before the current one is multiplied
  f16x8 kf[2 * KC], vf[DT];
  if (b0 + wave < b1) {
    const f16_t* kp = Kb + (long)(b0 + wave) * BLK + lane * 8;
    const f16_t* vp = Vb + (long)(b0 + wave) * BLK + (lane & 15) * 32 + g * 8;
#pragma unroll
    for (int f = 0; f < 2 * KC; f++) kf[f] = *reinterpret_cast<const f16x8*>(kp + f * 512);
#pragma unroll
    for (int dt = 0; dt < DT; dt++) vf[dt] = *reinterpret_cast<const f16x8*>(vp + dt * 512);
  }
  for (int b = b0 + wave; b < b1; b += 4) {
    f16x8 kn[2 * KC], vn[DT];
    if (b + 4 < b1) {
      const f16_t* kp = Kb + (long)(b + 4) * BLK + lane * 8;
      const f16_t* vp = Vb + (long)(b + 4) * BLK + (lane & 15) * 32 + g * 8;
#pragma unroll
      for (int f = 0; f < 2 * KC; f++) kn[f] = *reinterpret_cast<const f16x8*>(kp + f * 512);
#pragma unroll
      for (int dt = 0; dt < DT; dt++) vn[dt] = *reinterpret_cast<const f16x8*>(vp + dt * 512);
    }
#pragma unroll
    for (int t = 0; t < QT; t++) {
      // scores, transposed: sT[hb][i] = <K[key], Q[q]> for key = b*32 + hb*16 + g*4 + i, q = this lane's row
      f32x4 sT[2];
#pragma unroll
      for (int hb = 0; hb < 2; hb++) {
        f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kc = 0; kc < KC; kc++) z = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[hb * KC + kc], qf[t][kc], z, 0, 0, 0);
        sT[hb] = z;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int hb = 0; hb < 2; hb++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          int key = lapbase + b * 32 + hb * 16 + g * 4 + i;     // absolute position held by this slot
          key = key > maxlim ? key - ringn : key;
          const float v = (key <= lim[t] && key >= first[t]) ? sT[hb][i] * kScale : -INFINITY;
          sT[hb][i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(mrun[t], mx);
      const float msafe = mnew == -INFINITY ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(mrun[t] - msafe);   // exp2(-inf) = 0 on the first block
      mrun[t] = mnew;
      f16x8 pf;
      float psum = 0.f;
#pragma unroll
      for (int hb = 0; hb < 2; hb++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float p = __builtin_amdgcn_exp2f(sT[hb][i] - msafe);
          psum += p;
          pf[hb * 4 + i] = (f16_t)p;
        }
      lrun[t] = lrun[t] * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        o[t][dt] *= alpha;
        o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[dt], pf, o[t][dt], 0, 0, 0);   // O^T[dim][q]
      }
    }
    if (b + 4 < b1) {
#pragma unroll
      for (int f = 0; f < 2 * KC; f++) kf[f] = kn[f];
#pragma unroll
      for (int dt = 0; dt < DT; dt++) vf[dt] = vn[dt];
    }
  }
  // combine the four waves of the workgroup
#pragma unroll
  for (int t = 0; t < QT; t++) {
    float l = lrun[t];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (g == 0) { lm[wave][t * 16 + ql] = mrun[t]; ll[wave][t * 16 + ql] = l; }
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int i = 0; i < 4; i++) lo[wave][t * 16 + ql][dt * 16 + g * 4 + i] = o[t][dt][i];
  }
  __syncthreads();
  const long sh = (long)s * H + hh;
  float* part = ws + (sh * nsplit_cfg + split) * PSZ;   // slots are laid out for the configured split count
  for (int e = threadIdx.x; e < NQ * HD; e += 256) {
    const int qi = e / HD, dim = e % HD;
    const float M = fmaxf(fmaxf(lm[0][qi], lm[1][qi]), fmaxf(lm[2][qi], lm[3][qi]));
    const float Ms = M == -INFINITY ? 0.f : M;
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float f = __builtin_amdgcn_exp2f(lm[w][qi] - Ms);
      num += lo[w][qi][dim] * f;
      den += ll[w][qi] * f;
    }
    if (nsplit == 1) {
      if (qi < RPS) out[((long)s * RS + qi) * d + hh * HD + dim] = (f16_t)(den > 0.f ? num / den : 0.f);
    } else if (defer_merge == 1) {
      part[e] = num;
      if (dim == 0) { part[NQ * HD + qi] = M; part[NQ * HD + NQ + qi] = den; }
    } else {
      st_agent(part + e, num);
      if (dim == 0) { st_agent(part + NQ * HD + qi, M); st_agent(part + NQ * HD + NQ + qi, den); }
    }
  }
  if (nsplit == 1 || defer_merge == 1) return;     // deferred: k_attn_merge runs behind this launch
  if (defer_merge == 2) {
    // The partials went out as agent-scope stores (written through, not left in this die's L2), so they are visible to
    // the other dies once the stores have completed: wait for that instead of writing the whole L2 back.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  } else {
    publish_fence();
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned old = __hip_atomic_fetch_add(&counters[sh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == (unsigned)nsplit - 1);
    if (s_last) __hip_atomic_store(&counters[sh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!s_last) return;
  // last workgroup of this (sequence, head)
  attn_merge<QT, true, HD>(ms, ws + sh * nsplit_cfg * PSZ, nsplit, RPS, out + (long)s * RS * d + hh * HD, d);
}

template <int QT, int HD>
__global__ __launch_bounds__(256) void k_attn_mfma(const f16_t* __restrict__ q, const int* __restrict__ limit, int RPS, int RS,
                                                    const f16_t* __restrict__ Kc, const f16_t* __restrict__ Vc,
                                                    long seq_stride, int capb, f16_t* __restrict__ out, int H,
                                                    float* __restrict__ ws, unsigned* __restrict__ counters,
                                                    int nsplit_cfg, int defer_merge, const int* run_flag, int window) {
  if (run_flag && *run_flag == 0) return;
  attn_mfma_core<QT, HD>(q, limit, RPS, RS, Kc, Vc, seq_stride, capb, out, H, ws, counters, nsplit_cfg, defer_merge, window,
                     blockIdx.x, blockIdx.y, blockIdx.z);
}

// Up to three row sets per sequence, each attending to a cache of its own (the SP heads of the three levels read the
// coordinate-, point- and face-level caches of the last blocks, Eq. 1), in one launch: blockIdx.z = set * S + sequence.
// Workspace and counters of set z start at z * S * H * FM_ATTN_MAX_SPLIT * (32*64+64) floats and z * S * H counters.
struct AttnLevel {
  const f16_t* q;
  const int* limit;
  int RPS;                 // rows of the set per sequence (0: the set is empty)
  const f16_t *Kc, *Vc;
  long seq_stride;         // elements between the caches of two sequences
  int capb;
  f16_t* out;
  int nsplit_cfg, window;
};
struct AttnLevels { AttnLevel lv[3]; int S, RS; };   // sequences; rows per sequence in the q / limit / out buffers

__global__ __launch_bounds__(256) void k_attn_mfma_levels(AttnLevels L, int H, float* __restrict__ ws,
                                                           unsigned* __restrict__ counters, int defer_merge,
                                                           const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int z = blockIdx.z / L.S, sq = blockIdx.z % L.S;
  const AttnLevel A = z == 0 ? L.lv[0] : z == 1 ? L.lv[1] : L.lv[2];
  if (A.RPS == 0 || (int)blockIdx.x >= A.nsplit_cfg) return;
  attn_mfma_core<1>(A.q, A.limit, A.RPS, L.RS, A.Kc, A.Vc, A.seq_stride, A.capb, A.out, H,
                    ws + (size_t)z * L.S * H * FM_ATTN_MAX_SPLIT * (32 * 64 + 64), counters + z * L.S * H, A.nsplit_cfg,
                    defer_merge, A.window, blockIdx.x, blockIdx.y, sq);
}

// Second launch of the deferred form: one workgroup per (head, sequence) derives the split count exactly as the
// first launch did and merges; (sequence, head) pairs that fitted one split were already written there.
template <int QT, int HD = 64>
__device__ __forceinline__ void attn_merge_core(const int* __restrict__ limit, int RPS, int RS, int capb, int nsplit_cfg,
                                                f16_t* __restrict__ out, int H, const float* __restrict__ ws, int hh, int s) {
  constexpr int NQ = QT * 16;
  constexpr int PSZ = NQ * HD + 2 * NQ;
  __shared__ AttnMergeShared<QT> ms;
  const int d = H * HD;
  int maxlim = -1;
  for (int qi = 0; qi < RPS; qi++) maxlim = max(maxlim, limit[(long)s * RS + qi]);
  const int nblk = min((maxlim + 32) >> 5, capb);
  const int per = (capb + nsplit_cfg - 1) / nsplit_cfg;
  const int nsplit = max(1, (nblk + per - 1) / per);
  if (nsplit == 1) return;
  const long sh = (long)s * H + hh;
  attn_merge<QT, false, HD>(ms, ws + sh * nsplit_cfg * PSZ, nsplit, RPS, out + (long)s * RS * d + hh * HD, d);
}

template <int QT, int HD>
__global__ __launch_bounds__(256) void k_attn_merge(const int* __restrict__ limit, int RPS, int RS, int capb, int nsplit_cfg,
                                                     f16_t* __restrict__ out, int H, const float* __restrict__ ws,
                                                     const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  attn_merge_core<QT, HD>(limit, RPS, RS, capb, nsplit_cfg, out, H, ws, blockIdx.x, blockIdx.y);
}

__global__ __launch_bounds__(256) void k_attn_merge_levels(AttnLevels L, int H, const float* __restrict__ ws,
                                                            const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int z = blockIdx.y / L.S, sq = blockIdx.y % L.S;
  const AttnLevel A = z == 0 ? L.lv[0] : z == 1 ? L.lv[1] : L.lv[2];
  if (A.RPS == 0) return;
  attn_merge_core<1>(A.limit, A.RPS, L.RS, A.capb, A.nsplit_cfg, A.out, H,
                     ws + (size_t)z * L.S * H * FM_ATTN_MAX_SPLIT * (32 * 64 + 64), blockIdx.x, sq);
}

inline size_t mfma_attn_ws_floats(int S, int H, int hd = 64) {
  return (size_t)S * H * FM_ATTN_MAX_SPLIT * (32 * std::max(hd, 64) + 64);
}

template <typename T>
bool mfma_attn_launch(const MfmaRes&, const void*, const int*, int, int, const void*, const void*, long, int, void*, int,
                      const int*, bool, int, int, hipStream_t, int = 64) { return false; }

// `cap` = key capacity of the cache (positions); caches are laid out in 32-key blocks
template <>
inline bool mfma_attn_launch<f16_t>(const MfmaRes& res, const void* q, const int* limit, int rows, int RPS, const void* Kc,
                                    const void* Vc, long seq_stride, int cap, void* out, int H, const int* flag,
                                    bool dense, int key_bound, int window, hipStream_t st, int hd) {
  if (RPS < 1 || rows % RPS != 0) return false;
  if (hd != 64 && hd != 96 && hd != 128) return false;
  if (window > 0 && (cap % 32 != 0 || window > cap)) return false;     // a ring is a whole number of blocks
  const int S = rows / RPS;
  const int capb = (cap + 31) / 32;
  // The key axis is cut into fixed ranges of at least 8 blocks (two per wave), at most 64 of them, and no more than
  // give about 768 workgroups per launch (three per compute unit: measured best between 256 and 3072 for 8 x 16 and
  // 4 x 24 (sequence, head) pairs; with fewer pairs the ranges stay short).  The ranges depend on the capacity, the
  // head count and the batch size only, never on how far a sequence has grown.
  int nsplit = capb / 8;
  nsplit = nsplit < 1 ? 1 : nsplit;
  nsplit = nsplit > FM_ATTN_MAX_SPLIT ? FM_ATTN_MAX_SPLIT : nsplit;
  if (dense || res.attn_wgs > 0) {
    const int target = dense ? 768 : res.attn_wgs;
    const int want = target / (H * S) > 0 ? target / (H * S) : 1;
    nsplit = nsplit > want ? want : nsplit;
  }
  // `key_bound` is the host's upper bound on the visible keys: ranges past it hold nothing and are not launched
  const int per = (capb + nsplit - 1) / nsplit;
  const int bound_blocks = ((key_bound < cap ? key_bound : cap) + 31) / 32;
  int launched = (bound_blocks + per - 1) / per;
  launched = launched < 1 ? 1 : launched > nsplit ? nsplit : launched;
  dim3 grid(launched, H, S);
  // With many workgroups the in-kernel merge loses: every workgroup pays an agent-scope release fence (an L2
  // write-back, and those queue up per XCD).  Then the partials go out as plain stores and a second, tiny
  // launch merges them; the arithmetic is the same either way.
  const int defer = res.attn_merge == 2 ? 2 : (launched > 1 && (long)launched * H * S > 256) ? 1 : 0;
  // at most 32 query rows of a sequence per launch (16 for the wide heads, whose partial tiles would not fit the
  // LDS of a 32-row launch); longer row sets go out in chunks
  const int d = H * hd;
  const int chunk = hd == 64 ? 32 : 16;
#define FM_ATTN_GO(QTV, HDV)                                                                                       \
  {                                                                                                                \
    hipLaunchKernelGGL((k_attn_mfma<QTV, HDV>), grid, dim3(256), 0, st, qc, lc, rc, RPS, (const f16_t*)Kc, (const f16_t*)Vc, \
                       seq_stride, capb, oc, H, res.attn_ws, res.attn_counters, nsplit, defer, flag, window);     \
    if (defer == 1) hipLaunchKernelGGL((k_attn_merge<QTV, HDV>), dim3(H, S), dim3(256), 0, st, lc, rc, RPS, capb, nsplit, oc, H, res.attn_ws, flag); \
  }
  for (int r0 = 0; r0 < RPS; r0 += chunk) {
    const int rc = RPS - r0 < chunk ? RPS - r0 : chunk;
    const f16_t* qc = (const f16_t*)q + (long)r0 * d;
    const int* lc = limit + r0;
    f16_t* oc = (f16_t*)out + (long)r0 * d;
    if (hd == 96) FM_ATTN_GO(1, 96)
    else if (hd == 128) FM_ATTN_GO(1, 128)
    else if (rc <= 16) FM_ATTN_GO(1, 64)
    else FM_ATTN_GO(2, 64)
  }
#undef FM_ATTN_GO
  return true;
}

// One launch (plus the merge launch) for up to three row sets of one sequence, each with its own cache.
// `dense`, `key_bound`, `window` per set as in mfma_attn_launch.  Returns false if a set does not fit one q-tile.
// `rows` = rows of the set per sequence; q, limit and out point at the set's first row of sequence 0 in buffers with RS
// rows per sequence; S sequences.
struct AttnLevelHost {
  const void* q; const int* limit; int rows; const void *Kc, *Vc; long seq_stride; int cap; void* out; bool dense; int key_bound, window;
};
inline bool mfma_attn_launch_levels(const MfmaRes& res, const AttnLevelHost (&lv)[3], int S, int RS, int H, const int* flag,
                                    hipStream_t st) {
  AttnLevels L{};
  L.S = S; L.RS = RS;
  int gx = 1;
  long total = 0;
  for (int z = 0; z < 3; z++) {
    const AttnLevelHost& h = lv[z];
    AttnLevel& A = L.lv[z];
    A = AttnLevel{(const f16_t*)h.q, h.limit, h.rows, (const f16_t*)h.Kc, (const f16_t*)h.Vc, h.seq_stride, (h.cap + 31) / 32, (f16_t*)h.out, 1, h.window};
    if (h.rows == 0) continue;
    if (h.rows > 16) return false;
    if (h.window > 0 && (h.cap % 32 != 0 || h.window > h.cap)) return false;
    // the same partition of the key axis as mfma_attn_launch makes for one sequence
    int nsplit = A.capb / 8;
    nsplit = nsplit < 1 ? 1 : nsplit > FM_ATTN_MAX_SPLIT ? FM_ATTN_MAX_SPLIT : nsplit;
    if (h.dense || res.attn_wgs > 0) {
      const int target = h.dense ? 768 : res.attn_wgs;
      const int want = target / (H * S) > 0 ? target / (H * S) : 1;
      nsplit = nsplit > want ? want : nsplit;
    }
    A.nsplit_cfg = nsplit;
    const int per = (A.capb + nsplit - 1) / nsplit;
    const int bound_blocks = ((h.key_bound < h.cap ? h.key_bound : h.cap) + 31) / 32;
    int launched = (bound_blocks + per - 1) / per;
    launched = launched < 1 ? 1 : launched > nsplit ? nsplit : launched;
    gx = launched > gx ? launched : gx;
    total += (long)launched * H * S;
  }
  const int defer = res.attn_merge == 2 ? 2 : (gx > 1 && total > 256) ? 1 : 0;
  hipLaunchKernelGGL(k_attn_mfma_levels, dim3(gx, H, 3 * S), dim3(256), 0, st, L, H, res.attn_ws, res.attn_counters, defer, flag);
  if (defer == 1) hipLaunchKernelGGL(k_attn_merge_levels, dim3(H, 3 * S), dim3(256), 0, st, L, H, res.attn_ws, flag);
  return true;
}
