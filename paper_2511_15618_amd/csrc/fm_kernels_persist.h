// Persistent verify kernel for the half-precision path, one sequence, blocks of up to 32 tokens: the whole backbone
// forward of one verify pass is ONE launch.  Rows are handled in groups of 16 (one MFMA row tile): blocks of up to
// 16 tokens have one group per level, longer ones two at the coordinate level (template parameter QT).
//
// Why: at batch 1 a transformer block is ~10 dependent operations of 0.3-1 us of HBM time each; as
// separate launches every one costs ~4 us.  Here 256 resident workgroups walk a static schedule of
// stages (GEMM tiles, attention splits, merges, level transitions) and hand activations to each other
// through "tagged" exchange buffers: every 8-byte element carries 4 bytes of payload and a 4-byte tag
// (launch epoch, layer).  A consumer simply re-reads an element until its tag is the one it expects, so
// correctness never depends on the order in which stores become visible across XCDs, and there is no
// grid barrier.  Elements are written with agent-scope 8-byte atomic stores and read with agent-scope loads
// (8-byte atomics for single elements, 16-byte loads of two elements for bulk reads: each element still
// arrives whole), which bypass the per-XCD L2, not coherent across XCDs inside a launch.
// A workgroup that is not needed in a stage runs ahead and issues the weight loads of its next tile
// before it starts waiting, which is what keeps HBM busy across the dependency chain.
//
// Every wait is bounded (wall clock); on a time-out the kernel raises an abort word that every waiter
// polls, so all workgroups leave and the host reports an error instead of hanging.
//
// Arithmetic is kept batch-invariant exactly like the per-launch kernels: fixed 32-key blocks, fixed
// split ranges, fixed merge order, rows never mixed in a GEMM.
#pragma once
#include "fm_device.h"
#include "fm_kernels_mfma.h"
#include "fm_kernels_step.h"

typedef unsigned long long u64;

#define PK_NWG 256
#define PK_MAXSPLIT 64
#define PK_PART (16 * 64 + 32)            // per (head, split): 16x64 unnormalised O, 16 running maxima, 16 sums
#define PK_TIMEOUT_TICKS 20000000ull      // default bound of every wait: 200 ms of the 100 MHz wall clock

// A pointer read from a table in memory is generic to the compiler, and loads through it become FLAT instructions,
// which count against the LDS counter as well: every wait for an LDS read would then also wait for the weight
// or cache loads in flight.  The table therefore holds pointers that are typed as global.
#define PK_GLOBAL __attribute__((address_space(1)))
typedef const PK_GLOBAL f16_t* pk_cw_t;     // weights, condition-memory caches
typedef PK_GLOBAL f16_t* pk_w_t;            // self-attention caches (appended to by this kernel)
typedef const PK_GLOBAL float* pk_cf_t;     // gains

struct PkLayer {
  pk_cf_t g1, g2, g3;
  pk_cw_t wqkv, wo, cq, co, w1, w2;   // tiled; wqkv with rotary pairs inside one tile
  pk_w_t Kc, Vc;
  pk_cw_t Km, Vm;
  int level;      // 0 coordinate, 1 vertex, 2 face
  int tap;        // store the layer input to the level's tap ring (input of the last layer of a stack)
  int last;       // last layer of its stack: output goes to hT[stack] and to the stack's ring
  int stack;      // 0 cpre, 1 vpre, 2 face, 3 vpost, 4 cpost
};

struct PkArgs {
  const PkLayer* layers;
  int n_layers;
  int first[5], count[5];
  Dims D;
  int ff;
  float eps;
  int R[3];                 // row slots per level (<= RS)
  int RS;                   // rows the exchange buffers hold per region: 16, or 32 when the coordinate level has two row groups
  int capb[3], capbM;       // cache capacity in 32-key blocks per level / of the condition memory
  int nsplit[3], nsplitM;   // launch-time split counts (fixed partition of the key axis)
  int win[3];               // sliding window per level (0 = none); the self-attention caches are then rings of capb blocks
  const int* pos[3];
  const int* limx[3];
  const float2* cs[3];
  const int* vtok;
  float *ring_hc, *ring_hv, *ring_yf, *ring_yv;
  float* tap[3];
  const f16_t *emb, *short_cv, *short_vf, *lm;
  const float* gf;
  float* logits;
  // exchange buffers (u64 = payload | tag << 32)
  u64 *hA, *hB, *hC;        // [layers + 1][RS][d]: one region per layer, written once per launch
  u64* hT[4];               // outputs of cpre, vpre, face, vpost  [RS][d]
  u64 *xA, *xB, *xC;        // [layers (+ 1)][RS][d/2]: the same activations as hA, hB, hC rounded to half pairs, for the GEMMs
  u64 *q, *q2;              // [RS][d/2] rotated queries of the self- / cross-attention (half pairs)
  u64 *att, *att2;          // [layers][RS][d/2] attention outputs
  u64* pool;                // [2][16][d/2] pooled groups before the two shortening projections (coarse rows: at most 9)
  u64* mid;                 // [layers][RS][ff/2]
  u64 *newK, *newV;         // [H][RS][32]
  u64 *partS, *partX;       // [H][PK_MAXSPLIT][RS/16][PK_PART]
  u64* w2part;              // [d/16][RS/16][3][256]: partial tiles of the K-quarters 1..3 of the FFN down projection
  unsigned epoch;
  u64 timeout_ticks;        // bound of every wait (100 MHz wall clock)
  int two_phase;            // waits first watch one element per lane and only then read everything (0: the full read is the poll)
  unsigned test_skew;       // test hook: added to the tag the embedding publishes, so that nothing downstream ever arrives
  unsigned* abort_word;     // [0] abort flag, [1] earliest stage that gave up, [2] claim, [3..8] expected tag, tag seen,
                            // stage, workgroup, thread, element of the first missing value
  const int* run_flag;
  int prof_stage;           // stage whose inner phases are timed into prof[600..]
  u64* prof;                // optional [1 + stages]: earliest start, latest completion per stage (wall clock ticks)
};

template <int QT>
struct PkShared {
  f32x4 red[4][64];
  float ssq[4][16];
  float lo[4][16 * QT][65];
  float lm[4][16 * QT], ll[4][16 * QT];
};

__device__ __forceinline__ u64 pk_ld(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void pk_st(u64* p, unsigned payload, unsigned tag) {
  __hip_atomic_store(p, ((u64)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void pk_stf(u64* p, float v, unsigned tag) { pk_st(p, __float_as_uint(v), tag); }
__device__ __forceinline__ unsigned pk_pack(float lo, float hi) {
  const f16_t a = (f16_t)lo, b = (f16_t)hi;
  return (unsigned)__builtin_bit_cast(unsigned short, a) | ((unsigned)__builtin_bit_cast(unsigned short, b) << 16);
}
__device__ __forceinline__ bool pk_expired(const PkArgs& a, u64 t0, int stage) {
  // every waiter that gives up records its stage; the smallest one is where the chain broke
  if (__hip_atomic_load(a.abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
    atomicMin(a.abort_word + 1, (unsigned)stage);
    return true;
  }
  if (wall_clock64() - t0 > a.timeout_ticks) {
    __hip_atomic_store(a.abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    atomicMin(a.abort_word + 1, (unsigned)stage);
    return true;
  }
  return false;
}

// Wave-wide fetch of N tagged elements per lane (addresses from `addr(i)`, i < n <= N); inactive lanes get 0.
// All loads are issued before any is checked; the whole set is re-read until every tag matches.
template <int N, class F>
__device__ __forceinline__ bool pk_fetch(unsigned (&out)[N], int n, bool active, unsigned tag, F addr, const PkArgs& a, int stage) {
  const u64 t0 = wall_clock64();
  int it = 0;
  // (a.two_phase: watch one element per lane first; otherwise the full read comes first and the watching only starts
  // after a read that came back incomplete)
  auto watch = [&]() -> bool {
    while (true) {
      bool ok = true;
      if (active && n > 0) ok = (unsigned)(pk_ld(addr(0)) >> 32) == tag;
      if (__all(ok)) return true;
      if ((++it & 7) == 0 && pk_expired(a, t0, stage)) return false;
      __builtin_amdgcn_s_sleep(4);
    }
  };
  if (N > 1 && a.two_phase && !watch()) return false;
  // phase 2: read everything, again until complete
  while (true) {
    // all loads are issued back to back (the compiler keeps agent-scope loads in program order and would
    // otherwise wait for each one before the next), only then are the tags looked at
    u64 v[N];
#pragma unroll
    for (int i = 0; i < N; i++) {
      v[i] = 0;
      if (active && i < n) v[i] = pk_ld(addr(i));
    }
    bool ok = true;
#pragma unroll
    for (int i = 0; i < N; i++) {
      out[i] = (unsigned)v[i];
      if (active && i < n) ok = ok && ((unsigned)(v[i] >> 32) == tag);
    }
    if (__all(ok)) return true;
    if ((++it & 3) == 0 && pk_expired(a, t0, stage)) {
      // diagnostics of the first element found missing: expected tag, tag seen, stage, workgroup, thread
      if (!ok && atomicCAS(a.abort_word + 2, 0u, 1u) == 0u) {
        unsigned seen = 0, idx = 0;
        for (int i = 0; i < N; i++)
          if (active && i < n) { const u64 v = pk_ld(addr(i)); if ((unsigned)(v >> 32) != tag) { seen = (unsigned)(v >> 32); idx = i; break; } }
        a.abort_word[3] = tag; a.abort_word[4] = seen; a.abort_word[5] = (unsigned)stage;
        a.abort_word[6] = blockIdx.x; a.abort_word[7] = threadIdx.x; a.abort_word[8] = idx;
      }
      return false;
    }
    if (N > 1) { if (!watch()) return false; }
    else __builtin_amdgcn_s_sleep(2);
  }
}

// A level transition must not publish anything before the stack below it has finished with the shared
// exchange buffers, even when its own rows are inactive or only need data of earlier passes: it first
// waits for row 0 of the stack output from EVERY tile (a tile stores only after its last read).
__device__ __forceinline__ bool pk_wait_stack(const PkArgs& a, const u64* hT, unsigned tag, int stage, int rows);

#define PK_TAG(a, l) ((a).epoch * 64u + (unsigned)(l) + 1u)

__device__ __forceinline__ bool pk_wait_stack(const PkArgs& a, const u64* hT, unsigned tag, int stage, int rows) {
  unsigned s4[4];
  const int d = a.D.d;
  const int n = (d - (int)threadIdx.x + 255) / 256;     // columns threadIdx.x, +256, ... below d (d <= 1024)
  bool ok = pk_fetch<4>(s4, n, n > 0, tag, [&](int i) { return hT + threadIdx.x + 256 * i; }, a, stage);
  // a second row group is written by units of its own: their first row (16) as well
  if (rows > 16) ok = pk_fetch<4>(s4, n, n > 0, tag, [&](int i) { return hT + 16l * d + threadIdx.x + 256 * i; }, a, stage) && ok;
  return ok;
}

// phase timing inside the units of one chosen stage (debug): latest time each phase was reached
#define PK_MARK(k) do { if (a.prof && stage == a.prof_stage && threadIdx.x == 0) atomicMax(a.prof + 600 + (k), (u64)wall_clock64()); } while (0)

// ------------------------------------------------------------------------------------------
// GEMM tile: C[16 rows x 16 cols] = A[16 x K] * W_tile^T, four waves split K (K <= 1024), result in wave 0.
// A is a half-pair exchange buffer [16][K/2].  ASRC 1: the rows are RMS-normalised (gain g) on the fly; they are
// the half-rounded copy that the producers of the fp32 residual stream write next to it.
// Every wave takes the MFMA A-fragments of its K-quarter straight from the exchange buffer: lane (r, g) of
// fragment f needs the 8 consecutive values k0 = f*32 + g*8 .. +8 of row r, which are 32 contiguous bytes of
// tagged half pairs, i.e. two 16-byte agent-scope loads.  No LDS staging, no barrier before the multiplication;
// the tags are checked per lane and the whole set is re-read until complete.
// ------------------------------------------------------------------------------------------
template <int ASRC, class SH>
__device__ __forceinline__ bool pk_gemm_tile(const PkArgs& a, SH& sh, pk_cw_t Wt, int KT, const u64* A,
                                             unsigned tagA, pk_cf_t gain, int R, f32x4& result, int stage,
                                             int lda = 0) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  constexpr int NL = 2;       // 16-byte loads per fragment and lane
  constexpr int EF = 16;      // tagged elements (half pairs) per fragment row
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int r = lane & 15, g = lane >> 4;
  const bool on = r < R;
  const int FW = KT >> 2;                  // fragments per wave (host guarantees KT % 4 == 0, KT <= 32)
  const int K = KT * 32;
  if (lda == 0) lda = K >> 1;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  // weights and gains go out before the wait for the activations: they depend on nothing
  f16x8 wf[8];
#pragma unroll
  for (int f = 0; f < 8; f++)
    if (f < FW) wf[f] = *(const PK_GLOBAL f16x8*)(Wt + ((long)(wave * FW + f) * 64 + lane) * 8);
  f32x4 gl[ASRC == 1 ? 16 : 1];
  if (ASRC == 1) {
#pragma unroll
    for (int f = 0; f < 8; f++)
      if (f < FW) {
        const pk_cf_t gp = gain + (wave * FW + f) * 32 + g * 8;
        gl[2 * f] = *(const PK_GLOBAL f32x4*)gp;
        gl[2 * f + 1] = *(const PK_GLOBAL f32x4*)(gp + 4);
      }
  }
  // this wave's part of the rows: element (wave*FW + f)*EF + g*(EF/4) of row r is where fragment f starts
  const u64* Aw = A + (long)(wave * FW) * EF;
  const u64* mine = Aw + (long)min(r, R - 1) * lda + g * (EF / 4);
  const u64 t0 = wall_clock64();
  int it = 0;
  bool good = true;
  // The full fragment read is its own validity check, so a unit whose input is already there pays one round trip.
  // When a read comes back incomplete the wave falls back to watching one element per lane (lane l: fragment l/8, its
  // first or second half - a producer tile owns half a fragment row - in one of the last four rows) and reads the
  // fragments again once those show the tag: waiting costs the memory system 64 small loads per round, not 32 KiB.
  const int fs_ = min(lane >> 3, FW - 1), hs_ = (lane >> 2) & 1, rs_ = max(R - 1 - (lane & 3), 0);
#define PK_WATCH(AW)                                                                                          \
  {                                                                                                           \
    const u64* sent = (AW) + (long)rs_ * lda + fs_ * EF + hs_ * (EF / 2);                                     \
    while (good) {                                                                                            \
      const bool okw = (unsigned)(pk_ld(sent) >> 32) == tagA;                                                 \
      if (__all(okw)) break;                                                                                  \
      if ((++it & 7) == 0 && pk_expired(a, t0, stage)) { good = false; break; }                               \
      __builtin_amdgcn_s_sleep(4);                                                                            \
    }                                                                                                         \
  }
  if (a.two_phase) PK_WATCH(Aw)
  PK_MARK(1);
  // phase 2: the fragments (inline asm loads: the wait is explicit, and every destination is passed through
  // an empty asm afterwards to pin its uses behind the wait)
  u32x4 v[8 * NL];
#define PK_FETCH_FRAGS(MINE, AW)                                                                              \
  while (good) {                                                                                              \
    _Pragma("unroll") for (int f = 0; f < 8; f++) {                                                           \
      _Pragma("unroll") for (int j = 0; j < NL; j++) {                                                        \
        v[f * NL + j] = u32x4{tagA, tagA, tagA, tagA};                                                        \
        if (f < FW && on) {                                                                                   \
          const u64* p = (MINE) + f * EF + 2 * j;                                                             \
          asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v[f * NL + j]) : "v"(p) : "memory");      \
        }                                                                                                     \
      }                                                                                                       \
    }                                                                                                         \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                                          \
    bool ok = true;                                                                                           \
    _Pragma("unroll") for (int i = 0; i < 8 * NL; i++) {                                                      \
      asm volatile("" : "+v"(v[i]));                                                                          \
      ok = ok && v[i][1] == tagA && v[i][3] == tagA;      /* unused slots were preset to the tag */           \
    }                                                                                                         \
    if (__all(ok)) break;                                                                                     \
    if ((++it & 3) == 0 && pk_expired(a, t0, stage)) { good = false; break; }                                 \
    PK_WATCH(AW)                                                                                              \
  }
  PK_FETCH_FRAGS(mine, Aw)
  PK_MARK(2);
  if (ASRC == 1) {
    // RMSNorm without a barrier in front of the multiplication: the MFMA runs on half(x * gain) and the per-row
    // factor 1/rms, a scalar per output row, is applied to the accumulated tile afterwards.  Row sums of
    // squares: this lane's 8*FW values, then the four k-groups of the wave; the four waves meet in LDS below.
    float ss = 0.f;
#pragma unroll
    for (int f = 0; f < 8; f++) {
      if (f < FW) {
        u32x4 pk = u32x4{0u, 0u, 0u, 0u};
        if (on && good) pk = u32x4{v[2 * f][0], v[2 * f][2], v[2 * f + 1][0], v[2 * f + 1][2]};
        const f16x8 xh = __builtin_bit_cast(f16x8, pk);
        f16x8 av;
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const float x = (float)xh[j];
          ss += x * x;
          av[j] = (f16_t)(x * gl[2 * f + (j >> 2)][j & 3]);
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, wf[f], acc, 0, 0, 0);
      }
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (g == 0) sh.ssq[wave][r] = ss;
  } else {
#pragma unroll
    for (int f = 0; f < 8; f++) {
      if (f < FW) {
        u32x4 pk = u32x4{0u, 0u, 0u, 0u};
        if (on && good) pk = u32x4{v[2 * f][0], v[2 * f][2], v[2 * f + 1][0], v[2 * f + 1][2]};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, pk), wf[f], acc, 0, 0, 0);
      }
    }
  }
#undef PK_FETCH_FRAGS
#undef PK_WATCH
  sh.red[wave][lane] = acc;
  if (__syncthreads_or(!good)) return false;
  PK_MARK(3);
  if (wave == 0) {
    result = sh.red[0][lane] + sh.red[1][lane] + sh.red[2][lane] + sh.red[3][lane];
    if (ASRC == 1) {
#pragma unroll
      for (int i = 0; i < 4; i++) {      // result[i] belongs to row g*4 + i
        const int row = g * 4 + i;
        const float tot = sh.ssq[0][row] + sh.ssq[1][row] + sh.ssq[2][row] + sh.ssq[3][row];
        result[i] *= 1.0f / sqrtf(tot / (float)K + a.eps);
      }
    }
  }
  return true;
}

// residual epilogue (wave 0): out[r][n] = old[r][n] + c; optional copies into position-indexed rings
// The residual operand of a tile (complete long before the tile's GEMM input is) is fetched by wave 0 at the
// start of the unit, so that its latency hides behind the wait for the GEMM input.
__device__ __forceinline__ bool pk_res_prefetch(const PkArgs& a, int nt, const u64* hold, unsigned tag_old, int R,
                                                const int* pos, unsigned (&old)[4], int (&prow)[4], int stage) {
  const int lane = threadIdx.x & 63, g = lane >> 4, n = nt * 16 + (lane & 15);
  const int d = a.D.d;
#pragma unroll
  for (int i = 0; i < 4; i++) prow[i] = pos[min(g * 4 + i, R - 1)];    // positions of the lane's rows, for the ring copies
  return pk_fetch<4>(old, 4, true, tag_old, [&](int i) { return hold + (long)min(g * 4 + i, R - 1) * d + n; }, a, stage);
}

__device__ __forceinline__ void pk_epi_residual(const PkArgs& a, const f32x4& c, int nt, const unsigned (&old)[4],
                                                u64* hout, u64* xout, unsigned tag_out, int R, const int (&prow)[4],
                                                float* tap_ring, float* out_ring, int ring_size) {
  const int lane = threadIdx.x & 63, g = lane >> 4, n = nt * 16 + (lane & 15);
  const int d = a.D.d;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int r = g * 4 + i;
    if (r < R) {
      const float ho = __uint_as_float(old[i]);
      const float v = ho + c[i];
      pk_stf(hout + (long)r * d + n, v, tag_out);
      if (xout) {        // half-pair copy for the GEMM that normalises this row next (r < R holds for the lane pair alike)
        const float w = __shfl_xor(v, 1, 64);
        if ((lane & 1) == 0) pk_st(xout + (long)r * (d >> 1) + (n >> 1), pk_pack(v, w), tag_out);
      }
      const int p = prow[i];
      if (p >= 0) {
        if (tap_ring) tap_ring[(long)(p & (ring_size - 1)) * d + n] = ho;
        if (out_ring) out_ring[(long)(p & (ring_size - 1)) * d + n] = v;
      }
    }
  }
}

// half-pair epilogue (wave 0): dst[r][n/2] = (c[n], c[n+1]) as halves, optional GELU
__device__ __forceinline__ void pk_epi_half(const f32x4& c, int nt, u64* dst, int ld2, unsigned tag, int R, bool gelu) {
  const int lane = threadIdx.x & 63, g = lane >> 4, n = nt * 16 + (lane & 15);
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const float v = gelu ? gelu_tanh_f(c[i]) : c[i];
    const float w = __shfl_xor(v, 1, 64);
    const int r = g * 4 + i;
    if ((lane & 1) == 0 && r < R) {
      pk_st(dst + (long)r * ld2 + (n >> 1), pk_pack(v, w), tag);
    }
  }
}

// QKV epilogue (wave 0).  Tiles of the q and k parts hold 8 rotary pairs: columns 0..7 = dims qd*8.., columns
// 8..15 = the same dims + 32.  q -> exchange buffer; k, v -> cache (for later passes) and exchange buffers.
struct PkQkvPre {     // what the QKV epilogue needs besides the tile: requested before the tile's input arrives
  float2 t[4];        // rotary (cos, sin) of the lane's pair for its four rows
  int p[4];           // positions of those rows
};
__device__ __forceinline__ void pk_qkv_prefetch(int nt, int d, int R, const int* pos, const float2* cs, PkQkvPre& pre) {
  const int lane = threadIdx.x & 63, g = lane >> 4, col = lane & 15;
  const int part = (nt * 16) / d, cp = (nt * 16) % d;
  const int qd = (cp & 63) >> 4;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int rr = min(g * 4 + i, R - 1);
    pre.p[i] = pos[rr];
    pre.t[i] = part < 2 ? cs[(long)rr * 32 + qd * 8 + (col & 7)] : float2{1.f, 0.f};
  }
}
template <int QT>
__device__ __forceinline__ void pk_epi_qkv(const PkArgs& a, const PkLayer& L, const f32x4& c, int nt, unsigned tag, int R,
                                           const PkQkvPre& pre, int capb, int row0) {
  const int lane = threadIdx.x & 63, g = lane >> 4, col = lane & 15;
  const int d = a.D.d;
  const int part = (nt * 16) / d, cp = (nt * 16) % d;
  const int hh = cp >> 6, qd = (cp & 63) >> 4;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int r = g * 4 + i;
    float v = c[i];
    int dim;
    if (part < 2) {
      const int j = qd * 8 + (col & 7);
      const float2 t = pre.t[i];
      const float o = __shfl_xor(v, 8, 64);
      v = col < 8 ? v * t.x - o * t.y : v * t.x + o * t.y;
      dim = col < 8 ? j : j + 32;
    } else {
      dim = qd * 16 + col;
    }
    const float w = __shfl_xor(v, 1, 64);       // neighbour dim (dim ^ 1 sits in lane ^ 1 in every layout above)
    const int p = pre.p[i];
    if (r < R) {
      if (part == 0) {
        if ((lane & 1) == 0) pk_st(a.q + (long)(row0 + r) * (d >> 1) + ((hh * 64 + dim) >> 1), pk_pack(v, w), tag);
      } else {
        u64* nb = (part == 1 ? a.newK : a.newV) + ((long)hh * (QT * 16) + row0 + r) * 32;
        if ((lane & 1) == 0) pk_st(nb + (dim >> 1), pk_pack(v, w), tag);
        if (p >= 0) {
          const int ps = p % (capb * 32);      // the cache is a ring when a window is set
          const long base = (long)hh * capb * 2048;
          if (part == 1) L.Kc[base + kblk_off(ps, dim)] = (f16_t)v;
          else L.Vc[base + vblk_off(ps, dim)] = (f16_t)v;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Attention over one key range of one head (flash-decoding split), same arithmetic as k_attn_mfma<QT>: QT tiles of
// 16 query rows share every K/V block that is loaded.  Keys of this pass (positions >= P0) are taken from the
// exchange buffers, older keys from the cache.  lim[t]: last key the lane's row of tile t may see (-1: unused slot).
// Partial results: tile t of (head, split) at part + t * PK_PART.
// ------------------------------------------------------------------------------------------
template <int QT, class SH>
__device__ __forceinline__ bool pk_attn_unit(const PkArgs& a, SH& sh, const u64* qbuf, const int (&lim)[QT], int maxlim, int R,
                                             pk_cw_t Kc, pk_cw_t Vc, int capb, int nsplit_cfg, int hh, int split,
                                             bool overlay, int P0, u64* part, unsigned tag, int stage, int window) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int g = lane >> 4, ql = lane & 15;
  const int d = a.D.d;
  const float kScale = 0.125f * 1.4426950408889634f;
  // With a window the cache is a ring of capb blocks (a multiple of four): position p lives in slot p mod (32 capb);
  // seen from the newest visible position, slot j holds lapbase + j if that is <= maxlim, else the position one
  // lap earlier.  Without a window lapbase = 0 and nothing wraps.
  const int nblk = min((maxlim + 32) >> 5, capb);
  const int ringn = capb * 32;
  const int lapbase = max(maxlim, 0) / ringn * ringn;
  auto held = [&](int slot) { const int k = lapbase + slot; return k > maxlim ? k - ringn : k; };
  bool on[QT];
  int first[QT];
#pragma unroll
  for (int t = 0; t < QT; t++) {
    on[t] = t * 16 + ql < R;
    first[t] = window > 0 ? max(lim[t] - window + 1, 0) : 0;
  }
  const int per = (capb + nsplit_cfg - 1) / nsplit_cfg;
  const int nsplit = max(1, (nblk + per - 1) / per);
  if (split >= nsplit) return true;      // nothing visible in this range: the merge knows the same count
  const int b0 = split * per, b1 = min(b0 + per, nblk);

  // The wave's query fragments and, if one of its blocks holds rows written by this pass, those rows, in ONE
  // batch.  K fragment f = (hb, dh) holds key b*32 + hb*16 + lane%16, dims dh*32 + g*8..+8 (4 elements);
  // V fragment dt holds dim dt*16 + lane%16 and the 8 slots g*8 + j <-> key b*32 + (j/4)*16 + g*4 + j%4.
  int bov = -1;
  if (overlay) {
    const int cand[2] = {(P0 % ringn) >> 5, ((P0 + R - 1) % ringn) >> 5};     // slot blocks of the rows of this pass
#pragma unroll
    for (int k = 0; k < 2; k++) {
      const int b = cand[k];
      if (b >= b0 + wave && b < b1 && ((b - b0 - wave) & 3) == 0) bov = b;
    }
  }
  // the first K/V block of this wave depends on nothing from this pass: request it before waiting for q
  pk_cw_t Kb = Kc + (long)hh * capb * 2048;
  pk_cw_t Vb = Vc + (long)hh * capb * 2048;
  f16x8 kf[4], vf[4];
  if (b0 + wave < b1) {
    pk_cw_t kp = Kb + (long)(b0 + wave) * 2048 + lane * 8;
    pk_cw_t vp = Vb + (long)(b0 + wave) * 2048 + (lane & 15) * 32 + g * 8;
#pragma unroll
    for (int f = 0; f < 4; f++) kf[f] = *(const PK_GLOBAL f16x8*)(kp + f * 512);
#pragma unroll
    for (int dt = 0; dt < 4; dt++) vf[dt] = *(const PK_GLOBAL f16x8*)(vp + dt * 512);
  }
  // q of this lane: dims g*8..+8 and 32 + g*8..+8 of the head = two runs of four tagged elements = four 16-byte
  // agent-scope loads per query tile, simply repeated until every tag matches (small enough to poll with the data itself)
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  f16x8 qf0[QT], qf1[QT];
  bool ok = true;
  {
    const u64* qp[QT];
#pragma unroll
    for (int t = 0; t < QT; t++) qp[t] = qbuf + (long)(on[t] ? t * 16 + ql : 0) * (d >> 1) + ((hh * 64 + g * 8) >> 1);
    const u64 t0 = wall_clock64();
    int it = 0;
    u32x4 qv[QT][4];
    while (true) {
#pragma unroll
      for (int t = 0; t < QT; t++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const u64* p = qp[t] + (j >> 1) * 16 + (j & 1) * 2;
          asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(qv[t][j]) : "v"(p) : "memory");
        }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      bool okq = true;
#pragma unroll
      for (int t = 0; t < QT; t++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          asm volatile("" : "+v"(qv[t][j]));
          okq = okq && qv[t][j][1] == tag && qv[t][j][3] == tag;
        }
      if (__all(okq)) break;
      if ((++it & 7) == 0 && pk_expired(a, t0, stage)) { ok = false; break; }
    }
#pragma unroll
    for (int t = 0; t < QT; t++) {
      u32x4 lo4 = u32x4{qv[t][0][0], qv[t][0][2], qv[t][1][0], qv[t][1][2]};
      u32x4 hi4 = u32x4{qv[t][2][0], qv[t][2][2], qv[t][3][0], qv[t][3][2]};
      if (!on[t]) { lo4 = u32x4{0u, 0u, 0u, 0u}; hi4 = lo4; }
      qf0[t] = __builtin_bit_cast(f16x8, lo4);
      qf1[t] = __builtin_bit_cast(f16x8, hi4);
    }
  }
  // rows written by this pass that fall into one of this wave's blocks (at most one block)
  unsigned raw[48];
  if (bov >= 0) {
    ok = pk_fetch<48>(raw, 48, true, tag, [&](int i) {
      if (i < 16) {
        const int f = i >> 2;
        int nr = held(bov * 32 + (f >> 1) * 16 + (lane & 15)) - P0;
        nr = nr < 0 ? 0 : (nr >= R ? R - 1 : nr);
        return (const u64*)(a.newK + ((long)hh * (QT * 16) + nr) * 32 + (((f & 1) * 32 + g * 8) >> 1) + (i & 3));
      }
      const int j = (i - 16) & 7, dt = (i - 16) >> 3;
      int nr = held(bov * 32 + (j >> 2) * 16 + g * 4 + (j & 3)) - P0;
      nr = nr < 0 ? 0 : (nr >= R ? R - 1 : nr);
      return (const u64*)(a.newV + ((long)hh * (QT * 16) + nr) * 32 + ((dt * 16 + (lane & 15)) >> 1));
    }, a, stage) && ok;
  }

  float mrun[QT], lrun[QT];
  f32x4 o[QT][4];
#pragma unroll
  for (int t = 0; t < QT; t++) {
    mrun[t] = -INFINITY;
    lrun[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  for (int b = b0 + wave; b < b1; b += 4) {
    // the next block of this wave is requested before the current one is multiplied
    f16x8 kn[4], vn[4];
    if (b + 4 < b1) {
      pk_cw_t kp = Kb + (long)(b + 4) * 2048 + lane * 8;
      pk_cw_t vp = Vb + (long)(b + 4) * 2048 + (lane & 15) * 32 + g * 8;
#pragma unroll
      for (int f = 0; f < 4; f++) kn[f] = *(const PK_GLOBAL f16x8*)(kp + f * 512);
#pragma unroll
      for (int dt = 0; dt < 4; dt++) vn[dt] = *(const PK_GLOBAL f16x8*)(vp + dt * 512);
    }
    if (b == bov) {
#pragma unroll
      for (int f = 0; f < 4; f++) {
        const int nr = held(b * 32 + (f >> 1) * 16 + (lane & 15)) - P0;
        if (nr >= 0 && nr < R) kf[f] = __builtin_bit_cast(f16x8, (u32x4{raw[f * 4], raw[f * 4 + 1], raw[f * 4 + 2], raw[f * 4 + 3]}));
      }
#pragma unroll
      for (int dt = 0; dt < 4; dt++) {
        const int dim = dt * 16 + (lane & 15);
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const int nr = held(b * 32 + (j >> 2) * 16 + g * 4 + (j & 3)) - P0;
          if (nr >= 0 && nr < R) {
            const unsigned w = raw[16 + dt * 8 + j];
            const unsigned short hbits = (dim & 1) ? (unsigned short)(w >> 16) : (unsigned short)(w & 0xFFFFu);
            vf[dt][j] = __builtin_bit_cast(f16_t, hbits);
          }
        }
      }
    }
#pragma unroll
    for (int t = 0; t < QT; t++) {
      f32x4 sT[2];
#pragma unroll
      for (int hb = 0; hb < 2; hb++) {
        f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
        z = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[hb * 2], qf0[t], z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[hb * 2 + 1], qf1[t], z, 0, 0, 0);
        sT[hb] = z;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int hb = 0; hb < 2; hb++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int key = held(b * 32 + hb * 16 + g * 4 + i);      // absolute position
          const float v = (key <= lim[t] && key >= first[t]) ? sT[hb][i] * kScale : -INFINITY;
          sT[hb][i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(mrun[t], mx);
      const float msafe = mnew == -INFINITY ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f(mrun[t] - msafe);
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
      for (int dt = 0; dt < 4; dt++) {
        o[t][dt] *= alpha;
        o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[dt], pf, o[t][dt], 0, 0, 0);
      }
    }
    if (b + 4 < b1) {
#pragma unroll
      for (int f = 0; f < 4; f++) { kf[f] = kn[f]; vf[f] = vn[f]; }
    }
  }
#pragma unroll
  for (int t = 0; t < QT; t++) {
    float l = lrun[t];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (g == 0) { sh.lm[wave][t * 16 + ql] = mrun[t]; sh.ll[wave][t * 16 + ql] = l; }
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int i = 0; i < 4; i++) sh.lo[wave][t * 16 + ql][dt * 16 + g * 4 + i] = o[t][dt][i];
  }
  if (__syncthreads_or(!ok)) return false;
  for (int e = threadIdx.x; e < QT * 16 * 64; e += 256) {
    const int qi = e >> 6, dim = e & 63;
    const float M = fmaxf(fmaxf(sh.lm[0][qi], sh.lm[1][qi]), fmaxf(sh.lm[2][qi], sh.lm[3][qi]));
    const float Ms = M == -INFINITY ? 0.f : M;
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float f = __builtin_amdgcn_exp2f(sh.lm[w][qi] - Ms);
      num += sh.lo[w][qi][dim] * f;
      den += sh.ll[w][qi] * f;
    }
    if (qi < R) {
      u64* pt = part + (long)(qi >> 4) * PK_PART;      // the row's tile
      const int ql16 = qi & 15;
      pk_stf(pt + ql16 * 64 + dim, num, tag);
      if (dim == 0) { pk_stf(pt + 16 * 64 + ql16, M, tag); pk_stf(pt + 16 * 64 + 16 + ql16, den, tag); }
    }
  }
  __syncthreads();
  return true;
}

// merge of the splits of one head (one quarter of its dims per unit) into the half-pair attention output;
// thread = (row, dim), splits summed in a fixed order
// (rg: the row group, R: its rows; the split count comes from the largest limit of the whole level, as in the units
// that wrote the partial results)
template <int QT>
__device__ __forceinline__ bool pk_merge_unit(const PkArgs& a, int maxlim, int R, int rg, int capb, int nsplit_cfg,
                                              int hh, int dq, const u64* parts, u64* att, unsigned tag, int stage) {
  const int d = a.D.d;
  const int nblk = min((maxlim + 32) >> 5, capb);
  const int per = (capb + nsplit_cfg - 1) / nsplit_cfg;
  const int nsplit = max(1, (nblk + per - 1) / per);
  const long rec = (long)QT * PK_PART;                 // one (head, split) record: a tile per row group
  const u64* base = parts + (long)hh * PK_MAXSPLIT * rec + (long)rg * PK_PART;
  const int qi = threadIdx.x >> 4, dim = dq * 16 + (threadIdx.x & 15);
  const bool on = qi < R;
  bool ok = true;
  // splits are folded in a fixed order, 16 at a time, with the usual running-maximum rescale
  float M = -INFINITY, num = 0.f, den = 0.f;
  for (int k0 = 0; k0 < nsplit; k0 += 16) {
    unsigned raw[48];
    const int n = min(16, nsplit - k0);
    ok = pk_fetch<48>(raw, 3 * n, on, tag, [&](int i) {
      const u64* p = base + (long)(k0 + i / 3) * rec;
      const int w = i % 3;
      return w == 0 ? p + 16 * 64 + qi : w == 1 ? p + 16 * 64 + 16 + qi : p + qi * 64 + dim;
    }, a, stage) && ok;
    float Mc = M;
#pragma unroll
    for (int i = 0; i < 16; i++) if (i < n && on) Mc = fmaxf(Mc, __uint_as_float(raw[3 * i]));
    const float Ms = Mc == -INFINITY ? 0.f : Mc;
    const float scale = __builtin_amdgcn_exp2f(M - Ms);     // exp2(-inf) = 0 for the first chunk
    num *= scale;
    den *= scale;
    M = Mc;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      if (i < n && on) {
        const float f = __builtin_amdgcn_exp2f(__uint_as_float(raw[3 * i]) - Ms);
        den += __uint_as_float(raw[3 * i + 1]) * f;
        num += __uint_as_float(raw[3 * i + 2]) * f;
      }
    }
  }
  const float v = den > 0.f ? num / den : 0.f;
  const float w = __shfl_xor(v, 1, 64);
  if (on && (dim & 1) == 0) pk_st(att + (long)(rg * 16 + qi) * (d >> 1) + ((hh * 64 + dim) >> 1), pk_pack(v, w), tag);
  if (__syncthreads_or(!ok)) return false;
  return true;
}

// ------------------------------------------------------------------------------------------
// The kernel
// ------------------------------------------------------------------------------------------
#define PK_MINE(units) for (int u = (int)((blockIdx.x + PK_NWG - (rr % PK_NWG)) % PK_NWG); u < (units) && (worked = true); u += PK_NWG)
#define PK_NEXT(units)                                                                              \
  do {                                                                                              \
    if (a.prof && worked && threadIdx.x == 0) atomicMax(a.prof + 1 + stage, (u64)wall_clock64());   \
    worked = false;                                                                                 \
    rr += (units);                                                                                  \
    stage++;                                                                                        \
  } while (0)

template <int QT>
__global__ __launch_bounds__(256) void k_verify_persist(PkArgs a) {
  if (*a.run_flag == 0) return;
  __shared__ PkShared<QT> sh;
  const int RS = QT * 16, RH = QT * 8;     // rows of an exchange region (= a.RS), and half of it: the row count of a half-pair region in units of d
  const int d = a.D.d, H = a.D.H, ff = a.ff;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned rr = 0;     // round-robin origin of the current stage (same in every workgroup)
  int stage = 0;
  bool worked = false;
  if (a.prof && threadIdx.x == 0) atomicMin(a.prof, (u64)wall_clock64());

  // Per level and the same for all of its layers: the last visible key of this lane's query row in the
  // self-attention (its own position) and in the cross-attention, the block maxima, the first position of the pass.
  // (QT query tiles of 16 rows: tile t holds rows t*16 .. t*16+15 of the level)
  int limS[3][QT], limX[3][QT], maxS[3], maxX[3], firstP[3];
#pragma unroll
  for (int lv = 0; lv < 3; lv++) {
    const int ql = threadIdx.x & 15;
    int ms = -1, mx = -1, fp = 0x3fffffff;
#pragma unroll
    for (int t = 0; t < QT; t++) {
      const bool onl = t * 16 + ql < a.R[lv];
      limS[lv][t] = onl ? a.pos[lv][t * 16 + ql] : -1;
      limX[lv][t] = onl ? a.limx[lv][t * 16 + ql] : -1;
      ms = max(ms, limS[lv][t]);
      mx = max(mx, limX[lv][t]);
      if (limS[lv][t] >= 0) fp = min(fp, limS[lv][t]);
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      ms = max(ms, __shfl_xor(ms, o, 64));
      mx = max(mx, __shfl_xor(mx, o, 64));
      fp = min(fp, __shfl_xor(fp, o, 64));
    }
    maxS[lv] = ms; maxX[lv] = mx; firstP[lv] = fp;
  }

  // ---- embedding: one unit per coordinate row -> hA of layer 0
  PK_MINE(a.R[0]) {
    const int r = u;
    const bool onr = a.pos[0][r] >= 0;
    const f16_t* e = a.emb + (long)a.vtok[r] * d;
    for (int i = threadIdx.x; i < d; i += 256) {     // region of layer 0, and its half-pair copy (d is a multiple of 128)
      const float v = onr ? (float)e[i] : 0.f;
      pk_stf(a.hA + (long)r * d + i, v, PK_TAG(a, 0) + a.test_skew);
      const float w = __shfl_xor(v, 1, 64);
      if ((i & 1) == 0) pk_st(a.xA + (long)r * (d >> 1) + (i >> 1), pk_pack(v, w), PK_TAG(a, 0) + a.test_skew);
    }
  }
  PK_NEXT(a.R[0]);

  for (int st = 0; st < 5; st++) {
    for (int li = 0; li < a.count[st]; li++) {
      const int l = a.first[st] + li;
      const PkLayer& L = a.layers[l];
      const int lev = L.level, R = a.R[lev];
      const unsigned tag = PK_TAG(a, l);
      const int* pos = a.pos[lev];
      const int capb = a.capb[lev];
      // this layer's own regions of the exchange buffers
      u64* const hA_l = a.hA + (long)l * RS * d;
      u64* const hA_n = a.hA + (long)(l + 1) * RS * d;
      u64* const hB_l = a.hB + (long)l * RS * d;
      u64* const hC_l = a.hC + (long)l * RS * d;
      u64* const xA_l = a.xA + (long)l * RH * d;
      u64* const xA_n = a.xA + (long)(l + 1) * RH * d;
      u64* const xB_l = a.xB + (long)l * RH * d;
      u64* const xC_l = a.xC + (long)l * RH * d;
      u64* const att_l = a.att + (long)l * RH * d;
      u64* const att2_l = a.att2 + (long)l * RH * d;
      u64* const mid_l = a.mid + (long)l * RH * ff;
      // GEMM and merge units take the rows in groups of 16: unit = (tile, row group); a group's rows are contiguous
      // in every exchange buffer, so a unit is the one-group code on offset pointers
      const int RG = QT == 1 ? 1 : (R + 15) >> 4;      // a compile-time 1 for blocks of up to 16 tokens
      const long hd = d >> 1;
      // ---- QKV (norm1 on the fly, rotary, q / new K,V out, cache append)
      PK_MINE(3 * d / 16 * RG) {
        const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
        f32x4 c;
        PkQkvPre pre;
        if (wave == 0) pk_qkv_prefetch(nt, d, Rl, pos + row0, a.cs[lev] + (long)row0 * 32, pre);
        if (!pk_gemm_tile<1>(a, sh, L.wqkv + (long)nt * (d / 32) * 512, d / 32, xA_l + row0 * hd, tag, L.g1, Rl, c, stage)) return;
        if (wave == 0) pk_epi_qkv<QT>(a, L, c, nt, tag, Rl, pre, capb, row0);
        __syncthreads();
      }
      PK_NEXT(3 * d / 16 * RG);
      // ---- self-attention splits
      {
        const int ns = a.nsplit[lev];
        const int P0 = firstP[lev];
        PK_MINE(H * ns) {
          // range-major: the ranges that hold keys come first, so that with more ranges than a workgroup can take at once
          // the non-empty ones still spread over all workgroups
          const int hh = u % H, sp = u / H;
          if (!pk_attn_unit<QT>(a, sh, a.q, limS[lev], maxS[lev], R, L.Kc, L.Vc, capb, ns, hh, sp, true, P0,
                                a.partS + ((long)hh * PK_MAXSPLIT + sp) * (RS >> 4) * PK_PART, tag, stage, a.win[lev])) return;
        }
        PK_NEXT(H * ns);
        PK_MINE(4 * H * RG) {
          const int v = u / RG, rg = u % RG;
          if (!pk_merge_unit<QT>(a, maxS[lev], min(16, R - rg * 16), rg, capb, ns, v >> 2, v & 3, a.partS, att_l, tag, stage)) return;
        }
        PK_NEXT(4 * H * RG);
      }
      // ---- Wo + residual -> hB (tap: the layer input is what the draft heads of this level start from)
      PK_MINE(d / 16 * RG) {
        const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
        f32x4 c;
        unsigned old[4];
        int prow[4];
        bool okr = true;
        if (wave == 0) okr = pk_res_prefetch(a, nt, hA_l + (long)row0 * d, tag, Rl, pos + row0, old, prow, stage);
        if (!pk_gemm_tile<0>(a, sh, L.wo + (long)nt * (d / 32) * 512, d / 32, att_l + row0 * hd, tag, nullptr, Rl, c, stage)) return;
        if (wave == 0 && okr)
          pk_epi_residual(a, c, nt, old, hB_l + (long)row0 * d, xB_l + row0 * hd, tag, Rl, prow, L.tap ? a.tap[lev] : nullptr, nullptr,
                          lev == 0 ? 32 : lev == 1 ? 16 : 8);
        if (__syncthreads_or(!okr)) return;
      }
      PK_NEXT(d / 16 * RG);
      // ---- cross-attention query (norm2 on the fly)
      PK_MINE(d / 16 * RG) {
        const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
        f32x4 c;
        if (!pk_gemm_tile<1>(a, sh, L.cq + (long)nt * (d / 32) * 512, d / 32, xB_l + row0 * hd, tag, L.g2, Rl, c, stage)) return;
        if (wave == 0) pk_epi_half(c, nt, a.q2 + row0 * hd, d >> 1, tag, Rl, false);
        __syncthreads();
      }
      PK_NEXT(d / 16 * RG);
      // ---- cross-attention over the condition memory
      {
        const int ns = a.nsplitM;
        PK_MINE(H * ns) {
          const int hh = u / ns, sp = u % ns;
          if (!pk_attn_unit<QT>(a, sh, a.q2, limX[lev], maxX[lev], R, L.Km, L.Vm, a.capbM, ns, hh, sp, false, 0,
                                a.partX + ((long)hh * PK_MAXSPLIT + sp) * (RS >> 4) * PK_PART, tag, stage, 0)) return;
        }
        PK_NEXT(H * ns);
        PK_MINE(4 * H * RG) {
          const int v = u / RG, rg = u % RG;
          if (!pk_merge_unit<QT>(a, maxX[lev], min(16, R - rg * 16), rg, a.capbM, ns, v >> 2, v & 3, a.partX, att2_l, tag, stage)) return;
        }
        PK_NEXT(4 * H * RG);
      }
      // ---- cross output projection + residual -> hC
      PK_MINE(d / 16 * RG) {
        const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
        f32x4 c;
        unsigned old[4];
        int prow[4];
        bool okr = true;
        if (wave == 0) okr = pk_res_prefetch(a, nt, hB_l + (long)row0 * d, tag, Rl, pos + row0, old, prow, stage);
        if (!pk_gemm_tile<0>(a, sh, L.co + (long)nt * (d / 32) * 512, d / 32, att2_l + row0 * hd, tag, nullptr, Rl, c, stage)) return;
        if (wave == 0 && okr) pk_epi_residual(a, c, nt, old, hC_l + (long)row0 * d, xC_l + row0 * hd, tag, Rl, prow, nullptr, nullptr, 8);
        if (__syncthreads_or(!okr)) return;
      }
      PK_NEXT(d / 16 * RG);
      // ---- FFN up (norm3 on the fly, GELU)
      PK_MINE(ff / 16 * RG) {
        const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
        f32x4 c;
        if (!pk_gemm_tile<1>(a, sh, L.w1 + (long)nt * (d / 32) * 512, d / 32, xC_l + row0 * hd, tag, L.g3, Rl, c, stage)) return;
        if (wave == 0) pk_epi_half(c, nt, mid_l + (long)row0 * (ff >> 1), ff >> 1, tag, Rl, true);
        __syncthreads();
      }
      PK_NEXT(ff / 16 * RG);
      // ---- FFN down + residual -> next layer input, or the stack output (+ its ring for later passes).
      // K = ff is four times longer than in the other GEMMs, so a tile is computed by four units, one per
      // K-quarter; quarters 1..3 hand their partial tile to quarter 0, which adds them in a fixed order.
      PK_MINE(4 * (d / 16) * RG) {
        const int uv = u / RG, rg = u % RG, row0 = rg * 16, Rl = min(16, R - row0);
        const int nt = uv >> 2, kq = uv & 3;
        const int KTq = ff / 128;                       // fragments of one K-quarter
        u64* const w2p = a.w2part + ((long)nt * RG + rg) * 3 * 256;
        f32x4 c;
        unsigned old[4];
        int prow[4];
        bool okr = true;
        if (wave == 0 && kq == 0) okr = pk_res_prefetch(a, nt, hC_l + (long)row0 * d, tag, Rl, pos + row0, old, prow, stage);
        if (!pk_gemm_tile<0>(a, sh, L.w2 + ((long)nt * (ff / 32) + (long)kq * KTq) * 512, KTq,
                             mid_l + (long)row0 * (ff >> 1) + (long)kq * (ff / 8), tag, nullptr, Rl, c, stage, ff >> 1)) return;
        if (wave == 0) {
          const int lane = threadIdx.x & 63;
          if (kq > 0) {
#pragma unroll
            for (int i = 0; i < 4; i++) pk_stf(w2p + (long)(kq - 1) * 256 + i * 64 + lane, c[i], tag);
          } else {
            unsigned pr[12];
            okr = pk_fetch<12>(pr, 12, true, tag, [&](int i) { return w2p + (long)(i >> 2) * 256 + (i & 3) * 64 + lane; },
                               a, stage) && okr;
            if (okr) {
#pragma unroll
              for (int k = 0; k < 3; k++)
#pragma unroll
                for (int i = 0; i < 4; i++) c[i] += __uint_as_float(pr[k * 4 + i]);
              u64* dst = hA_n;
              u64* xdst = xA_n;
              float* ring = nullptr;
              int rs = 8;
              if (L.last && st < 4) {
                dst = a.hT[st];
                xdst = nullptr;        // a stack output feeds a level transition, not a GEMM
                ring = st == 0 ? a.ring_hc : st == 1 ? a.ring_hv : st == 2 ? a.ring_yf : a.ring_yv;
                rs = st == 0 ? 32 : st == 2 ? 8 : 16;
              }
              pk_epi_residual(a, c, nt, old, dst + (long)row0 * d, xdst ? xdst + row0 * hd : nullptr, PK_TAG(a, l + 1), Rl, prow,
                              nullptr, ring, rs);
            }
          }
        }
        if (__syncthreads_or(!okr)) return;
      }
      PK_NEXT(4 * (d / 16) * RG);
    }
    // ---- level transition after stack st; everything it produces carries the tag of the next layer
    const int ln = a.first[st] + a.count[st];
    const unsigned tagn = PK_TAG(a, ln);
    if (st == 0 || st == 1) {
      // shorten: coarse slot k pools fine positions 3j-2..3j (this pass: stack output; older: ring; before the start: 0)
      const int fl = st, cl = st + 1;
      const float* ring = st == 0 ? a.ring_hc : a.ring_hv;
      const int rs = st == 0 ? 32 : 16;
      const int Rf_ = a.R[fl], Rc_ = a.R[cl];
      int F0 = 0x3fffffff;   // first fine position of this pass
      for (int r = 0; r < Rf_; r++) if (a.pos[fl][r] >= 0) F0 = min(F0, a.pos[fl][r]);
      PK_MINE(Rc_) {
        const int j = a.pos[cl][u];
        bool ok = pk_wait_stack(a, a.hT[st], tagn, stage, QT == 1 ? 16 : Rf_);
        for (int i0 = 0; i0 < d; i0 += 512) {
          const int i = i0 + 2 * threadIdx.x;       // two adjacent columns per thread
          float s0 = 0.f, s1 = 0.f;
          if (j >= 0 && i < d) {
            for (int p = 3 * j - 2; p <= 3 * j; p++) {
              if (p < 0) continue;
              if (p >= F0) {
                unsigned raw[2];
                const u64* src = a.hT[st] + (long)(p - F0) * d + i;
                ok = pk_fetch<2>(raw, 2, true, tagn, [&](int t) { return src + t; }, a, stage) && ok;
                s0 += __uint_as_float(raw[0]); s1 += __uint_as_float(raw[1]);
              } else {
                s0 += ring[(long)(p & (rs - 1)) * d + i]; s1 += ring[(long)(p & (rs - 1)) * d + i + 1];
              }
            }
          }
          if (i < d) pk_st(a.pool + (long)st * 8 * d + (long)u * (d >> 1) + (i >> 1), pk_pack(s0 / 3.0f, s1 / 3.0f), tagn);
        }
        if (__syncthreads_or(!ok)) return;
      }
      PK_NEXT(Rc_);
      PK_MINE(d / 16) {
        f32x4 c;
        pk_cw_t W = (pk_cw_t)(st == 0 ? a.short_cv : a.short_vf) + (long)u * (d / 32) * 512;
        if (!pk_gemm_tile<0>(a, sh, W, d / 32, a.pool + (long)st * 8 * d, tagn, nullptr, Rc_, c, stage)) return;
        if (wave == 0) {
          const int lane = threadIdx.x & 63, g = lane >> 4, n = u * 16 + (lane & 15);
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const float w = __shfl_xor(c[i], 1, 64);
            if (g * 4 + i < Rc_) {
              pk_stf(a.hA + (long)ln * RS * d + (long)(g * 4 + i) * d + n, c[i], tagn);
              if ((lane & 1) == 0) pk_st(a.xA + (long)ln * RH * d + (long)(g * 4 + i) * (d >> 1) + (n >> 1), pk_pack(c[i], w), tagn);
            }
          }
        }
        __syncthreads();
      }
      PK_NEXT(d / 16);
    } else if (st == 2 || st == 3) {
      // upsample: fine row = skip (output of the level's first half) + coarse output of slot floor(pos/3)
      const int fl = st == 2 ? 1 : 0, cl = fl + 1;
      const u64* skip = a.hT[st == 2 ? 1 : 0];
      const unsigned tag_skip = PK_TAG(a, a.first[st == 2 ? 1 : 0] + a.count[st == 2 ? 1 : 0]);
      const float* ring = st == 2 ? a.ring_yf : a.ring_yv;
      const int rs = st == 2 ? 8 : 16;
      const int Rf_ = a.R[fl], Rc_ = a.R[cl];
      PK_MINE(Rf_) {
        const int p = a.pos[fl][u];
        int slot = -1;
        if (p >= 0) for (int r = 0; r < Rc_; r++) if (a.pos[cl][r] == p / 3) slot = r;
        bool ok = pk_wait_stack(a, a.hT[st], tagn, stage, QT == 1 ? 16 : Rc_);
        for (int i = threadIdx.x; i < d; i += 256) {
          unsigned r0[1], r1[1];
          ok = pk_fetch<1>(r0, 1, true, tag_skip, [&](int) { return skip + (long)u * d + i; }, a, stage) && ok;
          float v = __uint_as_float(r0[0]);
          if (p >= 0) {
            if (slot >= 0) {
              ok = pk_fetch<1>(r1, 1, true, tagn, [&](int) { return a.hT[st] + (long)slot * d + i; }, a, stage) && ok;
              v += __uint_as_float(r1[0]);
            } else {
              v += ring[(long)((p / 3) & (rs - 1)) * d + i];
            }
          }
          pk_stf(a.hA + (long)ln * RS * d + (long)u * d + i, v, tagn);
          const float w = __shfl_xor(v, 1, 64);
          if ((i & 1) == 0) pk_st(a.xA + (long)ln * RH * d + (long)u * (d >> 1) + (i >> 1), pk_pack(v, w), tagn);
        }
        if (__syncthreads_or(!ok)) return;
      }
      PK_NEXT(Rf_);
    }
  }
  // ---- output head: final norm on the fly, logits to plain memory (later launches read them)
  {
    const int l = a.n_layers, R = a.R[0];
    const int NT = (a.D.V + 15) / 16, RG = QT == 1 ? 1 : (R + 15) >> 4;
    PK_MINE(NT * RG) {
      const int nt = u / RG, row0 = (u % RG) * 16, Rl = min(16, R - row0);
      f32x4 c;
      if (!pk_gemm_tile<1>(a, sh, (pk_cw_t)a.lm + (long)nt * (d / 32) * 512, d / 32, a.xA + (long)l * RH * d + (long)row0 * (d >> 1),
                           PK_TAG(a, l), (pk_cf_t)a.gf, Rl, c, stage)) return;
      if (wave == 0) {
        const int lane = threadIdx.x & 63, g = lane >> 4, n = nt * 16 + (lane & 15);
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (g * 4 + i < Rl && n < a.D.V) a.logits[(long)(row0 + g * 4 + i) * a.D.V + n] = c[i];
      }
      __syncthreads();
    }
  }
}
