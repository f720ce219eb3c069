// Generic kernels (fp32 arithmetic, storage type T = float or half).  They are the whole path for
// fp32 configurations and the small/irregular pieces of the half-precision path; its hot kernels (MFMA
// GEMM and attention) live in fm_kernels_mfma.h.
//
// Row convention: a "row set" has S * RPS slots, slot r belongs to sequence r / RPS.  Each set has
// an int array `pos` (level-local position, -1 = inactive slot) and/or `limit` (last visible key).
#pragma once
#include "fm_device.h"

// ------------------------------------------------------------------------------------------
// Skinny GEMM  Y[g][m][n] = epilogue( sum_k X[g][m][k] * W[g][n][k] )       (W is [out, in])
// One wave per output column, lanes split K, rows in chunks of 8.
// ------------------------------------------------------------------------------------------
struct GemmArgs {
  const void* X; long ldx, gsx;   // activations (type T), row stride, group stride (elements)
  const void* W; long gsw;        // weights [N, K] (type T), group stride
  void* Y; long ldy, gsy;         // output: float (EPI_F32) or T
  const float* R; long ldr, gsr;  // optional residual added in EPI_F32 (may alias Y)
  int M, N, K;
  const int* run_flag;            // optional: whole launch is skipped when *run_flag == 0
  const float* gain;              // MFMA path only: when set, X is the fp32 residual stream and the GEMM applies
  float eps;                      // RMSNorm(gain, eps) to its rows on the fly
  // EPI_QKV (MFMA path, fused q,k,v projection whose q and k tiles hold whole rotary pairs): rotary on q and k,
  // q -> Y as half [M, d]; k, v -> the blocked caches at the rows' positions (rows with position < 0 are not cached)
  const float2* cs;               // [M][32] (cos, sin) of each row's position
  const int* pos;                 // [M] positions
  int RPS;                        // rows per sequence
  void *Kc, *Vc;                  // caches, `seq_stride` elements per sequence, `capb` 32-key blocks per head
  long seq_stride;
  int capb, H;
};
enum { EPI_F32 = 0, EPI_GELU_T = 2, EPI_T = 3, EPI_QKV = 4 };

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_simple(GemmArgs a) {
  if (a.run_flag && *a.run_flag == 0) return;
  const int g = blockIdx.y;
  const T* X = (const T*)a.X + (long)g * a.gsx;
  const T* W = (const T*)a.W + (long)g * a.gsw;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  if (n >= a.N) return;
  const T* w = W + (long)n * a.K;
  for (int r0 = 0; r0 < a.M; r0 += 8) {
    float acc[8];
#pragma unroll
    for (int r = 0; r < 8; r++) acc[r] = 0.f;
    for (int k = lane * 8; k < a.K; k += 512) {
      float wv[8];
      Store<T>::ld8(w + k, wv);
#pragma unroll
      for (int r = 0; r < 8; r++) {
        if (r0 + r < a.M) {
          float xv[8];
          Store<T>::ld8(X + (long)(r0 + r) * a.ldx + k, xv);
#pragma unroll
          for (int j = 0; j < 8; j++) acc[r] = fmaf(wv[j], xv[j], acc[r]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 8; r++) {
      float v = wave_sum(acc[r]);
      if (lane == r && r0 + r < a.M) {
        const long m = r0 + r;
        if (EPI == EPI_F32) {
          float* Y = (float*)a.Y + (long)g * a.gsy + m * a.ldy + n;
          if (a.R) v += a.R[(long)g * a.gsr + m * a.ldr + n];
          *Y = v;
        } else {
          T* Y = (T*)a.Y + (long)g * a.gsy + m * a.ldy + n;
          Store<T>::st(Y, EPI == EPI_GELU_T ? gelu_tanh_f(v) : v);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// RMSNorm of gathered rows:  out[r] = T( src[r] / sqrt(mean(src[r]^2) + eps) * gain[g(r)] )
// src rows come either from a dense buffer (srcptr == nullptr) or from a per-row pointer table.
// Optionally copies the raw row to `keep` (fp32) for a later residual add.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float* __restrict__ src, const float* const* __restrict__ srcptr,
                                                  const float* __restrict__ gain, int gain_mod, T* __restrict__ out,
                                                  float* __restrict__ keep, int d, float eps, const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  const int r = blockIdx.x;
  const float* x = srcptr ? srcptr[r] : src + (long)r * d;
  const float* g = gain + (long)(gain_mod ? (r % gain_mod) : 0) * d;
  __shared__ float red[4];
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { float v = x[i]; ss += v * v; }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = red[0] + red[1] + red[2] + red[3];
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = x[i];
    if (keep) keep[(long)r * d + i] = v;
    Store<T>::st(out + (long)r * d + i, v * inv * g[i]);
  }
}

// ------------------------------------------------------------------------------------------
// Embedding lookup (inactive slots become zero rows)
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_embed(const int* __restrict__ tok, const int* __restrict__ pos, const T* __restrict__ emb,
                        float* __restrict__ h, int d) {
  const int r = blockIdx.x;
  const bool on = pos[r] >= 0;
  const T* e = emb + (long)tok[r] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(long)r * d + i] = on ? Store<T>::ld(e + i) : 0.f;
}

// ------------------------------------------------------------------------------------------
// Rotary position + K/V append.  qkv fp32 [R][3d] -> q (T) [R][d]; K/V caches [S][H][cap][HD].
// cs[r][i] = (cos, sin) of pos * base^(-i/(HD/2)), i < HD/2; pair (i, i + HD/2).
// ------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ void k_rope_append(const float* __restrict__ qkv, long ldq, const float2* __restrict__ cs,
                              const int* __restrict__ pos, int RPS, T* __restrict__ q, T* __restrict__ Kc,
                              T* __restrict__ Vc, int H, int cap, const int* run_flag) {
  if (run_flag && *run_flag == 0) return;
  constexpr int HP = HD / 2;
  const int r = blockIdx.x;
  const int p = pos[r];
  const int d = H * HD;
  const int s = r / RPS;
  for (int idx = threadIdx.x; idx < H * HP; idx += blockDim.x) {
    const int hh = idx / HP, i = idx % HP;
    const float2 c = cs[(long)r * HP + i];
    const float* row = qkv + (long)r * ldq;
    const float qa = row[hh * HD + i], qb = row[hh * HD + HP + i];
    Store<T>::st(q + (long)r * d + hh * HD + i, qa * c.x - qb * c.y);
    Store<T>::st(q + (long)r * d + hh * HD + HP + i, qb * c.x + qa * c.y);
    if (Kc && p >= 0) {
      const float ka = row[d + hh * HD + i], kb = row[d + hh * HD + HP + i];
      const long o = (((long)s * H + hh) * cap + p % cap) * HD;     // the cache is a ring when a window is set
      Store<T>::st(Kc + o + i, ka * c.x - kb * c.y);
      Store<T>::st(Kc + o + HP + i, kb * c.x + ka * c.y);
      Store<T>::st(Vc + o + i, row[2 * d + hh * HD + i]);
      Store<T>::st(Vc + o + HP + i, row[2 * d + hh * HD + HP + i]);
    }
  }
}

// Condition-memory keys/values: kv fp32 [M][2d] -> caches [H][M][HD] of one sequence (no rotary).
template <typename T, int HD>
__global__ void k_mem_kv_store(const float* __restrict__ kv, T* __restrict__ Kc, T* __restrict__ Vc, int H, int M) {
  const int m = blockIdx.x;
  const int d = H * HD;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const int hh = i / HD, e = i % HD;
    const long o = ((long)hh * M + m) * HD + e;
    Store<T>::st(Kc + o, kv[(long)m * 2 * d + i]);
    Store<T>::st(Vc + o, kv[(long)m * 2 * d + d + i]);
  }
}

template <typename T>
__global__ void k_convert(const float* __restrict__ src, T* __restrict__ dst, long n) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
    Store<T>::st(dst + i, src[i]);
}

// ------------------------------------------------------------------------------------------
// Attention, one workgroup per (row, head): softmax(q K^T / sqrt(HD)) V over keys [0, limit[row]].
// Threads stride over the keys with a private online softmax and merge at the end.
// Caches: [S][H][cap][HD] (seq_stride = H*cap*HD; 0 for a cache shared by every sequence).
// ------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ __launch_bounds__(256) void k_attn_simple(const T* __restrict__ q, const int* __restrict__ limit, int RPS,
                                                      const T* __restrict__ Kc, const T* __restrict__ Vc, long seq_stride,
                                                      int cap, T* __restrict__ out, int H, const int* run_flag, int window) {
  if (run_flag && *run_flag == 0) return;
  const int r = blockIdx.x, hh = blockIdx.y;
  const int d = H * HD;
  const int lim = limit[r];
  const float kScale = HD == 64 ? 0.125f : 1.0f / sqrtf((float)HD);
  T* o = out + (long)r * d + hh * HD;
  if (lim < 0) {
    if (threadIdx.x < HD) Store<T>::st(o + threadIdx.x, 0.f);
    return;
  }
  const int s = r / RPS;
  const T* K = Kc + (long)s * seq_stride + (long)hh * cap * HD;
  const T* V = Vc + (long)s * seq_stride + (long)hh * cap * HD;
  float qv[HD];
#pragma unroll
  for (int i = 0; i < HD; i += 8) Store<T>::ld8(q + (long)r * d + hh * HD + i, qv + i);
  float m = -INFINITY, l = 0.f, acc[HD];
#pragma unroll
  for (int i = 0; i < HD; i++) acc[i] = 0.f;
  // window > 0: keys lim - window + 1 .. lim, stored at slot (position mod cap)
  const int first = window > 0 ? max(lim - window + 1, 0) : 0;
  for (int ka = first + threadIdx.x; ka <= lim; ka += 256) {
    const int j = window > 0 ? ka % cap : ka;
    float kv[HD];
#pragma unroll
    for (int i = 0; i < HD; i += 8) Store<T>::ld8(K + (long)j * HD + i, kv + i);
    float sc = 0.f;
#pragma unroll
    for (int i = 0; i < HD; i++) sc = fmaf(qv[i], kv[i], sc);
    sc *= kScale;
    const float mn = fmaxf(m, sc);
    const float a = __expf(m - mn), p = __expf(sc - mn);
#pragma unroll
    for (int i = 0; i < HD; i += 8) Store<T>::ld8(V + (long)j * HD + i, kv + i);
    l = l * a + p;
#pragma unroll
    for (int i = 0; i < HD; i++) acc[i] = acc[i] * a + p * kv[i];
    m = mn;
  }
  __shared__ float sm[4], sl[4], so[4][HD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float wm = wave_max(m);
  const float f = (m == -INFINITY) ? 0.f : __expf(m - wm);
  l = wave_sum(l * f);
#pragma unroll
  for (int i = 0; i < HD; i++) {
    float v = wave_sum(acc[i] * f);
    if (lane == 0) so[wave][i] = v;
  }
  if (lane == 0) { sm[wave] = wm; sl[wave] = l; }
  __syncthreads();
  if (threadIdx.x < HD) {
    const float gm = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float ff = (sm[w] == -INFINITY) ? 0.f : __expf(sm[w] - gm);
      num += so[w][threadIdx.x] * ff;
      den += sl[w] * ff;
    }
    Store<T>::st(o + threadIdx.x, num / den);
  }
}

// ------------------------------------------------------------------------------------------
// Hourglass plumbing: rings indexed by absolute level position (ring size RS, power of two)
// ------------------------------------------------------------------------------------------
__global__ void k_ring_save(const float* __restrict__ src, float* __restrict__ ring, const int* __restrict__ pos,
                            int RPS, int RS, int d) {
  const int r = blockIdx.x, p = pos[r];
  if (p < 0) return;
  float* dst = ring + ((long)(r / RPS) * RS + (p & (RS - 1))) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = src[(long)r * d + i];
}

// coarse slot j pools fine rows 3j-2, 3j-1, 3j (rows before the start count as zero; always / 3)
template <typename T>
__global__ void k_pool3(const float* __restrict__ ring_fine, int RSf, const int* __restrict__ pos_coarse, int RPS,
                        T* __restrict__ out, int d) {
  const int r = blockIdx.x, j = pos_coarse[r];
  const int s = r / RPS;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    float acc = 0.f;
    if (j >= 0) {
      for (int k = 3 * j - 2; k <= 3 * j; k++)
        if (k >= 0) acc += ring_fine[((long)s * RSf + (k & (RSf - 1))) * d + i];
    }
    Store<T>::st(out + (long)r * d + i, acc / 3.0f);
  }
}

// fine row at position p receives the coarse output of slot floor(p/3)
__global__ void k_upsample_add(float* __restrict__ h, const int* __restrict__ pos, int RPS,
                               const float* __restrict__ ring_coarse, int RSc, int d) {
  const int r = blockIdx.x, p = pos[r];
  if (p < 0) return;
  const float* c = ring_coarse + ((long)(r / RPS) * RSc + ((p / 3) & (RSc - 1))) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(long)r * d + i] += c[i];
}

// ------------------------------------------------------------------------------------------
// Greedy choice per row: lowest index among exact ties, over [0, nlim)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void argmax_merge(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__device__ __forceinline__ int block_argmax(float bv, int bi, float* sv, int* si) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(bv, o, 64);
    int oi = __shfl_xor(bi, o, 64);
    argmax_merge(bv, bi, ov, oi);
  }
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) { sv[wave] = bv; si[wave] = bi; }
  __syncthreads();
  bv = sv[0]; bi = si[0];
  for (int w = 1; w < nw; w++) argmax_merge(bv, bi, sv[w], si[w]);
  __syncthreads();
  return bi;
}

// `nonfinite` (may be null): counts the rows whose admissible logits hold an infinity or a NaN - half-precision
// activations beyond 65504 overflow silently on the way, and this is where it shows
__global__ __launch_bounds__(256) void k_argmax_rows(const float* __restrict__ logits, int V, int nlim, int* __restrict__ y,
                                                      unsigned long long* __restrict__ nonfinite) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const float* x = logits + (long)blockIdx.x * V;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  int bad = 0;
  for (int i = threadIdx.x; i < nlim; i += 256) {
    const float v = x[i];
    bad |= !(fabsf(v) <= 3.0e38f);
    argmax_merge(bv, bi, v, i);
  }
  bad = __syncthreads_or(bad);
  const int b = block_argmax(bv, bi, sv, si);
  if (threadIdx.x == 0) {
    y[blockIdx.x] = b;
    if (bad && nonfinite) atomicAdd(nonfinite, 1ull);
  }
}
