// Control kernels of one decode step: row bookkeeping for the verify pass, acceptance, commit,
// draft-row set-up, distribution store and the merge that builds the next block.  Integer work
// and a little fp32; every kernel is a single small launch.
#pragma once
#include "fm_device.h"
#include "fm_kernels_basic.h"

struct InvFreq { double v[64]; };  // base^(-i/(hd/2)) for the hd/2 rotary pairs of a head, computed in double on the host

struct Dims {
  int d, H, V, S, Bm, VB, FB, M;
  int hd;                // head width d / H: 64 (both storage types), 96 or 128 (fp32 storage only)
  int capc, capv, capf;  // K/V cache slots per level (rings when a window is set)
  int maxtok;            // longest stream (positions 1 .. maxtok)
  int wc, wv, wf;        // attention window per level in its own positions, 0 = unbounded
  int Dc, m, n;          // draft configuration
  int nspv, nspf;        // SP heads at the point / face level
  int nhfc, nhfv;        // HF parameter sets at the coordinate / vertex level
  int nbins, ban, eos, pad;
  int ruleA;             // rule (A) of the supplement: no point-level prediction at a face split node
  int t0, j0;            // rule (B): first coordinate offset (3, or 0 with the rule off) and first vertex offset (1 / 0)
                         // that own an HF parameter set; offsets below them are left to the coordinate level
};

struct StateDev {
  int *P, *main, *fin, *firedv, *firedf, *basec, *basev, *basef;
  int *vlen, *vtok, *y, *acc;
  int* hist;          // [S][maxtok + 1], hist[p] = x_p
  int* budget;        // [1]
  int* alive;         // [1] unfinished sequences; doubles as the run flag of the step
  unsigned long long* acc_hist;  // [3][32]: accepted lengths of steps whose block carried coordinate-level drafts only /
                                 // a fresh point-level prediction / a fresh face-level prediction
  unsigned long long* counters;  // [0] steps, [1] tokens, [2] verify rows with a non-finite logit
  int* kind;                     // [S] which of the three the block built by the last draft was
};

__device__ __forceinline__ int eff_block_len(const StateDev& st, const Dims& D, int s, const int* block_len) {
  if (st.fin[s]) return 0;
  int len = block_len[s];
  len = min(len, D.Bm);
  len = min(len, st.budget[0] - st.P[s]);
  return max(len, 0);
}

// (any number of workgroups: every entry is computed from the committed state alone)
__global__ __launch_bounds__(256) void k_verify_setup(StateDev st, Dims D, InvFreq inv, const int* __restrict__ block_tok,
                                                       const int* __restrict__ block_len, int* pos_c, int* pos_v, int* pos_f,
                                                       int* limx_c, int* limx_v, int* limx_f, float2* cs_c, float2* cs_v,
                                                       float2* cs_f) {
  const int tid = blockIdx.x * 256 + threadIdx.x, nth = gridDim.x * 256;
  // position of row idx of a level, -1 for a row the block does not reach
  auto row_c = [&](int idx) {
    const int s = idx / D.Bm, i = idx % D.Bm;
    return i < eff_block_len(st, D, s, block_len) ? st.P[s] + i : -1;
  };
  auto row_v = [&](int idx) {
    const int s = idx / D.VB, k = idx % D.VB;
    const int len = eff_block_len(st, D, s, block_len), P = st.P[s];
    const int j = (P + 2) / 3 + k;
    return 3 * j < P + len ? j : -1;
  };
  auto row_f = [&](int idx) {
    const int s = idx / D.FB, k = idx % D.FB;
    const int len = eff_block_len(st, D, s, block_len), P = st.P[s];
    const int f = (P + 8) / 9 + k;
    return 9 * f < P + len ? f : -1;
  };
  for (int idx = tid; idx < D.S * D.Bm; idx += nth) {
    const int s = idx / D.Bm, i = idx % D.Bm;
    const int p = row_c(idx);
    pos_c[idx] = p;
    limx_c[idx] = p >= 0 ? D.M - 1 : -1;
    int t = p >= 0 ? block_tok[idx] : D.pad;
    if (t < 0 || t >= D.V) t = D.pad;
    st.vtok[idx] = t;
    if (i == 0) st.vlen[s] = eff_block_len(st, D, s, block_len);
  }
  for (int idx = tid; idx < D.S * D.VB; idx += nth) {
    const int p = row_v(idx);
    pos_v[idx] = p;
    limx_v[idx] = p >= 0 ? D.M - 1 : -1;
  }
  for (int idx = tid; idx < D.S * D.FB; idx += nth) {
    const int p = row_f(idx);
    pos_f[idx] = p;
    limx_f[idx] = p >= 0 ? D.M - 1 : -1;
  }
  const int np = D.hd >> 1;      // rotary pairs per head
  for (int idx = tid; idx < D.S * D.Bm * np; idx += nth) {
    const int p = row_c(idx / np);
    const double a = (p < 0 ? 0.0 : (double)p) * inv.v[idx % np];
    cs_c[idx] = make_float2((float)cos(a), (float)sin(a));
  }
  for (int idx = tid; idx < D.S * D.VB * np; idx += nth) {
    const int p = row_v(idx / np);
    const double a = (p < 0 ? 0.0 : (double)p) * inv.v[idx % np];
    cs_v[idx] = make_float2((float)cos(a), (float)sin(a));
  }
  for (int idx = tid; idx < D.S * D.FB * np; idx += nth) {
    const int p = row_f(idx / np);
    const double a = (p < 0 ? 0.0 : (double)p) * inv.v[idx % np];
    cs_f[idx] = make_float2((float)cos(a), (float)sin(a));
  }
}

// accepted = 1 + number of leading drafts that equal the backbone's greedy prediction; with sampled decoding
// (accflag != null) 1 + number of leading drafts that passed the rejection test (flag of row i is about draft i + 1)
// (failed != null and *failed != 0: the forward pass gave up and its logits mean nothing; every accepted length is 0)
__global__ void k_accept(StateDev st, Dims D, int* __restrict__ accepted_out, const int* __restrict__ accflag,
                         const unsigned* __restrict__ failed) {
  const int s = threadIdx.x;
  if (s >= D.S) return;
  const int len = st.vlen[s];
  int a = 0;
  if (len > 0 && !(failed && *failed)) {
    a = 1;
    if (accflag) while (a < len && accflag[s * D.Bm + a - 1]) a++;
    else while (a < len && st.vtok[s * D.Bm + a] == st.y[s * D.Bm + a - 1]) a++;
  }
  st.acc[s] = a;
  if (accepted_out) accepted_out[s] = a;
}

// An accepted length of 0 (a pass that did not complete) leaves the sequence as it is.
__global__ void k_commit(StateDev st, Dims D, const int* __restrict__ accepted, const unsigned* __restrict__ failed) {
  const int s = threadIdx.x;
  __shared__ int any_live;
  if (failed && *failed) return;
  if (s == 0) any_live = 0;
  __syncthreads();
  if (s < D.S) {
    const int len = st.vlen[s];
    if (len > 0 && accepted[s] > 0) {
      any_live = 1;
      int a = accepted[s];
      a = min(a, len);
      for (int i = 1; i < a; i++)
        if (st.vtok[s * D.Bm + i] == D.eos) { a = i; break; }   // an accepted EOS draft is not fed: it becomes the main token
      int P = st.P[s];
      int* h = st.hist + (long)s * (D.maxtok + 1);
      for (int i = 0; i < a; i++) h[P + i] = st.vtok[s * D.Bm + i];
      P += a;
      const int mainTok = st.y[s * D.Bm + a - 1];
      h[P] = mainTok;
      st.P[s] = P;
      st.main[s] = mainTok;
      st.fin[s] = (mainTok == D.eos || P >= st.budget[0]) ? 1 : 0;
      st.vlen[s] = 0;
      atomicAdd(&st.acc_hist[min(max(st.kind[s], 0), 2) * 32 + min(a, 31)], 1ull);
      atomicAdd(&st.counters[1], (unsigned long long)a);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int alive = 0;
    for (int i = 0; i < D.S; i++) alive += st.fin[i] ? 0 : 1;
    st.alive[0] = alive;
    if (any_live) st.counters[0] += 1;
  }
}

// New token budget: sequences that have not ended with EOS become live again if they are below it.
__global__ void k_set_budget(StateDev st, Dims D, int budget) {
  if (threadIdx.x != 0) return;
  st.budget[0] = budget;
  int alive = 0;
  for (int i = 0; i < D.S; i++) {
    if (st.P[i] >= 0 && st.hist[(long)i * (D.maxtok + 1)] == D.nbins)   // sequence has been prefilled
      st.fin[i] = (st.main[i] == D.eos || st.P[i] >= budget) ? 1 : 0;
    alive += st.fin[i] ? 0 : 1;
  }
  st.alive[0] = alive;
}

// Reset one sequence to x_0 = BOS with empty caches and no draft rows.
__global__ void k_reset_seq(StateDev st, Dims D, int s, int bos) {
  if (threadIdx.x != 0) return;
  st.P[s] = 0; st.main[s] = bos; st.fin[s] = 0;
  st.firedv[s] = -1; st.firedf[s] = -1;
  st.basec[s] = -1000000; st.basev[s] = -1; st.basef[s] = -1;
  st.vlen[s] = 0; st.acc[s] = 0;
  st.hist[(long)s * (D.maxtok + 1)] = bos;
  int alive = 0;
  for (int i = 0; i < D.S; i++) alive += st.fin[i] ? 0 : 1;
  st.alive[0] = alive;
}


// ------------------------------------------------------------------------------------------
// Sampled decoding with non-greedy verification: drafts drawn from the averaged draft distributions, the
// rejection test of speculative sampling on the backbone's tempered softmax, residual resampling.
// Uniforms are counter based: (seed, sequence, absolute position of the token decided, purpose).
// ------------------------------------------------------------------------------------------
#define FM_U_DRAFT 0
#define FM_U_ACCEPT 1
#define FM_U_RESAMPLE 2

struct Sampling {
  float temperature;            // 0 = greedy decoding
  unsigned long long seed;
  float* qrow;                  // [S][Bm][V] averaged draft distribution behind draft index i (unnormalised over the admissible tokens)
  float* qsum;                  // [S][Bm]    its sum over the admissible tokens
  int* qtok;                    // [S][Bm]    the token drawn from it (-1: none)
  int* accflag;                 // [S][Bm]    row i: draft i + 1 passed the rejection test
  int keep_rows;                // test hook: greedy decoding also leaves the averaged rows in qrow (read by fm_debug_draft)
};

__device__ __forceinline__ float sample_uniform(unsigned long long seed, int purpose, int seq, int pos);

// Inverse CDF in index order over n weights, by one workgroup of up to 1024 threads: thread t owns the contiguous
// chunk [t*chunk, (t+1)*chunk); `wf(i)` gives weight i.  Returns the smallest i whose cumulative weight exceeds
// u * total (the last index with weight if rounding leaves none), the same in every thread.  sh: blockDim + 2 floats
// (the total is left in sh[blockDim]), si: 1 int.
template <class F>
__device__ __forceinline__ int block_inverse_cdf(int n, float u, F wf, float* sh, int* si) {
  const int t = threadIdx.x, nt = blockDim.x;
  const int chunk = (n + nt - 1) / nt;
  const int i0 = min(t * chunk, n), i1 = min(i0 + chunk, n);
  float local = 0.f;
  for (int i = i0; i < i1; i++) local += wf(i);
  sh[t] = local;
  if (t == 0) *si = -1;
  __syncthreads();
  if (t == 0) {
    float run = 0.f;
    for (int k = 0; k < nt; k++) { const float v = sh[k]; sh[k] = run; run += v; }
    sh[nt] = run;
  }
  __syncthreads();
  const float thr = u * sh[nt];
  const float excl = sh[t];
  if (i0 < i1 && excl <= thr && excl + local > thr) {
    float run = excl;
    for (int i = i0; i < i1; i++) {
      run += wf(i);
      if (run > thr) { *si = i; break; }
    }
  }
  __syncthreads();
  if (*si < 0 && t == 0) {
    int last = 0;
    for (int i = 0; i < n; i++)
      if (wf(i) > 0.f) last = i;
    *si = last;
  }
  __syncthreads();
  const int r = *si;
  __syncthreads();
  return r;
}

// ------------------------------------------------------------------------------------------
// Draft stage
// ------------------------------------------------------------------------------------------
struct DraftRows {
  // five row sets: 0 SP coordinate, 1 SP point, 2 SP face, 3 HF vertex, 4 HF coordinate
  const float** src[5];
  int* pos[5];
  int* lim[5];
  int* limx[5];
  float2* cs[5];
  int *alive, *firev, *firef;   // [S]
  int* flags;                   // [0] any alive with P > 0, [1] any point firing, [2] any face firing
  int rs[5];                    // rows per sequence in the tables of a set: row (sequence s, head k) = s * rs + k.  The
                                // set's own head count, or for the three SP sets the head count of all three together
                                // when their tables are one table (point, face, coordinate heads behind each other)
};

struct DraftBufs {
  const float *tap_c, *tap_v, *tap_f, *ring_yf;   // rings
  const float *spv_out, *spf_out, *hfv_out;        // head outputs feeding the HF blocks
  int spv_rs, spf_rs;                               // rows per sequence in spv_out / spf_out (as DraftRows::rs)
};

__device__ __forceinline__ void set_row(const DraftRows& R, int set, int r, const float* src, int pos, int lim, int M,
                                        const InvFreq& inv, int lane32, int np = 32) {
  if (lane32 == 0) {
    R.src[set][r] = src;
    R.pos[set][r] = lim >= 0 ? pos : -1;
    R.lim[set][r] = lim;
    R.limx[set][r] = lim >= 0 ? M - 1 : -1;
  }
  for (int i = lane32; i < np; i += 32) {        // np = rotary pairs per head
    const double a = (lim >= 0 ? (double)pos : 0.0) * inv.v[i];
    R.cs[set][(long)r * np + i] = make_float2((float)cos(a), (float)sin(a));
  }
}

// One workgroup per sequence, 32 threads per row at a time.  The three launch flags (any sequence alive / firing at the
// point level / at the face level) depend on the committed state only, so every workgroup could derive them; workgroup 0
// does, for all sequences, and writes them.
__global__ __launch_bounds__(256) void k_draft_setup(StateDev st, Dims D, InvFreq inv, DraftRows R, DraftBufs B) {
  const int lane32 = threadIdx.x & 31, grp = threadIdx.x >> 5;  // 8 groups of 32
  const int d = D.d;
  auto predicates = [&](int s, bool& alive, bool& firev, bool& firef, int& spos, int& v, int& f) {
    const int P = st.P[s];
    alive = !st.fin[s] && P > 0;
    spos = P - 1;
    v = alive ? spos / 3 : 0;
    f = alive ? spos / 9 : 0;
    firev = alive && D.m > 0 && ((v % 3) != 0 || !D.ruleA) && st.firedv[s] != v;
    firef = alive && D.n > 0 && st.firedf[s] != f;
  };
  if (blockIdx.x == 0) {
    __shared__ int f_any[3];
    if (threadIdx.x < 3) f_any[threadIdx.x] = 0;
    __syncthreads();
    for (int s = threadIdx.x; s < D.S; s += blockDim.x) {
      bool alive, firev, firef; int spos, v, f;
      predicates(s, alive, firev, firef, spos, v, f);
      if (alive) atomicOr(&f_any[0], 1);
      if (firev) atomicOr(&f_any[1], 1);
      if (firef) atomicOr(&f_any[2], 1);
    }
    __syncthreads();
    if (threadIdx.x < 3) R.flags[threadIdx.x] = f_any[threadIdx.x];
  }
  {
    const int s = blockIdx.x;
    bool alive, firev, firef; int spos, v, f;
    predicates(s, alive, firev, firef, spos, v, f);
    if (threadIdx.x == 0) { R.alive[s] = alive; R.firev[s] = firev; R.firef[s] = firef; }
    const float* tapc = B.tap_c + ((long)s * 32 + (spos & 31)) * d;
    const float* tapv = B.tap_v + ((long)s * 16 + (v & 15)) * d;
    const float* tapf = B.tap_f + ((long)s * 8 + (f & 7)) * d;
    const float* yf = B.ring_yf + ((long)s * 8 + (f & 7)) * d;
    // set 0: coordinate SP heads k = 1..Dc on the coordinate tap at s
    for (int k = grp; k < D.Dc; k += 8) set_row(R, 0, s * R.rs[0] + k, tapc, spos, alive ? spos : -1, D.M, inv, lane32, D.hd >> 1);
    // set 1: point SP heads on the vertex tap of v
    for (int k = grp; k < D.nspv; k += 8) set_row(R, 1, s * R.rs[1] + k, tapv, v, firev ? v : -1, D.M, inv, lane32, D.hd >> 1);
    // set 2: face SP heads on the face tap of f
    for (int k = grp; k < D.nspf; k += 8) set_row(R, 2, s * R.rs[2] + k, tapf, f, firef ? f : -1, D.M, inv, lane32, D.hd >> 1);
    // set 3: vertex-level HF, vertex offsets j = j0..n/3-1 from vertex token 3f; input = face feature j/3
    for (int q = grp; q < D.nhfv; q += 8) {
      const int j = q + D.j0;
      const float* src = (j < 3) ? yf : B.spf_out + ((long)s * B.spf_rs + (j / 3 - 1)) * d;
      set_row(R, 3, s * D.nhfv + q, src, 3 * f + j, firef ? 3 * f : -1, D.M, inv, lane32, D.hd >> 1);
    }
    // set 4: coordinate-level HF, offsets t = t0..; pipe 0 = point pipeline, pipe 1 = face pipeline
    for (int q = grp; q < 2 * D.nhfc; q += 8) {
      const int pipe = q / D.nhfc, t = q % D.nhfc + D.t0;
      const int r = s * 2 * D.nhfc + q;
      if (pipe == 0) {
        const bool on = firev && t < D.m;
        // offsets 0..2 (rule (B) off) belong to the current vertex: its own feature; later ones to the SP head outputs
        const float* src = t < 3 ? tapv : B.spv_out + ((long)s * B.spv_rs + min(t / 3 - 1, max(D.nspv - 1, 0))) * d;
        set_row(R, 4, r, src, 3 * v + t, on ? 3 * v : -1, D.M, inv, lane32, D.hd >> 1);
      } else {
        const bool on = firef && t < D.n;
        const float* src = B.hfv_out + ((long)s * max(D.nhfv, 1) + min(max(t / 3 - D.j0, 0), max(D.nhfv - 1, 0))) * d;
        set_row(R, 4, r, src, 9 * f + t, on ? 9 * f : -1, D.M, inv, lane32, D.hd >> 1);
      }
    }
  }
}

// softmax of one LM row of the draft heads into the distribution store of its level
__global__ __launch_bounds__(256) void k_dist_store(const float* __restrict__ logits, Dims D, DraftRows R, float* dist_c,
                                                     float* dist_v, float* dist_f) {
  const int r = blockIdx.x;
  float* dst = nullptr;
  if (r < D.S * D.Dc) {
    const int s = r / D.Dc, k = r % D.Dc;
    if (R.alive[s]) dst = dist_c + ((long)s * D.Dc + k) * D.V;
  } else {
    const int rr = r - D.S * D.Dc;
    const int s = rr / (2 * D.nhfc), q = rr % (2 * D.nhfc);
    const int pipe = q / D.nhfc, t = q % D.nhfc + D.t0;
    if (pipe == 0 && R.firev[s] && t < D.m) dst = dist_v + ((long)s * D.nhfc + (t - D.t0)) * D.V;
    if (pipe == 1 && R.firef[s] && t < D.n) dst = dist_f + ((long)s * D.nhfc + (t - D.t0)) * D.V;
  }
  if (!dst) return;
  const float* x = logits + (long)r * D.V;
  __shared__ float red[4];
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < D.V; i += 256) mx = fmaxf(mx, x[i]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int i = threadIdx.x; i < D.V; i += 256) sum += expf(x[i] - mx);
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
  __syncthreads();
  sum = red[0] + red[1] + red[2] + red[3];
  const float inv = 1.0f / sum;
  for (int i = threadIdx.x; i < D.V; i += 256) dst[i] = expf(x[i] - mx) * inv;
}

struct Replay {
  const int* stream;  // [S][stride], stream[p - 1] = x_p
  int stride, n_valid;
  float keep;
  unsigned long long seed;
};

__device__ __forceinline__ float replay_uniform(unsigned long long seed, unsigned long long seq, unsigned long long pos) {
  unsigned long long z = seed * 0x9E3779B97F4A7C15ull + seq * 0xBF58476D1CE4E5B9ull + pos * 0x94D049BB133111EBull +
                         0x2545F4914F6CDD1Dull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  return (float)(z >> 40) * (1.0f / 16777216.0f);
}

__device__ __forceinline__ float sample_uniform(unsigned long long seed, int purpose, int seq, int pos) {
  return replay_uniform(seed * 3ull + (unsigned long long)purpose, (unsigned long long)seq, (unsigned long long)pos);
}

// One workgroup per verify row (sequence s, block index i): the backbone's distribution p = softmax(logits / T) over the
// admissible tokens, the rejection test for the draft at index i + 1 (u q(x) < p(x); a draft that is not the token
// drawn from the stored distribution counts as a proposal with all its mass on it), and the token emitted after this
// row if the accepted prefix ends here: from max(p - q, 0) after a rejection, from p after the last row.
__global__ __launch_bounds__(256) void k_sample_rows(StateDev st, Dims D, const float* __restrict__ logits, Sampling sm) {
  __shared__ float sh[260];
  __shared__ int si;
  const int row = blockIdx.x, s = row / D.Bm, i = row % D.Bm;
  const int len = st.vlen[s];
  if (i >= len) return;
  const int nlim = D.ban ? D.nbins : D.V;
  const float* x = logits + (long)row * D.V;
  const float invT = 1.0f / sm.temperature;
  // max and sum of exp((x - max) / T)
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < nlim; j += 256) mx = fmaxf(mx, x[j]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = threadIdx.x; j < nlim; j += 256) sum += expf((x[j] - mx) * invT);
  // an infinity or a NaN among the logits shows in the sum (inf - inf, or NaN itself)
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = sum;
  __syncthreads();
  const float invZp = 1.0f / (sh[0] + sh[1] + sh[2] + sh[3]);
  if (threadIdx.x == 0 && !(fabsf(invZp) <= 3.0e38f && fabsf(mx) <= 3.0e38f)) atomicAdd(st.counters + 2, 1ull);
  __syncthreads();
  auto pf = [&](int j) { return expf((x[j] - mx) * invT) * invZp; };
  const int pos = st.P[s] + i + 1;                       // the token this row decides
  const bool has_draft = i + 1 < len;
  const int xd = has_draft ? st.vtok[s * D.Bm + i + 1] : -1;
  const bool fromq = has_draft && xd == sm.qtok[s * D.Bm + i + 1] && xd >= 0 && xd < nlim;
  const float* q = sm.qrow + ((long)s * D.Bm + i + 1) * D.V;
  const float invZq = fromq ? 1.0f / sm.qsum[s * D.Bm + i + 1] : 0.f;
  bool accepted = false;
  if (has_draft && xd >= 0 && xd < nlim) {
    const float pa = pf(xd), qa = fromq ? q[xd] * invZq : 1.0f;
    accepted = sample_uniform(sm.seed, FM_U_ACCEPT, s, pos) * qa < pa;
  }
  const float u = sample_uniform(sm.seed, FM_U_RESAMPLE, s, pos);
  int y;
  if (!has_draft) {
    y = block_inverse_cdf(nlim, u, pf, sh, &si);
  } else {
    auto wf = [&](int j) { return fromq ? fmaxf(pf(j) - q[j] * invZq, 0.f) : (j == xd ? 0.f : pf(j)); };
    // all the mass can vanish only if p and q agree everywhere (or p sits on the draft alone): then p itself
    float tot = 0.f;
    for (int j = threadIdx.x; j < nlim; j += 256) tot += wf(j);
    tot = wave_sum(tot);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = tot;
    __syncthreads();
    tot = sh[0] + sh[1] + sh[2] + sh[3];
    __syncthreads();
    y = tot > 0.f ? block_inverse_cdf(nlim, u, wf, sh, &si) : block_inverse_cdf(nlim, u, pf, sh, &si);
  }
  if (threadIdx.x == 0) {
    st.y[row] = y;
    sm.accflag[row] = accepted ? 1 : 0;
  }
}

// One workgroup per sequence: update the draft bookkeeping, average the distributions that cover
// each future position, take the greedy token, stop at the first uncovered position.
__global__ __launch_bounds__(1024) void k_merge(StateDev st, Dims D, DraftRows R, const float* __restrict__ dist_c,
                                                const float* __restrict__ dist_v, const float* __restrict__ dist_f,
                                                Replay rp, int speculative, int* __restrict__ block_tok,
                                                int* __restrict__ block_len, Sampling sm) {
  __shared__ float sh[1026];
  __shared__ int sidx;
  if (sm.temperature > 0.f)
    for (int i = threadIdx.x; i < D.Bm; i += blockDim.x) sm.qtok[blockIdx.x * D.Bm + i] = -1;
  const int s = blockIdx.x;
  int* tok = block_tok + (long)s * D.Bm;
  if (st.fin[s]) {
    if (threadIdx.x == 0) block_len[s] = 0;
    return;
  }
  const int P = st.P[s], budget = st.budget[0];
  if (threadIdx.x == 0) tok[0] = st.main[s];
  if (P == 0 || !speculative) {
    if (threadIdx.x == 0) { block_len[s] = 1; st.kind[s] = 0; }
    return;
  }
  const int spos = P - 1;
  const int basec = spos;
  const int basev = R.firev[s] ? 3 * (spos / 3) : st.basev[s];
  const int basef = R.firef[s] ? 9 * (spos / 9) : st.basef[s];
  __syncthreads();   // every thread has read the old state
  if (threadIdx.x == 0) {
    st.basec[s] = basec; st.basev[s] = basev; st.basef[s] = basef;
    if (R.firev[s]) st.firedv[s] = spos / 3;
    if (R.firef[s]) st.firedf[s] = spos / 9;
    st.kind[s] = R.firef[s] ? 2 : R.firev[s] ? 1 : 0;
  }
  const int nlim = D.ban ? D.nbins : D.V;
  int len = 1;
  // the averaged distributions behind draft index idx (position spos + 1 + idx), if any level covers it
  auto rows_of = [&](int p, const float* (&rows)[3]) {
    int cnt = 0;
    const int kc = p - (basec + 2);
    if (kc >= 0 && kc < D.Dc) rows[cnt++] = dist_c + ((long)s * D.Dc + kc) * D.V;
    const int tv = p - 1 - basev;
    if (basev >= 0 && tv >= D.t0 && tv < D.m) rows[cnt++] = dist_v + ((long)s * D.nhfc + (tv - D.t0)) * D.V;
    const int tf = p - 1 - basef;
    if (basef >= 0 && tf >= D.t0 && tf < D.n) rows[cnt++] = dist_f + ((long)s * D.nhfc + (tf - D.t0)) * D.V;
    return cnt;
  };
  if (sm.temperature > 0.f) {
    // sampled decoding: keep the averaged distribution (the proposal the verify pass tests against) and draw from it
    for (int p = spos + 2; len < D.Bm && p < budget; p++) {
      const float* rows[3];
      const int cnt = rows_of(p, rows);
      if (cnt == 0) break;
      const float inv = 1.0f / (float)cnt;
      float* qr = sm.qrow + ((long)s * D.Bm + len) * D.V;
      for (int i = threadIdx.x; i < nlim; i += blockDim.x) {
        float a = rows[0][i];
        if (cnt > 1) a += rows[1][i];
        if (cnt > 2) a += rows[2][i];
        qr[i] = a * inv;
      }
      __syncthreads();
      const int b = block_inverse_cdf(nlim, sample_uniform(sm.seed, FM_U_DRAFT, s, p), [&](int i) { return qr[i]; }, sh, &sidx);
      if (threadIdx.x == 0) { tok[len] = b; sm.qtok[s * D.Bm + len] = b; sm.qsum[s * D.Bm + len] = sh[blockDim.x]; }
      __syncthreads();
      len++;
    }
  } else {
    // greedy: one wave per draft index, all indices at once; the block then ends at the first index nothing covers
    __shared__ int stok[32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int idx = 1 + wave; idx < D.Bm; idx += (int)(blockDim.x >> 6)) {
      const float* rows[3];
      const int cnt = rows_of(spos + 1 + idx, rows);
      int bi = -1;
      if (cnt > 0) {
        const float inv = 1.0f / (float)cnt;
        float bv = -INFINITY;
        bi = 0x7fffffff;
        // four strides of the vocabulary per step, all loads of a step in flight together
        for (int i0 = lane; i0 < nlim; i0 += 256) {
          float a[4];
#pragma unroll
          for (int k = 0; k < 4; k++) {
            const int i = i0 + 64 * k;
            a[k] = 0.f;
            if (i < nlim) {
              a[k] = rows[0][i];
              if (cnt > 1) a[k] += rows[1][i];
              if (cnt > 2) a[k] += rows[2][i];
            }
          }
#pragma unroll
          for (int k = 0; k < 4; k++)
            if (i0 + 64 * k < nlim) {
              argmax_merge(bv, bi, a[k] * inv, i0 + 64 * k);
              if (sm.keep_rows) sm.qrow[((long)s * D.Bm + idx) * D.V + i0 + 64 * k] = a[k] * inv;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
          const float ov = __shfl_xor(bv, o, 64);
          const int oi = __shfl_xor(bi, o, 64);
          argmax_merge(bv, bi, ov, oi);
        }
      }
      if (lane == 0) stok[idx] = bi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      while (len < D.Bm && spos + 1 + len < budget && stok[len] >= 0) { tok[len] = stok[len]; len++; }
      stok[0] = len;
    }
    __syncthreads();
    len = stok[0];
  }
  if (rp.stream) {
    // synthetic draft source: the known continuation, each token kept with probability `keep`
    int n = min(D.Bm - 1, min(budget - 1 - P, rp.n_valid - P));
    n = max(n, 0);
    const int t = threadIdx.x;
    if (t >= 1 && t <= n) {
      const int p = P + t;
      const int truth = rp.stream[(long)s * rp.stride + p - 1];
      const bool keep = replay_uniform(rp.seed, (unsigned long long)s, (unsigned long long)p) < rp.keep;
      tok[t] = keep ? truth : (truth + 1) % D.nbins;
    }
    len = 1 + n;
  }
  if (threadIdx.x == 0) block_len[s] = len;
}

// ------------------------------------------------------------------------------------------
// Correct stage (Sec. 3.2): label rows of the point-level features, then the integer correction of a draft block
// ------------------------------------------------------------------------------------------
// One wave per point-level feature: softmax of the three label logits W_label f.  Rows 0 .. S*nspv-1 are the
// point pipeline's SP head outputs (vertex v + k), the rest the face pipeline's vertex-level HF outputs (vertex
// 3f + j); a row is stored only when its pipeline fired for the sequence, so older rows stay usable like the
// token distributions do.
__global__ __launch_bounds__(64) void k_label_rows(Dims D, DraftRows R, const float* __restrict__ spv_out, int spv_rs,
                                                    const float* __restrict__ hfv_out, const float* __restrict__ W,
                                                    float* __restrict__ lab_v, float* __restrict__ lab_f) {
  const int r = blockIdx.x, lane = threadIdx.x;
  const float* src;
  float* dst;
  if (r < D.S * D.nspv) {
    const int s = r / D.nspv, k = r % D.nspv;
    if (!R.firev[s]) return;
    src = spv_out + ((long)s * spv_rs + k) * D.d;      // spv_rs rows per sequence in the SP output buffer
    dst = lab_v + (long)r * 3;
  } else {
    const int rr = r - D.S * D.nspv, s = rr / D.nhfv;
    if (!R.firef[s]) return;
    src = hfv_out + (long)rr * D.d;
    dst = lab_f + (long)rr * 3;
  }
  float z[3] = {0.f, 0.f, 0.f};
  for (int i = lane; i < D.d; i += 64) {
    const float x = src[i];
    z[0] = fmaf(W[i], x, z[0]);
    z[1] = fmaf(W[D.d + i], x, z[1]);
    z[2] = fmaf(W[2 * D.d + i], x, z[2]);
  }
#pragma unroll
  for (int k = 0; k < 3; k++) z[k] = wave_sum(z[k]);
  if (lane == 0) {
    const float mx = fmaxf(z[0], fmaxf(z[1], z[2]));
    const float e0 = expf(z[0] - mx), e1 = expf(z[1] - mx), e2 = expf(z[2] - mx);
    const float inv = 1.0f / (e0 + e1 + e2);
    dst[0] = e0 * inv; dst[1] = e1 * inv; dst[2] = e2 * inv;
  }
}

#define FM_LABEL_HIST 0
#define FM_LABEL_NEW 1
#define FM_LABEL_INTRA 2

// One thread per sequence (a block holds at most 27 tokens, i.e. 9 points): labels of the block's points from the
// stored rows, the historical / intra-batch moves in ascending vertex order, then the z-y-x re-sort of the faces
// that consist of draft tokens only.  Integer work on bin coordinates; the main token is never touched.
// Vertex u owns x_{3u+1..3u+3}; block token i is x_{P+i}.
__global__ void k_correct(StateDev st, Dims D, const float* __restrict__ lab_v, const float* __restrict__ lab_f,
                          int hist_vertices, int* __restrict__ block_tok, const int* __restrict__ block_len,
                          int* __restrict__ labels_out) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= D.S) return;
  int* tok = block_tok + (long)s * D.Bm;
  int* lout = labels_out ? labels_out + (long)s * D.Bm : nullptr;
  if (lout)
    for (int i = 0; i < D.Bm; i++) lout[i] = -1;
  if (st.fin[s]) return;
  const int P = st.P[s];
  int len = block_len[s];
  len = min(len, D.Bm);
  if (len < 4) return;
  const int u0 = (P + 2) / 3, u1 = (P + len - 4) / 3;
  if (u1 < u0) return;
  const int np = u1 - u0 + 1;                    // <= 9
  int lab[9];
  bool pt[9];
  const int basev = st.basev[s], basef = st.basef[s];
  for (int i = 0; i < np; i++) {
    const int u = u0 + i;
    float a[3] = {0.f, 0.f, 0.f};
    int cnt = 0;
    const int kv = basev >= 0 ? u - basev / 3 : 0;
    if (basev >= 0 && kv >= 1 && kv <= D.nspv) {
      const float* row = lab_v + ((long)s * D.nspv + kv - 1) * 3;
      a[0] += row[0]; a[1] += row[1]; a[2] += row[2];
      cnt++;
    }
    const int jf = basef >= 0 ? u - basef / 3 : 0;
    if (basef >= 0 && jf >= D.j0 && jf < D.j0 + D.nhfv) {
      const float* row = lab_f + ((long)s * D.nhfv + jf - D.j0) * 3;
      a[0] += row[0]; a[1] += row[1]; a[2] += row[2];
      cnt++;
    }
    int l = FM_LABEL_NEW;
    if (cnt > 0) {
      const float inv = 1.0f / (float)cnt;
      const float m0 = a[0] * inv, m1 = a[1] * inv, m2 = a[2] * inv;
      l = 0;
      float best = m0;
      if (m1 > best) { best = m1; l = 1; }
      if (m2 > best) { best = m2; l = 2; }
    }
    lab[i] = l;
    if (lout) lout[i] = l;
    const int* c = tok + 3 * u + 1 - P;
    pt[i] = c[0] >= 0 && c[0] < D.nbins && c[1] >= 0 && c[1] < D.nbins && c[2] >= 0 && c[2] < D.nbins;
  }
  const int* known = st.hist + (long)s * (D.maxtok + 1);     // x_0 .. x_P (the pending main token is x_P)
  const int nkv = P / 3;
  const int h0 = max(0, nkv - hist_vertices);
  for (int i = 0; i < np; i++) {
    if (!pt[i]) continue;
    int* c = tok + 3 * (u0 + i) + 1 - P;
    if (lab[i] == FM_LABEL_HIST) {
      long best = -1;
      int bh = -1;
      bool same = false;
      for (int h = h0; h < nkv; h++) {
        const int* k = known + 3 * h + 1;
        if (!(k[0] < D.nbins && k[1] < D.nbins && k[2] < D.nbins)) continue;
        const long dz = c[0] - k[0], dy = c[1] - k[1], dx = c[2] - k[2];
        const long dd = dz * dz + dy * dy + dx * dx;
        if (dd == 0) { same = true; break; }
        if (bh < 0 || dd < best) { best = dd; bh = h; }
      }
      if (!same && bh >= 0) { c[0] = known[3 * bh + 1]; c[1] = known[3 * bh + 2]; c[2] = known[3 * bh + 3]; }
    } else if (lab[i] == FM_LABEL_INTRA) {
      long best = -1;
      int bw = -1;
      bool same = false;
      for (int w = 0; w < np; w++) {
        if (w == i || !pt[w]) continue;
        const int* k = tok + 3 * (u0 + w) + 1 - P;
        const long dz = c[0] - k[0], dy = c[1] - k[1], dx = c[2] - k[2];
        const long dd = dz * dz + dy * dy + dx * dx;
        if (dd == 0) { same = true; break; }
        if (lab[w] == FM_LABEL_NEW && (u0 + w) / 3 != (u0 + i) / 3 && (bw < 0 || dd < best)) { best = dd; bw = w; }
      }
      if (!same && bw >= 0) {
        const int* k = tok + 3 * (u0 + bw) + 1 - P;
        c[0] = k[0]; c[1] = k[1]; c[2] = k[2];
      }
    }
  }
  // faces whose nine tokens are all drafts of this block: vertices in ascending (z, y, x) order
  for (int f = (u0 + 2) / 3; f < (u1 + 1) / 3; f++) {
    const int i0 = 3 * f - u0;
    if (!(pt[i0] && pt[i0 + 1] && pt[i0 + 2])) continue;
    int* c = tok + 3 * (3 * f) + 1 - P;
    for (int pass = 0; pass < 2; pass++)
      for (int j = 0; j < 2 - pass; j++) {
        int* a = c + 3 * j;
        int* b = a + 3;
        const bool gt = a[0] != b[0] ? a[0] > b[0] : a[1] != b[1] ? a[1] > b[1] : a[2] > b[2];
        if (gt)
          for (int k = 0; k < 3; k++) { const int t = a[k]; a[k] = b[k]; b[k] = t; }
      }
  }
}
