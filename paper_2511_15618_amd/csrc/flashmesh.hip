// C-ABI library: context, weight loading, and the enqueue logic of draft / verify / commit.
// See include/flashmesh.h for the contract of every entry point.
#include "../../include/flashmesh.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <cstdlib>
#include <string>
#include <type_traits>
#include <vector>

#include "fm_device.h"
#include "fm_kernels_basic.h"
#include "fm_kernels_step.h"
#include "fm_kernels_mfma.h"
#include "fm_kernels_persist.h"
#include "fm_kernels_prefill.h"

// Staging area of fm_prefill_condition_static: a file-scope device array instead of memory owned by a context, so that
// the call touches no allocator.  Every GPU the library runs on holds its own copy at its own address; the host-side
// name below is only a handle for hipGetSymbolAddress and is never passed to a kernel or a copy.
#define FM_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[FM_STATIC_SCRATCH_BYTES];

#define RS_C 32  // ring sizes (positions kept per sequence) at the coordinate / vertex / face level
#define RS_V 16
#define RS_F 8

namespace {

struct Layer {
  float *g1, *g2, *g3;
  void *wqkv, *wo, *cq, *ckv, *co, *w1, *w2;  // storage type T, [out, in]
  void* wqkv_rp;                               // persistent path: q/k tiles hold whole rotary pairs
  void *Kc, *Vc;                               // [S][H][cap][64]
  void *Km, *Vm;                               // [S][H][M][64]
  int level;                                   // 0 coordinate, 1 vertex, 2 face
};

struct SpLevel {  // SP heads of one level, head-major contiguous so that one grouped GEMM serves all heads
  int cnt;
  float* g;
  void *wq, *wo, *cq, *co, *lin;
};
struct HfLevel {
  int cnt;
  float* g;
  void *wq, *w1, *w2;
};

struct LoadItem { size_t blob_off, n; void* dst; bool f32; int N, K, perm; };  // N, K > 0: linear weight [N, K]

// device address of `scratch` on each GPU, looked up once per device (at the first fm_create on it)
std::mutex g_scratch_mu;
void* g_scratch_addr[64] = {};

}  // namespace

struct fm_ctx {
  fm_config cfg;
  Dims D;
  InvFreq inv;
  hipStream_t stream;
  bool bf16;
  size_t esz;
  int ff, hff, Vpad;
  int Rc, Rv, Rf;  // row slots per level
  std::string err;
  std::vector<void*> allocs;
  std::vector<LoadItem> items;
  size_t blob_elems;
  bool weights_loaded;
  std::vector<bool> prefilled;

  // parameters
  void* emb;
  std::vector<Layer> stacks[5];  // cpre, vpre, face, vpost, cpost
  void *short_cv, *short_vf, *lm;
  float* gf;
  SpLevel sp[3];
  SpLevel sp_all;          // the heads of all three levels as one group list, in memory order point, face, coordinate
  bool sp_merged = false;  // half path, 64-wide heads: the three SP chains run as one chain of grouped launches
  const float** lm_src = nullptr;   // rows of the output head's input: coordinate SP head outputs, then coordinate HF outputs
  HfLevel hfc, hfv;
  float* label_w;     // label head of the correct stage [3][d]
  float *lab_v, *lab_f;   // label distributions of the point pipeline [S][nspv][3] and the face pipeline [S][nhfv][3]
  Sampling smp;           // sampled decoding (temperature 0 = greedy): proposals kept between draft and verify
  int correct_hist = 0;   // historical vertices the correct stage looks at; 0 = stage off (no label rows are computed)

  // state
  StateDev st;
  // rings (fp32)
  float *ring_hc, *ring_hv, *ring_yf, *ring_yv, *tap_c, *tap_v, *tap_f;
  // verify scratch
  int *pos[3], *limx[3];
  float2* cs[3];
  float* h[3];
  void *xn, *qT, *attT, *mid;
  float *qkv, *logits;
  MfmaRes mres;       // workspaces of the MFMA kernels (half-precision path)
  float* stage;       // staging for weight conversion / prefill GEMM output
  size_t stage_elems;
  unsigned char* static_scratch = nullptr;   // this GPU's copy of the file-scope staging array
  // draft scratch
  DraftRows dr;
  DraftBufs db;
  float *spv_out, *spf_out, *hfv_out, *dh, *dkeep, *dtmp, *dlogits;
  float *dist_c, *dist_v, *dist_f;
  void *dxn, *dq, *datt, *dmid;
  Replay replay;
  int *gen_tok, *gen_len;  // block buffers used by fm_generate
  int* gen_acc;
  int* host_flag;          // pinned: [0] alive flag, [1..S] lagged copy of the committed lengths
  std::vector<int> len_bound;   // host upper bound on each sequence's committed coordinate length
  long commits = 0;             // fm_commit calls so far
  bool sticky_error = false;    // a launch wrapper refused its arguments (message in err); reported by the entry point
  // persistent verify kernel (one sequence, block <= 32, half-precision path)
  bool persist;
  int persist_failures = 0;   // times the single-launch kernel gave up (the context then left that path)
  PkArgs pk;
  PrefillLayer* pf_layers = nullptr;   // per-block table of the tiled prefill GEMM (null: per-block launches)
  int pf_n = 0, pf_grid = 0;           // blocks in the table; workgroups of its launch (one per compute unit, multiple of 8)
  unsigned pk_epoch;
  size_t pk_lds;           // dynamic LDS of the persistent kernel (none at present)
  double weight_bytes;
};

namespace {

int fail(fm_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  return code;
}

#define HIPCHK(c, expr)                                                                         \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) return fail(c, FM_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

template <typename U> int dalloc(fm_ctx* c, U** p, size_t n, bool zero = true) {
  void* q = nullptr;
  const size_t bytes = (n ? n : 1) * sizeof(U);
  if (hipMalloc(&q, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, FM_ENOMEM, "hipMalloc of %zu bytes failed", bytes);
  }
  if (zero && hipMemset(q, 0, bytes) != hipSuccess) return fail(c, FM_EHIP, "hipMemset failed");
  c->allocs.push_back(q);
  *p = (U*)q;
  return FM_OK;
}
int dalloc_t(fm_ctx* c, void** p, size_t n) {  // n elements of the storage type
  uint8_t* q;
  int rc = dalloc(c, &q, n * c->esz);
  *p = q;
  return rc;
}
#define TRY(x) do { int rc_ = (x); if (rc_ != FM_OK) return rc_; } while (0)

int level_cap(const fm_ctx* c, int level) { return level == 0 ? c->D.capc : level == 1 ? c->D.capv : c->D.capf; }
int level_window(const fm_ctx* c, int level) { return level == 0 ? c->D.wc : level == 1 ? c->D.wv : c->D.wf; }
// Upper bound on the keys any row of the next pass can see at `level`, from the host's bound on the committed
// lengths (a commit adds at most block_max tokens; fm_read_state and the generate loop tighten it).
int level_key_bound(const fm_ctx* c, int level) {
  int b = 0;
  for (int s = 0; s < c->D.S; s++) b = std::max(b, c->len_bound[s]);
  const long keys = (long)b + c->D.Bm;                  // positions P .. P + block_max - 1 are in the pass
  const long k = level == 0 ? keys : level == 1 ? (keys + 2) / 3 + 1 : (keys + 8) / 9 + 1;
  return (int)std::min<long>(k, level_cap(c, level));
}
const int kStackLevel[5] = {0, 1, 2, 1, 0};

// ------------------------------------------------------------------------------------------
// launch wrappers
// ------------------------------------------------------------------------------------------
template <typename T>
void gemm(fm_ctx* c, int epi, const void* X, long ldx, long gsx, const void* W, long gsw, void* Y, long ldy, long gsy,
          const float* R, long ldr, long gsr, int M, int N, int K, int groups, const int* flag) {
  GemmArgs a{X, ldx, gsx, W, gsw, Y, ldy, gsy, R, ldr, gsr, M, N, K, flag, nullptr, 0.f, nullptr, nullptr, 0, nullptr, nullptr, 0, 0, 0};
  if (mfma_gemm_launch<T>(c->mres, a, epi, groups, c->stream)) return;
  // the plain kernel reads row-major weights: only the fp32 path has those
  if (!std::is_same<T, float>::value) { fail(c, FM_EINVAL, "gemm: unsupported shape M=%d N=%d K=%d", M, N, K); c->sticky_error = true; return; }
  dim3 grid((N + 3) / 4, groups);
  if (epi == EPI_F32) hipLaunchKernelGGL((k_gemm_simple<T, EPI_F32>), grid, dim3(256), 0, c->stream, a);
  else if (epi == EPI_GELU_T) hipLaunchKernelGGL((k_gemm_simple<T, EPI_GELU_T>), grid, dim3(256), 0, c->stream, a);
  else hipLaunchKernelGGL((k_gemm_simple<T, EPI_T>), grid, dim3(256), 0, c->stream, a);
}

template <typename T>
void attention(fm_ctx* c, const void* q, const int* limit, int rows, int RPS, const void* Kc, const void* Vc,
               long seq_stride, int cap, void* out, const int* flag, bool dense = false, int key_bound = 1 << 30,
               int window = 0) {
  if (mfma_attn_launch<T>(c->mres, q, limit, rows, RPS, Kc, Vc, seq_stride, cap, out, c->D.H, flag, dense, key_bound, window, c->stream, c->D.hd)) return;
  // the plain kernel reads row-major caches: only the fp32 path has those
  if (!std::is_same<T, float>::value) { fail(c, FM_EINVAL, "attention: unsupported row set (%d rows, %d per sequence)", rows, RPS); c->sticky_error = true; return; }
#define FM_ATTN(HDV) hipLaunchKernelGGL((k_attn_simple<T, HDV>), dim3(rows, c->D.H), dim3(256), 0, c->stream, (const T*)q, limit, RPS, \
                                        (const T*)Kc, (const T*)Vc, seq_stride, cap, (T*)out, c->D.H, flag, window)
  if (c->D.hd == 64) FM_ATTN(64); else if (c->D.hd == 96) FM_ATTN(96); else FM_ATTN(128);
#undef FM_ATTN
}

template <typename T>
void rmsnorm(fm_ctx* c, const float* src, const float* const* srcptr, const float* gain, int gain_mod, void* out,
             float* keep, int rows, const int* flag) {
  hipLaunchKernelGGL((k_rmsnorm<T>), dim3(rows), dim3(256), 0, c->stream, src, srcptr, gain, gain_mod, (T*)out, keep,
                     c->D.d, c->cfg.rms_eps, flag);
}

// Y = RMSNorm(h; gain) W^T for the rows of the fp32 residual stream h [rows, d].  Half-precision path: one fused
// launch (the GEMM normalises on the fly); fp32 path: norm into `xn`, then the plain GEMM.
template <typename T>
void gemm_norm(fm_ctx* c, int epi, const float* h, const float* gain, const void* W, void* Y, long ldy, int rows, int N,
               const int* flag) {
  const int d = c->D.d;
  if (std::is_same<T, f16_t>::value) {
    GemmArgs a{h, d, 0, W, 0, Y, ldy, 0, nullptr, 0, 0, rows, N, d, flag, gain, c->cfg.rms_eps, nullptr, nullptr, 0, nullptr, nullptr, 0, 0, 0};
    if (mfma_gemm_launch<T>(c->mres, a, epi, 1, c->stream)) return;
    fail(c, FM_EINVAL, "gemm_norm: unsupported shape M=%d N=%d K=%d", rows, N, d);
    c->sticky_error = true;
    return;
  }
  rmsnorm<T>(c, h, nullptr, gain, 0, c->xn, nullptr, rows, flag);
  gemm<T>(c, epi, c->xn, d, 0, W, 0, Y, ldy, 0, nullptr, 0, 0, rows, N, d, 1, flag);
}

// rotary position on q (and k), conversion to the storage type, optional append to a K/V cache
template <typename T>
void rope_append(fm_ctx* c, const float* qkv, long ldq, const float2* cs, const int* pos, int rows, int RPS, void* q,
                 void* Kc, void* Vc, int cap, const int* flag) {
  if (std::is_same<T, f16_t>::value) {
#define FM_ROPEH(HDV) hipLaunchKernelGGL((k_rope_append_h<HDV>), dim3(rows), dim3(256), 0, c->stream, qkv, ldq, cs, pos, RPS, (f16_t*)q, \
                                         (f16_t*)Kc, (f16_t*)Vc, c->D.H, (cap + 31) / 32, flag)
    if (c->D.hd == 64) FM_ROPEH(64); else if (c->D.hd == 96) FM_ROPEH(96); else FM_ROPEH(128);
#undef FM_ROPEH
  } else {
#define FM_ROPE(HDV) hipLaunchKernelGGL((k_rope_append<float, HDV>), dim3(rows), dim3(256), 0, c->stream, qkv, ldq, cs, pos, RPS, (float*)q, \
                                        (float*)Kc, (float*)Vc, c->D.H, cap, flag)
    if (c->D.hd == 64) FM_ROPE(64); else if (c->D.hd == 96) FM_ROPE(96); else FM_ROPE(128);
#undef FM_ROPE
  }
}

// elements of one (sequence) slice of a K or V cache with `cap` key positions
size_t cache_seq_elems(const fm_ctx* c, int cap) {
  return c->bf16 ? (size_t)c->D.H * ((cap + 31) / 32) * 32 * c->D.hd : (size_t)c->D.H * cap * c->D.hd;
}

// one transformer block on the row set of `level` (Sec. 3.1: self-attention, cross-attention to c, FFN)
template <typename T>
void run_block(fm_ctx* c, const Layer& L, int level) {
  const Dims& D = c->D;
  const int d = D.d, rows = level == 0 ? c->Rc : level == 1 ? c->Rv : c->Rf;
  const int RPS = level == 0 ? D.Bm : level == 1 ? D.VB : D.FB;
  const int cap = level_cap(c, level);
  float* h = c->h[level];
  const int* flag = c->st.alive;
  if (std::is_same<T, f16_t>::value && D.hd == 64) {
    // norm1, fused q,k,v projection, rotary, q out and cache append in one launch (written for 64-wide heads; the
    // wider heads of the paper's own shapes take the two launches below)
    GemmArgs a{h, d, 0, L.wqkv, 0, c->qT, d, 0, nullptr, 0, 0, rows, 3 * d, d, flag, L.g1, c->cfg.rms_eps,
               c->cs[level], c->pos[level], RPS, L.Kc, L.Vc, (long)cache_seq_elems(c, cap), (cap + 31) / 32, D.H};
    if (!mfma_gemm_launch<T>(c->mres, a, EPI_QKV, 1, c->stream)) { fail(c, FM_EINVAL, "qkv: unsupported shape"); c->sticky_error = true; }
  } else {
    gemm_norm<T>(c, EPI_F32, h, L.g1, L.wqkv, c->qkv, 3 * d, rows, 3 * d, flag);
    rope_append<T>(c, c->qkv, (long)3 * d, c->cs[level], c->pos[level], rows, RPS, c->qT, L.Kc, L.Vc, cap, flag);
  }
  attention<T>(c, c->qT, c->pos[level], rows, RPS, L.Kc, L.Vc, (long)cache_seq_elems(c, cap), cap, c->attT, flag, false,
               level_key_bound(c, level), level_window(c, level));
  gemm<T>(c, EPI_F32, c->attT, d, 0, L.wo, 0, h, d, 0, h, d, 0, rows, d, d, 1, flag);
  gemm_norm<T>(c, EPI_T, h, L.g2, L.cq, c->qT, d, rows, d, flag);
  attention<T>(c, c->qT, c->limx[level], rows, RPS, L.Km, L.Vm, (long)cache_seq_elems(c, D.M), D.M, c->attT, flag, true);
  gemm<T>(c, EPI_F32, c->attT, d, 0, L.co, 0, h, d, 0, h, d, 0, rows, d, d, 1, flag);
  gemm_norm<T>(c, EPI_GELU_T, h, L.g3, L.w1, c->mid, c->ff, rows, c->ff, flag);
  gemm<T>(c, EPI_F32, c->mid, c->ff, 0, L.w2, 0, h, d, 0, h, d, 0, rows, d, c->ff, 1, flag);
}

void ring_save(fm_ctx* c, const float* src, float* ring, int level, int RS) {
  const Dims& D = c->D;
  const int rows = level == 0 ? c->Rc : level == 1 ? c->Rv : c->Rf;
  const int RPS = level == 0 ? D.Bm : level == 1 ? D.VB : D.FB;
  hipLaunchKernelGGL(k_ring_save, dim3(rows), dim3(256), 0, c->stream, src, ring, c->pos[level], RPS, RS, D.d);
}

template <typename T>
void run_stack(fm_ctx* c, int stack, float* tap_ring, int tap_rs) {
  const int level = kStackLevel[stack];
  const size_t n = c->stacks[stack].size();
  for (size_t i = 0; i < n; i++) {
    if (tap_ring && i == n - 1) ring_save(c, c->h[level], tap_ring, level, tap_rs);
    run_block<T>(c, c->stacks[stack][i], level);
  }
}

// Word that the single-launch verify kernel raises when one of its bounded waits gave up (null on the per-operator
// path): the acceptance and commit kernels then report 0 accepted tokens and change nothing.
const unsigned* pass_failed(const fm_ctx* c) { return c->persist ? c->pk.abort_word : nullptr; }

// per verify row: the backbone's greedy token (or, with sampled decoding, the rejection test and the resampled token),
// then the accepted length per sequence
void choose_and_accept(fm_ctx* c, const float* logits, int32_t* accepted) {
  const Dims& D = c->D;
  if (c->smp.temperature > 0.f) {
    hipLaunchKernelGGL(k_sample_rows, dim3(c->Rc), dim3(256), 0, c->stream, c->st, D, logits, c->smp);
    hipLaunchKernelGGL(k_accept, dim3(1), dim3(64), 0, c->stream, c->st, D, accepted, (const int*)c->smp.accflag, pass_failed(c));
  } else {
    hipLaunchKernelGGL(k_argmax_rows, dim3(c->Rc), dim3(256), 0, c->stream, logits, D.V, D.ban ? D.nbins : D.V, c->st.y, c->st.counters + 2);
    hipLaunchKernelGGL(k_accept, dim3(1), dim3(64), 0, c->stream, c->st, D, accepted, (const int*)nullptr, pass_failed(c));
  }
}

template <typename T>
int verify_impl(fm_ctx* c, const int32_t* block_tok, const int32_t* block_len, float* logits_out, int32_t* accepted) {
  const Dims& D = c->D;
  const int d = D.d;
  hipLaunchKernelGGL(k_verify_setup, dim3(std::min(16, (D.S * D.Bm * (D.hd / 2) + 255) / 256)), dim3(256), 0, c->stream, c->st, D, c->inv, block_tok, block_len,
                     c->pos[0], c->pos[1], c->pos[2], c->limx[0], c->limx[1], c->limx[2], c->cs[0], c->cs[1], c->cs[2]);
  if (c->persist) {
    // the whole backbone forward in one launch (see fm_kernels_persist.h), then greedy choice and acceptance
    float* lgp = logits_out ? logits_out : c->logits;
    c->pk.logits = lgp;
    c->pk.epoch = ++c->pk_epoch;
    if (c->pk.RS == 32) hipLaunchKernelGGL(k_verify_persist<2>, dim3(PK_NWG), dim3(256), c->pk_lds, c->stream, c->pk);
    else hipLaunchKernelGGL(k_verify_persist<1>, dim3(PK_NWG), dim3(256), c->pk_lds, c->stream, c->pk);
    choose_and_accept(c, lgp, accepted);
    HIPCHK(c, hipGetLastError());
    return FM_OK;
  }
  hipLaunchKernelGGL((k_embed<T>), dim3(c->Rc), dim3(256), 0, c->stream, c->st.vtok, c->pos[0], (const T*)c->emb,
                     c->h[0], d);
  const int* flag = c->st.alive;
  // coordinate level, first half
  run_stack<T>(c, 0, nullptr, 0);
  ring_save(c, c->h[0], c->ring_hc, 0, RS_C);
  // shorten coordinate -> vertex
  hipLaunchKernelGGL((k_pool3<T>), dim3(c->Rv), dim3(256), 0, c->stream, c->ring_hc, RS_C, c->pos[1], D.VB, (T*)c->xn, d);
  gemm<T>(c, EPI_F32, c->xn, d, 0, c->short_cv, 0, c->h[1], d, 0, nullptr, 0, 0, c->Rv, d, d, 1, flag);
  run_stack<T>(c, 1, nullptr, 0);
  ring_save(c, c->h[1], c->ring_hv, 1, RS_V);
  // shorten vertex -> face
  hipLaunchKernelGGL((k_pool3<T>), dim3(c->Rf), dim3(256), 0, c->stream, c->ring_hv, RS_V, c->pos[2], D.FB, (T*)c->xn, d);
  gemm<T>(c, EPI_F32, c->xn, d, 0, c->short_vf, 0, c->h[2], d, 0, nullptr, 0, 0, c->Rf, d, d, 1, flag);
  run_stack<T>(c, 2, c->tap_f, RS_F);
  ring_save(c, c->h[2], c->ring_yf, 2, RS_F);
  // upsample face -> vertex (repeat + skip), vertex level second half
  hipLaunchKernelGGL(k_upsample_add, dim3(c->Rv), dim3(256), 0, c->stream, c->h[1], c->pos[1], D.VB, c->ring_yf, RS_F, d);
  run_stack<T>(c, 3, c->tap_v, RS_V);
  ring_save(c, c->h[1], c->ring_yv, 1, RS_V);
  // upsample vertex -> coordinate, coordinate level second half
  hipLaunchKernelGGL(k_upsample_add, dim3(c->Rc), dim3(256), 0, c->stream, c->h[0], c->pos[0], D.Bm, c->ring_yv, RS_V, d);
  run_stack<T>(c, 4, c->tap_c, RS_C);
  // output head, greedy prediction, acceptance
  float* lg = logits_out ? logits_out : c->logits;
  gemm_norm<T>(c, EPI_F32, c->h[0], c->gf, c->lm, lg, D.V, c->Rc, D.V, flag);
  choose_and_accept(c, lg, accepted);
  HIPCHK(c, hipGetLastError());
  return FM_OK;
}

// SP head chain (Eq. 1) for the row set `set` of one level; writes fp32 features to out (row stride ldo)
template <typename T>
void run_sp(fm_ctx* c, int set, const SpLevel& sp, const Layer& last, int level, float* out, long ldo, long gso,
            const int* flag) {
  const Dims& D = c->D;
  const int d = D.d, G = sp.cnt, rows = D.S * G;
  if (G == 0) return;
  const int cap = level_cap(c, level);
  const long dd = (long)d * d;
  rmsnorm<T>(c, nullptr, c->dr.src[set], sp.g, G, c->dxn, c->dkeep, rows, flag);
  gemm<T>(c, EPI_F32, c->dxn, (long)G * d, d, sp.wq, dd, c->dtmp, (long)G * d, d, nullptr, 0, 0, D.S, d, d, G, flag);
  rope_append<T>(c, c->dtmp, (long)d, c->dr.cs[set], c->dr.pos[set], rows, G, c->dq, nullptr, nullptr, cap, flag);
  attention<T>(c, c->dq, c->dr.lim[set], rows, G, last.Kc, last.Vc, (long)cache_seq_elems(c, cap), cap, c->datt, flag, false,
               level_key_bound(c, level), level_window(c, level));
  gemm<T>(c, EPI_T, c->datt, (long)G * d, d, sp.wo, dd, c->dxn, (long)G * d, d, nullptr, 0, 0, D.S, d, d, G, flag);
  gemm<T>(c, EPI_T, c->dxn, (long)G * d, d, sp.cq, dd, c->dq, (long)G * d, d, nullptr, 0, 0, D.S, d, d, G, flag);
  attention<T>(c, c->dq, c->dr.limx[set], rows, G, last.Km, last.Vm, (long)cache_seq_elems(c, D.M), D.M, c->datt, flag, true);
  gemm<T>(c, EPI_T, c->datt, (long)G * d, d, sp.co, dd, c->dxn, (long)G * d, d, nullptr, 0, 0, D.S, d, d, G, flag);
  gemm<T>(c, EPI_F32, c->dxn, (long)G * d, d, sp.lin, dd, out, ldo, gso, c->dkeep, (long)G * d, d, D.S, d, d, G, flag);
}

// The SP chains (Eq. 1) of all three levels as one chain of grouped launches (half path): the row set is, per sequence,
// the point-, face- and coordinate-level rows behind each other, every GEMM is grouped over all heads (S rows per head),
// and the two attention launches take one cache per level.  Same arithmetic per row as run_sp.  Rows of a level that
// does not fire in this step carry limit -1 (no keys) and produce values nobody reads.
void run_sp_all(fm_ctx* c, const int* flag) {
  typedef f16_t T;
  const Dims& D = c->D;
  const SpLevel& A = c->sp_all;
  const int d = D.d, G = A.cnt, S = D.S, rows = S * G;
  if (G == 0) return;
  const long dd = (long)d * d, ld = (long)G * d;
  const int nrow[3] = {D.nspv, D.nspf, D.Dc}, lev[3] = {1, 2, 0}, set[3] = {1, 2, 0};
  const Layer* last[3] = {&c->stacks[3].back(), &c->stacks[2].back(), &c->stacks[4].back()};
  rmsnorm<T>(c, nullptr, c->dr.src[1], A.g, G, c->dxn, c->dkeep, rows, flag);
  gemm<T>(c, EPI_F32, c->dxn, ld, d, A.wq, dd, c->dtmp, ld, d, nullptr, 0, 0, S, d, d, G, flag);
  rope_append<T>(c, c->dtmp, (long)d, c->dr.cs[1], c->dr.pos[1], rows, G, c->dq, nullptr, nullptr, 32, flag);
  AttnLevelHost lv[3];
  long off = 0;
  for (int z = 0; z < 3; z++) {
    const int cap = level_cap(c, lev[z]);
    lv[z] = AttnLevelHost{(const f16_t*)c->dq + off * d, c->dr.lim[set[z]], nrow[z], last[z]->Kc, last[z]->Vc,
                          (long)cache_seq_elems(c, cap), cap, (f16_t*)c->datt + off * d, false, level_key_bound(c, lev[z]),
                          level_window(c, lev[z])};
    off += nrow[z];
  }
  if (!mfma_attn_launch_levels(c->mres, lv, S, G, D.H, flag, c->stream)) { fail(c, FM_EINVAL, "merged SP attention: unsupported row sets"); c->sticky_error = true; return; }
  gemm<T>(c, EPI_T, c->datt, ld, d, A.wo, dd, c->dxn, ld, d, nullptr, 0, 0, S, d, d, G, flag);
  gemm<T>(c, EPI_T, c->dxn, ld, d, A.cq, dd, c->dq, ld, d, nullptr, 0, 0, S, d, d, G, flag);
  off = 0;
  for (int z = 0; z < 3; z++) {
    lv[z] = AttnLevelHost{(const f16_t*)c->dq + off * d, c->dr.limx[set[z]], nrow[z], last[z]->Km, last[z]->Vm,
                          (long)cache_seq_elems(c, D.M), D.M, (f16_t*)c->datt + off * d, true, 1 << 30, 0};
    off += nrow[z];
  }
  if (!mfma_attn_launch_levels(c->mres, lv, S, G, D.H, flag, c->stream)) { fail(c, FM_EINVAL, "merged SP cross-attention: unsupported row sets"); c->sticky_error = true; return; }
  gemm<T>(c, EPI_T, c->datt, ld, d, A.co, dd, c->dxn, ld, d, nullptr, 0, 0, S, d, d, G, flag);
  // outputs: per sequence the point, face and coordinate rows behind each other (spv_out, spf_out and the rows the output
  // head's pointer table names)
  gemm<T>(c, EPI_F32, c->dxn, ld, d, A.lin, dd, c->spv_out, ld, d, c->dkeep, ld, d, S, d, d, G, flag);
}

// HF block chain (Eq. 3-6) for row set `set`: `per_seq` rows per sequence, `G` parameter sets, `mult`
// consecutive row groups of G sharing the sets (mult = 2 for the coordinate level: point and face pipelines)
template <typename T>
void run_hf(fm_ctx* c, int set, const HfLevel& hf, int mult, const Layer& last, int level, float* out, const int* flag) {
  const Dims& D = c->D;
  const int d = D.d, G = hf.cnt, per_seq = G * mult, rows = D.S * per_seq;
  if (G == 0) return;
  const int cap = level_cap(c, level);
  const long dd = (long)d * d, dh = (long)d * c->hff;
  const int Mg = D.S * mult;           // rows per parameter set
  const long ld = (long)G * d;         // stride between those rows
  rmsnorm<T>(c, nullptr, c->dr.src[set], hf.g, G, c->dxn, c->dkeep, rows, flag);
  gemm<T>(c, EPI_F32, c->dxn, ld, d, hf.wq, dd, c->dtmp, ld, d, nullptr, 0, 0, Mg, d, d, G, flag);
  rope_append<T>(c, c->dtmp, (long)d, c->dr.cs[set], c->dr.pos[set], rows, per_seq, c->dq, nullptr, nullptr, cap, flag);
  attention<T>(c, c->dq, c->dr.lim[set], rows, per_seq, last.Kc, last.Vc, (long)cache_seq_elems(c, cap), cap, c->datt, flag, false,
               level_key_bound(c, level), level_window(c, level));
  gemm<T>(c, EPI_GELU_T, c->datt, ld, d, hf.w1, dh, c->dmid, (long)G * c->hff, c->hff, nullptr, 0, 0, Mg, c->hff, d, G, flag);
  gemm<T>(c, EPI_F32, c->dmid, (long)G * c->hff, c->hff, hf.w2, dh, out, ld, d, c->dkeep, ld, d, Mg, d, c->hff, G, flag);
}

template <typename T>
int draft_impl(fm_ctx* c, int32_t* block_tok, int32_t* block_len, int speculative) {
  const Dims& D = c->D;
  const int d = D.d;
  if (speculative) {
    hipLaunchKernelGGL(k_draft_setup, dim3(D.S), dim3(256), 0, c->stream, c->st, D, c->inv, c->dr, c->db);
    const int *f_alive = c->dr.flags, *f_v = c->dr.flags + 1, *f_f = c->dr.flags + 2;
    const Layer& lastc = c->stacks[4].back();
    const Layer& lastv = c->stacks[3].back();
    const Layer& lastf = c->stacks[2].back();
    const int nLM = D.S * (D.Dc + 2 * D.nhfc);
    if (std::is_same<T, f16_t>::value && c->sp_merged) {
      run_sp_all(c, f_alive);
    } else {
      // coordinate level: SP heads straight to the output head
      run_sp<T>(c, 0, c->sp[0], lastc, 0, c->dh, (long)D.Dc * d, d, f_alive);
      // point level: SP heads on the vertex feature; their outputs feed the coordinate HF rows of pipe 0
      run_sp<T>(c, 1, c->sp[1], lastv, 1, c->spv_out, (long)D.nspv * d, d, f_v);
      // face level: SP heads on the face feature, vertex-level HF, then coordinate HF rows of pipe 1
      run_sp<T>(c, 2, c->sp[2], lastf, 2, c->spf_out, (long)D.nspf * d, d, f_f);
    }
    run_hf<T>(c, 3, c->hfv, 1, lastv, 1, c->hfv_out, f_f);
    if (c->correct_hist > 0 && D.nspv + D.nhfv > 0)     // label rows of the point-level features (Sec. 3.2)
      hipLaunchKernelGGL(k_label_rows, dim3(D.S * (D.nspv + D.nhfv)), dim3(64), 0, c->stream, D, c->dr, c->spv_out, c->db.spv_rs, c->hfv_out,
                         c->label_w, c->lab_v, c->lab_f);
    run_hf<T>(c, 4, c->hfc, 2, lastc, 0, c->dh + (long)D.S * D.Dc * d, f_alive);
    if (nLM > 0) {
      rmsnorm<T>(c, nullptr, c->lm_src, c->gf, 0, c->dxn, nullptr, nLM, f_alive);
      gemm<T>(c, EPI_F32, c->dxn, d, 0, c->lm, 0, c->dlogits, D.V, 0, nullptr, 0, 0, nLM, D.V, d, 1, f_alive);
      hipLaunchKernelGGL(k_dist_store, dim3(nLM), dim3(256), 0, c->stream, c->dlogits, D, c->dr, c->dist_c, c->dist_v,
                         c->dist_f);
    }
  }
  hipLaunchKernelGGL(k_merge, dim3(D.S), dim3(1024), 0, c->stream, c->st, D, c->dr, c->dist_c, c->dist_v, c->dist_f,
                     c->replay, speculative, block_tok, block_len, c->smp);
  HIPCHK(c, hipGetLastError());
  return FM_OK;
}

// staging bytes a prefill call needs: the memory in fragment order (tiled GEMM), or the memory in the storage type
// followed by the fp32 K/V rows of one block
size_t prefill_stage_bytes(const fm_ctx* c) {
  const size_t M = c->D.M, d = c->D.d;
  if (c->bf16 && c->pf_layers) return M * d * sizeof(f16_t);
  return M * d * c->esz + M * 2 * d * sizeof(float);
}

template <typename T>
int prefill_impl(fm_ctx* c, int seq, const float* mem_dev, void* stage_area) {
  const Dims& D = c->D;
  const int d = D.d;
  // condition memory in the storage type (dmid is large enough: M*d <= checked at create)
  if (std::is_same<T, f16_t>::value && c->pf_layers) {
    // memory -> MFMA fragment order (the same tiling as a weight matrix), then one launch for all blocks
    f16_t* Xt = (f16_t*)stage_area;
    hipLaunchKernelGGL(k_tile_weight, dim3(1024), dim3(256), 0, c->stream, mem_dev, Xt, D.M, d, D.M, 0);
#define FM_PREFILL(HDV) hipLaunchKernelGGL((k_prefill_kv<HDV>), dim3(c->pf_grid), dim3(256), PF_LDS_BYTES, c->stream, (const f16_t*)Xt, \
                                           (const PrefillLayer*)c->pf_layers, (long)((size_t)seq * cache_seq_elems(c, D.M)), d / 32, d, D.M, c->pf_n)
    if (D.hd == 64) FM_PREFILL(64); else if (D.hd == 96) FM_PREFILL(96); else FM_PREFILL(128);
#undef FM_PREFILL
    hipLaunchKernelGGL(k_reset_seq, dim3(1), dim3(64), 0, c->stream, c->st, D, seq, D.nbins);
    HIPCHK(c, hipGetLastError());
    return FM_OK;
  }
  T* memT = (T*)stage_area;  // [M*d] T followed by fp32 [M][2d]
  float* kv = (float*)((unsigned char*)stage_area + (size_t)D.M * d * sizeof(T));
  hipLaunchKernelGGL((k_convert<T>), dim3(512), dim3(256), 0, c->stream, mem_dev, memT, (long)D.M * d);
  for (int st = 0; st < 5; st++)
    for (auto& L : c->stacks[st]) {
      gemm<T>(c, EPI_F32, memT, d, 0, L.ckv, 0, kv, 2 * d, 0, nullptr, 0, 0, D.M, 2 * d, d, 1, nullptr);
      T* Km = (T*)L.Km + (size_t)seq * cache_seq_elems(c, D.M);
      T* Vm = (T*)L.Vm + (size_t)seq * cache_seq_elems(c, D.M);
      if (std::is_same<T, f16_t>::value) {
#define FM_MEMKVH(HDV) hipLaunchKernelGGL((k_mem_kv_store_h<HDV>), dim3(D.M), dim3(256), 0, c->stream, kv, (f16_t*)Km, (f16_t*)Vm, D.H, D.M, \
                                          (D.M + 31) / 32)
        if (D.hd == 64) FM_MEMKVH(64); else if (D.hd == 96) FM_MEMKVH(96); else FM_MEMKVH(128);
#undef FM_MEMKVH
      } else {
#define FM_MEMKV(HDV) hipLaunchKernelGGL((k_mem_kv_store<float, HDV>), dim3(D.M), dim3(256), 0, c->stream, kv, (float*)Km, (float*)Vm, D.H, D.M)
        if (D.hd == 64) FM_MEMKV(64); else if (D.hd == 96) FM_MEMKV(96); else FM_MEMKV(128);
#undef FM_MEMKV
      }
    }
  hipLaunchKernelGGL(k_reset_seq, dim3(1), dim3(64), 0, c->stream, c->st, D, seq, D.nbins);
  HIPCHK(c, hipGetLastError());
  return FM_OK;
}

// After a synchronisation: did the single-launch verify kernel give up waiting (it never hangs, it reports)?
// If so the passes enqueued since then have accepted nothing and committed nothing (k_accept / k_commit look at the
// same word), so the decode state is that of the last good commit.  The failure is reported once with its diagnosis,
// the words are re-armed, and the context continues on the per-operator path, which shares weights, caches and rings.
int check_persist(fm_ctx* c) {
  if (!c->persist) return FM_OK;
  unsigned w[9] = {0};
  HIPCHK(c, hipMemcpy(w, c->pk.abort_word, sizeof w, hipMemcpyDeviceToHost));
  if (!w[0]) return FM_OK;
  const unsigned rearm[9] = {0u, 0xFFFFFFFFu, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
  HIPCHK(c, hipMemcpy(c->pk.abort_word, rearm, sizeof rearm, hipMemcpyHostToDevice));
  c->persist = false;
  c->persist_failures++;
  return fail(c, FM_EHIP, "persistent verify kernel timed out: earliest stuck stage %u; first missing element: stage %u "
              "workgroup %u thread %u index %u expected tag %u saw %u (epoch %u); passes since then accepted nothing, the "
              "context continues with one launch per operator", w[1], w[5], w[6], w[7], w[8], w[3], w[4], c->pk_epoch);
}

// Build the parameter tables and the list of (blob range -> device destination) in manifest order.
int build_params(fm_ctx* c) {
  const Dims& D = c->D;
  const size_t d = D.d, ff = c->ff, hff = c->hff, V = D.V;
  size_t off = 0;
  auto item = [&](void* dst, size_t n, bool f32) { c->items.push_back({off, n, dst, f32, 0, 0, 0}); off += n; };
  auto lin = [&](void* dst, size_t N, size_t K) { c->items.push_back({off, N * K, dst, false, (int)N, (int)K, 0}); off += N * K; };
  auto at = [&](void* base, size_t elems) { return (void*)((uint8_t*)base + elems * c->esz); };

  TRY(dalloc_t(c, &c->emb, V * d));
  item(c->emb, V * d, false);
  const int counts[5] = {c->cfg.l_cpre, c->cfg.l_vpre, c->cfg.l_face, c->cfg.l_vpost, c->cfg.l_cpost};
  for (int st = 0; st < 5; st++) {
    const int level = kStackLevel[st];
    const size_t cap = level_cap(c, level);
    for (int i = 0; i < counts[st]; i++) {
      Layer L{};
      L.level = level;
      TRY(dalloc(c, &L.g1, d)); TRY(dalloc(c, &L.g2, d)); TRY(dalloc(c, &L.g3, d));
      TRY(dalloc_t(c, &L.wqkv, 3 * d * d)); TRY(dalloc_t(c, &L.wo, d * d)); TRY(dalloc_t(c, &L.cq, d * d));
      TRY(dalloc_t(c, &L.ckv, 2 * d * d)); TRY(dalloc_t(c, &L.co, d * d));
      TRY(dalloc_t(c, &L.w1, ff * d)); TRY(dalloc_t(c, &L.w2, d * ff));
      TRY(dalloc_t(c, &L.Kc, D.S * cache_seq_elems(c, cap))); TRY(dalloc_t(c, &L.Vc, D.S * cache_seq_elems(c, cap)));
      TRY(dalloc_t(c, &L.Km, D.S * cache_seq_elems(c, D.M))); TRY(dalloc_t(c, &L.Vm, D.S * cache_seq_elems(c, D.M)));
      item(L.g1, d, true);
      if (c->bf16 && D.hd == 64) {
        // half path: the q and k tiles of the fused projection hold whole rotary pairs (both verify paths apply
        // the rotation in the GEMM epilogue), so only the permuted tiling is kept
        c->items.push_back({off, 3 * d * d, L.wqkv, false, (int)(3 * d), (int)d, (int)d});
        L.wqkv_rp = L.wqkv;
        off += 3 * d * d;
      } else {
        lin(L.wqkv, 3 * d, d);   // wq, wk, wv are consecutive in the blob
      }
      lin(L.wo, d, d);
      item(L.g2, d, true);
      lin(L.cq, d, d);
      lin(L.ckv, 2 * d, d);    // ck, cv consecutive
      lin(L.co, d, d);
      item(L.g3, d, true);
      lin(L.w1, ff, d);
      lin(L.w2, d, ff);
      c->stacks[st].push_back(L);
    }
  }
  TRY(dalloc_t(c, &c->short_cv, d * d)); lin(c->short_cv, d, d);
  TRY(dalloc_t(c, &c->short_vf, d * d)); lin(c->short_vf, d, d);
  TRY(dalloc(c, &c->gf, d)); item(c->gf, d, true);
  TRY(dalloc_t(c, &c->lm, (size_t)c->Vpad * d)); lin(c->lm, V, d);
  const int spcnt[3] = {D.Dc, D.nspv, D.nspf};
  // The heads of the three levels lie behind each other in device memory (point, face, coordinate: the order of the
  // merged row set), so that one grouped launch can serve all of them; the blob keeps its own order.
  {
    SpLevel& A = c->sp_all;
    A.cnt = D.Dc + D.nspv + D.nspf;
    const size_t n = A.cnt;
    TRY(dalloc(c, &A.g, n * d));
    TRY(dalloc_t(c, &A.wq, n * d * d)); TRY(dalloc_t(c, &A.wo, n * d * d)); TRY(dalloc_t(c, &A.cq, n * d * d));
    TRY(dalloc_t(c, &A.co, n * d * d)); TRY(dalloc_t(c, &A.lin, n * d * d));
    const size_t first[3] = {(size_t)D.nspv + D.nspf, 0, (size_t)D.nspv};
    for (int l = 0; l < 3; l++) {
      SpLevel& s = c->sp[l];
      s.g = A.g + first[l] * d;
      s.wq = at(A.wq, first[l] * d * d); s.wo = at(A.wo, first[l] * d * d); s.cq = at(A.cq, first[l] * d * d);
      s.co = at(A.co, first[l] * d * d); s.lin = at(A.lin, first[l] * d * d);
    }
  }
  for (int l = 0; l < 3; l++) {
    SpLevel& s = c->sp[l];
    s.cnt = spcnt[l];
    const size_t n = s.cnt;
    for (size_t k = 0; k < n; k++) {
      item(s.g + k * d, d, true);
      lin(at(s.wq, k * d * d), d, d); lin(at(s.wo, k * d * d), d, d);
      lin(at(s.cq, k * d * d), d, d); lin(at(s.co, k * d * d), d, d);
      lin(at(s.lin, k * d * d), d, d);
    }
  }
  HfLevel* hfs[2] = {&c->hfc, &c->hfv};
  const int hfcnt[2] = {D.nhfc, D.nhfv};
  for (int l = 0; l < 2; l++) {
    HfLevel& h = *hfs[l];
    h.cnt = hfcnt[l];
    const size_t n = h.cnt;
    TRY(dalloc(c, &h.g, n * d));
    TRY(dalloc_t(c, &h.wq, n * d * d)); TRY(dalloc_t(c, &h.w1, n * hff * d)); TRY(dalloc_t(c, &h.w2, n * d * hff));
    for (size_t k = 0; k < n; k++) {
      item(h.g + k * d, d, true);
      lin(at(h.wq, k * d * d), d, d);
      lin(at(h.w1, k * hff * d), hff, d);
      lin(at(h.w2, k * d * hff), d, hff);
    }
  }
  // label head of the correct stage (Sec. 3.2): [3][d], kept in fp32 (three dot products per point)
  TRY(dalloc(c, &c->label_w, 3 * d));
  item(c->label_w, 3 * d, true);
  c->blob_elems = off;
  return FM_OK;
}

// exchange buffers, layer table and argument block of the persistent verify kernel
int build_persist(fm_ctx* c) {
  const Dims& D = c->D;
  const size_t d = D.d;
  PkArgs& a = c->pk;
  memset(&a, 0, sizeof a);
  std::vector<PkLayer> hl;
  for (int st = 0; st < 5; st++) {
    a.first[st] = (int)hl.size();
    a.count[st] = (int)c->stacks[st].size();
    for (size_t i = 0; i < c->stacks[st].size(); i++) {
      const Layer& L = c->stacks[st][i];
      PkLayer p{};
      p.g1 = (pk_cf_t)L.g1; p.g2 = (pk_cf_t)L.g2; p.g3 = (pk_cf_t)L.g3;
      p.wqkv = (pk_cw_t)L.wqkv_rp; p.wo = (pk_cw_t)L.wo; p.cq = (pk_cw_t)L.cq; p.co = (pk_cw_t)L.co;
      p.w1 = (pk_cw_t)L.w1; p.w2 = (pk_cw_t)L.w2;
      p.Kc = (pk_w_t)L.Kc; p.Vc = (pk_w_t)L.Vc; p.Km = (pk_cw_t)L.Km; p.Vm = (pk_cw_t)L.Vm;
      p.level = L.level;
      p.last = i + 1 == c->stacks[st].size();
      p.tap = p.last && (st == 2 || st == 3 || st == 4);
      p.stack = st;
      hl.push_back(p);
    }
  }
  a.n_layers = (int)hl.size();
  PkLayer* dl;
  TRY(dalloc(c, &dl, hl.size()));
  if (hipMemcpy(dl, hl.data(), hl.size() * sizeof(PkLayer), hipMemcpyHostToDevice) != hipSuccess) return fail(c, FM_EHIP, "layer table copy failed");
  a.layers = dl;
  a.D = D; a.ff = c->ff; a.eps = c->cfg.rms_eps;
  a.R[0] = D.Bm; a.R[1] = D.VB; a.R[2] = D.FB;
  const int caps[3] = {D.capc, D.capv, D.capf};
  for (int l = 0; l < 3; l++) {
    a.capb[l] = (caps[l] + 31) / 32;
    int ns = PK_NWG / D.H;                       // about one attention unit per workgroup
    if (const char* e = getenv("FM_PK_NSPLIT")) ns = std::max(1, atoi(e));       // measurement switch: key ranges per head
    ns = std::min(ns, std::max(1, a.capb[l] / 2));
    a.nsplit[l] = std::max(1, std::min(ns, PK_MAXSPLIT));
    a.pos[l] = c->pos[l]; a.limx[l] = c->limx[l]; a.cs[l] = c->cs[l];
    a.win[l] = level_window(c, l);
  }
  a.capbM = (D.M + 31) / 32;
  a.nsplitM = std::max(1, std::min(std::min(PK_NWG / D.H, std::max(1, a.capbM / 2)), PK_MAXSPLIT));
  a.vtok = c->st.vtok;
  a.ring_hc = c->ring_hc; a.ring_hv = c->ring_hv; a.ring_yf = c->ring_yf; a.ring_yv = c->ring_yv;
  a.tap[0] = c->tap_c; a.tap[1] = c->tap_v; a.tap[2] = c->tap_f;
  a.emb = (const f16_t*)c->emb; a.short_cv = (const f16_t*)c->short_cv; a.short_vf = (const f16_t*)c->short_vf;
  a.lm = (const f16_t*)c->lm; a.gf = c->gf; a.logits = c->logits;
  const size_t nl = hl.size();
  // GEMM inputs (fp32 residual stream and its half-pair copy, attention outputs, FFN hidden): one region per layer,
  // so that no address is written twice within a launch
  // rows per exchange region: one group of 16, or two when the block is longer than 16 tokens
  a.RS = D.Bm > 16 ? 32 : 16;
  const size_t RS = a.RS, RH = RS / 2, RG = RS / 16;
  TRY(dalloc(c, &a.hA, (nl + 1) * RS * d)); TRY(dalloc(c, &a.hB, nl * RS * d)); TRY(dalloc(c, &a.hC, nl * RS * d));
  for (int i = 0; i < 4; i++) TRY(dalloc(c, &a.hT[i], RS * d));
  TRY(dalloc(c, &a.xA, (nl + 1) * RH * d)); TRY(dalloc(c, &a.xB, nl * RH * d)); TRY(dalloc(c, &a.xC, nl * RH * d));
  TRY(dalloc(c, &a.q, RH * d)); TRY(dalloc(c, &a.att, nl * RH * d)); TRY(dalloc(c, &a.q2, RH * d));
  TRY(dalloc(c, &a.att2, nl * RH * d));
  TRY(dalloc(c, &a.pool, 2 * 8 * d)); TRY(dalloc(c, &a.mid, nl * RH * c->ff));
  TRY(dalloc(c, &a.newK, (size_t)D.H * RS * 32)); TRY(dalloc(c, &a.newV, (size_t)D.H * RS * 32));
  TRY(dalloc(c, &a.partS, (size_t)D.H * PK_MAXSPLIT * RG * PK_PART)); TRY(dalloc(c, &a.partX, (size_t)D.H * PK_MAXSPLIT * RG * PK_PART));
  TRY(dalloc(c, &a.w2part, (d / 16) * RG * 3 * 256));
  TRY(dalloc(c, &a.abort_word, 16));
  if (hipMemset(a.abort_word + 1, 0xFF, 4) != hipSuccess) return fail(c, FM_EHIP, "hipMemset failed");
  a.run_flag = c->st.alive;
  if (const char* e = getenv("FM_PROFILE")) {
    if (e[0] == '1') TRY(dalloc(c, &a.prof, 1024));
    if (const char* ps = getenv("FM_PROFILE_STAGE")) a.prof_stage = atoi(ps); else a.prof_stage = -1;
  }
  c->pk_epoch = 0;
  // test hooks for the bounded waits: a shorter bound, and an embedding that publishes under the wrong tag
  a.timeout_ticks = PK_TIMEOUT_TICKS;
  a.test_skew = 0;
  a.two_phase = 0;
  if (const char* e = getenv("FM_PK_TWO_PHASE")) a.two_phase = atoi(e);
  if (const char* e = getenv("FM_PK_TIMEOUT_TICKS")) a.timeout_ticks = strtoull(e, nullptr, 10);
  if (const char* e = getenv("FM_PK_TEST_SKEW")) a.test_skew = (unsigned)atoi(e);
  c->pk_lds = 0;   // the kernel uses static LDS only
  // all 256 workgroups must be resident at once: they wait for each other's results
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      (a.RS == 32 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_verify_persist<2>, 256, c->pk_lds)
                  : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_verify_persist<1>, 256, c->pk_lds)) != hipSuccess ||
      (long)cus * per_cu < PK_NWG) {
    (void)hipGetLastError();
    c->persist = false;   // fall back to the per-launch path
  }
  return FM_OK;
}

int build_buffers(fm_ctx* c) {
  const Dims& D = c->D;
  const size_t d = D.d, S = D.S;
  StateDev& st = c->st;
  TRY(dalloc(c, &st.P, S)); TRY(dalloc(c, &st.main, S)); TRY(dalloc(c, &st.fin, S));
  TRY(dalloc(c, &st.firedv, S)); TRY(dalloc(c, &st.firedf, S));
  TRY(dalloc(c, &st.basec, S)); TRY(dalloc(c, &st.basev, S)); TRY(dalloc(c, &st.basef, S));
  TRY(dalloc(c, &st.vlen, S)); TRY(dalloc(c, &st.vtok, S * D.Bm)); TRY(dalloc(c, &st.y, S * D.Bm)); TRY(dalloc(c, &st.acc, S));
  TRY(dalloc(c, &st.hist, S * (D.maxtok + 1))); TRY(dalloc(c, &st.budget, 1)); TRY(dalloc(c, &st.alive, 1));
  TRY(dalloc(c, &st.acc_hist, 3 * 32)); TRY(dalloc(c, &st.counters, 3)); TRY(dalloc(c, &st.kind, S));
  TRY(dalloc(c, &c->ring_hc, S * RS_C * d)); TRY(dalloc(c, &c->tap_c, S * RS_C * d));
  TRY(dalloc(c, &c->ring_hv, S * RS_V * d)); TRY(dalloc(c, &c->ring_yv, S * RS_V * d)); TRY(dalloc(c, &c->tap_v, S * RS_V * d));
  TRY(dalloc(c, &c->ring_yf, S * RS_F * d)); TRY(dalloc(c, &c->tap_f, S * RS_F * d));
  const size_t rows[3] = {(size_t)c->Rc, (size_t)c->Rv, (size_t)c->Rf};
  for (int l = 0; l < 3; l++) {
    TRY(dalloc(c, &c->pos[l], rows[l])); TRY(dalloc(c, &c->limx[l], rows[l]));
    TRY(dalloc(c, &c->cs[l], rows[l] * 64)); TRY(dalloc(c, &c->h[l], rows[l] * d));
  }
  TRY(dalloc_t(c, &c->xn, rows[0] * d)); TRY(dalloc_t(c, &c->qT, rows[0] * d)); TRY(dalloc_t(c, &c->attT, rows[0] * d));
  TRY(dalloc_t(c, &c->mid, rows[0] * c->ff));
  TRY(dalloc(c, &c->qkv, rows[0] * 3 * d)); TRY(dalloc(c, &c->logits, rows[0] * D.V));
  // staging: conversion of the largest tensor, or the prefill (memory in T + fp32 K/V of one layer)
  size_t big = std::max((size_t)c->ff * d, (size_t)c->hff * d);
  big = std::max(big, 3 * d * d);
  big = std::max(big, (size_t)D.V * d);
  c->stage_elems = std::max(big, (size_t)D.M * d + (size_t)D.M * 2 * d);
  TRY(dalloc(c, &c->stage, c->stage_elems));
  // draft rows
  const size_t nset[5] = {S * D.Dc, S * D.nspv, S * D.nspf, S * D.nhfv, S * 2 * D.nhfc};
  size_t maxset = 1;
  for (int i = 3; i < 5; i++) {
    maxset = std::max(maxset, nset[i]);
    TRY(dalloc(c, (const float***)&c->dr.src[i], nset[i])); TRY(dalloc(c, &c->dr.pos[i], nset[i]));
    TRY(dalloc(c, &c->dr.lim[i], nset[i])); TRY(dalloc(c, &c->dr.limx[i], nset[i]));
    TRY(dalloc(c, &c->dr.cs[i], nset[i] * 64));
  }
  const char* spm = getenv("FM_SP_MERGED");      // "0": one chain of launches per level
  c->sp_merged = c->bf16 && D.hd == 64 && D.Dc <= 16 && D.nspv <= 16 && D.nspf <= 16 && !(spm && spm[0] == '0');
  const int G_all = D.Dc + D.nspv + D.nspf;
  {
    // One table for the three SP row sets.  Merged chain: rows [sequence][point heads | face heads | coordinate heads],
    // as the heads lie in memory, so that a grouped launch over all heads sees S rows per head with one stride.
    // Otherwise the three sets behind each other, each [sequence][head].
    const size_t nsp = nset[0] + nset[1] + nset[2], np = (size_t)D.hd / 2;
    maxset = std::max(maxset, nsp);
    const float** src; int *pos, *lim, *limx; float2* cs;
    TRY(dalloc(c, (const float***)&src, nsp)); TRY(dalloc(c, &pos, nsp)); TRY(dalloc(c, &lim, nsp)); TRY(dalloc(c, &limx, nsp));
    TRY(dalloc(c, &cs, nsp * 64));
    const size_t first_m[3] = {(size_t)D.nspv + D.nspf, 0, (size_t)D.nspv}, first_s[3] = {nset[1] + nset[2], 0, nset[1]};
    const int cnt[5] = {D.Dc, D.nspv, D.nspf, D.nhfv, 2 * D.nhfc};
    for (int i = 0; i < 5; i++) c->dr.rs[i] = cnt[i];
    for (int i = 0; i < 3; i++) {
      const size_t first = c->sp_merged ? first_m[i] : first_s[i];
      if (c->sp_merged) c->dr.rs[i] = G_all;
      c->dr.src[i] = src + first; c->dr.pos[i] = pos + first; c->dr.lim[i] = lim + first;
      c->dr.limx[i] = limx + first; c->dr.cs[i] = cs + first * np;
    }
  }
  TRY(dalloc(c, &c->dr.alive, S)); TRY(dalloc(c, &c->dr.firev, S)); TRY(dalloc(c, &c->dr.firef, S)); TRY(dalloc(c, &c->dr.flags, 4));
  TRY(dalloc(c, &c->hfv_out, nset[3] * d));
  const size_t nLM = S * (D.Dc + 2 * D.nhfc);
  // Outputs of the SP heads.  Merged chain: one buffer [sequence][point | face | coordinate heads][d]; otherwise one
  // buffer per level, the coordinate level's being the first rows of the output head's input.  The output head reads its
  // rows (coordinate SP heads of every sequence, then the coordinate HF rows) through a pointer table either way.
  TRY(dalloc(c, &c->dh, nLM * d));
  int spv_rs = std::max(D.nspv, 1), spf_rs = D.nspf;
  if (c->sp_merged) {
    TRY(dalloc(c, &c->spv_out, (size_t)S * std::max(G_all, 1) * d));
    c->spf_out = c->spv_out + (size_t)D.nspv * d;
    spv_rs = spf_rs = G_all;
  } else {
    TRY(dalloc(c, &c->spv_out, nset[1] * d));
    TRY(dalloc(c, &c->spf_out, nset[2] * d));
  }
  {
    std::vector<const float*> tab(std::max<size_t>(nLM, 1));
    for (size_t i = 0; i < nLM; i++) {
      if (c->sp_merged && i < S * (size_t)D.Dc) tab[i] = c->spv_out + ((i / D.Dc) * G_all + D.nspv + D.nspf + i % D.Dc) * d;
      else tab[i] = c->dh + i * d;
    }
    TRY(dalloc(c, (const float***)&c->lm_src, tab.size()));
    HIPCHK(c, hipMemcpy(c->lm_src, tab.data(), tab.size() * sizeof(float*), hipMemcpyHostToDevice));
  }
  TRY(dalloc(c, &c->dlogits, nLM * D.V));
  const size_t rmax = std::max(maxset, nLM);
  TRY(dalloc(c, &c->dkeep, rmax * d)); TRY(dalloc(c, &c->dtmp, rmax * d));
  TRY(dalloc_t(c, &c->dxn, rmax * d)); TRY(dalloc_t(c, &c->dq, rmax * d)); TRY(dalloc_t(c, &c->datt, rmax * d));
  TRY(dalloc_t(c, &c->dmid, rmax * c->hff));
  TRY(dalloc(c, &c->dist_c, S * std::max(D.Dc, 1) * D.V));
  TRY(dalloc(c, &c->dist_v, S * std::max(D.nhfc, 1) * D.V)); TRY(dalloc(c, &c->dist_f, S * std::max(D.nhfc, 1) * D.V));
  TRY(dalloc(c, &c->lab_v, S * std::max(D.nspv, 1) * 3)); TRY(dalloc(c, &c->lab_f, S * std::max(D.nhfv, 1) * 3));
  c->smp = Sampling{0.f, 0ull, nullptr, nullptr, nullptr, nullptr, 0};
  TRY(dalloc(c, &c->smp.qrow, S * D.Bm * D.V)); TRY(dalloc(c, &c->smp.qsum, S * D.Bm));
  TRY(dalloc(c, &c->smp.qtok, S * D.Bm)); TRY(dalloc(c, &c->smp.accflag, S * D.Bm));
  c->db = DraftBufs{c->tap_c, c->tap_v, c->tap_f, c->ring_yf, c->spv_out, c->spf_out, c->hfv_out, spv_rs, spf_rs};
  TRY(dalloc(c, &c->gen_tok, S * D.Bm)); TRY(dalloc(c, &c->gen_len, S)); TRY(dalloc(c, &c->gen_acc, S));
  if (c->persist) TRY(build_persist(c));
  c->mres = MfmaRes{nullptr, nullptr, 0, 0, 0, 768, 0, 0};
  if (const char* e = getenv("FM_ATTN_MERGE")) c->mres.attn_merge = atoi(e);   // measurement switch, see MfmaRes
  if (const char* e = getenv("FM_ATTN_WGS")) c->mres.attn_wgs = atoi(e);       // measurement switch: workgroups per self-attention launch
  if (const char* e = getenv("FM_GEMM_NC")) c->mres.gemm_nc = atoi(e);         // measurement switch: 1 = one column tile per workgroup
  if (const char* e = getenv("FM_GEMM_WAVES")) c->mres.gemm_waves = atoi(e);   // measurement switch: 4, 8 or 16
  if (const char* e = getenv("FM_GEMM_MT_CAP")) c->mres.gemm_mt_cap = atoi(e); // measurement switch: up to 2, 3, 5 or 8 row tiles per workgroup
  if (c->bf16) {
    c->mres.attn_ws_floats = mfma_attn_ws_floats(3 * D.S, D.H, D.hd);       // 3: the merged SP launch has three row sets per sequence
    TRY(dalloc(c, &c->mres.attn_ws, c->mres.attn_ws_floats, false));
    TRY(dalloc(c, &c->mres.attn_counters, (size_t)3 * D.S * D.H));

    // tiled prefill GEMM: whole 256 x 128 output tiles only (keys x dims for V, dims x keys for K)
    const char* pt = getenv("FM_PREFILL_TILED");     // "0" forces the per-block GEMM + scatter launches
    if (D.M % 256 == 0 && d % 256 == 0 && !(pt && pt[0] == '0')) {
      std::vector<PrefillLayer> tab;
      for (int st = 0; st < 5; st++)
        for (auto& L : c->stacks[st]) tab.push_back(PrefillLayer{(const f16_t*)L.ckv, (f16_t*)L.Km, (f16_t*)L.Vm});
      uint8_t* raw = nullptr;
      TRY(dalloc(c, &raw, tab.size() * sizeof(PrefillLayer)));
      c->pf_layers = (PrefillLayer*)raw;
      HIPCHK(c, hipMemcpy(c->pf_layers, tab.data(), tab.size() * sizeof(PrefillLayer), hipMemcpyHostToDevice));
      c->pf_n = (int)tab.size();
      HIPCHK(c, hipFuncSetAttribute((const void*)k_prefill_kv<64>, hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS_BYTES));
      HIPCHK(c, hipFuncSetAttribute((const void*)k_prefill_kv<96>, hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS_BYTES));
      HIPCHK(c, hipFuncSetAttribute((const void*)k_prefill_kv<128>, hipFuncAttributeMaxDynamicSharedMemorySize, PF_LDS_BYTES));
      hipDeviceProp_t prop;
      int dev = 0;
      HIPCHK(c, hipGetDevice(&dev));
      HIPCHK(c, hipGetDeviceProperties(&prop, dev));
      c->pf_grid = std::max(8, prop.multiProcessorCount / 8 * 8);
    }
  }
  if (hipHostMalloc((void**)&c->host_flag, 64 + sizeof(int) * (size_t)c->D.S) != hipSuccess) return fail(c, FM_ENOMEM, "hipHostMalloc failed");
  return FM_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
extern "C" {

int fm_create(const fm_config* cfg, void* hip_stream, fm_ctx** out) {
  if (!cfg || !out) return FM_EINVAL;
  *out = nullptr;
  const fm_config& g = *cfg;
  if (g.d_model <= 0 || g.n_heads <= 0 || g.d_model % g.n_heads != 0) return FM_EINVAL;
  const int hd = g.d_model / g.n_heads;          // 64, or the paper's own widths 96 and 128
  if (hd != 64 && hd != 96 && hd != 128) return FM_EINVAL;
  if (g.ffn_mult < 1 || g.hf_ffn_mult < 1 || g.n_bins < 1 || g.mem_len < 1) return FM_EINVAL;
  if (g.l_cpre < 1 || g.l_cpost < 1 || g.l_vpre < 1 || g.l_vpost < 1 || g.l_face < 1) return FM_EINVAL;
  if (g.dtype != FM_DTYPE_F32 && g.dtype != FM_DTYPE_BF16) return FM_EINVAL;
  if (g.max_batch < 1 || g.max_batch > 64 || g.max_tokens < 9 || g.max_tokens % 9 != 0) return FM_EINVAL;
  if (g.draft_coord < 0 || g.draft_point < 0 || g.draft_face < 0) return FM_EINVAL;
  if (g.draft_point % 3 != 0 || g.draft_face % 9 != 0) return FM_EINVAL;
  if ((g.draft_point > 0 || g.draft_face > 0) && g.draft_coord < 2 && !(g.rules_off & 2)) return FM_EINVAL;  // rule (B) leaves 3 tokens to the coordinate level
  const int Bm = std::max(std::max(1 + g.draft_coord, g.draft_point), std::max(g.draft_face, 1));
  if (Bm > 27) return FM_EINVAL;  // rings hold 32 coordinate positions: block + 2 carried rows
  if (!(g.rope_base > 1.f) || !(g.rms_eps > 0.f)) return FM_EINVAL;
  if (g.window < 0 || g.window % 9 != 0) return FM_EINVAL;
  if (g.rules_off & ~3) return FM_EINVAL;

  fm_ctx* c = new (std::nothrow) fm_ctx();
  if (!c) return FM_ENOMEM;
  c->cfg = g;
  c->stream = (hipStream_t)hip_stream;
  c->bf16 = g.dtype == FM_DTYPE_BF16;
  c->esz = c->bf16 ? 2 : 4;
  c->ff = g.ffn_mult * g.d_model;
  c->hff = g.hf_ffn_mult * g.d_model;
  Dims& D = c->D;
  D.d = g.d_model; D.H = g.n_heads; D.hd = hd; D.V = g.n_bins + 3; D.S = g.max_batch; D.Bm = Bm;
  D.VB = (Bm + 2) / 3; D.FB = (Bm + 8) / 9; D.M = g.mem_len;
  D.maxtok = g.max_tokens;
  D.capc = g.max_tokens; D.capv = (g.max_tokens + 2) / 3 + 1; D.capf = (g.max_tokens + 8) / 9 + 1;
  D.wc = D.wv = D.wf = 0;
  if (g.window > 0 && g.window < g.max_tokens) {
    // rings: the window plus the rows of one pass (a rejected block leaves stale rows behind the committed
    // length; they must only ever overwrite positions that no later query can see), in groups of four 32-key
    // blocks (the rows of one pass then never meet twice in the blocks one wave of an attention range walks)
    D.wc = g.window; D.wv = g.window / 3; D.wf = g.window / 9;
    auto ring = [](int w, int rows) { return (w + rows + 2 + 127) / 128 * 128; };
    D.capc = ring(D.wc, D.Bm); D.capv = ring(D.wv, D.VB); D.capf = ring(D.wf, D.FB);
  }
  D.Dc = g.draft_coord; D.m = g.draft_point; D.n = g.draft_face;
  D.nspv = std::max(D.m / 3 - 1, 0); D.nspf = std::max(D.n / 9 - 1, 0);
  D.t0 = (g.rules_off & 2) ? 0 : 3; D.j0 = (g.rules_off & 2) ? 0 : 1;
  D.nhfc = std::max(std::max(D.m, D.n) - D.t0, 0); D.nhfv = std::max(D.n / 3 - D.j0, 0);
  D.ruleA = (g.rules_off & 1) ? 0 : 1;
  D.nbins = g.n_bins; D.ban = g.ban_specials ? 1 : 0; D.eos = g.n_bins + 1; D.pad = g.n_bins + 2;
  c->Vpad = (D.V + 63) / 64 * 64;
  c->Rc = D.S * D.Bm; c->Rv = D.S * D.VB; c->Rf = D.S * D.FB;
  for (int i = 0; i < 64; i++) c->inv.v[i] = std::pow((double)g.rope_base, -(double)i / (hd / 2.0));
  c->weights_loaded = false;
  c->prefilled.assign(D.S, false);
  c->len_bound.assign(D.S, D.maxtok);
  c->replay = Replay{nullptr, 0, 0, 0.f, 0ull};
  c->host_flag = nullptr;
  {
    const int nl = g.l_cpre + g.l_cpost + g.l_vpre + g.l_vpost + g.l_face;
    const char* env = getenv("FM_PERSIST");
    c->persist = c->bf16 && D.hd == 64 && D.S == 1 && D.Bm <= 32 && D.d % 128 == 0 && D.d <= 1024 && c->ff % 512 == 0 && nl < 62 &&
                 !(env && env[0] == '0');
  }
  int rc = build_params(c);
  if (rc == FM_OK) rc = build_buffers(c);
  if (rc == FM_OK) {
    // this GPU's copy of the static staging array: address looked up once per device, with that device current
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) rc = fail(c, FM_EHIP, "hipGetDevice failed");
    else {
      std::lock_guard<std::mutex> lk(g_scratch_mu);
      if (!g_scratch_addr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) rc = fail(c, FM_EHIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
        else g_scratch_addr[dev] = p;
      }
      c->static_scratch = (unsigned char*)g_scratch_addr[dev];
    }
  }
  if (rc == FM_OK) {
    const int budget = g.max_tokens;
    if (hipMemcpy(c->st.budget, &budget, sizeof(int), hipMemcpyHostToDevice) != hipSuccess) rc = FM_EHIP;
    // all sequences start finished until they are prefilled
    std::vector<int> ones(D.S, 1);
    if (hipMemcpy(c->st.fin, ones.data(), sizeof(int) * D.S, hipMemcpyHostToDevice) != hipSuccess) rc = FM_EHIP;
  }
  if (rc != FM_OK) {
    fprintf(stderr, "fm_create: %s\n", c->err.c_str());
    for (void* p : c->allocs) (void)hipFree(p);
    if (c->host_flag) (void)hipHostFree(c->host_flag);
    delete c;
    return rc;
  }
  // algorithmic weight bytes of one verify pass
  const double d2 = (double)D.d * D.d;
  const int nl = g.l_cpre + g.l_cpost + g.l_vpre + g.l_vpost + g.l_face;
  c->weight_bytes = c->esz * (nl * (6.0 + 2.0 * g.ffn_mult) * d2 + 2.0 * d2 + (double)D.V * D.d);
  *out = c;
  return FM_OK;
}

int fm_destroy(fm_ctx* c) {
  if (!c) return FM_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->host_flag) (void)hipHostFree(c->host_flag);
  delete c;
  return FM_OK;
}

const char* fm_last_error(const fm_ctx* c) { return c ? c->err.c_str() : "null context"; }
int32_t fm_block_max(const fm_ctx* c) { return c ? c->D.Bm : FM_EINVAL; }
int32_t fm_verify_path(const fm_ctx* c) { return c ? (c->persist ? 1 : 0) : FM_EINVAL; }
int64_t fm_blob_elems(const fm_ctx* c) { return c ? (int64_t)c->blob_elems : FM_EINVAL; }

int fm_load_weights(fm_ctx* c, const float* blob, size_t n_floats) {
  if (!c) return FM_EINVAL;
  if (!blob) return fail(c, FM_EINVAL, "null blob");
  if (n_floats != c->blob_elems) return fail(c, FM_EINVAL, "blob has %zu floats, expected %zu", n_floats, c->blob_elems);
  for (const LoadItem& it : c->items) {
    size_t done = 0;
    while (done < it.n) {
      const size_t n = std::min(it.n - done, c->stage_elems);
      if (it.f32) {
        HIPCHK(c, hipMemcpyAsync((float*)it.dst + done, blob + it.blob_off + done, n * 4, hipMemcpyHostToDevice, c->stream));
      } else {
        HIPCHK(c, hipMemcpyAsync(c->stage, blob + it.blob_off + done, n * 4, hipMemcpyHostToDevice, c->stream));
        if (c->bf16 && it.N > 0) {
          if (n != it.n) return fail(c, FM_EINVAL, "staging buffer smaller than a weight matrix");
          hipLaunchKernelGGL(k_tile_weight, dim3(1024), dim3(256), 0, c->stream, c->stage, (f16_t*)it.dst, it.N, it.K,
                             (it.N + 15) / 16 * 16, it.perm);
        } else if (c->bf16)
          hipLaunchKernelGGL((k_convert<f16_t>), dim3(1024), dim3(256), 0, c->stream, c->stage, (f16_t*)it.dst + done, (long)n);
        else
          hipLaunchKernelGGL((k_convert<float>), dim3(1024), dim3(256), 0, c->stream, c->stage, (float*)it.dst + done, (long)n);
      }
      HIPCHK(c, hipStreamSynchronize(c->stream));  // the staging buffer is reused
      done += n;
    }
  }
  HIPCHK(c, hipGetLastError());
  c->weights_loaded = true;
  return FM_OK;
}

int fm_prefill_condition(fm_ctx* c, int32_t seq, const float* mem_dev) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (seq < 0 || seq >= c->D.S) return fail(c, FM_EINVAL, "sequence %d out of range [0,%d)", seq, c->D.S);
  if (!mem_dev) return fail(c, FM_EINVAL, "null condition memory");
  int rc = c->bf16 ? prefill_impl<f16_t>(c, seq, mem_dev, c->stage) : prefill_impl<float>(c, seq, mem_dev, c->stage);
  if (rc == FM_OK) { c->prefilled[seq] = true; c->len_bound[seq] = 0; }
  return rc;
}

int fm_prefill_condition_static(fm_ctx* c, int32_t seq, const float* mem_dev) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (seq < 0 || seq >= c->D.S) return fail(c, FM_EINVAL, "sequence %d out of range [0,%d)", seq, c->D.S);
  if (!mem_dev) return fail(c, FM_EINVAL, "null condition memory");
  if (!c->static_scratch) return fail(c, FM_ESTATE, "no static staging area on this device");
  const size_t need = prefill_stage_bytes(c);
  if (need > FM_STATIC_SCRATCH_BYTES)
    return fail(c, FM_EINVAL, "condition memory of %d x %d needs %zu staging bytes, the static area holds %u: use fm_prefill_condition",
                c->D.M, c->D.d, need, (unsigned)FM_STATIC_SCRATCH_BYTES);
  int rc = c->bf16 ? prefill_impl<f16_t>(c, seq, mem_dev, c->static_scratch) : prefill_impl<float>(c, seq, mem_dev, c->static_scratch);
  if (rc == FM_OK) { c->prefilled[seq] = true; c->len_bound[seq] = 0; }
  return rc;
}

int fm_draft(fm_ctx* c, int32_t* block_tok, int32_t* block_len) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (!block_tok || !block_len) return fail(c, FM_EINVAL, "null block buffer");
  const int rc = c->bf16 ? draft_impl<f16_t>(c, block_tok, block_len, 1) : draft_impl<float>(c, block_tok, block_len, 1);
  return rc == FM_OK && c->sticky_error ? FM_EINVAL : rc;
}

int fm_set_sampling(fm_ctx* c, float temperature, uint64_t seed) {
  if (!c) return FM_EINVAL;
  if (!(temperature >= 0.f) || temperature > 1e4f) return fail(c, FM_EINVAL, "temperature %g outside [0, 1e4]", (double)temperature);
  c->smp.temperature = temperature;
  c->smp.seed = seed;
  return FM_OK;
}

int fm_set_correct(fm_ctx* c, int32_t hist_vertices) {
  if (!c) return FM_EINVAL;
  if (hist_vertices < 0) return fail(c, FM_EINVAL, "hist_vertices %d < 0", hist_vertices);
  c->correct_hist = hist_vertices;
  return FM_OK;
}

int fm_correct(fm_ctx* c, int32_t* block_tok, const int32_t* block_len, int32_t* labels_out) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (c->correct_hist <= 0) return fail(c, FM_ESTATE, "correct stage is off: call fm_set_correct before the fm_draft whose block is corrected");
  if (!block_tok || !block_len) return fail(c, FM_EINVAL, "null block buffer");
  hipLaunchKernelGGL(k_correct, dim3((c->D.S + 63) / 64), dim3(64), 0, c->stream, c->st, c->D, c->lab_v, c->lab_f, c->correct_hist,
                     block_tok, block_len, labels_out);
  HIPCHK(c, hipGetLastError());
  return FM_OK;
}

int fm_verify_block(fm_ctx* c, const int32_t* block_tok, const int32_t* block_len, float* logits, int32_t* accepted) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (!block_tok || !block_len || !accepted) return fail(c, FM_EINVAL, "null block / accepted buffer");
  const int rc = c->bf16 ? verify_impl<f16_t>(c, block_tok, block_len, logits, accepted)
                         : verify_impl<float>(c, block_tok, block_len, logits, accepted);
  return rc == FM_OK && c->sticky_error ? FM_EINVAL : rc;
}

int fm_commit(fm_ctx* c, const int32_t* accepted) {
  if (!c) return FM_EINVAL;
  if (!accepted) return fail(c, FM_EINVAL, "null accepted buffer");
  hipLaunchKernelGGL(k_commit, dim3(1), dim3(64), 0, c->stream, c->st, c->D, accepted, pass_failed(c));
  HIPCHK(c, hipGetLastError());
  for (int s = 0; s < c->D.S; s++) c->len_bound[s] = std::min(c->len_bound[s] + c->D.Bm, c->D.maxtok);
  c->commits++;
  return FM_OK;
}

int fm_set_budget(fm_ctx* c, int32_t max_faces) {
  if (!c) return FM_EINVAL;
  if (max_faces < 1 || 9 * max_faces > c->D.maxtok) return fail(c, FM_EINVAL, "max_faces %d outside [1,%d]", max_faces, c->D.maxtok / 9);
  hipLaunchKernelGGL(k_set_budget, dim3(1), dim3(64), 0, c->stream, c->st, c->D, 9 * max_faces);
  HIPCHK(c, hipGetLastError());
  return FM_OK;
}

int fm_set_draft_replay(fm_ctx* c, const int32_t* stream_dev, int32_t stride, int32_t n_valid, float keep_prob, uint64_t seed) {
  if (!c) return FM_EINVAL;
  if (stream_dev && (stride < n_valid || n_valid < 0 || !(keep_prob >= 0.f && keep_prob <= 1.f)))
    return fail(c, FM_EINVAL, "bad replay arguments");
  c->replay = Replay{stream_dev, stride, n_valid, keep_prob, (unsigned long long)seed};
  return FM_OK;
}

int fm_read_state(fm_ctx* c, int32_t* host_out) {
  if (!c || !host_out) return FM_EINVAL;
  const int S = c->D.S;
  std::vector<int> P(S), mn(S), fin(S);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(P.data(), c->st.P, S * 4, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(mn.data(), c->st.main, S * 4, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(fin.data(), c->st.fin, S * 4, hipMemcpyDeviceToHost));
  TRY(check_persist(c));
  for (int s = 0; s < S; s++) {
    c->len_bound[s] = P[s];
    host_out[s * 6 + 0] = P[s];
    host_out[s * 6 + 1] = (P[s] + 2) / 3;
    host_out[s * 6 + 2] = (P[s] + 8) / 9;
    host_out[s * 6 + 3] = mn[s];
    host_out[s * 6 + 4] = fin[s];
    host_out[s * 6 + 5] = P[s];
  }
  return FM_OK;
}

int fm_debug_profile(fm_ctx* c, uint64_t* host_out, int32_t n) {
  if (!c || !host_out || n < 1 || n > 1024) return FM_EINVAL;
  if (!c->persist || !c->pk.prof) return fail(c, FM_ESTATE, "stage profiling is off (FM_PROFILE=1 at fm_create, persistent path only)");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host_out, c->pk.prof, (size_t)n * 8, hipMemcpyDeviceToHost));
  std::vector<unsigned long long> init(1024, 0ull);
  init[0] = ~0ull;
  HIPCHK(c, hipMemcpy(c->pk.prof, init.data(), 1024 * 8, hipMemcpyHostToDevice));   // re-arm
  return FM_OK;
}

int fm_debug_draft(fm_ctx* c, int32_t which, float* host_out) {
  if (!c) return FM_EINVAL;
  const Dims& D = c->D;
  if (which == -1 || which == -2) { c->smp.keep_rows = which == -1 ? 1 : 0; return FM_OK; }
  if (!host_out) return fail(c, FM_EINVAL, "null output");
  const float* src = which == 0 ? c->smp.qrow : which == 1 ? c->lab_v : which == 2 ? c->lab_f : nullptr;
  if (!src) return fail(c, FM_EINVAL, "draft buffer %d out of range", which);
  const size_t n = which == 0 ? (size_t)D.S * D.Bm * D.V : which == 1 ? (size_t)D.S * std::max(D.nspv, 1) * 3 : (size_t)D.S * std::max(D.nhfv, 1) * 3;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host_out, src, n * sizeof(float), hipMemcpyDeviceToHost));
  return FM_OK;
}

int fm_debug_ring(fm_ctx* c, int32_t which, float* host_out) {
  if (!c || !host_out) return FM_EINVAL;
  float* src[7] = {c->ring_hc, c->ring_hv, c->ring_yf, c->ring_yv, c->tap_c, c->tap_v, c->tap_f};
  const int rs[7] = {RS_C, RS_V, RS_F, RS_V, RS_C, RS_V, RS_F};
  if (which < 0 || which >= 7) return fail(c, FM_EINVAL, "ring %d out of range", which);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(host_out, src[which], (size_t)c->D.S * rs[which] * c->D.d * sizeof(float), hipMemcpyDeviceToHost));
  return FM_OK;
}

int fm_debug_mem_kv(fm_ctx* c, int32_t seq, int32_t block, float* host_k, float* host_v) {
  if (!c || !host_k || !host_v) return FM_EINVAL;
  if (seq < 0 || seq >= c->D.S) return fail(c, FM_EINVAL, "sequence %d out of range", seq);
  if (!c->prefilled[seq]) return fail(c, FM_ESTATE, "sequence %d has no condition memory", seq);
  const Layer* L = nullptr;
  int left = block;
  for (int st = 0; st < 5 && !L && left >= 0; st++) {
    if (left < (int)c->stacks[st].size()) L = &c->stacks[st][left];
    else left -= (int)c->stacks[st].size();
  }
  if (block < 0 || !L) return fail(c, FM_EINVAL, "block %d out of range", block);
  const Dims& D = c->D;
  const size_t n = cache_seq_elems(c, D.M);
  std::vector<unsigned char> raw(n * c->esz);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int kv = 0; kv < 2; kv++) {
    const unsigned char* src = (const unsigned char*)(kv ? L->Vm : L->Km) + (size_t)seq * n * c->esz;
    HIPCHK(c, hipMemcpy(raw.data(), src, raw.size(), hipMemcpyDeviceToHost));
    float* out = kv ? host_v : host_k;
    const int hd = D.hd, capb = (D.M + 31) / 32;
    for (int m = 0; m < D.M; m++)
      for (int i = 0; i < D.d; i++) {
        const int hh = i / hd, e = i % hd;
        if (c->bf16) {
          // the blocked layouts of the half path: 32-key blocks of a head; K in MFMA fragment order, V as [dim][key slot]
          const int r = m & 31;
          size_t o = ((size_t)hh * capb + (m >> 5)) * 32 * hd;
          if (kv == 0) o += (size_t)((((r >> 4) * (hd / 32) + (e >> 5)) * 64 + (r & 15) + 16 * ((e & 31) >> 3)) * 8 + (e & 7));
          else o += (size_t)e * 32 + ((r & 15) >> 2) * 8 + (r >> 4) * 4 + (r & 3);
          out[(size_t)m * D.d + i] = (float)((const f16_t*)raw.data())[o];
        } else {
          out[(size_t)m * D.d + i] = ((const float*)raw.data())[((size_t)hh * D.M + m) * hd + e];
        }
      }
  }
  return FM_OK;
}

int fm_verify_bytes(fm_ctx* c, double* host_bytes) {
  if (!c || !host_bytes) return FM_EINVAL;
  const int S = c->D.S;
  std::vector<int> P(S), fin(S);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(P.data(), c->st.P, S * 4, hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(fin.data(), c->st.fin, S * 4, hipMemcpyDeviceToHost));
  double bytes = c->weight_bytes;
  const fm_config& g = c->cfg;
  for (int s = 0; s < S; s++) {
    if (fin[s]) continue;
    double Lc = P[s], Lv = (P[s] + 2) / 3, Lf = (P[s] + 8) / 9;
    const double M = c->D.M;
    if (c->D.wc > 0) { Lc = std::min<double>(Lc, c->D.wc); Lv = std::min<double>(Lv, c->D.wv); Lf = std::min<double>(Lf, c->D.wf); }
    bytes += c->esz * 2.0 * c->D.d *
             ((g.l_cpre + g.l_cpost) * (Lc + M) + (g.l_vpre + g.l_vpost) * (Lv + M) + g.l_face * (Lf + M));
  }
  *host_bytes = bytes;
  return FM_OK;
}

int fm_measure_peaks(fm_ctx* c, double* host_out) {
  if (!c || !host_out) return FM_EINVAL;
  const size_t bytes = (size_t)1 << 30;
  float4 *a = nullptr, *b = nullptr;
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = FM_OK;
  auto cleanup = [&]() {
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    if (sink) (void)hipFree(sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
#define PK_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); cleanup(); return fail(c, FM_EHIP, "peak probe: %s failed", #x); } } while (0)
  PK_TRY(hipStreamSynchronize(c->stream));
  PK_TRY(hipMalloc((void**)&a, bytes)); PK_TRY(hipMalloc((void**)&b, bytes)); PK_TRY(hipMalloc((void**)&sink, 1024 * 256 * 4));
  PK_TRY(hipMemsetAsync(a, 0, bytes, c->stream)); PK_TRY(hipMemsetAsync(b, 0, bytes, c->stream));
  PK_TRY(hipEventCreate(&e0)); PK_TRY(hipEventCreate(&e1));
  const long n16 = (long)(bytes / 16);
  const int reps = 5, iters = 4000, wgs = 1024;
  float ms = 0.f;
  // streaming read
  hipLaunchKernelGGL(k_probe_read, dim3(2048), dim3(256), 0, c->stream, a, sink, n16);
  PK_TRY(hipEventRecord(e0, c->stream));
  for (int i = 0; i < reps; i++) hipLaunchKernelGGL(k_probe_read, dim3(2048), dim3(256), 0, c->stream, a, sink, n16);
  PK_TRY(hipEventRecord(e1, c->stream)); PK_TRY(hipEventSynchronize(e1)); PK_TRY(hipEventElapsedTime(&ms, e0, e1));
  host_out[0] = (double)bytes * reps / (ms * 1e-3) / 1e9;
  // streaming copy (read + write bytes)
  hipLaunchKernelGGL(k_probe_copy, dim3(32768), dim3(256), 0, c->stream, a, b, n16);
  PK_TRY(hipEventRecord(e0, c->stream));
  for (int i = 0; i < reps; i++) hipLaunchKernelGGL(k_probe_copy, dim3(32768), dim3(256), 0, c->stream, a, b, n16);
  PK_TRY(hipEventRecord(e1, c->stream)); PK_TRY(hipEventSynchronize(e1)); PK_TRY(hipEventElapsedTime(&ms, e0, e1));
  host_out[1] = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;
  // MFMA loop
  hipLaunchKernelGGL(k_probe_mfma, dim3(wgs), dim3(256), 0, c->stream, sink, 100);
  PK_TRY(hipEventRecord(e0, c->stream));
  hipLaunchKernelGGL(k_probe_mfma, dim3(wgs), dim3(256), 0, c->stream, sink, iters);
  PK_TRY(hipEventRecord(e1, c->stream)); PK_TRY(hipEventSynchronize(e1)); PK_TRY(hipEventElapsedTime(&ms, e0, e1));
  host_out[2] = 2.0 * 32 * 32 * 16 * 8.0 * iters * 4.0 * wgs / (ms * 1e-3) / 1e12;
#undef PK_TRY
  cleanup();
  return rc;
}

int fm_measure_exchange(fm_ctx* c, int32_t workgroups, int32_t bytes, int32_t pingpong, double* host_out) {
  if (!c || !host_out) return FM_EINVAL;
  if (workgroups < 2 || workgroups > 256 || bytes < workgroups * 8 || bytes > 49152 || bytes % (workgroups * 16) != 0)
    return fail(c, FM_EINVAL, "exchange probe: 2..256 workgroups, bytes a multiple of 16 per workgroup, at most 49152");
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_probe_exchange, 256, 0) != hipSuccess || (long)cus * per_cu < workgroups) {
    (void)hipGetLastError();
    return fail(c, FM_ESTATE, "exchange probe: %d workgroups cannot be resident together on this device", workgroups);
  }
  const int vol = bytes / 8, nstage = 2000;
  unsigned long long *buf = nullptr, *ticks = nullptr;
  unsigned* words = nullptr;
  auto cleanup = [&]() {
    if (buf) (void)hipFree(buf);
    if (ticks) (void)hipFree(ticks);
    if (words) (void)hipFree(words);
  };
#define PK_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); cleanup(); return fail(c, FM_EHIP, "exchange probe: %s failed", #x); } } while (0)
  PK_TRY(hipStreamSynchronize(c->stream));
  PK_TRY(hipMalloc((void**)&buf, (size_t)3 * vol * 8)); PK_TRY(hipMalloc((void**)&ticks, 16)); PK_TRY(hipMalloc((void**)&words, 256));
  PK_TRY(hipMemsetAsync(buf, 0, (size_t)3 * vol * 8, c->stream)); PK_TRY(hipMemsetAsync(ticks, 0, 16, c->stream));
  PK_TRY(hipMemsetAsync(words, 0, 256, c->stream));
  hipLaunchKernelGGL(k_probe_exchange, dim3(workgroups), dim3(256), 0, c->stream, buf, words, words + 32, ticks, vol, nstage, pingpong ? 1 : 0);
  PK_TRY(hipStreamSynchronize(c->stream));
  unsigned long long t[2] = {0, 0};
  unsigned ab = 0;
  PK_TRY(hipMemcpy(t, ticks, 16, hipMemcpyDeviceToHost)); PK_TRY(hipMemcpy(&ab, words + 32, 4, hipMemcpyDeviceToHost));
#undef PK_TRY
  cleanup();
  if (ab) return fail(c, FM_EHIP, "exchange probe: a bounded wait expired");
  host_out[0] = (double)(t[1] - t[0]) * 0.01 / nstage;       // microseconds per round (100 MHz wall clock)
  return FM_OK;
}

int fm_measure_gemm(fm_ctx* c, int32_t rows, double* host_out) {
  if (!c || !host_out) return FM_EINVAL;
  if (!c->bf16 || !c->weights_loaded) return fail(c, FM_ESTATE, "GEMM probe needs the half-precision path with weights loaded");
  if (rows < 1 || rows > 65536) return fail(c, FM_EINVAL, "rows %d outside [1, 65536]", rows);
  const int d = c->D.d, N = c->ff;
  const Layer& L = c->stacks[0][0];
  f16_t *X = nullptr, *Y = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() {
    if (X) (void)hipFree(X);
    if (Y) (void)hipFree(Y);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
#define PK_TRY(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); cleanup(); return fail(c, FM_EHIP, "GEMM probe: %s failed", #x); } } while (0)
  PK_TRY(hipStreamSynchronize(c->stream));
  PK_TRY(hipMalloc((void**)&X, (size_t)rows * d * 2)); PK_TRY(hipMalloc((void**)&Y, (size_t)rows * N * 2));
  PK_TRY(hipMemsetAsync(X, 0, (size_t)rows * d * 2, c->stream));
  PK_TRY(hipEventCreate(&e0)); PK_TRY(hipEventCreate(&e1));
  // Y[rows, ff] = gelu(X[rows, d] W1^T): the FFN up projection of the first block, half in and out
  GemmArgs a{X, d, 0, L.w1, 0, Y, N, 0, nullptr, 0, 0, rows, N, d, nullptr, nullptr, 0.f, nullptr, nullptr, 0, nullptr, nullptr, 0, 0, 0};
  const int reps = rows <= 256 ? 50 : 10;
  float ms = 0.f;
  if (!mfma_gemm_launch<f16_t>(c->mres, a, EPI_GELU_T, 1, c->stream)) { cleanup(); return fail(c, FM_EINVAL, "GEMM probe: unsupported shape"); }
  // FM_GEMM_PROBE_CYCLE = n: successive launches walk the up projections of n different blocks (n x 8 d^2 bytes
  // of weights), which tells a last-level-cache hit from an L2 hit from HBM
  std::vector<const void*> ws;
  for (int st = 0; st < 5; st++) for (auto& Lx : c->stacks[st]) ws.push_back(Lx.w1);
  int cyc = 1;
  if (const char* e = getenv("FM_GEMM_PROBE_CYCLE")) cyc = std::max(1, std::min(atoi(e), (int)ws.size()));
  for (int i = 0; i < cyc; i++) { a.W = ws[i]; mfma_gemm_launch<f16_t>(c->mres, a, EPI_GELU_T, 1, c->stream); }
  PK_TRY(hipEventRecord(e0, c->stream));
  for (int i = 0; i < reps; i++) { a.W = ws[i % cyc]; mfma_gemm_launch<f16_t>(c->mres, a, EPI_GELU_T, 1, c->stream); }
  PK_TRY(hipEventRecord(e1, c->stream)); PK_TRY(hipEventSynchronize(e1)); PK_TRY(hipEventElapsedTime(&ms, e0, e1));
  host_out[0] = ms / reps;
  host_out[1] = 2.0 * rows * (double)N * d * reps / (ms * 1e-3) / 1e12;
#undef PK_TRY
  cleanup();
  return FM_OK;
}

int fm_generate(fm_ctx* c, int32_t max_faces, int32_t speculative, int32_t* out_tok, int32_t* out_len, fm_stats* stats) {
  if (!c) return FM_EINVAL;
  if (!c->weights_loaded) return fail(c, FM_ESTATE, "weights not loaded");
  if (!out_tok || !out_len) return fail(c, FM_EINVAL, "null output buffer");
  for (int s = 0; s < c->D.S; s++)
    if (!c->prefilled[s]) return fail(c, FM_ESTATE, "sequence %d has no condition memory", s);
  TRY(fm_set_budget(c, max_faces));
  const Dims& D = c->D;
  // events: whole loop, lagged flag copy, and the four phase marks of a sampled step; destroyed on every way out
  enum { E_BEGIN, E_END, E_FLAG, E_P0, E_P1, E_P2, E_P3, E_COUNT };
  struct Events {
    hipEvent_t e[E_COUNT] = {};
    ~Events() { for (hipEvent_t x : e) if (x) (void)hipEventDestroy(x); }
  } ev;
  for (int i = 0; i < E_COUNT; i++) HIPCHK(c, hipEventCreate(&ev.e[i]));
  HIPCHK(c, hipMemsetAsync(c->st.acc_hist, 0, 3 * 32 * sizeof(unsigned long long), c->stream));
  HIPCHK(c, hipMemsetAsync(c->st.counters, 0, 3 * sizeof(unsigned long long), c->stream));
  HIPCHK(c, hipEventRecord(ev.e[E_BEGIN], c->stream));
  const long max_steps = 9L * max_faces + 1 + 128;     // + the steps a failed pass of the single-launch kernel may void
  const int check_every = 32;
  bool pending = false, done = false, phase_pending = false;
  long commits_at_copy = 0, phase_samples = 0;
  double ms_phase[3] = {0.0, 0.0, 0.0};
  auto take_phases = [&]() -> int {
    float a = 0.f, b = 0.f, d = 0.f;
    HIPCHK(c, hipEventElapsedTime(&a, ev.e[E_P0], ev.e[E_P1]));
    HIPCHK(c, hipEventElapsedTime(&b, ev.e[E_P1], ev.e[E_P2]));
    HIPCHK(c, hipEventElapsedTime(&d, ev.e[E_P2], ev.e[E_P3]));
    ms_phase[0] += a; ms_phase[1] += b; ms_phase[2] += d;
    phase_samples++;
    phase_pending = false;
    return FM_OK;
  };
  int rc = FM_OK;
  for (long step = 0; step < max_steps && !done && rc == FM_OK; step++) {
    // one step per interval carries the phase marks, once the marks of the previous sample have been read
    bool sample = step % check_every == 1;
    if (sample && phase_pending) {
      if (hipEventQuery(ev.e[E_P3]) == hipSuccess) TRY(take_phases());
      else { (void)hipGetLastError(); sample = false; }
    }
    if (sample) HIPCHK(c, hipEventRecord(ev.e[E_P0], c->stream));
    rc = c->bf16 ? draft_impl<f16_t>(c, c->gen_tok, c->gen_len, speculative) : draft_impl<float>(c, c->gen_tok, c->gen_len, speculative);
    if (rc == FM_OK && speculative && c->correct_hist > 0) rc = fm_correct(c, c->gen_tok, c->gen_len, nullptr);
    if (rc == FM_OK && sample) HIPCHK(c, hipEventRecord(ev.e[E_P1], c->stream));
    if (rc == FM_OK)
      rc = c->bf16 ? verify_impl<f16_t>(c, c->gen_tok, c->gen_len, nullptr, c->gen_acc)
                   : verify_impl<float>(c, c->gen_tok, c->gen_len, nullptr, c->gen_acc);
    if (rc == FM_OK && sample) HIPCHK(c, hipEventRecord(ev.e[E_P2], c->stream));
    if (rc == FM_OK) rc = fm_commit(c, c->gen_acc);
    if (rc == FM_OK && sample) { HIPCHK(c, hipEventRecord(ev.e[E_P3], c->stream)); phase_pending = true; }
    if (rc == FM_OK && c->sticky_error) rc = FM_EINVAL;
    if (rc != FM_OK) break;
    if ((step + 1) % check_every == 0) {
      // look at the flag copied one interval ago, then queue the next copy: the device never waits for the host
      if (pending) {
        HIPCHK(c, hipEventSynchronize(ev.e[E_FLAG]));
        if (c->host_flag[0] == 0) done = true;
        // the lengths of one interval ago bound today's: every commit since then added at most block_max
        const long since = c->commits - commits_at_copy;
        for (int s = 0; s < D.S; s++)
          c->len_bound[s] = (int)std::min<long>(c->len_bound[s], c->host_flag[16 + s] + since * D.Bm);
        if (c->host_flag[1] != 0) {
          // the single-launch verify kernel gave up in some pass of the last interval: nothing was accepted or
          // committed since, so the loop simply goes on with one launch per operator (message kept in fm_last_error)
          HIPCHK(c, hipStreamSynchronize(c->stream));
          (void)check_persist(c);
          pending = false;
          continue;
        }
      }
      if (!done) {
        HIPCHK(c, hipMemcpyAsync(c->host_flag, c->st.alive, sizeof(int), hipMemcpyDeviceToHost, c->stream));
        if (c->persist)
          HIPCHK(c, hipMemcpyAsync(c->host_flag + 1, c->pk.abort_word, sizeof(int), hipMemcpyDeviceToHost, c->stream));
        else
          c->host_flag[1] = 0;
        HIPCHK(c, hipMemcpyAsync(c->host_flag + 16, c->st.P, sizeof(int) * (size_t)D.S, hipMemcpyDeviceToHost, c->stream));
        commits_at_copy = c->commits;
        HIPCHK(c, hipEventRecord(ev.e[E_FLAG], c->stream));
        pending = true;
      }
    }
  }
  if (rc != FM_OK) return rc;
  HIPCHK(c, hipEventRecord(ev.e[E_END], c->stream));
  // outputs: x_1 .. x_P per sequence
  for (int s = 0; s < D.S; s++)
    HIPCHK(c, hipMemcpyAsync(out_tok + (size_t)s * D.maxtok, c->st.hist + (size_t)s * (D.maxtok + 1) + 1, (size_t)D.maxtok * 4,
                             hipMemcpyDeviceToDevice, c->stream));
  HIPCHK(c, hipMemcpyAsync(out_len, c->st.P, (size_t)D.S * 4, hipMemcpyDeviceToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  TRY(check_persist(c));      // a failure in the very last interval: reported, the caller may call again
  if (phase_pending) TRY(take_phases());
  if (stats) {
    unsigned long long cnt[3], hist[3 * 32];
    HIPCHK(c, hipMemcpy(cnt, c->st.counters, sizeof cnt, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hist, c->st.acc_hist, sizeof hist, hipMemcpyDeviceToHost));
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, ev.e[E_BEGIN], ev.e[E_END]));
    stats->steps = (int64_t)cnt[0];
    stats->tokens = (int64_t)cnt[1];
    for (int k = 0; k < 3; k++)
      for (int i = 0; i < 32; i++) stats->acc_hist[k][i] = (int64_t)hist[k * 32 + i];
    stats->ms_total = ms;
    const double n = phase_samples > 0 ? (double)phase_samples : 1.0;
    stats->ms_draft = ms_phase[0] / n; stats->ms_verify = ms_phase[1] / n; stats->ms_commit = ms_phase[2] / n;
    stats->phase_samples = phase_samples;
    stats->nonfinite_rows = (int64_t)cnt[2];
  }
  return FM_OK;
}

}  // extern "C"
