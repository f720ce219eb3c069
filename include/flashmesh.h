/*
 * flashmesh.h - C ABI of the MI355X (gfx950) predict / verify / commit decode path of an
 * hourglass transformer over quantised mesh coordinate tokens.
 *
 * Token sequence: x_0 = BOS, then 9 coordinate tokens per face, 3 per vertex (supplement,
 * "Hourglass Transformer").  Input position n predicts x_{n+1}.  One decode step is
 *     fm_draft  ->  fm_verify_block  ->  fm_commit
 * i.e. the predict and verify stages of Sec. 3 ("Predict-Correct-Verify Paradigm"); the
 * correct stage only edits the draft block and plugs in between fm_draft and fm_verify_block
 * through the caller-visible block buffer.
 *
 * Conventions
 *  - Every function returns 0 on success or a negative FM_E* code; fm_last_error() gives a
 *    message for the last failure on that context.  Nothing throws or aborts across the ABI.
 *  - Pointers named *_dev are DEVICE pointers owned by the caller (the library borrows them for
 *    the duration of the enqueued work); pointers named host_* / *_host are HOST pointers.
 *  - All device work is enqueued on the hipStream_t given to fm_create.  Only fm_load_weights,
 *    fm_generate, fm_read_state and fm_destroy synchronise that stream.
 *  - Weights, K/V caches at the three hourglass levels, pooling / upsampling carries, tapped
 *    features and draft distributions are owned by the context.
 *  - Sequences are independent; `batch` sequences are processed together with ragged block
 *    lengths and ragged accepted lengths.
 */
#ifndef FLASHMESH_H
#define FLASHMESH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FM_OK 0
#define FM_EINVAL (-1) /* bad argument or configuration                       */
#define FM_ESTATE (-2) /* call out of order (e.g. weights not loaded)         */
#define FM_ENOMEM (-3) /* device or host allocation failed                    */
#define FM_EHIP (-4)   /* a HIP runtime call failed; see fm_last_error        */

#define FM_DTYPE_F32 0  /* fp32 storage and arithmetic                          */
#define FM_DTYPE_BF16 1 /* bf16-valued weights held as IEEE half (exact), half K/V and GEMM inputs, fp32 accumulation */

typedef struct fm_ctx fm_ctx; /* opaque, owned by the library */

/* Plain-old-data configuration, copied by fm_create.  head_dim = d_model / n_heads must be 64, 96 or 128 (96 and 128 are the
 * widths of the paper's own models, Sec. 5.1; they run one launch per operator in either storage type - the single-launch
 * verify kernel and the fused projection epilogue are written for 64-wide heads).
 * vocabulary = n_bins + 3 with BOS = n_bins, EOS = n_bins + 1, PAD = n_bins + 2. */
typedef struct {
  int32_t d_model, n_heads, ffn_mult, n_bins;
  int32_t l_cpre, l_cpost, l_vpre, l_vpost, l_face; /* transformer blocks per hourglass stack      */
  int32_t mem_len;                                  /* rows of the condition memory c               */
  int32_t dtype;                                    /* FM_DTYPE_*                                   */
  int32_t max_batch;                                /* sequences held by the context                */
  int32_t max_tokens;                               /* longest stream per sequence (multiple of 9); also the
                                                       coordinate-level K/V capacity unless `window` is set */
  int32_t draft_coord;  /* Dc: coordinate-level SP heads (Eq. 1), one future token each            */
  int32_t draft_point;  /* m : nominal point-level tokens, multiple of 3, 0 = level off            */
  int32_t draft_face;   /* n : nominal face-level tokens, multiple of 9, 0 = level off             */
  int32_t hf_ffn_mult;  /* width multiplier of FFN^(t) in the HF block (Eq. 6)                     */
  int32_t ban_specials; /* 1: argmax over the coordinate bins only (BOS/EOS/PAD never chosen)      */
  float rope_base, rms_eps;
  int32_t window;       /* sliding-window self-attention (Sec. 5.1 "window size"): 0 = a position sees the whole
                           context and max_tokens is also the K/V capacity; W > 0 (multiple of 9) = a position p
                           of the coordinate level sees keys [p-W+1, p], the vertex and face levels W/3 and W/9
                           of their own positions, the K/V caches are rings of W + block_max + 2 positions (rounded
                           up to 128) and max_tokens only bounds the length of the emitted stream                 */
  int32_t rules_off;    /* schedule rules of the supplement's "Optimizations" to switch OFF (0 = the paper's final schedule):
                           bit 0 = rule (A): the point level then also fires at face split nodes;
                           bit 1 = rule (B): the point and face levels then also predict their first three tokens (HF sets for
                           the coordinate offsets 0..2 and the vertex offset 0 join the blob), which are averaged with the
                           coordinate level's                                                                            */
} fm_config;

typedef struct {
  int64_t steps;             /* decode steps run by fm_generate                                   */
  int64_t tokens;            /* tokens emitted over all sequences (BOS excluded)                  */
  int64_t acc_hist[3][32];   /* histograms of accepted lengths (main token included) per (step, live sequence), by what the
                                block carried: [0] coordinate-level drafts only, [1] a fresh point-level prediction, [2] a
                                fresh face-level prediction.  Their sum is the histogram of all steps; the mean of
                                (length - 1) over [2] / [1] is the number of correctly verified tokens per draft prediction
                                at the face / point level (Sec. 5.4, Table "draft_num": Face-Acc, Point-Acc)                */
  double ms_total;           /* device time of the whole loop, hipEvent                            */
  double ms_draft, ms_verify, ms_commit; /* device time of the draft (+ correct), verify and commit phases of one step: mean
                                over the phase_samples steps that carried event marks (one step in 32)                      */
  int64_t phase_samples;
  int64_t nonfinite_rows;    /* verify rows whose logits held an infinity or a NaN (0 in a healthy run): with FM_DTYPE_BF16
                                activations, K/V and GEMM inputs are IEEE half, which overflows beyond 65504 without a trap */
} fm_stats;

/* Create a context for `cfg` bound to `hip_stream` (a hipStream_t; NULL = the null stream).
 * Allocates every device buffer up front.  FM_EINVAL for an unsupported configuration. */
int fm_create(const fm_config* cfg, void* hip_stream, fm_ctx** out);
int fm_destroy(fm_ctx* ctx);
const char* fm_last_error(const fm_ctx* ctx);

/* Largest verify block (main token + drafts) = max(1 + Dc, m, n): row stride of the block buffers. */
int32_t fm_block_max(const fm_ctx* ctx);
/* Number of float32 values fm_load_weights expects. */
int64_t fm_blob_elems(const fm_ctx* ctx);

/* Load all parameters from one HOST blob of float32 values in manifest order (embedding; per stack
 * cpre, vpre, face, vpost, cpost and per block g1,wq,wk,wv,wo,g2,cq,ck,cv,co,g3,w1,w2; shorten
 * coord->vertex, vertex->face; final gain, LM head; SP heads per level; HF sets per level; label head), linear
 * weights as [out,in].  Converts to the configured storage type on the device.  Synchronises. */
int fm_load_weights(fm_ctx* ctx, const float* host_blob, size_t n_floats);

/* Cross-attention keys/values of every block for sequence `seq` from its condition memory
 * mem_dev [mem_len, d_model] float32 (K_mem = W_k c, V_mem = W_v c; the condition c of Sec. 3.1),
 * and reset of the sequence to x_0 = BOS with empty caches. */
int fm_prefill_condition(fm_ctx* ctx, int32_t seq, const float* mem_dev);

/* fm_prefill_condition for callers that must not touch an allocator while they run (a serving loop that re-conditions
 * a sequence between requests, code under HIP graph capture, harnesses that forbid hipMalloc): the same kernels and the
 * same result, but the staging area of the call (the condition memory re-ordered for the matrix units, or, on the fp32
 * path, its converted copy and one block's K/V rows) lives in a 16 MiB device array that is part of the library image
 * instead of memory owned by the context.  The call allocates and frees nothing.  FM_EINVAL with a message when the
 * configuration needs more staging than 16 MiB (mem_len * d_model * 2 bytes in half precision with mem_len and d_model
 * multiples of 256, else mem_len * d_model * (element size + 8)).  Every GPU holds one such array for all contexts on
 * it: calls that overlap in time on one GPU (different streams or contexts) race on it; calls on one stream are safe. */
int fm_prefill_condition_static(fm_ctx* ctx, int32_t seq, const float* mem_dev);

/* Predict stage (Sec. 3.1, supplement "Three-Level Speculative Decoding"): from the features tapped
 * at the last committed position run the coordinate-level SP heads, and the point / face pipelines
 * (SP heads, draft upsample Eq. 2, HF blocks Eq. 3-6) where a split node was crossed (rules (A) and
 * (B) of the supplement), average the distributions that cover a position and take the argmax.
 * Writes block_tok_dev[seq*block_max + i] (i = 0 is the main token) and block_len_dev[seq]
 * (0 for a finished sequence).  Updates only the context's draft bookkeeping. */
int fm_draft(fm_ctx* ctx, int32_t* block_tok_dev, int32_t* block_len_dev);

/* Correct stage (Sec. 3.2 "Correction Mechanism"), between fm_draft and fm_verify_block; it edits draft tokens only,
 * never block_tok_dev[seq*block_max + 0], so the emitted stream is unchanged and only acceptance can move.
 * fm_set_correct(hist_vertices > 0) switches it on: fm_draft then also keeps, per point-level feature of the point and
 * face pipelines, the softmax of the linear label head (historical / new / intra-batch), and fm_generate runs the
 * stage in every speculative step; 0 switches it off.
 * fm_correct: the points of a block are the vertices whose three tokens (z, y, x) are all drafts and all coordinate
 * bins; a point's label is the arg max of the mean of the label rows held for it (new if none).  A historical point
 * that equals none of the last hist_vertices known vertices moves onto the nearest of them; an intra-batch point
 * that equals no other point of the block moves onto the nearest point labelled new in another face (squared
 * distance in bins, lowest vertex index on ties, no candidate: unchanged); faces made of draft tokens only are
 * re-sorted ascending in (z, y, x).  labels_out_dev ([batch, block_max] int32, may be NULL) receives the label of
 * the i-th point of each block, -1 beyond.  FM_ESTATE when the stage is off. */
int fm_set_correct(fm_ctx* ctx, int32_t hist_vertices);
int fm_correct(fm_ctx* ctx, int32_t* block_tok_dev, const int32_t* block_len_dev, int32_t* labels_out_dev);

/* Sampled decoding with non-greedy verification (the supplement's "Integrating the three levels" averages predicted
 * distributions; Sec. 3.3 evaluates a match test, which is temperature 0 here).  With temperature T > 0: fm_draft draws
 * every draft token from the averaged draft distribution q over the admissible tokens; fm_verify_block forms
 * p = softmax(logits / T) per row, accepts draft x while u q(x) < p(x) (a draft that is not the token drawn from q -
 * replayed, corrected or written by the caller - counts as a proposal with all its mass on it), and the next main token
 * comes from max(p - q, 0) after the first rejection, from p after a fully accepted block.  The emitted stream is then
 * distributed like token-by-token sampling from the backbone.  Uniforms are counter based, keyed by (seed, sequence,
 * absolute position, purpose), so a run is reproducible.  temperature = 0 (the default) is greedy decoding. */
int fm_set_sampling(fm_ctx* ctx, float temperature, uint64_t seed);

/* Verify stage (Sec. 3.3): one causal backbone forward over each sequence's block at positions
 * P .. P+len-1 against the K/V caches of all three levels.  logits_dev ([batch, block_max, vocab]
 * float32) may be NULL.  accepted_len_dev[seq] = 1 + number of leading drafts equal to the
 * backbone's own greedy prediction (0 for an empty block).  Committed state is not changed;
 * calling it twice with the same block gives the same result.
 * One sequence in half precision runs as a single launch of 256 workgroups that wait for each other's results and
 * must therefore all be resident: the library checks at fm_create that the kernel fits once per compute unit, but it
 * cannot see other work on the GPU.  A kernel of another stream or process that occupies compute units while a pass
 * runs can make a bounded wait (200 ms) expire.  Such a pass writes accepted_len_dev = 0 for every sequence, fm_commit
 * of it changes nothing, the next synchronising call (fm_read_state, fm_verify_bytes, fm_generate) returns FM_EHIP with
 * the diagnosis once, and from then on the context runs one launch per operator (fm_verify_path() = 0), so the caller
 * can simply draft and verify again. */
int fm_verify_block(fm_ctx* ctx, const int32_t* block_tok_dev, const int32_t* block_len_dev,
                    float* logits_dev, int32_t* accepted_len_dev);

/* Commit the first accepted_len_dev[seq] (1..len; 0 = leave the sequence as it is) tokens of the last verified block: advances the
 * committed lengths at all three levels (K/V rollback is implicit: rows past them are scratch), and
 * makes the backbone's prediction after the last accepted token the next main token. */
int fm_commit(fm_ctx* ctx, const int32_t* accepted_len_dev);

/* Whole loop, device side: repeat draft -> verify -> commit until every sequence has max_faces faces
 * or ended with EOS.  speculative = 0 runs plain one-token-per-step greedy decoding of the same
 * backbone.  out_tok_dev [batch, max_tokens] receives x_1.., out_len_dev [batch] their count.
 * host_stats may be NULL.  Sequences must have been prefetched with fm_prefill_condition. */
int fm_generate(fm_ctx* ctx, int32_t max_faces, int32_t speculative, int32_t* out_tok_dev,
                int32_t* out_len_dev, fm_stats* host_stats);

/* Test / measurement hooks ------------------------------------------------------------------- */

/* HOST out[seq*6 + k]: committed coordinate, vertex, face lengths, pending main token, finished flag,
 * tokens emitted.  Synchronises. */
int fm_read_state(fm_ctx* ctx, int32_t* host_out);

/* Synthetic draft source for throughput measurements with a prescribed acceptance pattern: when
 * stream_dev != NULL, fm_draft still runs every head but then replaces draft token x_p by
 * stream_dev[seq*stride + p - 1] (the known greedy continuation, x_1 first) when the counter-based
 * uniform u(seed, seq, p) < keep_prob, else by a wrong id.  NULL switches it off. */
int fm_set_draft_replay(fm_ctx* ctx, const int32_t* stream_dev, int32_t stride, int32_t n_valid,
                        float keep_prob, uint64_t seed);

/* Budget of 9*max_faces generated tokens per sequence for the step-wise API (default max_tokens):
 * blocks are clipped to it and a sequence that reaches it is finished; prefilled sequences below the
 * new budget that did not end with EOS become live again.  FM_EINVAL outside [1, max_tokens/9]. */
int fm_set_budget(fm_ctx* ctx, int32_t max_faces);

/* Stage timing of the persistent verify kernel (only when the context was created with the environment
 * variable FM_PROFILE=1): HOST out[0] = earliest workgroup start, out[1 + s] = latest completion of stage s of
 * the passes since the last call, in ticks of the 100 MHz wall clock; then re-arms.  Synchronises. */
int fm_debug_profile(fm_ctx* ctx, uint64_t* host_out, int32_t n);

/* HOST copy of one of the position-indexed carry rings, [batch][ring][d_model] float32; which: 0 coordinate
 * pre-stack outputs (32 entries), 1 vertex pre-stack outputs (16), 2 face outputs (8), 3 vertex outputs (16),
 * 4/5/6 tapped features of the coordinate (32) / vertex (16) / face (8) level.  Entry = position mod ring size.
 * Synchronises. */
int fm_debug_ring(fm_ctx* ctx, int32_t which, float* host_out);

/* Draft-stage buffers of the last fm_draft for element-wise parity checks.  which = -1 / -2 switches the keeping of the
 * averaged draft distributions on / off (greedy decoding does not need them and skips the stores by default; sampled
 * decoding always keeps them).  which = 0: HOST out [batch][block_max][vocab] float32, row i of a sequence = the
 * averaged distribution behind draft index i (supplement "Integrating the three levels"; entries at or above the
 * admissible token count and rows at or above the block length are unspecified).  which = 1 / 2: the label
 * distributions of the point pipeline [batch][max(m/3 - 1, 1)][3] / of the face pipeline [batch][max(n/3 - 1, 1)][3]
 * (Sec. 3.2; rows of pipelines that have not fired hold older values; with rule (B) off the face pipeline has n/3 rows).
 * Synchronises. */
int fm_debug_draft(fm_ctx* ctx, int32_t which, float* host_out);

/* Cross-attention keys and values of the condition memory as fm_prefill_condition left them (Sec. 3.1: K_mem = W_k c,
 * V_mem = W_v c), for element-wise parity checks: HOST k_out and v_out, each [mem_len][d_model] float32 in plain row-major
 * order (the library undoes its blocked cache layouts), for sequence `seq` and transformer block `block`, blocks counted
 * through the stacks in the order coordinate-pre, point-pre, face, point-post, coordinate-post.  Synchronises.
 * FM_EINVAL for an index out of range, FM_ESTATE if the sequence has not been prefilled. */
int fm_debug_mem_kv(fm_ctx* ctx, int32_t seq, int32_t block, float* host_k, float* host_v);

/* What this GPU sustains, for reporting next to the published peaks: HOST out[0] = streaming read GB/s, out[1] =
 * streaming copy GB/s (read + write bytes), out[2] = register-only MFMA loop TFLOP/s (fp16, 32x32x16).  Allocates
 * and frees 2 GiB of device memory for the duration of the call.  Synchronises. */
int fm_measure_peaks(fm_ctx* ctx, double* host_out);

/* Cost of one dependent all-to-all hand-off between resident workgroups, the step that the single-launch verify kernel
 * repeats about ten times per transformer block: 2000 rounds in which each of `workgroups` (2..256) workgroups publishes
 * its share of `bytes` (tagged 8-byte elements, agent-scope stores) and then reads all of them (agent-scope loads,
 * repeated until every tag matches), nothing else.  pingpong != 0: one element each way between two workgroups instead.
 * HOST out[0] = microseconds per round.  Allocates and frees its buffers; every wait in the kernel is bounded.
 * Synchronises. */
int fm_measure_exchange(fm_ctx* ctx, int32_t workgroups, int32_t bytes, int32_t pingpong, double* host_out);

/* Row sweep of the weight-streaming GEMM kernel that the per-operator path uses: times Y[rows, 4 d_model] =
 * gelu(X[rows, d_model] W1^T) with the FFN up projection of the first block (half-precision contexts only), back to
 * back on the context's stream.  HOST out[0] = milliseconds per launch, out[1] = TFLOP/s.  Allocates and frees its
 * operands.  Synchronises. */
int fm_measure_gemm(fm_ctx* ctx, int32_t rows, double* host_out);

/* Which implementation fm_verify_block runs for this context: 1 = the single persistent kernel (half-precision
 * storage, one sequence, block <= 32), 0 = one launch per operator.  Both compute the same function with the same
 * arithmetic per operator; they cut the key axis of the attention differently, so results agree to rounding, and
 * each is bit-reproducible in itself. */
int32_t fm_verify_path(const fm_ctx* ctx);

/* Algorithmic HBM bytes of one verify pass at the current committed lengths (weights once, self
 * and cross K/V once per block and sequence), for roofline reporting.  Synchronises. */
int fm_verify_bytes(fm_ctx* ctx, double* host_bytes);

#ifdef __cplusplus
}
#endif
#endif /* FLASHMESH_H */
