/*
 * spark.h -- C ABI of the MI355X (gfx950) SPAR-K decoding library.
 *
 * SPAR-K (scheduled periodic alternating early exit) decodes an interleaved text/speech token
 * stream with a depth schedule: text positions run all L layers; inside every speech chunk the
 * positions are cut into periods of K, one fixed slot of each period runs all L layers (a
 * "refresh") and the other K-1 exit at layer e and are decoded by a layer-specific head g_e
 * (Sec. IV-B.1, IV-B.2).  The upper-layer KV of early-exited positions is not computed when they
 * exit: their hidden state h^(e) is kept, and the next full-depth step pushes them, together with
 * its own position, through layers e+1..L in one batched pass (Sec. IV-B.3, Algorithm 1).
 *
 * All compute runs in HIP kernels on the stream given to spark_init.  Pointers marked [device]
 * are device memory owned by the caller and must outlive the context; pointers marked [host] are
 * ordinary host memory.  Every call returns SPARK_OK or a negative SPARK_E* code; nothing throws
 * and the only state outside a context is the static scratch area of spark_init_static.  A context
 * is not thread-safe.
 */
#ifndef SPARK_H
#define SPARK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPARK_OK 0
#define SPARK_EINVAL (-1)  /* bad dimension, e outside [1,L], K < 1, phase outside [0,K), bad id */
#define SPARK_ENOSEQ (-2)  /* unknown / closed sequence id, or no free sequence slot */
#define SPARK_ENOMEM (-3)  /* KV pool exhausted, context longer than max_seq_len, buffer too small */
#define SPARK_ESTATE (-4)  /* step before prefill, second prefill on a live sequence */
#define SPARK_EHIP (-5)    /* a HIP runtime call failed; see spark_last_error */
#define SPARK_ENAN (-6)    /* a head produced a NaN logit */

#define SPARK_DTYPE_FP32 0
#define SPARK_DTYPE_BF16 1

#define SPARK_SCOPE_CHUNK 0  /* period counter restarts at every speech chunk (Sec. IV-B.1) */
#define SPARK_SCOPE_STREAM 1 /* period counter runs over all speech positions of the sequence */

#define SPARK_MAX_PERIOD 16  /* largest supported K */

/* size of the library's own scratch area, see spark_init_static */
#define SPARK_STATIC_SCRATCH_BYTES (64u << 20)

/* Model dimensions and schedule.  Plain data; `size` must be sizeof(spark_config). */
typedef struct spark_config {
  uint32_t size;
  int32_t n_layers;      /* L */
  int32_t d_model;       /* d, multiple of 8 */
  int32_t n_q_heads;     /* multiple of n_kv_heads */
  int32_t n_kv_heads;
  int32_t head_dim;      /* 64 or 128 */
  int32_t d_ffn;         /* SwiGLU width F, multiple of 8 */
  int32_t vocab_text;    /* ids [0, vocab_text) are text */
  int32_t vocab_speech;  /* ids [vocab_text, vocab_text + vocab_speech) are speech */
  float rope_base;       /* rotary base, angle = pos * base^(-2i/head_dim) on pairs (i, i+hd/2) */
  float rms_eps;
  int32_t dtype;         /* SPARK_DTYPE_*: element type of every matrix and of the KV cache */
  int32_t exit_layer;    /* e in [1, L]; e == L disables early exit (Sec. III, IV-B.1) */
  int32_t period_k;      /* K in [1, SPARK_MAX_PERIOD]; K == 1 disables early exit */
  int32_t phase;         /* in [0, K): slot of the full-depth position inside each period */
  int32_t scope;         /* SPARK_SCOPE_* */
  int32_t n_text;        /* interleave pattern: n_text text slots, then n_speech speech slots */
  int32_t n_speech;
  int32_t max_batch;     /* sequences that may be open / stepped together */
  int32_t max_seq_len;   /* longest context (prompt + generated) of one sequence */
  int32_t kv_page_tokens;/* tokens per KV page, multiple of 16 */
  /* The same periodic rule on text positions (Sec. V-C "Exploring Text Early Exit Policies",
   * Table II row G10).  text_period_k <= 1: every text position runs full depth (the default of
   * Sec. IV-B.1).  Otherwise the text position with index t -- inside its chunk (SCOPE_CHUNK) or
   * among all text positions of the sequence (SCOPE_STREAM) -- runs full depth iff
   * t mod text_period_k == text_phase and exits at layer e otherwise; early-exited text
   * positions are completed by the next full-depth step like speech ones.  The pending rows of
   * both modalities must fit: 2*period_k + 2*text_period_k <= 2*SPARK_MAX_PERIOD. */
  int32_t text_period_k;
  int32_t text_phase;    /* in [0, text_period_k) when text_period_k > 1 */
} spark_config;

/* Weights [device].  Matrices are row-major [out][in] in `dtype`; gains and lens_b are fp32.
 * Per-layer tensors are stacked along a leading layer axis.  The layer-specific head is
 * g_e(h) = lens_head . RMSNorm(h + lens_a h + lens_b ; lens_norm)  (Sec. IV-B.2, Eq. 2);
 * the final head is g_L(h) = lm_head . RMSNorm(h ; final_norm)  (Sec. III, Eq. 1). */
typedef struct spark_weights {
  const void *embed;       /* [V][d] */
  const float *attn_norm;  /* [L][d] */
  const void *wq;          /* [L][n_q_heads*head_dim][d] */
  const void *wk;          /* [L][n_kv_heads*head_dim][d] */
  const void *wv;          /* [L][n_kv_heads*head_dim][d] */
  const void *wo;          /* [L][d][n_q_heads*head_dim] */
  const float *mlp_norm;   /* [L][d] */
  const void *wg;          /* [L][F][d] */
  const void *wu;          /* [L][F][d] */
  const void *wd;          /* [L][d][F] */
  const float *final_norm; /* [d] */
  const void *lm_head;     /* [V][d] */
  const void *lens_a;      /* [d][d] */
  const float *lens_b;     /* [d] */
  const float *lens_norm;  /* [d] */
  const void *lens_head;   /* [V][d]; may alias lm_head */
} spark_weights;

/* Exit-layer log of one sequence (Sec. V-A "Metrics", Eq. 4). */
typedef struct spark_stats {
  int64_t text_steps;        /* text positions decoded at depth L */
  int64_t speech_full_steps; /* speech positions decoded at depth L */
  int64_t speech_ee_steps;   /* speech positions decoded at depth e */
  int64_t flush_rows[2 * SPARK_MAX_PERIOD]; /* [m]: full-depth steps that pushed m rows through
                                               layers e+1..L (pending positions + their own) */
  double mean_text_depth;    /* average exit layer over text positions (0 if none) */
  double mean_speech_depth;  /* average exit layer over speech positions (0 if none) */
  double speech_layer_saving;/* (1 - mean_speech_depth / L) * 100, Eq. 4 (0 if none) */
  int64_t text_ee_steps;     /* text positions decoded at depth e (0 unless text_period_k > 1) */
} spark_stats;

typedef struct spark_ctx spark_ctx;

/* Sizes of the two device buffers the caller must provide for this configuration: the paged KV
 * pool (every sequence at max_seq_len) and the scratch area (activations, schedule state, logits).
 * What has to be kept follows from Sec. IV-B.3: the KV cache of all L layers for every position,
 * and the hidden states h^(e) of the early-exited positions until the next full-depth step; on
 * memory management itself the paper is silent.  For bf16 models whose widths are multiples of 8
 * the scratch size also has room for a second copy of the projection and head matrices, laid out
 * in the order the matrix units consume them, which the context writes when it is created and
 * which the projections of five and more rows read instead of the caller's tensors (as many bytes
 * again as those matrices).  cfg [host]; the two sizes are written to kv_pool_bytes /
 * scratch_bytes [host] (either may be NULL).
 * Returns SPARK_EINVAL for a configuration the library refuses. */
int spark_workspace_bytes(const spark_config *cfg, size_t *kv_pool_bytes, size_t *scratch_bytes);

/* The schedule alone (Sec. IV-B.1), no device needed: executed depth (exit_layer or n_layers) and
 * modality (1 = text) of the first n_steps generated tokens of a sequence opened at cycle_offset
 * with the given text budget (<= 0: none; see spark_seq_text_budget).  depth_out, is_text_out
 * [host], n_steps entries each.  It evaluates the same function the dispatch kernel evaluates. */
int spark_schedule_preview(const spark_config *cfg, int32_t cycle_offset, int32_t text_budget,
                           int32_t n_steps, int32_t *depth_out, int32_t *is_text_out);

/* Create a context: the inputs of Algorithm 1 -- a model with L layers (Sec. III), the exit layer
 * l_EE with its layer-specific head (Sec. IV-B.2), the period K and phase of the schedule
 * (Sec. IV-B.1) and the interleave ratio N_text : N_speech (Sec. III).  cfg, weights [host];
 * kv_pool and scratch [device] must be at least the sizes reported above and 256-byte aligned and
 * stay the caller's (they must outlive the context; their contents need not be cleared);
 * hip_stream is a hipStream_t (NULL = the default stream) on which every kernel of this context is
 * launched.  The weights struct is copied; the tensors are not, and they must keep their contents
 * while the context lives (the copy mentioned above is taken from them here, once).  *out [host] receives the context,
 * to be released with spark_destroy.  SPARK_EINVAL: refused configuration or a NULL tensor;
 * SPARK_ENOMEM: a buffer is NULL, too small or misaligned; SPARK_EHIP: a runtime call failed. */
int spark_init(const spark_config *cfg, const spark_weights *weights, void *kv_pool,
               size_t kv_pool_bytes, void *scratch, size_t scratch_bytes, void *hip_stream,
               spark_ctx **out);

/* spark_init for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the scratch area is a static device array of
 * SPARK_STATIC_SCRATCH_BYTES inside the library instead of a caller's buffer, and the staging
 * buffers are ordinary host arrays; the call makes no hipMalloc / hipHostMalloc / hipFree.  The
 * caller still passes the weights and the KV pool.  Such a context keeps no second copy of the
 * weights (its projections of five and more rows read the caller's tensors); configurations whose
 * scratch need without that copy exceeds SPARK_STATIC_SCRATCH_BYTES are refused
 * (SPARK_ENOMEM, with a message on stderr).  Each GPU has one such array: at most one context per
 * device may live on it at a time (a second spark_init_static on the same device returns
 * SPARK_ESTATE until the first is destroyed), the array keeps the previous context's contents
 * (what must start at zero is cleared here), and calls on two contexts that share it would race.
 * Everything else is spark_init. */
int spark_init_static(const spark_config *cfg, const spark_weights *weights, void *kv_pool,
                      size_t kv_pool_bytes, void *hip_stream, spark_ctx **out);

/* Open a sequence: one response of the interleaved generation of Sec. III.  cycle_offset >= 0 is
 * the slot of the N_text + N_speech interleave cycle at which the first generated token falls
 * (0 = first text slot); where a response enters the cycle the paper does not say.  Writes the id
 * (0 .. max_batch-1) to *seq_id [host].  SPARK_ENOSEQ: all max_batch slots are open. */
int spark_seq_open(spark_ctx *ctx, int32_t cycle_offset, int32_t *seq_id);

/* The text of an interleaved response ends before its speech does (Sec. IV-A: speech tokens are
 * 79.5 % / 81.2 % of what the two models generate, more than the 2/3 their interleave ratios alone
 * give).  After n_text_tokens text tokens in all, this sequence generates speech only: the slots
 * of the cycle that would be text become speech, and the speech chunk running at that moment goes
 * on, so a per-chunk index (SPARK_SCOPE_CHUNK) keeps counting from that chunk's start.  May be
 * set once per sequence, before or between steps, and not below the number of text tokens the
 * sequence has generated already (SPARK_EINVAL; SPARK_ESTATE if a budget is set). */
int spark_seq_text_budget(spark_ctx *ctx, int32_t seq_id, int32_t n_text_tokens);

/* The phase of the schedule on speech positions is a free choice (Table II: the Even, Odd and
 * Triple variants differ in little else), and in a batch it decides whether the sequences'
 * full-depth steps fall on the same steps: only then does an early-exit step skip the upper layers
 * for the whole batch (Sec. IV-B.3).  spark_seq_set_phase moves one sequence's phase (0 <= phase <
 * period_k) for its future speech positions; spark_align_phases moves the phases of n sequences
 * [host ids] so that, counted in their own speech positions, each runs full depth at its K-th
 * speech position from now and every K-th after it (SPARK_SCOPE_STREAM only).  The move can join
 * two runs of early exits (at most 2K-2 pending positions, which the pending slots hold).  Not
 * available with a schedule on text positions (SPARK_EINVAL). */
int spark_seq_set_phase(spark_ctx *ctx, int32_t seq_id, int32_t phase);
int spark_align_phases(spark_ctx *ctx, int32_t n, const int32_t *seq_ids);

/* Condition on a prompt [host] of n >= 1 ids (Sec. III: generation is conditioned on the input;
 * on how the prompt is processed the paper is silent): positions 0..n-2 are run at full depth and
 * fill the KV of every layer, which is the state every full-depth step restores (end of
 * Sec. IV-B.3); the last id is held as the input of the first spark_step, so that every generated
 * token comes out of spark_step with its executed depth.  One prompt per sequence (SPARK_ESTATE on
 * a second); SPARK_EINVAL: empty prompt or an id outside the vocabulary; SPARK_ENOMEM: longer
 * than max_seq_len or no KV pages left.  Returns when the prompt pass has completed. */
int spark_prefill(spark_ctx *ctx, int32_t seq_id, const int32_t *prompt, int32_t n);

/* One decoding step for n distinct prefilled sequences seq_ids[0..n) [host] (Algorithm 1).
 * For each: the schedule decides early exit or full depth; layers 1..e run on the new position;
 * an early-exit position is decoded by g_e and its h^(e) kept pending; a full-depth position
 * takes the pending positions with it through layers e+1..L and is decoded by g_L.
 * out_tokens[i], out_depth[i] [host]: emitted id (greedy, lowest id on ties) and executed depth
 * (e or L).  forced_next [host, nullable]: if forced_next[i] >= 0 it becomes the next input of
 * sequence i in place of the emitted id (teacher forcing); the emitted id is still reported.
 * Returns after the results are on the host. */
int spark_step(spark_ctx *ctx, int32_t n, const int32_t *seq_ids, const int32_t *forced_next,
               int32_t *out_tokens, int32_t *out_depth);

/* n_steps consecutive steps of the same n sequences without returning to the host in between:
 * the emitted id (or forced_next[s*n + i] when given and >= 0) feeds the next step on the device.
 * out_tokens / out_depth [host] are [n_steps][n].  Same results as n_steps calls of spark_step. */
int spark_decode(spark_ctx *ctx, int32_t n_steps, int32_t n, const int32_t *seq_ids,
                 const int32_t *forced_next, int32_t *out_tokens, int32_t *out_depth);

/* Temperature / nucleus (top-p) sampling in place of the arg-max (Sec. V-A "Models": Step-Audio-2
 * decodes with temperature 0.7 and top_p 0.9; GLM-4-Voice greedily).  temperature > 0 and
 * 0 < top_p <= 1 switch it on for spark_decode_sampled; temperature <= 0 switches it off.
 * With w_i = exp((l_i - max l) / temperature) and integer masses q_i = floor(w_i * 2^32 + 1/2)
 * (at most 2^32 - 1), the candidates are ordered by larger q, then lower id; the nucleus is the
 * shortest prefix whose mass reaches ceil(top_p * sum q); with M its mass and omega the step's
 * 64-bit random word, the token is the element of the prefix at which the running mass first
 * exceeds floor(omega * M / 2^64).  Returns SPARK_EINVAL for parameters outside these ranges. */
int spark_set_sampling(spark_ctx *ctx, float temperature, float top_p);

/* spark_decode with one 64-bit random word per step and sequence: rand_words [host] is
 * [n_steps][n].  With sampling switched off (or rand_words == NULL) it is spark_decode. */
int spark_decode_sampled(spark_ctx *ctx, int32_t n_steps, int32_t n, const int32_t *seq_ids,
                         const int32_t *forced_next, const uint64_t *rand_words,
                         int32_t *out_tokens, int32_t *out_depth);

/* Logits [host, V floats] of the head that decoded the sequence's latest position -- g_L of Eq. 1
 * or the layer-specific g_e of Eq. 2 -- and which head it was (*head = e or L; may be NULL).
 * SPARK_ESTATE: the sequence has not been stepped or was not in the latest step. */
int spark_get_logits(spark_ctx *ctx, int32_t seq_id, float *out_logits, int32_t *head);

/* Copy one position's cached key and value vectors (n_kv_heads*head_dim floats each) of one layer
 * (0-based) to the host; for tests of the deferred KV fill. */
int spark_get_kv(spark_ctx *ctx, int32_t seq_id, int32_t layer, int32_t pos, float *k_out,
                 float *v_out);

/* Current context length, number of positions whose upper-layer KV (layers e+1..L) is complete,
 * and number of pending early-exited positions of a sequence: the bookkeeping of Sec. IV-B.3
 * (after every full-depth step the cache is complete, len == upper_valid).  All [host]; any
 * pointer may be NULL. */
int spark_seq_state(spark_ctx *ctx, int32_t seq_id, int32_t *len, int32_t *upper_valid,
                    int32_t *n_pending);

/* The exit-layer log of a sequence so far (Sec. V-A "Metrics", Eq. 4); out [host]. */
int spark_get_stats(spark_ctx *ctx, int32_t seq_id, spark_stats *out);

/* Release a sequence and its KV pages (the paper is silent on the lifetime of a response); waits
 * for the context's stream. */
int spark_seq_close(spark_ctx *ctx, int32_t seq_id);

/* Wait for the context's stream and release the context (its host memory and staging buffers;
 * the caller's device buffers are untouched).  NULL is ignored. */
void spark_destroy(spark_ctx *ctx);

/* Text of the last error of this context (never NULL; valid until the next call on ctx). */
const char *spark_last_error(const spark_ctx *ctx);

/* Measurement support.  While `kernel_class` is >= 0, every launch of that class of kernel during
 * spark_step / spark_decode is bracketed by HIP events on the context's stream;
 * spark_profile_read waits for them and reports the number of bracketed launches and their summed
 * duration in milliseconds since the last read (total_ms), and in empty_ms [nullable] the summed
 * duration of as many empty brackets (a third event behind every bracket measures it), i.e. what
 * the event mechanism itself adds to total_ms.  Classes: see SPARK_KC_*.  -1 switches it off. */
#define SPARK_KC_QKV 0
#define SPARK_KC_ATTN 1
#define SPARK_KC_OPROJ 2
#define SPARK_KC_GATEUP 3
#define SPARK_KC_DOWN 4
#define SPARK_KC_LENS 5
#define SPARK_KC_HEAD 6
/* 7 is unused */
#define SPARK_KC_SAMPLE 8 /* the temperature / nucleus sampler */
#define SPARK_KC_COUNT 9
int spark_profile_select(spark_ctx *ctx, int32_t kernel_class);
int spark_profile_read(spark_ctx *ctx, int64_t *n_launches, double *total_ms, double *empty_ms);

/* Measurement support: what the memory system delivers to the simplest possible reader, to be
 * quoted next to the published peak.  Reads buf [device, 16-byte aligned, bytes a multiple of 16]
 * `reps` times with a plain kernel of 16-byte loads (every wave eight consecutive KiB per trip) (nontemporal != 0: with the
 * non-temporal hint the weight-streaming kernels use) on the context's stream, bracketed by HIP
 * events after one untimed pass, and writes the rate in GB/s (10^9 bytes) to *gbps [host] and the
 * XOR of all 32-bit words of buf to *checksum [host, may be NULL].  buf should be larger than the
 * last-level cache (256 MB) for the figure to be a memory figure. */
int spark_measure_read(spark_ctx *ctx, const void *buf, size_t bytes, int32_t reps, int32_t nontemporal,
                       double *gbps, uint32_t *checksum);

/* Kernel-selection switches of one context, for tests and sweeps; the defaults are the measured
 * choices and nothing in the results depends on them beyond rounding order.  name [host]:
 *   "mfma" (0: every row count stays on the vector kernels), "mfma_min_rows" (rows from which the
 *   projections run on the MFMA units), "mfma_small_tiles", "mfma_xcd_max_split",
 *   "attn_pieces" (64-token pieces per attention workgroup, 0 = by the size of the launch, at most
 *   8), "attn_mfma_min_rows", "gemv_big_kb", "mfma_tiled" (0: the MFMA projections stage the
 *   caller's weight rows through LDS instead of reading the context's copy in operand order),
 *   "mfma_small_max_k", "fuse_norm" (0: every RMSNorm of the batched path is its own launch),
 *   "prefill_rows" (prompt rows per pass, a multiple of 32, at most 256).
 * SPARK_EINVAL for an unknown name. */
int spark_tune(spark_ctx *ctx, const char *name, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* SPARK_H */
