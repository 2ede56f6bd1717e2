/*
 * spark_oracle.c -- plain CPU oracle for SPAR-K decoding.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the HIP library computes.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by nothing
 * else: the product path never links, loads or calls it, and it shares no code, table or
 * constant with the HIP sources.  Nothing here is blocked, fused or reordered: every function
 * is the paper's step (or the textbook definition of a transformer block) written out.
 *
 * What it computes
 *   - the SPAR-K early-exit scheduler            (Sec. IV-B.1, "SPAR-K Early Exit Scheduler")
 *   - prediction from an intermediate layer with a layer-specific head g_l
 *                                                (Sec. IV-B.2, Eq. 2)
 *   - deferred parallel decoding of missing upper-layer KV
 *                                                (Sec. IV-B.3, Algorithm 1)
 *   - standard full-depth decoding               (Sec. III, Eq. 1)
 *   - exit-layer logging                         (Sec. V-A "Metrics", Eq. 4)
 *
 * Arithmetic type: `real`, float by default (the target fixes fp32 for the oracle); compile with
 * -DORA_REAL=double for the fp64 twin used to bound the oracle's own rounding noise.
 *
 * Pins (tests/test_oracle_*.py): schedule against the exit-layer column of Table II and the
 * closed-form count of full-depth slots; primitives against closed forms and library routines;
 * standard decoding against a full-recompute definition in numpy (oracle/definition.py);
 * SPAR-K with e = L or K = 1 against standard decoding; teacher-forced SPAR-K KV and logits
 * against standard decoding (the invariant stated at the end of Sec. IV-B.3).
 * The form of the layer-specific head (affine translator + norm + unembedding) is a reading of
 * "layer-specific LM head [tuned lens]" that the paper does not spell out: PARITY UNPINNED for
 * that choice of form; its arithmetic is pinned to the numpy definition.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORA_REAL
#define ORA_REAL float
#endif
typedef ORA_REAL real;

#define ORA_OK 0
#define ORA_EINVAL (-1)
#define ORA_ESTATE (-2)
#define ORA_ENOMEM (-3)
#define ORA_ENAN (-4)

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn;
  int32_t vocab_text, vocab_speech;
  float rope_base, rms_eps;
  int32_t dtype;          /* 0: matrices are float, 1: matrices are bf16 bit patterns (uint16) */
  int32_t exit_layer;     /* e in [1, L] */
  int32_t period_k;       /* K >= 1 */
  int32_t phase;          /* slot of the full-depth position inside a period, in [0, K) */
  int32_t scope;          /* 0: period counter restarts at each speech chunk; 1: runs on */
  int32_t n_text, n_speech;
  int32_t max_seq_len;
  int32_t kv_round_bf16;  /* diagnostic: round cached K/V to bf16 precision when stored */
  /* the same periodic rule on text positions (Sec. V-C "Exploring Text Early Exit Policies",
   * Table II row G10): K_text <= 1 keeps every text position at full depth */
  int32_t text_period_k;
  int32_t text_phase;     /* in [0, K_text) */
} ora_config;

typedef struct {
  const void *embed;                 /* [V][d] */
  const float *attn_norm;            /* [L][d] */
  const void *wq, *wk, *wv, *wo;     /* [L][nq*hd][d], [L][nkv*hd][d] x2, [L][d][nq*hd] */
  const float *mlp_norm;             /* [L][d] */
  const void *wg, *wu, *wd;          /* [L][F][d] x2, [L][d][F] */
  const float *final_norm;           /* [d] */
  const void *lm_head;               /* [V][d] */
  const void *lens_a;                /* [d][d] */
  const float *lens_b, *lens_norm;   /* [d], [d] */
  const void *lens_head;             /* [V][d] */
} ora_weights;

typedef struct {
  ora_config c;
  ora_weights w;
  real *inv_freq; /* [hd/2] */
} ora_model;

typedef struct {
  ora_model *m;
  int cycle_offset;
  int len;          /* positions 0..len-1 have KV in layers 1..e (and an id in tokens[]) */
  int upper_valid;  /* positions 0..upper_valid-1 have KV in layers e+1..L */
  int g;            /* number of tokens emitted so far */
  int j_stream;     /* number of speech tokens emitted so far */
  int texts;        /* number of text tokens emitted so far */
  int run;          /* speech positions since the last text position (= index inside the chunk) */
  int text_budget;  /* > 0: after this many text tokens every position is speech */
  int speech_phase; /* the sequence's phase on speech positions (the configuration's unless moved) */
  int n_pending;    /* early-exited positions whose upper KV is deferred */
  real *pend_h;     /* [2K][d]: h^(e) of the pending positions, oldest first, then the current */
  int *pend_pos;    /* [2K] */
  int next_input, has_input;
  real **K, **V;    /* [L] -> [max_seq_len][nkv*hd] */
  int64_t n_text_steps, n_speech_full, n_speech_ee, n_text_ee;
  int64_t *flush_hist; /* [pend_cap]: how many full-depth steps processed m rows */
} ora_seq;

/* ------------------------------------------------------------------ element access */

static inline real bf16_widen(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (real)f;
}

static inline real round_to_bf16(real x) { /* round-to-nearest-even on the fp32 value */
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  memcpy(&f, &u, 4);
  return (real)f;
}

static inline real welem(const void *base, size_t i, int dtype) {
  return dtype ? bf16_widen(((const uint16_t *)base)[i]) : (real)((const float *)base)[i];
}

/* ------------------------------------------------------------------ primitives */

/* y[i] = sum_j W[i][j] x[j]; W is [n_out][n_in] row-major starting at element `off` of base */
static void matvec(const void *base, size_t off, int dtype, int n_out, int n_in, const real *x,
                   real *y) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < n_out; ++i) {
    real acc = 0;
    size_t row = off + (size_t)i * (size_t)n_in;
    for (int j = 0; j < n_in; ++j) acc += welem(base, row + j, dtype) * x[j];
    y[i] = acc;
  }
}

/* out = x / sqrt(mean(x^2) + eps) * gamma */
static void rmsnorm(const real *x, const float *gamma, int d, real eps, real *out) {
  real ss = 0;
  for (int i = 0; i < d; ++i) ss += x[i] * x[i];
  real inv = (real)1 / (real)sqrt((double)(ss / (real)d + eps));
  for (int i = 0; i < d; ++i) out[i] = x[i] * inv * (real)gamma[i];
}

/* rotary embedding on one head vector, pairs (i, i + hd/2), angle = pos * base^(-2i/hd) */
static void rope(real *v, int hd, int pos, const real *inv_freq) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    real ang = (real)pos * inv_freq[i];
    real c = (real)cos((double)ang), s = (real)sin((double)ang);
    real a = v[i], b = v[i + half];
    v[i] = a * c - b * s;
    v[i + half] = b * c + a * s;
  }
}

static inline real silu(real x) { return x / ((real)1 + (real)exp(-(double)x)); }

/* one query head over cached keys/values 0..n_ctx-1 of one kv head.
 * kcache/vcache: [.][stride] rows, head slice starts at column `col`. */
static void attend_head(const real *q, const real *kcache, const real *vcache, int stride, int col,
                        int hd, int n_ctx, real *scores, real *out) {
  real scale = (real)1 / (real)sqrt((double)hd);
  real mx = -INFINITY;
  for (int t = 0; t < n_ctx; ++t) {
    const real *k = kcache + (size_t)t * stride + col;
    real s = 0;
    for (int i = 0; i < hd; ++i) s += q[i] * k[i];
    s *= scale;
    scores[t] = s;
    if (s > mx) mx = s;
  }
  real den = 0;
  for (int t = 0; t < n_ctx; ++t) {
    scores[t] = (real)exp((double)(scores[t] - mx));
    den += scores[t];
  }
  for (int i = 0; i < hd; ++i) out[i] = 0;
  for (int t = 0; t < n_ctx; ++t) {
    const real *v = vcache + (size_t)t * stride + col;
    real p = scores[t] / den;
    for (int i = 0; i < hd; ++i) out[i] += p * v[i];
  }
}

/* argmax with lowest index winning ties; returns -1 if a NaN is met */
static int argmax_lowest(const real *x, int n) {
  int best = 0;
  for (int i = 0; i < n; ++i) {
    if (x[i] != x[i]) return -1;
    if (x[i] > x[best]) best = i;
  }
  return best;
}

/* ------------------------------------------------------------------ nucleus sampling */

/* Temperature / nucleus (top-p) sampling from a vector of logits (Sec. V-A "Models": Step-Audio-2
 * decodes with temperature 0.7 and top_p 0.9).  The paper fixes neither tie handling nor how the
 * random draw is mapped to a token; the definition used here makes both exact:
 *   w_i = exp((l_i - max l) / T);  q_i = floor(w_i * 2^32 + 1/2), at most 2^32 - 1  (integer masses)
 *   order: larger q first, lower index first among equal q
 *   nucleus: the shortest prefix of that order whose mass reaches ceil(top_p * sum q); M = its mass
 *   x = floor(omega * M / 2^64) for the 64-bit random word omega of the step
 *   token: the element of the prefix at which the running mass first exceeds x.
 * Returns the token (-1 on a NaN logit or bad parameters).  nucleus_out: size of the nucleus;
 * gap_out: how far, as a fraction of the total mass, the two decisions are from going the other
 * way -- the smaller of (a) the distance of x to the edges of the chosen element's interval and
 * (b) the distance of the nucleus' mass before and after its last element to the threshold. */
typedef struct { uint64_t q; int32_t idx; } ora_mass;
static int mass_order(const void *a, const void *b) {
  const ora_mass *x = a, *y = b;
  if (x->q != y->q) return x->q > y->q ? -1 : 1;
  return x->idx < y->idx ? -1 : (x->idx > y->idx);
}
int ora_sample(const double *logits, int V, double temperature, double top_p, uint64_t omega,
               int32_t *nucleus_out, double *gap_out) {
  if (V < 1 || !(temperature > 0.0) || !(top_p > 0.0) || top_p > 1.0) return -1;
  double mx = logits[0];
  for (int i = 0; i < V; ++i) {
    if (logits[i] != logits[i]) return -1;
    if (logits[i] > mx) mx = logits[i];
  }
  ora_mass *e = malloc((size_t)V * sizeof(*e));
  if (!e) return -1;
  uint64_t total = 0;
  for (int i = 0; i < V; ++i) {
    double w = exp((logits[i] - mx) / temperature);
    double scaled = floor(w * 4294967296.0 + 0.5);
    e[i].q = scaled >= 4294967295.0 ? 4294967295ull : (uint64_t)scaled;
    e[i].idx = i;
    total += e[i].q;
  }
  qsort(e, (size_t)V, sizeof(*e), mass_order);
  uint64_t target = (uint64_t)ceil(top_p * (double)total);
  if (target < 1) target = 1;
  if (target > total) target = total;
  uint64_t run = 0;
  int cut = 0;
  for (int i = 0; i < V; ++i) {
    run += e[i].q;
    if (run >= target) { cut = i; break; }
  }
  const uint64_t M = run;
  const uint64_t x = (uint64_t)(((__uint128_t)omega * M) >> 64);
  /* (with the whole vocabulary in the nucleus there is no cut that could move) */
  double gap = target == total ? 1.0
                               : fmin((double)(M - target), (double)(target - (M - e[cut].q))) / (double)total;
  run = 0;
  int tok = e[cut].idx;
  for (int i = 0; i <= cut; ++i) {
    if (run + e[i].q > x) {
      tok = e[i].idx;
      gap = fmin(gap, fmin((double)(x - run), (double)(run + e[i].q - 1 - x)) / (double)total);
      break;
    }
    run += e[i].q;
  }
  if (nucleus_out) *nucleus_out = cut + 1;
  if (gap_out) *gap_out = gap;
  free(e);
  return tok;
}

/* ------------------------------------------------------------------ model pieces */

static size_t lofs(const ora_model *m, int l, size_t rows, size_t cols) {
  (void)m;
  return (size_t)l * rows * cols;
}

/* q,k,v of one row at layer l from the normed input; rope at the row's own position; store K,V */
static void qkv_row(ora_seq *s, int l, const real *h, int pos, real *q /*[nq*hd]*/, real *n_buf) {
  const ora_model *m = s->m;
  const ora_config *c = &m->c;
  int d = c->d_model, hd = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads;
  int kvw = nkv * hd;
  rmsnorm(h, m->w.attn_norm + (size_t)l * d, d, (real)c->rms_eps, n_buf);
  real *k = s->K[l] + (size_t)pos * kvw, *v = s->V[l] + (size_t)pos * kvw;
  matvec(m->w.wq, lofs(m, l, (size_t)nq * hd, d), c->dtype, nq * hd, d, n_buf, q);
  matvec(m->w.wk, lofs(m, l, kvw, d), c->dtype, kvw, d, n_buf, k);
  matvec(m->w.wv, lofs(m, l, kvw, d), c->dtype, kvw, d, n_buf, v);
  for (int hq = 0; hq < nq; ++hq) rope(q + hq * hd, hd, pos, m->inv_freq);
  for (int hk = 0; hk < nkv; ++hk) rope(k + hk * hd, hd, pos, m->inv_freq);
  if (c->kv_round_bf16)
    for (int i = 0; i < kvw; ++i) {
      k[i] = round_to_bf16(k[i]);
      v[i] = round_to_bf16(v[i]);
    }
}

/* attention of one row (all query heads) over positions 0..pos, then h += Wo a */
static void attn_out_row(ora_seq *s, int l, const real *q, int pos, real *h, real *a_buf,
                         real *score_buf, real *o_buf) {
  const ora_model *m = s->m;
  const ora_config *c = &m->c;
  int d = c->d_model, hd = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads;
  int group = nq / nkv, kvw = nkv * hd;
  /* the query heads are independent of each other: one thread each, with its own score buffer
   * (score_buf holds max_seq_len entries per thread); the arithmetic of a head is unchanged */
#pragma omp parallel for schedule(static)
  for (int hq = 0; hq < nq; ++hq) {
    int hk = hq / group; /* grouped-query attention: consecutive query heads share a kv head */
    attend_head(q + hq * hd, s->K[l], s->V[l], kvw, hk * hd, hd, pos + 1,
                score_buf + (size_t)omp_get_thread_num() * c->max_seq_len, a_buf + hq * hd);
  }
  matvec(m->w.wo, lofs(m, l, d, (size_t)nq * hd), c->dtype, d, nq * hd, a_buf, o_buf);
  for (int i = 0; i < d; ++i) h[i] += o_buf[i];
}

/* h += Wd (silu(Wg n) * (Wu n)), n = RMSNorm(h; mlp_norm_l) */
static void mlp_row(const ora_model *m, int l, real *h, real *n_buf, real *g_buf, real *u_buf,
                    real *o_buf) {
  const ora_config *c = &m->c;
  int d = c->d_model, F = c->d_ffn;
  rmsnorm(h, m->w.mlp_norm + (size_t)l * d, d, (real)c->rms_eps, n_buf);
  matvec(m->w.wg, lofs(m, l, F, d), c->dtype, F, d, n_buf, g_buf);
  matvec(m->w.wu, lofs(m, l, F, d), c->dtype, F, d, n_buf, u_buf);
  for (int i = 0; i < F; ++i) g_buf[i] = silu(g_buf[i]) * u_buf[i];
  matvec(m->w.wd, lofs(m, l, d, F), c->dtype, d, F, g_buf, o_buf);
  for (int i = 0; i < d; ++i) h[i] += o_buf[i];
}

typedef struct {
  real *n, *q, *a, *o, *g, *u, *scores, *logits, *t;
} ora_tmp;

static int tmp_alloc(const ora_config *c, int rows, ora_tmp *t) {
  int d = c->d_model, qw = c->n_q_heads * c->head_dim;
  t->n = malloc(sizeof(real) * d);
  t->q = malloc(sizeof(real) * (size_t)qw * rows);
  t->a = malloc(sizeof(real) * qw);
  t->o = malloc(sizeof(real) * d);
  t->g = malloc(sizeof(real) * c->d_ffn);
  t->u = malloc(sizeof(real) * c->d_ffn);
  t->scores = malloc(sizeof(real) * (size_t)c->max_seq_len * (size_t)omp_get_max_threads());
  t->logits = malloc(sizeof(real) * (size_t)(c->vocab_text + c->vocab_speech));
  t->t = malloc(sizeof(real) * d);
  return (t->n && t->q && t->a && t->o && t->g && t->u && t->scores && t->logits && t->t) ? 0 : -1;
}
static void tmp_free(ora_tmp *t) {
  free(t->n); free(t->q); free(t->a); free(t->o); free(t->g); free(t->u);
  free(t->scores); free(t->logits); free(t->t);
}

/* one standard transformer block on one row: pre-norm attention + pre-norm SwiGLU MLP */
static void block_row(ora_seq *s, int l, real *h, int pos, ora_tmp *t) {
  qkv_row(s, l, h, pos, t->q, t->n);
  attn_out_row(s, l, t->q, pos, h, t->a, t->scores, t->o);
  mlp_row(s->m, l, h, t->n, t->g, t->u, t->o);
}

static void embed_row(const ora_model *m, int tok, real *h) {
  int d = m->c.d_model;
  for (int i = 0; i < d; ++i) h[i] = welem(m->w.embed, (size_t)tok * d + i, m->c.dtype);
}

/* final head g_L: logits = W_L RMSNorm(h; final_norm)   (Eq. 1) */
static void head_final(const ora_model *m, const real *h, ora_tmp *t) {
  const ora_config *c = &m->c;
  rmsnorm(h, m->w.final_norm, c->d_model, (real)c->rms_eps, t->n);
  matvec(m->w.lm_head, 0, c->dtype, c->vocab_text + c->vocab_speech, c->d_model, t->n, t->logits);
}

/* layer-specific head g_e: logits = W_e RMSNorm(h + A h + b; lens_norm)   (Eq. 2) */
static void head_lens(const ora_model *m, const real *h, ora_tmp *t) {
  const ora_config *c = &m->c;
  int d = c->d_model;
  matvec(m->w.lens_a, 0, c->dtype, d, d, h, t->o);
  for (int i = 0; i < d; ++i) t->t[i] = h[i] + t->o[i] + (real)m->w.lens_b[i];
  rmsnorm(t->t, m->w.lens_norm, d, (real)c->rms_eps, t->n);
  matvec(m->w.lens_head, 0, c->dtype, c->vocab_text + c->vocab_speech, d, t->n, t->logits);
}

/* ------------------------------------------------------------------ scheduler (Sec. IV-B.1) */

/* The schedule as a small state machine over the positions a sequence generates.  The
 * interleave pattern is a fixed cycle of n_text text slots followed by n_speech speech slots,
 * entered at cycle_offset.  A speech chunk is cut into periods of K slots; the slot with index
 * phase inside each period runs full depth, the other K-1 exit at layer e.  Text runs full depth,
 * unless a text period K_text > 1 is given: then text positions follow the same rule with
 * (K_text, text_phase), indexed inside their chunk (scope 0) or over all text positions so far
 * (scope 1).
 * The text of a response ends before its speech does (Sec. IV-A: speech is 79.5 % / 81.2 % of
 * the generated tokens, more than the 2/3 an interleave of 1:2 or 13:26 alone gives): with a text
 * budget B > 0, once B text tokens have been emitted every further position is speech, and the
 * chunk that is running then simply goes on (its index keeps counting). */
typedef struct {
  int g, j_stream, texts;
  int run; /* speech positions since the last text position */
} sched_state;

static void sched_start(const ora_config *c, int cycle_offset, sched_state *st) {
  int slot = cycle_offset % (c->n_text + c->n_speech);
  st->g = st->j_stream = st->texts = 0;
  st->run = slot >= c->n_text ? slot - c->n_text : 0;   /* entered inside a speech chunk */
}

/* modality and depth of the position about to be generated */
static void sched_decide(const ora_config *c, int cycle_offset, int text_budget, int speech_phase,
                         const sched_state *st, int *is_text, int *full) {
  int cyc = c->n_text + c->n_speech;
  int slot = (int)(((int64_t)st->g + cycle_offset) % cyc);
  int text_over = text_budget > 0 && st->texts >= text_budget;
  *is_text = slot < c->n_text && !text_over;
  if (c->exit_layer == c->n_layers) {
    *full = 1;
  } else if (*is_text) {
    int t = (c->scope == 0) ? slot : st->texts;
    *full = c->text_period_k <= 1 || (t % c->text_period_k == c->text_phase);
  } else {
    /* inside a chunk: the slot's place in it; after the text has ended the running chunk goes on */
    int j = (c->scope == 1) ? st->j_stream : (text_over ? st->run : slot - c->n_text);
    *full = c->period_k == 1 || (j % c->period_k == speech_phase);
  }
}

static void sched_advance(sched_state *st, int is_text) {
  st->g += 1;
  if (is_text) {
    st->texts += 1;
    st->run = 0;
  } else {
    st->j_stream += 1;
    st->run += 1;
  }
}

/* rows the pending buffer holds: between two full-depth steps at most K-1 speech positions exit
 * early inside a chunk; with no full-depth slot between them a chunk's tail (<= K-1) and the next
 * chunk's head (<= K-1) can join: 2K-1 rows with the current one.  Text periods add the same. */
static int pend_cap(const ora_config *c) {
  return 2 * c->period_k + (c->text_period_k > 1 ? 2 * c->text_period_k : 0);
}

static int config_ok(const ora_config *c) {
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return 0;
  if (c->n_q_heads % c->n_kv_heads) return 0;
  if (c->head_dim < 2 || (c->head_dim & 1) || c->d_ffn < 1) return 0;
  if (c->vocab_text < 0 || c->vocab_speech < 0 || c->vocab_text + c->vocab_speech < 1) return 0;
  if (c->exit_layer < 1 || c->exit_layer > c->n_layers) return 0;
  if (c->period_k < 1 || c->phase < 0 || c->phase >= c->period_k) return 0;
  if (c->scope != 0 && c->scope != 1) return 0;
  if (c->n_text < 0 || c->n_speech < 0 || c->n_text + c->n_speech < 1) return 0;
  if (c->dtype != 0 && c->dtype != 1) return 0;
  if (c->text_period_k < 0) return 0;
  if (c->text_period_k > 1 && (c->text_phase < 0 || c->text_phase >= c->text_period_k)) return 0;
  /* With counters that restart per chunk the pattern repeats with the cycle: a cycle without a
   * full-depth slot would never complete its KV, and the longest run of early exits must fit the
   * pending buffer.  (Counters over the stream reach every phase: runs hold at most K-1 speech
   * and K_text-1 text positions.) */
  if (c->scope == 0 && c->exit_layer < c->n_layers) {
    int cyc = c->n_text + c->n_speech, run = 0, longest = 0, any_full = 0;
    sched_state st;
    sched_start(c, 0, &st);
    for (int g = 0; g < 2 * cyc; ++g) {
      int is_text, full;
      sched_decide(c, 0, 0, c->phase, &st, &is_text, &full);
      sched_advance(&st, is_text);
      if (full) { any_full = 1; run = 0; } else if (++run > longest) longest = run;
    }
    if (!any_full || longest + 1 > pend_cap(c)) return 0;
  }
  return 1;
}

/* depth_out[i] = executed depth of generated token i, is_text_out[i] = its modality; no model.
 * text_budget <= 0: the text never ends. */
int ora_schedule_run_budget(const ora_config *c, int cycle_offset, int text_budget, int n_steps,
                            int32_t *depth_out, int32_t *is_text_out) {
  if (!config_ok(c) || cycle_offset < 0) return ORA_EINVAL;
  sched_state st;
  sched_start(c, cycle_offset, &st);
  for (int g = 0; g < n_steps; ++g) {
    int is_text, full;
    sched_decide(c, cycle_offset, text_budget, c->phase, &st, &is_text, &full);
    depth_out[g] = full ? c->n_layers : c->exit_layer;
    is_text_out[g] = is_text;
    sched_advance(&st, is_text);
  }
  return ORA_OK;
}

/* the same with the speech phase moved on the way: before generated token move_step[i] is decided
 * the phase becomes move_phase[i] (move_step ascending) */
int ora_schedule_run_moves(const ora_config *c, int cycle_offset, int text_budget, int n_steps, int n_moves,
                           const int32_t *move_step, const int32_t *move_phase, int32_t *depth_out,
                           int32_t *is_text_out) {
  if (!config_ok(c) || cycle_offset < 0 || (n_moves > 0 && c->text_period_k > 1)) return ORA_EINVAL;
  for (int i = 0; i < n_moves; ++i)
    if (move_phase[i] < 0 || move_phase[i] >= c->period_k) return ORA_EINVAL;
  sched_state st;
  sched_start(c, cycle_offset, &st);
  int phase = c->phase, next = 0;
  for (int g = 0; g < n_steps; ++g) {
    while (next < n_moves && move_step[next] <= g) phase = move_phase[next++];
    int is_text, full;
    sched_decide(c, cycle_offset, text_budget, phase, &st, &is_text, &full);
    depth_out[g] = full ? c->n_layers : c->exit_layer;
    is_text_out[g] = is_text;
    sched_advance(&st, is_text);
  }
  return ORA_OK;
}

int ora_schedule_run(const ora_config *c, int cycle_offset, int n_steps, int32_t *depth_out,
                     int32_t *is_text_out) {
  return ora_schedule_run_budget(c, cycle_offset, 0, n_steps, depth_out, is_text_out);
}

/* LayerSaving of Eq. 4, in percent, from logged depths */
double ora_layer_saving(const int32_t *depth, int n, int n_layers) {
  if (n <= 0) return 0.0;
  double sum = 0;
  for (int i = 0; i < n; ++i) sum += depth[i];
  return (1.0 - (sum / n) / n_layers) * 100.0;
}

/* ------------------------------------------------------------------ lifetime */

ora_model *ora_create(const ora_config *c, const ora_weights *w) {
  if (!config_ok(c) || c->max_seq_len < 1) return NULL;
  ora_model *m = calloc(1, sizeof(*m));
  if (!m) return NULL;
  m->c = *c;
  m->w = *w;
  int half = c->head_dim / 2;
  m->inv_freq = malloc(sizeof(real) * half);
  for (int i = 0; i < half; ++i)
    m->inv_freq[i] = (real)pow((double)c->rope_base, -2.0 * i / (double)c->head_dim);
  return m;
}

void ora_destroy(ora_model *m) {
  if (!m) return;
  free(m->inv_freq);
  free(m);
}

ora_seq *ora_seq_open(ora_model *m, int cycle_offset) {
  if (!m || cycle_offset < 0) return NULL;
  const ora_config *c = &m->c;
  ora_seq *s = calloc(1, sizeof(*s));
  if (!s) return NULL;
  s->m = m;
  s->cycle_offset = cycle_offset;
  s->speech_phase = c->phase;
  {
    sched_state st;
    sched_start(c, cycle_offset, &st);
    s->run = st.run;
  }
  size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
  s->K = calloc(c->n_layers, sizeof(real *));
  s->V = calloc(c->n_layers, sizeof(real *));
  for (int l = 0; l < c->n_layers; ++l) {
    s->K[l] = calloc((size_t)c->max_seq_len * kvw, sizeof(real));
    s->V[l] = calloc((size_t)c->max_seq_len * kvw, sizeof(real));
    if (!s->K[l] || !s->V[l]) return NULL;
  }
  s->pend_h = calloc((size_t)pend_cap(c) * c->d_model, sizeof(real));
  s->pend_pos = calloc((size_t)pend_cap(c), sizeof(int));
  s->flush_hist = calloc((size_t)pend_cap(c), sizeof(int64_t));
  return s;
}

void ora_seq_close(ora_seq *s) {
  if (!s) return;
  for (int l = 0; l < s->m->c.n_layers; ++l) {
    free(s->K[l]);
    free(s->V[l]);
  }
  free(s->K); free(s->V); free(s->pend_h); free(s->pend_pos); free(s->flush_hist);
  free(s);
}

/* ------------------------------------------------------------------ prefill */

/* The prompt is conditioned on at full depth: positions 0..n-2 get KV in every layer; the last
 * prompt token is held back as the input of the first decoding step. */
int ora_prefill(ora_seq *s, const int32_t *prompt, int n) {
  const ora_config *c = &s->m->c;
  int V = c->vocab_text + c->vocab_speech;
  if (s->has_input || s->len) return ORA_ESTATE;
  if (n < 1 || n > c->max_seq_len) return ORA_EINVAL;
  for (int i = 0; i < n; ++i)
    if (prompt[i] < 0 || prompt[i] >= V) return ORA_EINVAL;
  ora_tmp t;
  if (tmp_alloc(c, 1, &t)) return ORA_ENOMEM;
  real *h = malloc(sizeof(real) * c->d_model);
  for (int p = 0; p < n - 1; ++p) {
    embed_row(s->m, prompt[p], h);
    for (int l = 0; l < c->n_layers; ++l) block_row(s, l, h, p, &t);
  }
  s->len = s->upper_valid = n - 1;
  s->next_input = prompt[n - 1];
  s->has_input = 1;
  free(h);
  tmp_free(&t);
  return ORA_OK;
}

static void copy_out(const real *src, double *dst, int n) {
  if (dst)
    for (int i = 0; i < n; ++i) dst[i] = (double)src[i];
}

/* ------------------------------------------------------------------ standard decoding (Eq. 1) */

/* One full-depth step with a KV cache.  Optionally reports the residual stream after layer
 * capture_layer (1-based) of the processed position. */
int ora_step_standard(ora_seq *s, int forced_next, int32_t *tok_out, double *logits_out,
                      int capture_layer, double *h_capture) {
  const ora_config *c = &s->m->c;
  int V = c->vocab_text + c->vocab_speech, d = c->d_model;
  if (!s->has_input || s->n_pending) return ORA_ESTATE;
  if (s->len >= c->max_seq_len) return ORA_ENOMEM;
  if (forced_next >= V) return ORA_EINVAL;
  ora_tmp t;
  if (tmp_alloc(c, 1, &t)) return ORA_ENOMEM;
  real *h = malloc(sizeof(real) * d);
  int pos = s->len;
  embed_row(s->m, s->next_input, h);
  for (int l = 0; l < c->n_layers; ++l) {
    block_row(s, l, h, pos, &t);
    if (l + 1 == capture_layer) copy_out(h, h_capture, d);
  }
  head_final(s->m, h, &t);
  int y = argmax_lowest(t.logits, V);
  copy_out(t.logits, logits_out, V);
  free(h);
  tmp_free(&t);
  if (y < 0) return ORA_ENAN;
  s->len = s->upper_valid = pos + 1;
  s->g += 1;
  *tok_out = y;
  s->next_input = forced_next >= 0 ? forced_next : y;
  return ORA_OK;
}

/* ------------------------------------------------------------------ SPAR-K decoding (Alg. 1) */

/* One decoding step under the schedule.  tok_out: emitted token; depth_out: e or L;
 * logits_out (nullable, [V]): logits of the head that produced the token. */
int ora_step(ora_seq *s, int forced_next, int32_t *tok_out, int32_t *depth_out,
             double *logits_out) {
  ora_model *m = s->m;
  const ora_config *c = &m->c;
  int V = c->vocab_text + c->vocab_speech, d = c->d_model, L = c->n_layers, e = c->exit_layer;
  int qw = c->n_q_heads * c->head_dim;
  if (!s->has_input) return ORA_ESTATE;
  if (s->len >= c->max_seq_len) return ORA_ENOMEM;
  if (forced_next >= V) return ORA_EINVAL;

  int is_text, full;
  sched_state st = {s->g, s->j_stream, s->texts, s->run};
  sched_decide(c, s->cycle_offset, s->text_budget, s->speech_phase, &st, &is_text, &full);

  ora_tmp t;
  if (tmp_alloc(c, pend_cap(c), &t)) return ORA_ENOMEM;
  int pos = s->len;
  /* the current position's hidden state lives in the slot after the pending ones */
  real *h = s->pend_h + (size_t)s->n_pending * d;
  s->pend_pos[s->n_pending] = pos;

  /* run layers 1..e on the new position; cache lower KV; h now holds h^(e) */
  embed_row(m, s->next_input, h);
  for (int l = 0; l < e; ++l) block_row(s, l, h, pos, &t);
  s->len = pos + 1;

  int y;
  if (!full) {
    /* early exit: predict from h^(e) with g_e, keep h^(e), defer the upper KV */
    head_lens(m, h, &t);
    y = argmax_lowest(t.logits, V);
    s->n_pending += 1;
    *depth_out = e;
    if (is_text) s->n_text_ee += 1; else s->n_speech_ee += 1;
  } else {
    /* full depth: pending positions and the current one go through layers e+1..L together;
     * each row keeps its own position, attention is causal inside the batch because row r only
     * reads cache entries 0..pos_r, all of which are written before any row attends. */
    int rows = s->n_pending + 1;
    for (int l = e; l < L; ++l) {
      for (int r = 0; r < rows; ++r)
        qkv_row(s, l, s->pend_h + (size_t)r * d, s->pend_pos[r], t.q + (size_t)r * qw, t.n);
      for (int r = 0; r < rows; ++r)
        attn_out_row(s, l, t.q + (size_t)r * qw, s->pend_pos[r], s->pend_h + (size_t)r * d, t.a,
                     t.scores, t.o);
      for (int r = 0; r < rows; ++r)
        mlp_row(m, l, s->pend_h + (size_t)r * d, t.n, t.g, t.u, t.o);
    }
    /* only the current position is decoded; the pending rows keep their early-exit tokens */
    head_final(m, s->pend_h + (size_t)(rows - 1) * d, &t);
    y = argmax_lowest(t.logits, V);
    s->flush_hist[rows] += 1;
    s->n_pending = 0;
    s->upper_valid = pos + 1;
    *depth_out = L;
    if (is_text) s->n_text_steps += 1; else s->n_speech_full += 1;
  }
  copy_out(t.logits, logits_out, V);
  tmp_free(&t);
  if (y < 0) return ORA_ENAN;
  sched_advance(&st, is_text);
  s->g = st.g;
  s->j_stream = st.j_stream;
  s->texts = st.texts;
  s->run = st.run;
  *tok_out = y;
  s->next_input = forced_next >= 0 ? forced_next : y;
  return ORA_OK;
}

/* ------------------------------------------------------------------ inspection */

/* After `budget` text tokens in all, the sequence generates speech only.  To be set once, and not
 * below the number of text tokens already generated. */
int ora_seq_text_budget(ora_seq *s, int budget) {
  if (!s || budget < 1 || s->text_budget > 0 || budget < s->texts) return ORA_EINVAL;
  s->text_budget = budget;
  return ORA_OK;
}

/* The phase on speech positions is free (Table II's Even / Odd / Triple variants): a caller may
 * move it for a sequence's future positions, e.g. to line up the full-depth steps of a batch.
 * Not with early exits on text positions (the joined runs of early exits would outgrow the
 * pending buffer). */
int ora_seq_set_phase(ora_seq *s, int phase) {
  if (!s || phase < 0 || phase >= s->m->c.period_k || s->m->c.text_period_k > 1) return ORA_EINVAL;
  s->speech_phase = phase;
  return ORA_OK;
}

int ora_seq_j_stream(const ora_seq *s) { return s->j_stream; }

int ora_seq_len(const ora_seq *s) { return s->len; }
int ora_seq_upper_valid(const ora_seq *s) { return s->upper_valid; }
int ora_seq_pending(const ora_seq *s) { return s->n_pending; }

/* stats: [0] full-depth text steps, [1] full-depth speech steps, [2] early-exit speech steps,
 * then flush_hist[1..pend_cap-1], then [2 + pend_cap] early-exit text steps */
void ora_seq_stats(const ora_seq *s, int64_t *out) {
  const int cap = pend_cap(&s->m->c);
  out[0] = s->n_text_steps;
  out[1] = s->n_speech_full;
  out[2] = s->n_speech_ee;
  for (int i = 1; i < cap; ++i) out[2 + i] = s->flush_hist[i];
  out[2 + cap] = s->n_text_ee;
}
int ora_pend_cap(const ora_config *c) { return pend_cap(c); }

int ora_get_kv(const ora_seq *s, int layer /*0-based*/, int pos, double *k_out, double *v_out) {
  const ora_config *c = &s->m->c;
  if (layer < 0 || layer >= c->n_layers || pos < 0 || pos >= c->max_seq_len) return ORA_EINVAL;
  int kvw = c->n_kv_heads * c->head_dim;
  copy_out(s->K[layer] + (size_t)pos * kvw, k_out, kvw);
  copy_out(s->V[layer] + (size_t)pos * kvw, v_out, kvw);
  return ORA_OK;
}

/* logits of g_e on an arbitrary hidden state */
int ora_lens_logits(ora_model *m, const double *h_in, double *logits_out) {
  const ora_config *c = &m->c;
  ora_tmp t;
  if (tmp_alloc(c, 1, &t)) return ORA_ENOMEM;
  real *h = malloc(sizeof(real) * c->d_model);
  for (int i = 0; i < c->d_model; ++i) h[i] = (real)h_in[i];
  head_lens(m, h, &t);
  copy_out(t.logits, logits_out, c->vocab_text + c->vocab_speech);
  free(h);
  tmp_free(&t);
  return ORA_OK;
}

int ora_real_bytes(void) { return (int)sizeof(real); }

/* threads the row loops of matvec run on */
int ora_num_threads(void) {
  int n = 1;
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
  return n;
}

/* ------------------------------------------------------------------ primitive probes (for pins) */

void ora_prim_matvec(const void *w, int dtype, int n_out, int n_in, const double *x, double *y) {
  real *xr = malloc(sizeof(real) * n_in), *yr = malloc(sizeof(real) * n_out);
  for (int i = 0; i < n_in; ++i) xr[i] = (real)x[i];
  matvec(w, 0, dtype, n_out, n_in, xr, yr);
  copy_out(yr, y, n_out);
  free(xr); free(yr);
}

void ora_prim_rmsnorm(const double *x, const float *gamma, int d, double eps, double *out) {
  real *xr = calloc(d, sizeof(real)), *yr = calloc(d, sizeof(real));
  for (int i = 0; i < d; ++i) xr[i] = (real)x[i];
  rmsnorm(xr, gamma, d, (real)eps, yr);
  copy_out(yr, out, d);
  free(xr); free(yr);
}

void ora_prim_rope(double *v, int hd, int pos, double base) {
  int half = hd / 2;
  real *f = calloc(half, sizeof(real)), *vr = calloc(hd, sizeof(real));
  for (int i = 0; i < half; ++i) f[i] = (real)pow(base, -2.0 * i / (double)hd);
  for (int i = 0; i < hd; ++i) vr[i] = (real)v[i];
  rope(vr, hd, pos, f);
  copy_out(vr, v, hd);
  free(f); free(vr);
}

double ora_prim_silu(double x) { return (double)silu((real)x); }

/* q: [hd]; k, v: [n_ctx][hd] */
void ora_prim_attend(const double *q, const double *k, const double *v, int hd, int n_ctx,
                     double *out) {
  real *qr = malloc(sizeof(real) * hd), *kr = malloc(sizeof(real) * hd * n_ctx);
  real *vr = malloc(sizeof(real) * hd * n_ctx), *sc = malloc(sizeof(real) * n_ctx);
  real *o = malloc(sizeof(real) * hd);
  for (int i = 0; i < hd; ++i) qr[i] = (real)q[i];
  for (int i = 0; i < hd * n_ctx; ++i) { kr[i] = (real)k[i]; vr[i] = (real)v[i]; }
  attend_head(qr, kr, vr, hd, 0, hd, n_ctx, sc, o);
  copy_out(o, out, hd);
  free(qr); free(kr); free(vr); free(sc); free(o);
}

int ora_prim_argmax(const double *x, int n) {
  real *xr = malloc(sizeof(real) * n);
  for (int i = 0; i < n; ++i) xr[i] = (real)x[i];
  int r = argmax_lowest(xr, n);
  free(xr);
  return r;
}

double ora_prim_bf16_round(double x) { return (double)round_to_bf16((real)x); }
