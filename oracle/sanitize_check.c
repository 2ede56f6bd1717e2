/*
 * sanitize_check.c -- runs every entry point of the CPU oracle on a tiny model, for a build with
 * -fsanitize=address,undefined (oracle/build_oracle.py, build_sanitized).  TEST INFRASTRUCTURE ONLY.
 *
 * The oracle's source is included as it is, so the instrumented code is the code the tests use.
 * Exit status 0 and no sanitizer report: no out-of-bounds access, use after free, leak, signed
 * overflow or misaligned access on the paths below (both element types, chunk and stream scope,
 * early exits on text positions, a text budget, a moved phase, the sampler, the primitive probes).
 */
#include "spark_oracle.c"

#include <stdio.h>

static uint32_t lcg_state = 12345u;
static float lcg_unit(void) { /* uniform in [-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(lcg_state >> 8) / 8388608.0f - 1.0f;
}

static uint16_t to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static void *matrix(size_t n, int dtype, float scale) {
  if (dtype) {
    uint16_t *p = malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = to_bf16(lcg_unit() * scale);
    return p;
  }
  float *p = malloc(n * sizeof(float));
  for (size_t i = 0; i < n; ++i) p[i] = lcg_unit() * scale;
  return p;
}

static float *gains(size_t n) {
  float *p = malloc(n * sizeof(float));
  for (size_t i = 0; i < n; ++i) p[i] = 1.0f + 0.1f * lcg_unit();
  return p;
}

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "sanitize_check: %s failed at line %d\n", #cond, __LINE__); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static int run_model(int dtype, int scope, int K, int phase, int n_text, int n_speech, int e,
                     int text_period, int kv_round) {
  ora_config c;
  memset(&c, 0, sizeof(c));
  c.n_layers = 3; c.d_model = 32; c.n_q_heads = 4; c.n_kv_heads = 2; c.head_dim = 8; c.d_ffn = 48;
  c.vocab_text = 24; c.vocab_speech = 16;
  c.rope_base = 10000.0f; c.rms_eps = 1e-6f;
  c.dtype = dtype; c.exit_layer = e; c.period_k = K; c.phase = phase; c.scope = scope;
  c.n_text = n_text; c.n_speech = n_speech; c.max_seq_len = 48; c.kv_round_bf16 = kv_round;
  c.text_period_k = text_period; c.text_phase = 0;
  const int L = c.n_layers, d = c.d_model, F = c.d_ffn, V = c.vocab_text + c.vocab_speech;
  const int qw = c.n_q_heads * c.head_dim, kvw = c.n_kv_heads * c.head_dim;
  ora_weights w;
  void *mats[12];
  float *gs[5];
  mats[0] = matrix((size_t)V * d, dtype, 0.5f);          w.embed = mats[0];
  mats[1] = matrix((size_t)L * qw * d, dtype, 0.2f);     w.wq = mats[1];
  mats[2] = matrix((size_t)L * kvw * d, dtype, 0.2f);    w.wk = mats[2];
  mats[3] = matrix((size_t)L * kvw * d, dtype, 0.2f);    w.wv = mats[3];
  mats[4] = matrix((size_t)L * d * qw, dtype, 0.2f);     w.wo = mats[4];
  mats[5] = matrix((size_t)L * F * d, dtype, 0.2f);      w.wg = mats[5];
  mats[6] = matrix((size_t)L * F * d, dtype, 0.2f);      w.wu = mats[6];
  mats[7] = matrix((size_t)L * d * F, dtype, 0.2f);      w.wd = mats[7];
  mats[8] = matrix((size_t)V * d, dtype, 0.3f);          w.lm_head = mats[8];
  mats[9] = matrix((size_t)d * d, dtype, 0.1f);          w.lens_a = mats[9];
  mats[10] = matrix((size_t)V * d, dtype, 0.3f);         w.lens_head = mats[10];
  mats[11] = matrix((size_t)d, 0, 0.1f);                 w.lens_b = mats[11];
  gs[0] = gains((size_t)L * d); w.attn_norm = gs[0];
  gs[1] = gains((size_t)L * d); w.mlp_norm = gs[1];
  gs[2] = gains(d);             w.final_norm = gs[2];
  gs[3] = gains(d);             w.lens_norm = gs[3];
  gs[4] = NULL;

  ora_model *m = ora_create(&c, &w);
  CHECK(m != NULL);
  int32_t prompt[6] = {1, 30, 7, 25, 39, 0};
  double *logits = malloc(sizeof(double) * V), *kbuf = malloc(sizeof(double) * kvw),
         *vbuf = malloc(sizeof(double) * kvw), *hbuf = malloc(sizeof(double) * d);

  /* SPAR-K decoding, free running and teacher forced, a text budget and a moved phase on the way */
  ora_seq *s = ora_seq_open(m, 1);
  CHECK(s != NULL);
  CHECK(ora_prefill(s, prompt, 6) == ORA_OK);
  CHECK(ora_prefill(s, prompt, 6) == ORA_ESTATE);
  for (int i = 0; i < 40; ++i) {
    int32_t tok = -1, depth = -1;
    if (i == 9 && n_text > 0) CHECK(ora_seq_text_budget(s, 8) == ORA_OK);
    if (i == 14 && text_period <= 1) CHECK(ora_seq_set_phase(s, (phase + 1) % K) == ORA_OK);
    int rc = ora_step(s, (i % 3) ? -1 : (i * 7) % V, &tok, &depth, (i & 1) ? logits : NULL);
    CHECK(rc == ORA_OK);
    CHECK(tok >= 0 && tok < V && (depth == e || depth == L));
    CHECK(ora_seq_upper_valid(s) + ora_seq_pending(s) == ora_seq_len(s));
    CHECK(ora_get_kv(s, L - 1, ora_seq_len(s) - 1, kbuf, vbuf) == ORA_OK);
  }
  {
    int32_t tok, depth;
    CHECK(ora_seq_len(s) == 45);
    for (int i = 0; i < 3; ++i) CHECK(ora_step(s, -1, &tok, &depth, NULL) == ORA_OK);
    CHECK(ora_step(s, -1, &tok, &depth, NULL) == ORA_ENOMEM);   /* max_seq_len reached */
  }
  int64_t *stats = calloc((size_t)3 + ora_pend_cap(&c), sizeof(int64_t));
  ora_seq_stats(s, stats);
  CHECK(stats[0] + stats[1] + stats[2] + stats[2 + ora_pend_cap(&c)] == 43);
  CHECK(ora_seq_j_stream(s) >= 0);
  ora_seq_close(s);

  /* standard decoding with a captured hidden state, then the layer-specific head on it */
  s = ora_seq_open(m, 0);
  CHECK(s != NULL && ora_prefill(s, prompt, 3) == ORA_OK);
  for (int i = 0; i < 5; ++i) {
    int32_t tok = -1;
    CHECK(ora_step_standard(s, -1, &tok, logits, e, hbuf) == ORA_OK);
    CHECK(ora_lens_logits(m, hbuf, logits) == ORA_OK);
  }
  ora_seq_close(s);

  /* the scheduler alone */
  int32_t depth[64], is_text[64], mstep[2] = {5, 17}, mphase[2] = {0, 0};
  mphase[1] = K - 1;
  CHECK(ora_schedule_run(&c, 2, 64, depth, is_text) == ORA_OK);
  CHECK(ora_schedule_run_budget(&c, 0, n_text > 0 ? 3 : 0, 64, depth, is_text) == ORA_OK);
  if (text_period <= 1)
    CHECK(ora_schedule_run_moves(&c, 1, 0, 64, 2, mstep, mphase, depth, is_text) == ORA_OK);
  double saving = ora_layer_saving(depth, 64, L);
  CHECK(saving >= 0.0 && saving <= 100.0);

  /* sampler and primitive probes */
  for (int i = 0; i < V; ++i) logits[i] = (double)lcg_unit() * 3.0;
  int32_t nucleus = 0;
  double gap = 0;
  int tok = ora_sample(logits, V, 0.7, 0.9, 0x9e3779b97f4a7c15ull, &nucleus, &gap);
  CHECK(tok >= 0 && tok < V && nucleus >= 1 && nucleus <= V);
  CHECK(ora_sample(logits, V, 0.0, 0.9, 1ull, NULL, NULL) == -1);
  double x[32], y[32], q[8], kk[5 * 8], vv[5 * 8], o[8];
  for (int i = 0; i < 32; ++i) x[i] = lcg_unit();
  for (int i = 0; i < 8; ++i) q[i] = lcg_unit();
  for (int i = 0; i < 40; ++i) { kk[i] = lcg_unit(); vv[i] = lcg_unit(); }
  ora_prim_matvec(mats[9], dtype, d, d, x, y);
  ora_prim_rmsnorm(x, gs[2], d, 1e-6, y);
  ora_prim_rope(x, 8, 11, 10000.0);
  ora_prim_attend(q, kk, vv, 8, 5, o);
  CHECK(ora_prim_argmax(x, 32) >= 0);
  CHECK(ora_prim_silu(0.0) == 0.0 && ora_prim_bf16_round(1.0) == 1.0);
  CHECK(ora_real_bytes() == (int)sizeof(real) && ora_num_threads() >= 1);

  free(stats); free(logits); free(kbuf); free(vbuf); free(hbuf);
  ora_destroy(m);
  for (int i = 0; i < 12; ++i) free(mats[i]);
  for (int i = 0; i < 4; ++i) free(gs[i]);
  return 0;
}

int main(void) {
  int bad = 0;
  /* dtype, scope, K, phase, n_text, n_speech, e, K_text, kv rounding */
  bad |= run_model(0, 0, 4, 3, 2, 4, 2, 0, 0);   /* per-chunk counter, K divides the chunk */
  bad |= run_model(1, 1, 4, 3, 1, 2, 2, 0, 1);   /* stream counter, chunk shorter than the period */
  bad |= run_model(1, 0, 3, 0, 1, 4, 1, 0, 1);   /* Triple on a 4-slot chunk: truncated last period */
  bad |= run_model(0, 1, 2, 1, 3, 5, 2, 2, 0);   /* early exits on text positions too */
  bad |= run_model(1, 1, 1, 0, 1, 2, 2, 0, 1);   /* K = 1: every position full depth */
  bad |= run_model(0, 1, 4, 0, 1, 2, 3, 0, 0);   /* e = L */
  if (bad) return 1;
  printf("sanitize_check: ok\n");
  return 0;
}
