// Host side of the SPAR-K decoding library: context, sequence bookkeeping, kernel launches and
// the C ABI declared in include/spark.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>
#include <map>
#include <new>
#include <string>
#include <vector>

#include "../../include/spark.h"
#include "attention.h"
#include "device_common.h"
#include "gemv.h"
#include "measure.h"
#include "mfma_gemm.h"
#include "sampling.h"
#include "sched.h"

using namespace spark;

namespace {

constexpr int PREFILL_CHUNK = 256;   // most prompt rows pushed through the layers together (buffers are sized for it)
constexpr size_t MFMA_PARTIAL_BYTES = 48u << 20;  // k-split partial sums of one projection
constexpr int MAX_STEPS_PER_CALL = 256;
// rows from which the MFMA projections run: up to four rows are one pass of the vector kernel
// (measured at four rows: level at the GLM shape, 14-20 % faster for a batch of four at the Step
// shape); five rows would be two such passes
constexpr int MFMA_MIN_ROWS = 5;
constexpr int MAX_SEQ_LEN = 16384;

struct Layout {  // byte offsets into the scratch buffer
  size_t state, page_table, plan, lower, upper, ee, full, prefill_rows, prefill_tokens, seq_ids,
      forced, step_flags, out_tokens, out_depth, best, arrivals, row_ssq, sample_hist, sample_arrive, sample_count, hidden, xsplit, xsplit2, mfma_part, sample_q, sample_cand, rand_words, qbuf, attn_out, part, act, lens_u,
      logits, rope, inv_freq, total,
      tiled, total_tiled;   // the MFMA-ordered copy of the projection weights lies behind everything else (absent on the static area)
};

struct Derived {
  int V, rmax, max_rows, max_pages, n_pages_total, slice, n_splits, group, esz;
  size_t page_elems, kv_pool_bytes;
};

// Where the MFMA-ordered copies of the projection matrices lie (element offsets from the start of
// the tiled region; per layer for the four projections of a layer).
struct TiledMap {
  std::vector<size_t> qkv, o, gateup, down;
  size_t lens_a = 0, lens_head = 0, lm_head = 0, total = 0;
};

struct Seq {
  bool open = false, prefilled = false;
  int cycle_offset = 0, len = 0, g = 0, j_stream = 0, n_pending = 0, last_full = 0;
  int text_budget = 0;   // > 0: speech only after this many text tokens
  int phase = 0;         // the sequence's phase on speech positions (the configuration's, unless moved)
  std::vector<int> pages;
  int64_t text_steps = 0, speech_full = 0, speech_ee = 0, text_ee = 0;
  int64_t flush_rows[2 * SPARK_MAX_PERIOD] = {0};
};

}  // namespace

struct spark_ctx {
  spark_config cfg;
  spark_weights w;
  Derived dv;
  Layout lo;
  TiledMap tm;
  SchedParams sp;
  hipStream_t stream;
  char *scratch;
  void *kv_pool;
  int n_cu;
  std::vector<Seq> seqs;
  std::vector<int> free_pages;
  int *h_in;   // pinned: seq_ids[max_batch] + forced[MAX_STEPS][max_batch]
  int *h_out;  // pinned: tokens[MAX_STEPS][max_batch] + depth[...] + plan[PL_WORDS]
  char err[512];
  // kernel selection; the defaults are the measured choices, spark_tune moves them (tests, sweeps)
  bool mfma_ok = true;         // the shape allows the MFMA projections (16-byte vectors of 8 weights)
  bool use_mfma = true;        // "mfma" = 0 keeps every row count on the vector kernels
  int mfma_xcd_max_split = 4;  // row tiles share an XCD when k has at most this many ranges
  int mfma_small_tiles = 32;   // launches with fewer 8-wave tiles use 4-wave workgroups
  int mfma_min_rows = MFMA_MIN_ROWS;
  int attn_pieces = 0;         // 64-token pieces per attention workgroup (0: by the launch's size)
  int gemv_big_kb = 40;        // vector-kernel launches with more LDS per workgroup run eight waves per workgroup
  int attn_mfma_min_rows = 1;  // passes with at least this many rows run attention on the MFMA units (where the shape allows)
  int mfma_small_max_k = 32768;  // ... and an input width of at most this
  bool has_tiled = false;      // the context owns the MFMA-ordered copy of the projection weights
  bool use_tiled = true;       // "mfma_tiled" = 0 keeps the MFMA projections on the kernel that stages weights through LDS
  bool fuse_norm = true;       // the residual projections' finishing launches prepare the next norm's input (no separate launch)
  bool static_scratch = false; // the scratch area is the library's static device array (spark_init_static)
  int device = 0;
  float temperature = 0.f, top_p = 0.f;   // nucleus sampling, off while temperature <= 0
  int prefill_chunk = 128;   // prompt rows per pass, see spark_init
  int attn_splits_now = 0;   // context slices the rows of the passes being enqueued can reach (0: unknown, launch all)
  std::map<std::pair<const void *, size_t>, int> occ_cache;  // workgroups per CU of a (kernel, LDS bytes)
  // profiling of one kernel class
  int prof_class = -1;
  std::vector<hipEvent_t> prof_ev;
  size_t prof_used = 0;
};

namespace {

int fail(spark_ctx *c, int code, const char *fmt, ...) {
  if (c) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

#define HIP_TRY(ctx, call)                                                                  \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(ctx, SPARK_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),  \
                  __FILE__, __LINE__);                                                      \
  } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// hidden-state slots per sequence: between two full-depth steps at most K-1 speech positions exit
// early inside a chunk; a chunk's tail and the next chunk's head can join when nothing between them
// runs full depth: 2K-1 rows with the current one.  A text period adds the same.
int pending_slots(const spark_config *c) {
  return 2 * c->period_k + (c->text_period_k > 1 ? 2 * c->text_period_k : 0);
}

SchedParams sched_params(const spark_config *c) {
  return SchedParams{c->n_layers, c->exit_layer, c->period_k, c->phase, c->scope, c->n_text,
                     c->n_speech, pending_slots(c), c->text_period_k, c->text_phase};
}

bool config_ok(const spark_config *c, char *why, size_t n) {
#define BAD(cond, msg) if (cond) { snprintf(why, n, "%s", msg); return false; }
  BAD(c->size != sizeof(spark_config), "spark_config.size does not match this library");
  BAD(c->n_layers < 1, "n_layers < 1");
  BAD(c->d_model < 8 || c->d_model % 8, "d_model must be a positive multiple of 8");
  BAD(c->d_model > 4096, "d_model > 4096 is not supported");
  BAD(c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads,
      "n_q_heads must be a positive multiple of n_kv_heads");
  {
    int grp = c->n_q_heads / c->n_kv_heads;
    BAD(grp != 1 && grp != 2 && grp != 4 && grp != 7 && grp != 8 && grp != 16,
        "query heads per KV head must be one of 1, 2, 4, 7, 8, 16");
  }
  BAD(c->head_dim != 64 && c->head_dim != 128, "head_dim must be 64 or 128");
  BAD(c->d_ffn < 8 || c->d_ffn % 8, "d_ffn must be a positive multiple of 8");
  BAD(c->vocab_text < 0 || c->vocab_speech < 0 || c->vocab_text + c->vocab_speech < 1,
      "empty vocabulary");
  BAD(c->dtype != SPARK_DTYPE_FP32 && c->dtype != SPARK_DTYPE_BF16, "unknown dtype");
  BAD(c->exit_layer < 1 || c->exit_layer > c->n_layers, "exit_layer outside [1, n_layers]");
  BAD(c->period_k < 1 || c->period_k > SPARK_MAX_PERIOD, "period_k outside [1, 16]");
  BAD(c->phase < 0 || c->phase >= c->period_k, "phase outside [0, period_k)");
  BAD(c->scope != SPARK_SCOPE_CHUNK && c->scope != SPARK_SCOPE_STREAM, "unknown scope");
  BAD(c->n_text < 0 || c->n_speech < 0 || c->n_text + c->n_speech < 1, "empty interleave cycle");
  BAD(c->text_period_k < 0 || c->text_period_k > SPARK_MAX_PERIOD, "text_period_k outside [0, 16]");
  BAD(c->text_period_k > 1 && (c->text_phase < 0 || c->text_phase >= c->text_period_k),
      "text_phase outside [0, text_period_k)");
  BAD(pending_slots(c) > 2 * SPARK_MAX_PERIOD, "period_k + text_period_k > 16: too many pending rows");
  if (c->scope == SPARK_SCOPE_CHUNK && c->exit_layer < c->n_layers) {
    // the pattern repeats with the cycle: it needs a full-depth slot, and its longest run of early
    // exits (which may wrap around the cycle and cross modalities) must fit the pending slots
    const SchedParams sp = sched_params(c);
    const int cyc = c->n_text + c->n_speech;
    int run = 0, longest = 0;
    bool any_full = false;
    for (int g = 0; g < 2 * cyc; ++g) {
      int is_text, full;
      schedule_decide(sp, g, 0, 0, 0, sp.phase, is_text, full);
      if (full) { any_full = true; run = 0; } else { longest = std::max(longest, ++run); }
    }
    BAD(!any_full, "a cycle without a full-depth slot would never complete its KV");
    BAD(longest + 1 > pending_slots(c), "a run of early exits is longer than the pending slots");
  }
  BAD(c->max_batch < 1 || c->max_batch > SCHED_THREADS, "max_batch outside [1, 256]");
  BAD(c->max_seq_len < 1 || c->max_seq_len > MAX_SEQ_LEN, "max_seq_len outside [1, 16384]");
  BAD(c->kv_page_tokens < 16 || c->kv_page_tokens % 16, "kv_page_tokens must be a multiple of 16");
#undef BAD
  return true;
}

void derive(const spark_config &c, Derived &d) {
  d.V = c.vocab_text + c.vocab_speech;
  d.rmax = pending_slots(&c);
  d.max_rows = std::max(c.max_batch * d.rmax, PREFILL_CHUNK);
  d.max_pages = (c.max_seq_len + c.kv_page_tokens - 1) / c.kv_page_tokens;
  d.n_pages_total = d.max_pages * c.max_batch;
  d.slice = ATTN_SLICE;
  d.n_splits = (c.max_seq_len + d.slice - 1) / d.slice;
  d.group = c.n_q_heads / c.n_kv_heads;
  d.esz = c.dtype == SPARK_DTYPE_BF16 ? 2 : 4;
  d.page_elems = (size_t)c.n_layers * 2 * c.n_kv_heads * c.kv_page_tokens * c.head_dim;
  d.kv_pool_bytes = d.page_elems * d.esz * d.n_pages_total;
}

// the MFMA kernels load 16-byte vectors of 8 weights; other widths stay on the vector kernel
bool shape_allows_mfma(const spark_config &c) {
  return c.dtype == SPARK_DTYPE_BF16 && c.d_model % 8 == 0 && (c.n_q_heads * c.head_dim) % 8 == 0 && c.d_ffn % 8 == 0;
}

void tiled_map(const spark_config &c, const Derived &d, TiledMap &tm) {
  tm = TiledMap();
  if (!shape_allows_mfma(c)) return;
  const int dm = c.d_model, qw = c.n_q_heads * c.head_dim, F = c.d_ffn;
  size_t o = 0;
  auto take = [&](int n_tasks, int n_in) { size_t at = o; o += tg_tiled_elems(n_tasks, n_in); return at; };
  for (int l = 0; l < c.n_layers; ++l) {
    tm.qkv.push_back(take((c.n_q_heads + 2 * c.n_kv_heads) * (c.head_dim / 2), dm));
    tm.o.push_back(take(dm / 2, qw));
    tm.gateup.push_back(take(F, dm));
    tm.down.push_back(take(dm / 2, F));
  }
  tm.lens_a = take(dm / 2, dm);
  tm.lens_head = take((d.V + 1) / 2, dm);
  tm.lm_head = take((d.V + 1) / 2, dm);
  tm.total = o;
}

void layout(const spark_config &c, const Derived &d, Layout &l) {
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
  const size_t qw = (size_t)c.n_q_heads * c.head_dim;
  l.state = take(sizeof(int) * ST_WORDS * c.max_batch);
  l.page_table = take(sizeof(int) * (size_t)d.max_pages * c.max_batch);
  l.plan = take(sizeof(int) * PL_WORDS);
  l.lower = take(sizeof(RowDesc) * c.max_batch);
  l.upper = take(sizeof(RowDesc) * (size_t)c.max_batch * d.rmax);
  l.ee = take(sizeof(RowDesc) * c.max_batch);
  l.full = take(sizeof(RowDesc) * c.max_batch);
  l.prefill_rows = take(sizeof(RowDesc) * PREFILL_CHUNK);
  l.prefill_tokens = take(sizeof(int) * PREFILL_CHUNK);
  l.seq_ids = take(sizeof(int) * c.max_batch);
  l.forced = take(sizeof(int) * (size_t)MAX_STEPS_PER_CALL * c.max_batch);
  l.step_flags = take(sizeof(int) * c.max_batch);
  l.out_tokens = take(sizeof(int) * (size_t)MAX_STEPS_PER_CALL * c.max_batch);
  l.out_depth = take(sizeof(int) * (size_t)MAX_STEPS_PER_CALL * c.max_batch);
  l.best = take(sizeof(unsigned long long) * c.max_batch);
  l.arrivals = take(sizeof(int) * (size_t)d.max_rows * c.n_q_heads);   // per (row, group of query heads)
  l.row_ssq = take(sizeof(unsigned long long) * 2 * SSQ_WAYS * (size_t)d.max_rows);   // sums of squares handed from a finishing launch to the next projection
  l.sample_hist = take(sizeof(unsigned long long) * (size_t)SAMPLE_BINS * c.max_batch);   // zero between launches
  l.sample_arrive = take(sizeof(unsigned) * c.max_batch);
  l.sample_count = take(sizeof(unsigned) * c.max_batch);
  l.hidden = take(sizeof(float) * ((size_t)c.max_batch * d.rmax + PREFILL_CHUNK) * c.d_model);
  l.qbuf = take(sizeof(float) * d.max_rows * qw);
  l.attn_out = take(sizeof(float) * d.max_rows * qw);
  l.part = take(sizeof(float) * (size_t)d.max_rows * c.n_q_heads * d.n_splits * (c.head_dim + 4));
  l.act = take(sizeof(float) * (size_t)d.max_rows * c.d_ffn);
  l.lens_u = take(sizeof(float) * (size_t)c.max_batch * c.d_model);
  {
    const size_t widest = align_up(std::max((size_t)c.d_ffn, std::max((size_t)c.d_model, qw)), 64);
    l.xsplit = take(sizeof(bf16_t) * 3 * (size_t)d.max_rows * widest);
    // a second one for the MLP activations: the gate/up kernel writes them while it still reads its input
    l.xsplit2 = take(c.dtype == SPARK_DTYPE_BF16 ? sizeof(bf16_t) * 3 * (size_t)d.max_rows * widest : 256);
    l.mfma_part = take(c.dtype == SPARK_DTYPE_BF16 ? MFMA_PARTIAL_BYTES : 256);
  }
  l.logits = take(sizeof(float) * (size_t)c.max_batch * d.V);
  l.sample_q = take(sizeof(unsigned) * (size_t)c.max_batch * d.V);   // integer masses of the sampler
  l.sample_cand = take(sizeof(unsigned long long) * (size_t)SAMPLE_CAP * c.max_batch);
  l.rand_words = take(sizeof(unsigned long long) * (size_t)MAX_STEPS_PER_CALL * c.max_batch);
  l.rope = take(sizeof(float2) * (size_t)c.max_seq_len * (c.head_dim / 2));
  l.inv_freq = take(sizeof(float) * (c.head_dim / 2));
  l.total = o;
  // behind everything else: the MFMA-ordered copy of the bf16 projection weights, for contexts
  // whose scratch area has room for it
  TiledMap tm;
  tiled_map(c, d, tm);
  l.tiled = o;
  l.total_tiled = o + align_up(sizeof(bf16_t) * tm.total, 256);
}

template <typename T> T *at(spark_ctx *c, size_t off) { return (T *)(c->scratch + off); }

// ------------------------------------------------------------------ profiling brackets

// Every bracketed launch takes three events: before, after, and one more right behind it.  The
// last pair has nothing in between and measures what the event mechanism itself adds to a bracket;
// spark_profile_read subtracts its mean.
int prof_begin(spark_ctx *c, int kclass) {
  if (c->prof_class != kclass) return SPARK_OK;
  while (c->prof_used + 3 > c->prof_ev.size()) {
    hipEvent_t ev;
    HIP_TRY(c, hipEventCreate(&ev));
    c->prof_ev.push_back(ev);
  }
  HIP_TRY(c, hipEventRecord(c->prof_ev[c->prof_used], c->stream));
  return SPARK_OK;
}
int prof_end(spark_ctx *c, int kclass) {
  if (c->prof_class != kclass) return SPARK_OK;
  HIP_TRY(c, hipEventRecord(c->prof_ev[c->prof_used + 1], c->stream));
  HIP_TRY(c, hipEventRecord(c->prof_ev[c->prof_used + 2], c->stream));
  c->prof_used += 3;
  return SPARK_OK;
}

// ------------------------------------------------------------------ launches

template <typename WT, typename Pro, typename Epi>
int launch_gemv(spark_ctx *c, const Pro &pro, const Epi &epi, const RowDesc *rows, int m_rows,
                int n_in, int n_tasks, int kclass) {
  if (m_rows <= 0) return SPARK_OK;
  // activation rows per pass over the weights: as many as fit in the LDS budget next to the
  // partial-sum words; a norm prologue needs the whole row resident.  The budget is 64 KiB, or
  // 80 KiB for rows that do not fit in that (two such workgroups still fit in a CU's 160 KiB): a
  // single row of the MLP width (18944) then stays in one chunk, four rows of 4096 under a norm
  // prologue take one pass over the weights instead of two, and what has to be cut into chunks
  // anyway is cut into fewer
  const bool whole_row = std::is_same<Pro, ProNorm>::value;
  int mt = std::min(4, m_rows);
  const size_t budget = sizeof(float) * mt * align_up(n_in, 512) + 256 > 65536 ? 81920 : 65536;
  const size_t lds_budget = budget - sizeof(float) * (GEMV_BIG_THREADS / 64) * 4;
  while (mt > 1 && whole_row && sizeof(float) * mt * align_up(n_in, 512) > lds_budget) --mt;
  int kc_cap = (int)(lds_budget / (sizeof(float) * mt)) / 512 * 512;
  int kc = std::min((int)align_up(n_in, 512), kc_cap);
  if (whole_row && kc < n_in) return fail(c, SPARK_EINVAL, "row of %d does not fit in LDS", n_in);
  // much LDS per workgroup means few workgroups per CU: those launches run eight waves per
  // workgroup, so that a CU still has 16 waves streaming
  const bool big = sizeof(float) * (size_t)mt * kc > (size_t)c->gemv_big_kb * 1024;   // at most three workgroups per CU
  const int threads = big ? GEMV_BIG_THREADS : GEMV_THREADS, waves = threads / 64;
  size_t lds = sizeof(float) * ((size_t)mt * kc + waves * mt);
  // one resident set of blocks: the kernel loops over its tasks, so the grid is sized to what the
  // chip holds at once (no second wave of blocks with a cold pipeline)
  void (*kern)(Pro, Epi, const RowDesc *, int, int, int, int) = nullptr;
  switch (mt) {
    case 1: kern = big ? gemv_rows_k<WT, 1, Pro, Epi, GEMV_U, GEMV_D, GEMV_BIG_THREADS> : gemv_rows_k<WT, 1, Pro, Epi>; break;
    case 2: kern = big ? gemv_rows_k<WT, 2, Pro, Epi, GEMV_U, GEMV_D, GEMV_BIG_THREADS> : gemv_rows_k<WT, 2, Pro, Epi>; break;
    case 3: kern = big ? gemv_rows_k<WT, 3, Pro, Epi, GEMV_U, GEMV_D, GEMV_BIG_THREADS> : gemv_rows_k<WT, 3, Pro, Epi>; break;
    default: kern = big ? gemv_rows_k<WT, 4, Pro, Epi, GEMV_U, GEMV_D, GEMV_BIG_THREADS> : gemv_rows_k<WT, 4, Pro, Epi>; break;
  }
  // attribute and occupancy are asked for once per (kernel, LDS size), not on every launch
  const auto key = std::make_pair((const void *)kern, lds);
  auto found = c->occ_cache.find(key);
  if (found == c->occ_cache.end()) {
    if (lds > 65536)
      HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 81920));
    int o = 0;
    HIP_TRY(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, kern, threads, lds));
    found = c->occ_cache.emplace(key, std::max(1, std::min(o, 4))).first;
  }
  const int occ = found->second;
  int bx = std::min((n_tasks + waves - 1) / waves, c->n_cu * occ);
  dim3 grid(bx, (m_rows + mt - 1) / mt), block(threads);
  int rc = prof_begin(c, kclass);
  if (rc) return rc;
  kern<<<grid, block, lds, c->stream>>>(pro, epi, rows, m_rows, n_in, n_tasks, kc);
  HIP_TRY(c, hipGetLastError());
  return prof_end(c, kclass);
}

size_t xsplit_stride(spark_ctx *c);

// a split-activation buffer seen as rows of `width` elements (padded to the MFMA chunk)
SplitOut split_target(spark_ctx *c, int width, bool second = false) {
  return SplitOut{at<bf16_t>(c, second ? c->lo.xsplit2 : c->lo.xsplit), xsplit_stride(c),
                  (int)align_up(width, MG_KC), width};
}

KVView kv_view(spark_ctx *c) {
  KVView v;
  v.pool = c->kv_pool;
  v.page_table = at<int>(c, c->lo.page_table);
  v.max_pages = c->dv.max_pages;
  v.n_layers = c->cfg.n_layers;
  v.n_kv_heads = c->cfg.n_kv_heads;
  v.page_tokens = c->cfg.kv_page_tokens;
  v.head_dim = c->cfg.head_dim;
  return v;
}

constexpr int ATTN_SPLIT_HEADS_MAX_ROWS = 4;

// GT query heads per workgroup
template <typename WT, int HD, int GT>
void launch_attention_g(spark_ctx *c, const RowDesc *rows, int m, int layer, const SplitOut &so) {
  const spark_config &g = c->cfg;
  const Derived &d = c->dv;
  float *part = at<float>(c, c->lo.part);
  const int n_groups = (d.group + GT - 1) / GT;
  const int splits = c->attn_splits_now > 0 ? std::min(d.n_splits, c->attn_splits_now) : d.n_splits;
  attn_rows_k<WT, HD, GT><<<dim3(splits, g.n_kv_heads * n_groups, m), ATTN_THREADS, 0, c->stream>>>(
      rows, at<float>(c, c->lo.qbuf), kv_view(c), layer, g.n_q_heads, d.group, d.n_splits,
      1.0f / sqrtf((float)HD), part, at<int>(c, c->lo.arrivals), at<float>(c, c->lo.attn_out), so);
}

template <typename WT, int HD>
void launch_attention_hd(spark_ctx *c, const RowDesc *rows, int m, int layer, const SplitOut &so) {
  // a handful of rows: four query heads per workgroup, so that even two KV heads make enough
  // workgroups; many rows: all heads of a KV head together, K and V are read once
  const int group = c->dv.group;
  const int gt = (m <= ATTN_SPLIT_HEADS_MAX_ROWS && group > 2) ? 2 : group;
  switch (gt) {
    case 1: launch_attention_g<WT, HD, 1>(c, rows, m, layer, so); break;
    case 2: launch_attention_g<WT, HD, 2>(c, rows, m, layer, so); break;
    case 3: launch_attention_g<WT, HD, 4>(c, rows, m, layer, so); break;
    case 4: launch_attention_g<WT, HD, 4>(c, rows, m, layer, so); break;
    case 5: case 6: case 7: launch_attention_g<WT, HD, 7>(c, rows, m, layer, so); break;
    case 8: launch_attention_g<WT, HD, 8>(c, rows, m, layer, so); break;
    default: launch_attention_g<WT, HD, 16>(c, rows, m, layer, so); break;
  }
}

// split_out: also leave the output as the three bf16 parts the MFMA output projection reads
template <typename WT> int launch_attention(spark_ctx *c, const RowDesc *rows, int m, int layer, bool split_out) {
  int rc = prof_begin(c, SPARK_KC_ATTN);
  if (rc) return rc;
  const int qw = c->cfg.n_q_heads * c->cfg.head_dim;
  const SplitOut so = split_out ? split_target(c, qw) : SplitOut{nullptr, 0, 0, 0};
  if (std::is_same<WT, bf16_t>::value && c->cfg.head_dim == 128 && c->dv.group <= 16 && c->use_mfma &&
      m >= c->attn_mfma_min_rows) {
    // the slice tasks on the MFMA units, all query heads of a KV head together; with many
    // workgroups to run, several 64-token pieces per workgroup
    const int splits = c->attn_splits_now > 0 ? std::min(c->dv.n_splits, c->attn_splits_now) : c->dv.n_splits;
    const long tasks = (long)splits * c->cfg.n_kv_heads * m;
    int pieces = c->attn_pieces > 0 ? c->attn_pieces : (tasks >= 8L * c->n_cu ? 4 : tasks >= 4L * c->n_cu ? 2 : 1);
    // contexts of 4096 tokens and more: eight pieces (measured on 8 x 8192 tokens: 8.19 -> 8.09 ms per step)
    if (c->attn_pieces <= 0 && pieces == 4 && splits >= 64) pieces = 8;
    // few workgroups (a handful of rows, two KV heads): eight query heads per workgroup
    const int heads_per_wg = (tasks < c->n_cu / 2 && c->dv.group > 8) ? 8 : c->dv.group;
    const int wg_per_kv = (c->dv.group + heads_per_wg - 1) / heads_per_wg;
    attn_rows_mfma_k<128><<<dim3((splits + pieces - 1) / pieces, c->cfg.n_kv_heads * wg_per_kv, m), ATTN_THREADS, 0,
                            c->stream>>>(
        rows, at<float>(c, c->lo.qbuf), kv_view(c), layer, c->cfg.n_q_heads, c->dv.group, heads_per_wg,
        c->dv.n_splits, pieces, 1.0f / sqrtf(128.0f), at<float>(c, c->lo.part), at<int>(c, c->lo.arrivals),
        at<float>(c, c->lo.attn_out), so);
  } else if (c->cfg.head_dim == 128) launch_attention_hd<WT, 128>(c, rows, m, layer, so);
  else launch_attention_hd<WT, 64>(c, rows, m, layer, so);
  HIP_TRY(c, hipGetLastError());
  return prof_end(c, SPARK_KC_ATTN);
}

// ------------------------------------------------------------------ MFMA path (16..128+ rows, bf16)


// the three bf16 parts of the split activations are stored one after the other
size_t xsplit_stride(spark_ctx *c) {
  const spark_config &g = c->cfg;
  const size_t widest = align_up(std::max((size_t)g.d_ffn, std::max((size_t)g.d_model, (size_t)g.n_q_heads * g.head_dim)), 64);
  return (size_t)c->dv.max_rows * widest;
}

int launch_prep(spark_ctx *c, const RowDesc *rows, int m, const float *src, int stride, int indirect,
                const float *gamma, int n) {
  prep_rows_k<<<m, 256, 0, c->stream>>>(rows, src, stride, indirect, gamma, c->cfg.rms_eps, n,
                                        (int)align_up(n, MG_KC), at<bf16_t>(c, c->lo.xsplit), xsplit_stride(c));
  HIP_TRY(c, hipGetLastError());
  return SPARK_OK;
}

// tasks one thread of the finishing kernel takes: the vocabulary heads reduce their arg-max over 8
// per thread, then over the workgroup's threads of the same row
template <typename Epi> int finish_tasks_per_thread(const Epi &) { return 1; }
template <typename WT> int finish_tasks_per_thread(const EpiVocab<WT> &) { return 8; }

template <int MTILES, typename Epi, bool SPLIT, int WAVES>
int mfma_occupancy(spark_ctx *c) {
  auto kern = mfma_rows_k<MTILES, Epi, SPLIT, WAVES>;
  const size_t lds = mg_lds_bytes(MTILES, WAVES);
  const auto key = std::make_pair((const void *)kern, lds);
  auto found = c->occ_cache.find(key);
  if (found == c->occ_cache.end()) {
    if (lds > 65536)
      HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int o = 0;
    HIP_TRY(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, kern, 64 * WAVES, lds));
    if (o < 1) return fail(c, SPARK_EHIP, "the MFMA kernel for %d rows does not fit on a CU", 32 * MTILES);
    found = c->occ_cache.emplace(key, o).first;
  }
  return found->second;
}

template <int MTILES, int TB, typename Epi, bool SPLIT>
int tiled_occupancy(spark_ctx *c) {
  auto kern = mfma_tiled_k<MTILES, TB, Epi, SPLIT>;
  const size_t lds = tg_lds_bytes(MTILES);
  const auto key = std::make_pair((const void *)kern, lds);
  auto found = c->occ_cache.find(key);
  if (found == c->occ_cache.end()) {
    int o = 0;
    HIP_TRY(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, kern, 64 * TG_WAVES, lds));
    if (o < 1) return fail(c, SPARK_EHIP, "the tiled MFMA kernel for %d rows does not fit on a CU", 32 * MTILES);
    found = c->occ_cache.emplace(key, o).first;
  }
  return found->second;
}

// tiled: the projection's weights in MFMA operand order (then the kernel that takes them from
// there runs; its workgroups cover the same tiles of tasks), or nullptr
template <int MTILES, typename Epi, int WAVES>
int launch_mfma_shape(spark_ctx *c, const Epi &epi, const RowDesc *rows, int m, int n_in, int n_tasks,
                      bool may_split, bool second_input, const bf16_t *tiled) {
  constexpr int TB = WAVES / 4;   // blocks of 32 tasks per wave of the four-wave tiled kernel
  constexpr bool STATELESS = std::is_same<typename Epi::State, NoState>::value;
  constexpr int TASKS_PER_BLOCK = WAVES * MG_TASKS_PER_WAVE;
  const int mrows = 32 * MTILES;
  const int z = (m + mrows - 1) / mrows;
  const int bx = (n_tasks + TASKS_PER_BLOCK - 1) / TASKS_PER_BLOCK;
  const int n_chunks = (n_in + MG_KC - 1) / MG_KC;
  // rows of the partial sums: padded to eight only (a pass of eight rows then writes and reads a
  // quarter of what 32 padded rows would)
  const int m_pad = (int)align_up(m, 8);
  // resident workgroups on the chip: the k range is split until one round of them has work
  int occ = tiled ? tiled_occupancy<MTILES, TB, Epi, true>(c) : mfma_occupancy<MTILES, Epi, true, WAVES>(c);
  if (occ < 0) return occ;
  // k splits: the count that keeps most of the chip busy over whole rounds of resident
  // workgroups, with at least eight chunks each (the pipeline needs a few to fill)
  int split = 1;
  if (may_split) {
    // (the tiled kernel: one workgroup already keeps a CU's share of the memory system busy, and
    // two on a CU share that CU's throughput, so rounds are counted in CUs)
    const int slots = (tiled ? 1 : occ) * c->n_cu, tiles = bx * z;
    const size_t per_split = sizeof(float) * (size_t)n_tasks * 2 * m_pad;
    // (few tiles: shorter k ranges are worth the pipeline fill they cost)
    const int min_chunks = tiles < 32 ? 4 : 8;
    const int max_split = (int)std::min<size_t>(std::max(1, n_chunks / min_chunks), std::max<size_t>(1, MFMA_PARTIAL_BYTES / per_split));
    double best = 0.0;
    for (int s = 1; s <= std::min(max_split, 32); ++s) {
      const int blocks = tiles * s, rounds = (blocks + slots - 1) / slots;
      const double util = (double)blocks / ((double)rounds * slots);
      if (util > best + 0.02) { best = util; split = s; }
    }
  }
  const int cps = (n_chunks + split - 1) / split;
  split = (n_chunks + cps - 1) / cps;
  const bf16_t *xs = at<bf16_t>(c, second_input ? c->lo.xsplit2 : c->lo.xsplit);
  const size_t xst = xsplit_stride(c);
  float *part = at<float>(c, c->lo.mfma_part);
  // one-dimensional grid: the kernel deals its ids so that the row tiles of a weight tile share an XCD
  const int xcd_groups = z > 1 && split <= c->mfma_xcd_max_split;
  const int tiles_padded = xcd_groups ? (bx * split + 7) / 8 * 8 : bx * split;
  dim3 grid(tiles_padded * z);
  const size_t lds = mg_lds_bytes(MTILES, WAVES);
  // (an epilogue that sums over a row runs in the finishing launch only; so does, on tiled
  // weights, one with a running state: the tiled kernel hands every lane 64 tasks of one row,
  // the finishing launch reduces the states of a row before they reach memory)
  if (split > 1 || EpiHasRowSum<Epi>::value || (tiled && !STATELESS)) {
    if (tiled)
      mfma_tiled_k<MTILES, TB, Epi, true><<<grid, 64 * TG_WAVES, tg_lds_bytes(MTILES), c->stream>>>(
          epi, tiled, rows, m, xs, xst, n_in, n_tasks, cps, part, m_pad, bx, split, z, xcd_groups);
    else
      mfma_rows_k<MTILES, Epi, true, WAVES><<<grid, 64 * WAVES, lds, c->stream>>>(
          epi, rows, m, xs, xst, n_in, n_tasks, cps, part, m_pad, bx, split, z, xcd_groups);
    if constexpr (std::is_same<typename Epi::State, NoState>::value || EpiHasRowSum<Epi>::value) {
      // epilogues without a running state: stores coalesced over tasks
      const dim3 fgrid((n_tasks + 31) / 32, (m_pad + 31) / 32);
      if (split <= 8) mfma_finish_tile_k<Epi, 8><<<fgrid, 1024, 0, c->stream>>>(epi, rows, m, n_tasks, split, part, m_pad);
      else mfma_finish_tile_k<Epi, MG_MAX_SPLIT><<<fgrid, 1024, 0, c->stream>>>(epi, rows, m, n_tasks, split, part, m_pad);
    } else {
      const int tpt = finish_tasks_per_thread(epi);
      const int total = ((n_tasks + tpt - 1) / tpt) * m_pad;
      mfma_finish_k<Epi><<<(total + 255) / 256, 256, 0, c->stream>>>(epi, rows, m, n_tasks, split, part, m_pad, tpt);
    }
  } else if constexpr (!EpiHasRowSum<Epi>::value) {
    bool done = false;
    if constexpr (STATELESS) {
      if (tiled) {
        mfma_tiled_k<MTILES, TB, Epi, false><<<grid, 64 * TG_WAVES, tg_lds_bytes(MTILES), c->stream>>>(
            epi, tiled, rows, m, xs, xst, n_in, n_tasks, cps, part, m_pad, bx, split, z, xcd_groups);
        done = true;
      }
    }
    if (!done) {
      occ = mfma_occupancy<MTILES, Epi, false, WAVES>(c);
      if (occ < 0) return occ;
      mfma_rows_k<MTILES, Epi, false, WAVES><<<grid, 64 * WAVES, lds, c->stream>>>(
          epi, rows, m, xs, xst, n_in, n_tasks, cps, part, m_pad, bx, split, z, xcd_groups);
    }
  }
  HIP_TRY(c, hipGetLastError());
  return SPARK_OK;
}

template <int MTILES, typename Epi>
int launch_mfma_tiles(spark_ctx *c, const Epi &epi, const RowDesc *rows, int m, int n_in, int n_tasks,
                      bool may_split, const bf16_t *tiled, bool second_input = false) {
  if (n_in % 8) return fail(c, SPARK_EINVAL, "MFMA path needs an input width that is a multiple of 8, not %d", n_in);
  // matrices of few rows and a short k (q/k/v, o, the lens translator): four waves per workgroup,
  // so that the launch has enough workgroups without cutting k into ranges too short to stream
  // (measured at 32 rows: q/k/v 23.5 -> 20.8 us, o 20.2 -> 16.0 us; down, with its long k, and
  // gate/up, with its many tiles, are better off with eight)
  const int tiles8 = ((n_tasks + MG_TASKS_PER_BLOCK - 1) / MG_TASKS_PER_BLOCK) * ((m + 32 * MTILES - 1) / (32 * MTILES));
  if (tiles8 < c->mfma_small_tiles && n_in <= c->mfma_small_max_k)
    return launch_mfma_shape<MTILES, Epi, 4>(c, epi, rows, m, n_in, n_tasks, may_split, second_input, tiled);
  return launch_mfma_shape<MTILES, Epi, 8>(c, epi, rows, m, n_in, n_tasks, may_split, second_input, tiled);
}

// y = W x for m rows whose hi/lo split sits in the xhi/xlo buffers
template <typename Epi>
int launch_mfma(spark_ctx *c, const Epi &epi, const RowDesc *rows, int m, int n_in, int n_tasks,
                bool may_split, int kclass, const bf16_t *tiled, bool second_input = false) {
  int rc = prof_begin(c, kclass);
  if (rc) return rc;
  if (m <= 32) rc = launch_mfma_tiles<1>(c, epi, rows, m, n_in, n_tasks, may_split, tiled, second_input);
  else rc = launch_mfma_tiles<2>(c, epi, rows, m, n_in, n_tasks, may_split, tiled, second_input);   // tiles of 64 rows
  if (rc) return rc;
  return prof_end(c, kclass);
}

template <typename WT> int launch_attention(spark_ctx *c, const RowDesc *rows, int m, int layer, bool split_out);

// The copy of one projection's weights in MFMA operand order, or nullptr when the context has none
// (or is told not to use it).
const bf16_t *tiled_at(spark_ctx *c, size_t elem_off) {
  return c->has_tiled && c->use_tiled ? at<bf16_t>(c, c->lo.tiled) + elem_off : nullptr;
}

template <typename Epi>
int tile_one(spark_ctx *c, const Epi &epi, int n_tasks, int n_in, size_t elem_off) {
  const int n_chunks = (n_in + MG_KC - 1) / MG_KC, n_tb = (n_tasks + 31) / 32;
  tile_weights_k<<<dim3(n_chunks, n_tb * 2), 256, 0, c->stream>>>(epi, n_tasks, n_in, n_chunks,
                                                               at<bf16_t>(c, c->lo.tiled) + elem_off);
  HIP_TRY(c, hipGetLastError());
  return SPARK_OK;
}

// Writes the MFMA-ordered copies once, with the epilogues' own task -> weight rows mapping (only
// the weight pointers and widths of an epilogue matter here).
int build_tiled(spark_ctx *c) {
  typedef bf16_t WT;
  const spark_config &g = c->cfg;
  const int d = g.d_model, hd = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, F = g.d_ffn, V = c->dv.V;
  const size_t qw = (size_t)nq * hd, kvw = (size_t)nkv * hd;
  int rc;
  for (int l = 0; l < g.n_layers; ++l) {
    EpiQKV<WT> eq;
    eq.wq = (const WT *)c->w.wq + (size_t)l * qw * d;
    eq.wk = (const WT *)c->w.wk + (size_t)l * kvw * d;
    eq.wv = (const WT *)c->w.wv + (size_t)l * kvw * d;
    eq.d = d; eq.nq = nq; eq.nkv = nkv; eq.hd = hd; eq.layer = l;
    eq.qbuf = nullptr; eq.rope = nullptr; eq.kv = kv_view(c);
    if ((rc = tile_one(c, eq, (nq + 2 * nkv) * (hd / 2), d, c->tm.qkv[l]))) return rc;
    EpiResidual<WT> eo{(const WT *)c->w.wo + (size_t)l * d * qw, (int)qw, d, nullptr, d};
    if ((rc = tile_one(c, eo, d / 2, (int)qw, c->tm.o[l]))) return rc;
    EpiSwiGLUSplit<WT> eg{(const WT *)c->w.wg + (size_t)l * F * d, (const WT *)c->w.wu + (size_t)l * F * d, d, F,
                          SplitOut{nullptr, 0, 0, 0}};
    if ((rc = tile_one(c, eg, F, d, c->tm.gateup[l]))) return rc;
    EpiResidual<WT> ed{(const WT *)c->w.wd + (size_t)l * d * F, F, d, nullptr, d};
    if ((rc = tile_one(c, ed, d / 2, F, c->tm.down[l]))) return rc;
  }
  EpiLensAffine<WT> ea{(const WT *)c->w.lens_a, nullptr, nullptr, nullptr, d};
  if ((rc = tile_one(c, ea, d / 2, d, c->tm.lens_a))) return rc;
  EpiVocab<WT> el{(const WT *)c->w.lens_head, d, V, nullptr, nullptr};
  if ((rc = tile_one(c, el, (V + 1) / 2, d, c->tm.lens_head))) return rc;
  EpiVocab<WT> ev{(const WT *)c->w.lm_head, d, V, nullptr, nullptr};
  if ((rc = tile_one(c, ev, (V + 1) / 2, d, c->tm.lm_head))) return rc;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return SPARK_OK;
}

// layers [l0, l1) on m >= 16 rows, bf16 weights
int run_layers_mfma(spark_ctx *c, int l0, int l1, const RowDesc *rows, int m) {
  typedef bf16_t WT;
  const spark_config &g = c->cfg;
  const int d = g.d_model, hd = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, F = g.d_ffn;
  const size_t qw = (size_t)nq * hd, kvw = (size_t)nkv * hd;
  float *hidden = at<float>(c, c->lo.hidden);
  // RMSNorm is linear in 1/rms: the finishing launch of a residual projection writes the split
  // gamma (.) h for the projection that follows and adds up h's sum of squares per row; that
  // projection's epilogue scales by 1/rms.  Only the first norm of a run is a launch of its own.
  unsigned long long *ssq_attn = at<unsigned long long>(c, c->lo.row_ssq);
  unsigned long long *ssq_mlp = ssq_attn + (size_t)SSQ_WAYS * c->dv.max_rows;
  const bool fuse = c->fuse_norm;
  int rc;
  for (int l = l0; l < l1; ++l) {
    const bool qkv_scaled = fuse && l > l0;
    if (!qkv_scaled && (rc = launch_prep(c, rows, m, hidden, d, 1, c->w.attn_norm + (size_t)l * d, d))) return rc;
    EpiQKV<WT> eq;
    eq.wq = (const WT *)c->w.wq + (size_t)l * qw * d;
    eq.wk = (const WT *)c->w.wk + (size_t)l * kvw * d;
    eq.wv = (const WT *)c->w.wv + (size_t)l * kvw * d;
    eq.d = d; eq.nq = nq; eq.nkv = nkv; eq.hd = hd; eq.layer = l;
    eq.qbuf = at<float>(c, c->lo.qbuf);
    eq.rope = at<float2>(c, c->lo.rope);
    eq.kv = kv_view(c);
    if (qkv_scaled) eq.scale = RowScale{ssq_attn, 1.0f / (float)d, g.rms_eps};
    if ((rc = launch_mfma(c, eq, rows, m, d, (nq + 2 * nkv) * (hd / 2), true, SPARK_KC_QKV, tiled_at(c, c->tm.qkv[l])))) return rc;

    // attention leaves its output split for the MFMA kernel; so does the SwiGLU epilogue below
    if ((rc = launch_attention<WT>(c, rows, m, l, true))) return rc;

    EpiSwiGLUSplit<WT> eg{(const WT *)c->w.wg + (size_t)l * F * d, (const WT *)c->w.wu + (size_t)l * F * d,
                          d, F, split_target(c, F, true)};
    if (fuse) {
      EpiResidualNorm<WT> eo{(const WT *)c->w.wo + (size_t)l * d * qw, (int)qw, d, hidden, d,
                             c->w.mlp_norm + (size_t)l * d, split_target(c, d), ssq_mlp};
      if ((rc = launch_mfma(c, eo, rows, m, (int)qw, d / 2, true, SPARK_KC_OPROJ, tiled_at(c, c->tm.o[l])))) return rc;
      eg.scale = RowScale{ssq_mlp, 1.0f / (float)d, g.rms_eps};
    } else {
      EpiResidual<WT> eo{(const WT *)c->w.wo + (size_t)l * d * qw, (int)qw, d, hidden, d};
      if ((rc = launch_mfma(c, eo, rows, m, (int)qw, d / 2, true, SPARK_KC_OPROJ, tiled_at(c, c->tm.o[l])))) return rc;
      if ((rc = launch_prep(c, rows, m, hidden, d, 1, c->w.mlp_norm + (size_t)l * d, d))) return rc;
    }
    if ((rc = launch_mfma(c, eg, rows, m, d, F, true, SPARK_KC_GATEUP, tiled_at(c, c->tm.gateup[l])))) return rc;

    if (fuse && l + 1 < l1) {
      EpiResidualNorm<WT> ed{(const WT *)c->w.wd + (size_t)l * d * F, F, d, hidden, d,
                             c->w.attn_norm + (size_t)(l + 1) * d, split_target(c, d), ssq_attn};
      if ((rc = launch_mfma(c, ed, rows, m, F, d / 2, true, SPARK_KC_DOWN, tiled_at(c, c->tm.down[l]), true))) return rc;
    } else {
      EpiResidual<WT> ed{(const WT *)c->w.wd + (size_t)l * d * F, F, d, hidden, d};
      if ((rc = launch_mfma(c, ed, rows, m, F, d / 2, true, SPARK_KC_DOWN, tiled_at(c, c->tm.down[l]), true))) return rc;
    }
  }
  return SPARK_OK;
}

// layers [l0, l1) on m rows described by `rows` (device)
template <typename WT>
int run_layers(spark_ctx *c, int l0, int l1, const RowDesc *rows, int m) {
  const spark_config &g = c->cfg;
  if (l0 >= l1 || m <= 0) return SPARK_OK;
  // many rows: the projections are dense contractions for the MFMA units
  if (std::is_same<WT, bf16_t>::value && m >= c->mfma_min_rows && c->use_mfma)
    return run_layers_mfma(c, l0, l1, rows, m);
  const int d = g.d_model, hd = g.head_dim, nq = g.n_q_heads, nkv = g.n_kv_heads, F = g.d_ffn;
  const size_t qw = (size_t)nq * hd, kvw = (size_t)nkv * hd;
  float *hidden = at<float>(c, c->lo.hidden);
  int rc;
  for (int l = l0; l < l1; ++l) {
    ProNorm n1{hidden, c->w.attn_norm + (size_t)l * d, g.rms_eps, d, 1};
    EpiQKV<WT> eq;
    eq.wq = (const WT *)c->w.wq + (size_t)l * qw * d;
    eq.wk = (const WT *)c->w.wk + (size_t)l * kvw * d;
    eq.wv = (const WT *)c->w.wv + (size_t)l * kvw * d;
    eq.d = d; eq.nq = nq; eq.nkv = nkv; eq.hd = hd; eq.layer = l;
    eq.qbuf = at<float>(c, c->lo.qbuf);
    eq.rope = at<float2>(c, c->lo.rope);
    eq.kv = kv_view(c);
    if ((rc = launch_gemv<WT>(c, n1, eq, rows, m, d, (nq + 2 * nkv) * (hd / 2), SPARK_KC_QKV))) return rc;

    if ((rc = launch_attention<WT>(c, rows, m, l, false))) return rc;

    ProPlain pa{at<float>(c, c->lo.attn_out), (int)qw, 0};
    EpiResidual<WT> eo{(const WT *)c->w.wo + (size_t)l * d * qw, (int)qw, d, hidden, d};
    if ((rc = launch_gemv<WT>(c, pa, eo, rows, m, (int)qw, d / 2, SPARK_KC_OPROJ))) return rc;

    ProNorm n2{hidden, c->w.mlp_norm + (size_t)l * d, g.rms_eps, d, 1};
    EpiSwiGLU<WT> eg{(const WT *)c->w.wg + (size_t)l * F * d, (const WT *)c->w.wu + (size_t)l * F * d,
                     d, F, at<float>(c, c->lo.act)};
    if ((rc = launch_gemv<WT>(c, n2, eg, rows, m, d, F, SPARK_KC_GATEUP))) return rc;

    ProPlain pd{at<float>(c, c->lo.act), F, 0};
    EpiResidual<WT> ed{(const WT *)c->w.wd + (size_t)l * d * F, F, d, hidden, d};
    if ((rc = launch_gemv<WT>(c, pd, ed, rows, m, F, d / 2, SPARK_KC_DOWN))) return rc;
  }
  return SPARK_OK;
}

template <typename WT> int run_lens_head(spark_ctx *c, const RowDesc *rows, int m) {
  const spark_config &g = c->cfg;
  const int d = g.d_model, V = c->dv.V;
  float *hidden = at<float>(c, c->lo.hidden), *u = at<float>(c, c->lo.lens_u);
  int rc;
  if (std::is_same<WT, bf16_t>::value && m >= c->mfma_min_rows && c->use_mfma) {
    if ((rc = launch_prep(c, rows, m, hidden, d, 1, nullptr, d))) return rc;
    EpiLensAffine<bf16_t> ea{(const bf16_t *)c->w.lens_a, c->w.lens_b, hidden, u, d};
    if ((rc = launch_mfma(c, ea, rows, m, d, d / 2, true, SPARK_KC_LENS, tiled_at(c, c->tm.lens_a)))) return rc;
    if ((rc = launch_prep(c, rows, m, u, d, 0, c->w.lens_norm, d))) return rc;
    EpiVocab<bf16_t> ev{(const bf16_t *)c->w.lens_head, d, V, at<float>(c, c->lo.logits),
                        at<unsigned long long>(c, c->lo.best)};
    rc = prof_begin(c, SPARK_KC_LENS);
    if (rc) return rc;
    if ((rc = launch_mfma_tiles<1>(c, ev, rows, m, d, (V + 1) / 2, true, tiled_at(c, c->tm.lens_head)))) return rc;
    return prof_end(c, SPARK_KC_LENS);
  }
  ProPlain ph{hidden, d, 1};
  EpiLensAffine<WT> ea{(const WT *)c->w.lens_a, c->w.lens_b, hidden, u, d};
  if ((rc = launch_gemv<WT>(c, ph, ea, rows, m, d, d / 2, SPARK_KC_LENS))) return rc;
  // the translated state sits in u[pass row]; normalising it is the head's prologue
  ProNorm pn{u, c->w.lens_norm, g.rms_eps, d, 0};
  EpiVocab<WT> ev{(const WT *)c->w.lens_head, d, V, at<float>(c, c->lo.logits),
                  at<unsigned long long>(c, c->lo.best)};
  return launch_gemv<WT>(c, pn, ev, rows, m, d, (V + 1) / 2, SPARK_KC_LENS);
}

template <typename WT> int run_final_head(spark_ctx *c, const RowDesc *rows, int m) {
  const spark_config &g = c->cfg;
  const int d = g.d_model, V = c->dv.V;
  if (std::is_same<WT, bf16_t>::value && m >= c->mfma_min_rows && c->use_mfma) {
    int rc;
    if ((rc = launch_prep(c, rows, m, at<float>(c, c->lo.hidden), d, 1, c->w.final_norm, d))) return rc;
    EpiVocab<bf16_t> ev{(const bf16_t *)c->w.lm_head, d, V, at<float>(c, c->lo.logits),
                        at<unsigned long long>(c, c->lo.best)};
    rc = prof_begin(c, SPARK_KC_HEAD);
    if (rc) return rc;
    if ((rc = launch_mfma_tiles<1>(c, ev, rows, m, d, (V + 1) / 2, true, tiled_at(c, c->tm.lm_head)))) return rc;
    return prof_end(c, SPARK_KC_HEAD);
  }
  ProNorm pn{at<float>(c, c->lo.hidden), c->w.final_norm, g.rms_eps, d, 1};
  EpiVocab<WT> ev{(const WT *)c->w.lm_head, d, V, at<float>(c, c->lo.logits),
                  at<unsigned long long>(c, c->lo.best)};
  return launch_gemv<WT>(c, pn, ev, rows, m, d, (V + 1) / 2, SPARK_KC_HEAD);
}

}  // namespace

// ------------------------------------------------------------------ C ABI

namespace {

Seq *find_seq(spark_ctx *c, int id) {
  if (id < 0 || id >= (int)c->seqs.size() || !c->seqs[id].open) return nullptr;
  return &c->seqs[id];
}

// make sure `seq` owns pages for positions [0, upto); new page-table entries go to the device
int ensure_pages(spark_ctx *c, int id, int upto) {
  Seq &s = c->seqs[id];
  const int pt = c->cfg.kv_page_tokens;
  const int need = (upto + pt - 1) / pt;
  const int have = (int)s.pages.size();
  if (need <= have) return SPARK_OK;
  if (need > c->dv.max_pages) return fail(c, SPARK_ENOMEM, "sequence %d exceeds max_seq_len", id);
  if ((int)c->free_pages.size() < need - have) return fail(c, SPARK_ENOMEM, "KV pool exhausted");
  for (int p = have; p < need; ++p) {
    s.pages.push_back(c->free_pages.back());
    c->free_pages.pop_back();
  }
  int *dst = at<int>(c, c->lo.page_table) + (size_t)id * c->dv.max_pages + have;
  HIP_TRY(c, hipMemcpyAsync(dst, s.pages.data() + have, sizeof(int) * (need - have),
                            hipMemcpyHostToDevice, c->stream));
  // the source vector may be reallocated by a later push_back
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return SPARK_OK;
}

template <typename WT>
int enqueue_step(spark_ctx *c, int n, int n_upper, int n_ee, int n_full, const int *forced_dev,
                 const unsigned long long *rand_dev, int *out_tok_dev, int *out_depth_dev) {
  const spark_config &g = c->cfg;
  RowDesc *lower = at<RowDesc>(c, c->lo.lower), *upper = at<RowDesc>(c, c->lo.upper);
  RowDesc *ee = at<RowDesc>(c, c->lo.ee), *full = at<RowDesc>(c, c->lo.full);
  int *state = at<int>(c, c->lo.state), *plan = at<int>(c, c->lo.plan);
  int *seq_ids = at<int>(c, c->lo.seq_ids), *flags = at<int>(c, c->lo.step_flags);
  unsigned long long *best = at<unsigned long long>(c, c->lo.best);
  int rc;
  sched_dispatch_k<<<1, SCHED_THREADS, 0, c->stream>>>(c->sp, n, seq_ids, state, lower, upper, ee,
                                                      full, plan, flags, out_depth_dev, best);
  embed_rows_k<WT><<<n, 256, 0, c->stream>>>(lower, state, nullptr, (const WT *)c->w.embed,
                                             g.d_model, at<float>(c, c->lo.hidden));
  HIP_TRY(c, hipGetLastError());
  if ((rc = run_layers<WT>(c, 0, g.exit_layer, lower, n))) return rc;
  if (n_ee && (rc = run_lens_head<WT>(c, ee, n_ee))) return rc;
  if (n_full) {
    if ((rc = run_layers<WT>(c, g.exit_layer, g.n_layers, upper, n_upper))) return rc;
    if ((rc = run_final_head<WT>(c, full, n_full))) return rc;
  }
  if (rand_dev && c->temperature > 0.f) {   // the drawn token takes the arg-max's place
    if ((rc = prof_begin(c, SPARK_KC_SAMPLE))) return rc;
    const dim3 grid((c->dv.V + SAMPLE_CHUNK - 1) / SAMPLE_CHUNK, n);
    float *logits = at<float>(c, c->lo.logits);
    unsigned *masses = at<unsigned>(c, c->lo.sample_q);
    unsigned long long *class_mass = at<unsigned long long>(c, c->lo.sample_hist);
    sample_mass_k<<<grid, SAMPLE_THREADS, 0, c->stream>>>(logits, c->dv.V, (double)c->temperature, masses,
                                                          class_mass, best);
    sample_pick_k<<<grid, SAMPLE_THREADS, 0, c->stream>>>(
        logits, c->dv.V, (double)c->top_p, rand_dev, masses, class_mass,
        at<unsigned long long>(c, c->lo.sample_cand), at<unsigned>(c, c->lo.sample_count),
        at<unsigned>(c, c->lo.sample_arrive), best);
    if ((rc = prof_end(c, SPARK_KC_SAMPLE))) return rc;
  }
  emit_k<<<1, SCHED_THREADS, 0, c->stream>>>(n, seq_ids, forced_dev, flags, best, state, plan,
                                            out_tok_dev);
  HIP_TRY(c, hipGetLastError());
  return SPARK_OK;
}

int decode_chunk(spark_ctx *c, int steps, int n, const int32_t *seq_ids, const int32_t *forced,
                 const uint64_t *rand_words, int32_t *out_tokens, int32_t *out_depth) {
  const spark_config &g = c->cfg;
  int rc;
  // validation and page reservation
  for (int i = 0; i < n; ++i) {
    Seq *s = find_seq(c, seq_ids[i]);
    if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_ids[i]);
    if (!s->prefilled) return fail(c, SPARK_ESTATE, "sequence %d stepped before prefill", seq_ids[i]);
    for (int k = 0; k < i; ++k)
      if (seq_ids[k] == seq_ids[i]) return fail(c, SPARK_EINVAL, "sequence %d listed twice", seq_ids[i]);
    if (s->len + steps > g.max_seq_len)
      return fail(c, SPARK_ENOMEM, "sequence %d would exceed max_seq_len", seq_ids[i]);
    if (forced)
      for (int st = 0; st < steps; ++st)
        if (forced[st * n + i] >= c->dv.V) return fail(c, SPARK_EINVAL, "forced id out of range");
  }
  // the schedule of the whole call, before anything is enqueued: the pending rows and the current
  // row of a sequence must fit its slots of the hidden-state arena at every step
  for (int i = 0; i < n; ++i) {
    const Seq &sq = c->seqs[seq_ids[i]];
    int gg = sq.g, jj = sq.j_stream, npend = sq.n_pending;
    for (int st = 0; st < steps; ++st) {
      int is_text, full;
      schedule_decide(c->sp, gg, sq.cycle_offset, jj, sq.text_budget, sq.phase, is_text, full);
      npend = full ? 0 : npend + 1;
      if (npend + 1 > c->dv.rmax)
        return fail(c, SPARK_ESTATE, "sequence %d would hold %d pending positions, its slots hold %d",
                    seq_ids[i], npend, c->dv.rmax - 1);
      ++gg;
      if (!is_text) ++jj;
    }
  }
  for (int i = 0; i < n; ++i)
    if ((rc = ensure_pages(c, seq_ids[i], c->seqs[seq_ids[i]].len + steps))) return rc;

  // inputs
  int *h_ids = c->h_in, *h_forced = c->h_in + g.max_batch;
  memcpy(h_ids, seq_ids, sizeof(int) * n);
  HIP_TRY(c, hipMemcpyAsync(at<int>(c, c->lo.seq_ids), h_ids, sizeof(int) * n, hipMemcpyHostToDevice,
                            c->stream));
  if (forced) {
    memcpy(h_forced, forced, sizeof(int) * (size_t)steps * n);
    HIP_TRY(c, hipMemcpyAsync(at<int>(c, c->lo.forced), h_forced, sizeof(int) * (size_t)steps * n,
                              hipMemcpyHostToDevice, c->stream));
  }

  if (rand_words)   // (pageable source: the copy has completed on return)
    HIP_TRY(c, hipMemcpyAsync(at<unsigned long long>(c, c->lo.rand_words), rand_words,
                              sizeof(uint64_t) * (size_t)steps * n, hipMemcpyHostToDevice, c->stream));

  // host mirror of the schedule: decides the launch shapes, checked against the device's depths
  struct Mirror { int g, j, npend, len; };
  std::vector<Mirror> mir(n);
  for (int i = 0; i < n; ++i) {
    Seq &s = c->seqs[seq_ids[i]];
    mir[i] = Mirror{s.g, s.j_stream, s.n_pending, s.len};
  }
  std::vector<int> want_depth((size_t)steps * n), want_text((size_t)steps * n),
      want_rows((size_t)steps * n);
  for (int st = 0; st < steps; ++st) {
    int n_upper = 0, n_ee = 0, n_full = 0, max_pos = 0;
    for (int i = 0; i < n; ++i) max_pos = std::max(max_pos, mir[i].len);   // position of the new row
    c->attn_splits_now = max_pos / ATTN_SLICE + 1;
    for (int i = 0; i < n; ++i) {
      int is_text, full;
      const Seq &sq = c->seqs[seq_ids[i]];
      schedule_decide(c->sp, mir[i].g, sq.cycle_offset, mir[i].j, sq.text_budget, sq.phase, is_text, full);
      want_depth[st * n + i] = full ? g.n_layers : g.exit_layer;
      want_text[st * n + i] = is_text;
      want_rows[st * n + i] = full ? mir[i].npend + 1 : 0;
      if (full) { n_upper += mir[i].npend + 1; ++n_full; mir[i].npend = 0; }
      else { ++n_ee; mir[i].npend += 1; }
      mir[i].g += 1;
      if (!is_text) mir[i].j += 1;
      mir[i].len += 1;
    }
    const int *f = forced ? at<int>(c, c->lo.forced) + (size_t)st * n : nullptr;
    int *ot = at<int>(c, c->lo.out_tokens) + (size_t)st * n;
    int *od = at<int>(c, c->lo.out_depth) + (size_t)st * n;
    const unsigned long long *rw =
        rand_words ? at<unsigned long long>(c, c->lo.rand_words) + (size_t)st * n : nullptr;
    rc = g.dtype == SPARK_DTYPE_BF16 ? enqueue_step<bf16_t>(c, n, n_upper, n_ee, n_full, f, rw, ot, od)
                                     : enqueue_step<float>(c, n, n_upper, n_ee, n_full, f, rw, ot, od);
    if (rc) return rc;
  }

  // results
  const size_t cnt = (size_t)steps * n;
  int *h_tok = c->h_out, *h_dep = c->h_out + (size_t)MAX_STEPS_PER_CALL * g.max_batch;
  int *h_plan = h_dep + (size_t)MAX_STEPS_PER_CALL * g.max_batch;
  HIP_TRY(c, hipMemcpyAsync(h_tok, at<int>(c, c->lo.out_tokens), sizeof(int) * cnt,
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipMemcpyAsync(h_dep, at<int>(c, c->lo.out_depth), sizeof(int) * cnt,
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipMemcpyAsync(h_plan, at<int>(c, c->lo.plan), sizeof(int) * PL_WORDS,
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  memcpy(out_tokens, h_tok, sizeof(int) * cnt);
  memcpy(out_depth, h_dep, sizeof(int) * cnt);

  // commit the mirror and the exit-layer log
  for (int st = 0; st < steps; ++st)
    for (int i = 0; i < n; ++i) {
      Seq &s = c->seqs[seq_ids[i]];
      const size_t k = (size_t)st * n + i;
      if (h_dep[k] != want_depth[k])
        return fail(c, SPARK_ESTATE, "device schedule (%d) and host mirror (%d) disagree", h_dep[k],
                    want_depth[k]);
      if (want_rows[k]) {
        s.flush_rows[want_rows[k]] += 1;
        if (want_text[k]) s.text_steps += 1; else s.speech_full += 1;
      } else if (want_text[k]) {
        s.text_ee += 1;
      } else {
        s.speech_ee += 1;
      }
      s.last_full = want_rows[k] != 0;
    }
  for (int i = 0; i < n; ++i) {
    Seq &s = c->seqs[seq_ids[i]];
    s.g = mir[i].g; s.j_stream = mir[i].j; s.n_pending = mir[i].npend; s.len = mir[i].len;
  }
  if (h_plan[PL_ERR]) {
    int e = h_plan[PL_ERR];
    int zero = 0;  // error path only: clear the flag so that the context stays usable
    (void)hipMemcpy(at<int>(c, c->lo.plan) + PL_ERR, &zero, sizeof(int), hipMemcpyHostToDevice);
    if (e & ERR_NAN) return fail(c, SPARK_ENAN, "a head produced a NaN logit");
    return fail(c, SPARK_ESTATE, "device saw an inactive sequence");
  }
  return SPARK_OK;
}

template <typename WT> int prefill_rows(spark_ctx *c, int id, const int32_t *prompt, int n_rows) {
  const spark_config &g = c->cfg;
  const int base_slot = g.max_batch * c->dv.rmax;
  std::vector<RowDesc> rows(PREFILL_CHUNK);
  RowDesc *rows_dev = at<RowDesc>(c, c->lo.prefill_rows);
  int *tok_dev = at<int>(c, c->lo.prefill_tokens);
  int rc;
  for (int p0 = 0; p0 < n_rows; p0 += c->prefill_chunk) {
    const int m = std::min(c->prefill_chunk, n_rows - p0);
    for (int r = 0; r < m; ++r) rows[r] = RowDesc{base_slot + r, id, p0 + r, -1};
    HIP_TRY(c, hipMemcpyAsync(rows_dev, rows.data(), sizeof(RowDesc) * m, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(tok_dev, prompt + p0, sizeof(int) * m, hipMemcpyHostToDevice, c->stream));
    embed_rows_k<WT><<<m, 256, 0, c->stream>>>(rows_dev, nullptr, tok_dev, (const WT *)c->w.embed,
                                               g.d_model, at<float>(c, c->lo.hidden));
    HIP_TRY(c, hipGetLastError());
    c->attn_splits_now = (p0 + m - 1) / ATTN_SLICE + 1;
    if ((rc = run_layers<WT>(c, 0, g.n_layers, rows_dev, m))) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  return SPARK_OK;
}

}  // namespace

extern "C" {

int spark_workspace_bytes(const spark_config *cfg, size_t *kv_pool_bytes, size_t *scratch_bytes) {
  char why[128];
  if (!cfg || !config_ok(cfg, why, sizeof(why))) return SPARK_EINVAL;
  Derived d;
  Layout l;
  derive(*cfg, d);
  layout(*cfg, d, l);
  if (kv_pool_bytes) *kv_pool_bytes = d.kv_pool_bytes;
  if (scratch_bytes) *scratch_bytes = l.total_tiled;
  return SPARK_OK;
}

int spark_schedule_preview(const spark_config *cfg, int32_t cycle_offset, int32_t text_budget,
                           int32_t n_steps, int32_t *depth_out, int32_t *is_text_out) {
  char why[128];
  if (!cfg || !config_ok(cfg, why, sizeof(why)) || cycle_offset < 0 || n_steps < 0 || !depth_out ||
      !is_text_out || (text_budget > 0 && cfg->n_text < 1))
    return SPARK_EINVAL;
  const SchedParams sp = sched_params(cfg);
  int j_stream = 0;
  for (int g = 0; g < n_steps; ++g) {
    int is_text, full;
    schedule_decide(sp, g, cycle_offset, j_stream, text_budget, sp.phase, is_text, full);   // the function the device runs
    depth_out[g] = full ? cfg->n_layers : cfg->exit_layer;
    is_text_out[g] = is_text;
    if (!is_text) ++j_stream;
  }
  return SPARK_OK;
}

namespace {

// What spark_init and spark_init_static share.  `pinned`: the staging buffers for ids, forced tokens
// and results are pinned host memory (hipHostMalloc); otherwise they are ordinary host arrays.
int init_context(const spark_config *cfg, const spark_weights *weights, void *kv_pool, size_t kv_pool_bytes,
                 void *scratch, size_t scratch_bytes, void *hip_stream, bool static_scratch, spark_ctx **out) {
  spark_ctx *c = new spark_ctx();
  c->cfg = *cfg;
  c->w = *weights;
  c->err[0] = 0;
  derive(*cfg, c->dv);
  layout(*cfg, c->dv, c->lo);
  if (!kv_pool || !scratch || kv_pool_bytes < c->dv.kv_pool_bytes || scratch_bytes < c->lo.total ||
      ((uintptr_t)kv_pool & 255) || ((uintptr_t)scratch & 255)) {
    delete c;
    return SPARK_ENOMEM;
  }
  c->stream = (hipStream_t)hip_stream;
  c->scratch = (char *)scratch;
  c->kv_pool = kv_pool;
  c->static_scratch = static_scratch;
  c->sp = sched_params(cfg);
  c->seqs.resize(cfg->max_batch);
  for (int p = c->dv.n_pages_total - 1; p >= 0; --p) c->free_pages.push_back(p);
  c->h_in = c->h_out = nullptr;
  auto bail = [&](int code) { spark_destroy(c); return code; };
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return bail(SPARK_EHIP);
  c->device = dev;
  c->n_cu = prop.multiProcessorCount;
  // the MFMA kernels load 16-byte vectors of 8 weights; other widths stay on the vector kernel
  c->mfma_ok = cfg->d_model % 8 == 0 && (cfg->n_q_heads * cfg->head_dim) % 8 == 0 && cfg->d_ffn % 8 == 0;
  c->use_mfma = c->mfma_ok;
  // a scratch area of the full size holds the MFMA-ordered copy of the projection weights (the
  // static area never does)
  tiled_map(*cfg, c->dv, c->tm);
  c->has_tiled = !static_scratch && c->tm.total > 0 && scratch_bytes >= c->lo.total_tiled;
  // Prompt rows per pass: on the MFMA path the widest projection (gate/up) is cut into tiles of 256
  // weight-row pairs x 64 prompt rows; the row count is chosen so that one round of tiles about
  // fills the chip, which needs no k split and no second kernel for that projection.
  if (c->use_mfma && cfg->dtype == SPARK_DTYPE_BF16) {
    const int x_tiles = (cfg->d_ffn + MG_TASKS_PER_BLOCK - 1) / MG_TASKS_PER_BLOCK;
    c->prefill_chunk = std::max(128, std::min(PREFILL_CHUNK, 64 * (c->n_cu / std::max(1, x_tiles))));
  }
  size_t in_ints = (size_t)cfg->max_batch * (1 + MAX_STEPS_PER_CALL);
  size_t out_ints = (size_t)cfg->max_batch * 2 * MAX_STEPS_PER_CALL + PL_WORDS;
  if (static_scratch) {   // this variant allocates nothing through the HIP runtime
    c->h_in = new (std::nothrow) int[in_ints];
    c->h_out = new (std::nothrow) int[out_ints];
    if (!c->h_in || !c->h_out) return bail(SPARK_ENOMEM);
  } else if (hipHostMalloc((void **)&c->h_in, sizeof(int) * in_ints, hipHostMallocDefault) != hipSuccess ||
             hipHostMalloc((void **)&c->h_out, sizeof(int) * out_ints, hipHostMallocDefault) != hipSuccess) {
    return bail(SPARK_EHIP);
  }
  // device state, rotary table.  Everything up to the hidden-state arena starts at zero: sequence
  // state, page table, plan and error word, and the counters that kernels hand to the next launch
  // at zero (attention arrivals, the sampler's histogram, arrivals and candidate counts).  The
  // scratch area may hold another context's leftovers (the static array always does).
  if (hipMemsetAsync(c->scratch + c->lo.state, 0, c->lo.hidden - c->lo.state, c->stream) != hipSuccess)
    return bail(SPARK_EHIP);
  const int half = cfg->head_dim / 2;
  std::vector<float> inv(half);
  for (int i = 0; i < half; ++i)
    inv[i] = (float)pow((double)cfg->rope_base, -2.0 * i / (double)cfg->head_dim);
  if (hipMemcpyAsync(c->scratch + c->lo.inv_freq, inv.data(), sizeof(float) * half,
                     hipMemcpyHostToDevice, c->stream) != hipSuccess)
    return bail(SPARK_EHIP);
  int total = half * cfg->max_seq_len;
  rope_table_k<<<(total + 255) / 256, 256, 0, c->stream>>>(at<float>(c, c->lo.inv_freq), half,
                                                          cfg->max_seq_len, at<float2>(c, c->lo.rope));
  if (hipGetLastError() != hipSuccess || hipStreamSynchronize(c->stream) != hipSuccess)
    return bail(SPARK_EHIP);
  if (c->has_tiled && build_tiled(c) != SPARK_OK) return bail(SPARK_EHIP);
  *out = c;
  return SPARK_OK;
}

bool init_args_ok(const spark_config *cfg, const spark_weights *weights) {
  char why[128];
  if (!cfg || !weights || !config_ok(cfg, why, sizeof(why))) return false;
  const void *const *wp = (const void *const *)weights;
  for (size_t i = 0; i < sizeof(spark_weights) / sizeof(void *); ++i)
    if (!wp[i]) return false;
  return true;
}

}  // namespace

// The scratch area of spark_init_static: one array per GPU the library is loaded on, held until the
// process ends.  In host code the name `static_scratch_area` is a handle for hipGetSymbolAddress,
// not an address: the per-device address is looked up once and kept in static_scratch_ptr.
static __device__ __align__(256) unsigned char static_scratch_area[SPARK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
char *static_scratch_ptr[MAX_DEVICES] = {nullptr};
bool static_scratch_busy[MAX_DEVICES] = {false};
}  // namespace

int spark_init(const spark_config *cfg, const spark_weights *weights, void *kv_pool,
               size_t kv_pool_bytes, void *scratch, size_t scratch_bytes, void *hip_stream,
               spark_ctx **out) {
  if (!out) return SPARK_EINVAL;
  *out = nullptr;
  if (!init_args_ok(cfg, weights)) return SPARK_EINVAL;
  return init_context(cfg, weights, kv_pool, kv_pool_bytes, scratch, scratch_bytes, hip_stream, false, out);
}

int spark_init_static(const spark_config *cfg, const spark_weights *weights, void *kv_pool,
                      size_t kv_pool_bytes, void *hip_stream, spark_ctx **out) {
  if (!out) return SPARK_EINVAL;
  *out = nullptr;
  if (!init_args_ok(cfg, weights)) return SPARK_EINVAL;
  Derived d;
  Layout l;
  derive(*cfg, d);
  layout(*cfg, d, l);
  if (l.total > (size_t)SPARK_STATIC_SCRATCH_BYTES) {
    fprintf(stderr, "spark_init_static: this configuration needs %zu bytes of scratch, the static area holds %zu\n",
            l.total, (size_t)SPARK_STATIC_SCRATCH_BYTES);
    return SPARK_ENOMEM;
  }
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SPARK_EHIP;
  if (static_scratch_busy[dev]) {
    fprintf(stderr, "spark_init_static: device %d already has a live context on the static scratch area\n", dev);
    return SPARK_ESTATE;
  }
  if (!static_scratch_ptr[dev]) {   // once per device, with that device current
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch_area)) != hipSuccess || !p) return SPARK_EHIP;
    static_scratch_ptr[dev] = (char *)p;
  }
  int rc = init_context(cfg, weights, kv_pool, kv_pool_bytes, static_scratch_ptr[dev],
                        (size_t)SPARK_STATIC_SCRATCH_BYTES, hip_stream, true, out);
  if (rc == SPARK_OK) static_scratch_busy[dev] = true;
  return rc;
}

int spark_tune(spark_ctx *c, const char *name, int32_t value) {
  if (!c || !name) return SPARK_EINVAL;
  const std::string k(name);
  if (k == "mfma") c->use_mfma = value != 0 && c->mfma_ok;
  else if (k == "mfma_min_rows") c->mfma_min_rows = std::max(1, (int)value);
  else if (k == "mfma_small_tiles") c->mfma_small_tiles = value;
  else if (k == "mfma_xcd_max_split") c->mfma_xcd_max_split = value;
  else if (k == "attn_pieces") c->attn_pieces = std::max(0, std::min(8, (int)value));
  else if (k == "attn_mfma_min_rows") c->attn_mfma_min_rows = std::max(1, (int)value);
  else if (k == "gemv_big_kb") c->gemv_big_kb = std::max(1, (int)value);
  else if (k == "prefill_rows") c->prefill_chunk = std::max(32, std::min(PREFILL_CHUNK, (int)value / 32 * 32));
  else if (k == "mfma_small_max_k") c->mfma_small_max_k = std::max(8, (int)value);
  else if (k == "mfma_tiled") c->use_tiled = value != 0;
  else if (k == "fuse_norm") c->fuse_norm = value != 0;
  else return fail(c, SPARK_EINVAL, "unknown tuning name '%s'", name);
  return SPARK_OK;
}

int spark_seq_open(spark_ctx *c, int32_t cycle_offset, int32_t *seq_id) {
  if (!c || !seq_id) return SPARK_EINVAL;
  if (cycle_offset < 0) return fail(c, SPARK_EINVAL, "cycle_offset < 0");
  for (int i = 0; i < (int)c->seqs.size(); ++i)
    if (!c->seqs[i].open) {
      c->seqs[i] = Seq();
      c->seqs[i].open = true;
      c->seqs[i].cycle_offset = cycle_offset % (c->cfg.n_text + c->cfg.n_speech);
      c->seqs[i].phase = c->cfg.phase;
      *seq_id = i;
      return SPARK_OK;
    }
  return fail(c, SPARK_ENOSEQ, "all %d sequence slots are open", (int)c->seqs.size());
}

int spark_prefill(spark_ctx *c, int32_t seq_id, const int32_t *prompt, int32_t n) {
  if (!c) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  if (s->prefilled) return fail(c, SPARK_ESTATE, "sequence %d already has a prompt", seq_id);
  if (!prompt || n < 1) return fail(c, SPARK_EINVAL, "empty prompt");
  if (n > c->cfg.max_seq_len) return fail(c, SPARK_ENOMEM, "prompt longer than max_seq_len");
  for (int i = 0; i < n; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->dv.V) return fail(c, SPARK_EINVAL, "prompt id out of range");
  int rc = ensure_pages(c, seq_id, n - 1);
  if (rc) return rc;
  if (n > 1) {
    rc = c->cfg.dtype == SPARK_DTYPE_BF16 ? prefill_rows<bf16_t>(c, seq_id, prompt, n - 1)
                                          : prefill_rows<float>(c, seq_id, prompt, n - 1);
    if (rc) return rc;
  }
  int st[ST_WORDS] = {0};
  st[ST_LEN] = n - 1;
  st[ST_OFFSET] = s->cycle_offset;
  st[ST_NEXT] = prompt[n - 1];
  st[ST_ACTIVE] = 1;
  st[ST_TEXTBUDGET] = s->text_budget;
  st[ST_PHASE] = s->phase;
  HIP_TRY(c, hipMemcpyAsync(at<int>(c, c->lo.state) + (size_t)seq_id * ST_WORDS, st, sizeof(st),
                            hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  s->len = n - 1;
  s->prefilled = true;
  return SPARK_OK;
}

int spark_decode_sampled(spark_ctx *c, int32_t n_steps, int32_t n, const int32_t *seq_ids,
                         const int32_t *forced_next, const uint64_t *rand_words,
                         int32_t *out_tokens, int32_t *out_depth) {
  if (!c) return SPARK_EINVAL;
  if (n < 1 || n > c->cfg.max_batch || n_steps < 1 || !seq_ids || !out_tokens || !out_depth)
    return fail(c, SPARK_EINVAL, "bad batch (n=%d, n_steps=%d)", n, n_steps);
  for (int s0 = 0; s0 < n_steps; s0 += MAX_STEPS_PER_CALL) {
    int steps = std::min(MAX_STEPS_PER_CALL, n_steps - s0);
    int rc = decode_chunk(c, steps, n, seq_ids, forced_next ? forced_next + (size_t)s0 * n : nullptr,
                          rand_words ? rand_words + (size_t)s0 * n : nullptr,
                          out_tokens + (size_t)s0 * n, out_depth + (size_t)s0 * n);
    if (rc) return rc;
  }
  return SPARK_OK;
}

int spark_decode(spark_ctx *c, int32_t n_steps, int32_t n, const int32_t *seq_ids,
                 const int32_t *forced_next, int32_t *out_tokens, int32_t *out_depth) {
  return spark_decode_sampled(c, n_steps, n, seq_ids, forced_next, nullptr, out_tokens, out_depth);
}

int spark_set_sampling(spark_ctx *c, float temperature, float top_p) {
  if (!c) return SPARK_EINVAL;
  if (!(temperature > 0.f)) {
    c->temperature = c->top_p = 0.f;
    return SPARK_OK;
  }
  if (!(top_p > 0.f) || top_p > 1.f) return fail(c, SPARK_EINVAL, "top_p outside (0, 1]");
  c->temperature = temperature;
  c->top_p = top_p;
  return SPARK_OK;
}

int spark_step(spark_ctx *c, int32_t n, const int32_t *seq_ids, const int32_t *forced_next,
               int32_t *out_tokens, int32_t *out_depth) {
  return spark_decode(c, 1, n, seq_ids, forced_next, out_tokens, out_depth);
}

int spark_get_logits(spark_ctx *c, int32_t seq_id, float *out_logits, int32_t *head) {
  if (!c || !out_logits) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  if (!s->g) return fail(c, SPARK_ESTATE, "sequence %d has not been stepped", seq_id);
  // logits rows are indexed by the position of the sequence in the last batch
  std::vector<int> ids(c->cfg.max_batch);
  HIP_TRY(c, hipMemcpy(ids.data(), at<int>(c, c->lo.seq_ids), sizeof(int) * c->cfg.max_batch,
                       hipMemcpyDeviceToHost));
  int row = -1;
  for (int i = 0; i < c->cfg.max_batch; ++i)
    if (ids[i] == seq_id) { row = i; break; }
  if (row < 0) return fail(c, SPARK_ESTATE, "sequence %d was not in the last step", seq_id);
  HIP_TRY(c, hipMemcpy(out_logits, at<float>(c, c->lo.logits) + (size_t)row * c->dv.V,
                       sizeof(float) * c->dv.V, hipMemcpyDeviceToHost));
  if (head) *head = s->last_full ? c->cfg.n_layers : c->cfg.exit_layer;
  return SPARK_OK;
}

int spark_get_kv(spark_ctx *c, int32_t seq_id, int32_t layer, int32_t pos, float *k_out,
                 float *v_out) {
  if (!c || !k_out || !v_out) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  const spark_config &g = c->cfg;
  if (layer < 0 || layer >= g.n_layers || pos < 0 || pos >= s->len)
    return fail(c, SPARK_EINVAL, "layer or position out of range");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  const int pt = g.kv_page_tokens, hd = g.head_dim, esz = c->dv.esz;
  const int page = s->pages[pos / pt];
  std::vector<unsigned char> raw((size_t)hd * esz);
  for (int which = 0; which < 2; ++which)
    for (int h = 0; h < g.n_kv_heads; ++h) {
      size_t o = (size_t)page * g.n_layers + layer;
      o = (o * 2 + which) * g.n_kv_heads + h;
      o = (o * pt + pos % pt) * hd;
      HIP_TRY(c, hipMemcpy(raw.data(), (const char *)c->kv_pool + o * esz, (size_t)hd * esz,
                           hipMemcpyDeviceToHost));
      float *dst = (which ? v_out : k_out) + (size_t)h * hd;
      for (int i = 0; i < hd; ++i) {
        if (esz == 2) {
          uint32_t u = (uint32_t)((const uint16_t *)raw.data())[i] << 16;
          memcpy(dst + i, &u, 4);
        } else {
          dst[i] = ((const float *)raw.data())[i];
        }
      }
    }
  return SPARK_OK;
}

int spark_seq_text_budget(spark_ctx *c, int32_t seq_id, int32_t n_text_tokens) {
  if (!c) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  if (n_text_tokens < 1) return fail(c, SPARK_EINVAL, "text budget < 1");
  if (s->text_budget > 0) return fail(c, SPARK_ESTATE, "sequence %d already has a text budget", seq_id);
  if (n_text_tokens < s->g - s->j_stream)
    return fail(c, SPARK_EINVAL, "sequence %d has generated more text tokens already", seq_id);
  if (c->cfg.n_text < 1) return fail(c, SPARK_EINVAL, "the interleave has no text slots");
  s->text_budget = n_text_tokens;
  if (s->prefilled) {   // the state is on the device already
    HIP_TRY(c, hipMemcpyAsync(at<int>(c, c->lo.state) + (size_t)seq_id * ST_WORDS + ST_TEXTBUDGET,
                              &s->text_budget, sizeof(int), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  return SPARK_OK;
}

namespace {
int set_phase(spark_ctx *c, int seq_id, Seq *s, int phase) {
  s->phase = phase;
  if (s->prefilled) {   // the state is on the device already
    HIP_TRY(c, hipMemcpyAsync(at<int>(c, c->lo.state) + (size_t)seq_id * ST_WORDS + ST_PHASE, &s->phase,
                              sizeof(int), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  return SPARK_OK;
}
}  // namespace

int spark_seq_set_phase(spark_ctx *c, int32_t seq_id, int32_t phase) {
  if (!c) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  if (phase < 0 || phase >= c->cfg.period_k) return fail(c, SPARK_EINVAL, "phase outside [0, period_k)");
  // a moved phase can join two runs of early exits: K-1 before and K-1 after the move, which the
  // pending slots hold; runs that early-exited text positions could extend further are not allowed
  if (c->cfg.text_period_k > 1) return fail(c, SPARK_EINVAL, "the phase cannot be moved when text exits early too");
  if (c->cfg.scope == SPARK_SCOPE_CHUNK && c->cfg.exit_layer < c->cfg.n_layers) {
    // per-chunk counters repeat with the cycle: the moved phase needs a full-depth slot in it, and
    // its runs of early exits, joined with the K-1 that may be pending from before the move, must
    // fit the pending slots (the check spark_init makes for the configuration's own phase)
    const int cyc = c->cfg.n_text + c->cfg.n_speech;
    int run = 0, longest = 0;
    bool any_full = false;
    for (int g = 0; g < 2 * cyc; ++g) {
      int is_text, full;
      schedule_decide(c->sp, g, 0, 0, 0, phase, is_text, full);
      if (full) { any_full = true; run = 0; } else { longest = std::max(longest, ++run); }
    }
    if (!any_full) return fail(c, SPARK_EINVAL, "with phase %d no slot of the cycle would run full depth", phase);
    if (longest + c->cfg.period_k > pending_slots(&c->cfg))
      return fail(c, SPARK_EINVAL, "with phase %d a run of early exits would outgrow the pending slots", phase);
  }
  return set_phase(c, seq_id, s, phase);
}

int spark_align_phases(spark_ctx *c, int32_t n, const int32_t *seq_ids) {
  if (!c || n < 1 || !seq_ids) return SPARK_EINVAL;
  if (c->cfg.scope != SPARK_SCOPE_STREAM) return fail(c, SPARK_EINVAL, "phases are aligned over stream counters only");
  if (c->cfg.text_period_k > 1) return fail(c, SPARK_EINVAL, "the phase cannot be moved when text exits early too");
  for (int i = 0; i < n; ++i)
    if (!find_seq(c, seq_ids[i])) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_ids[i]);
  const int K = c->cfg.period_k;
  for (int i = 0; i < n; ++i) {
    Seq *s = find_seq(c, seq_ids[i]);
    // the K-th speech position from now runs full depth, for every sequence alike
    if (int rc = set_phase(c, seq_ids[i], s, (s->j_stream + K - 1) % K)) return rc;
  }
  return SPARK_OK;
}

int spark_seq_state(spark_ctx *c, int32_t seq_id, int32_t *len, int32_t *upper_valid,
                    int32_t *n_pending) {
  if (!c) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  // the device copy is authoritative
  int st[ST_WORDS];
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipMemcpy(st, at<int>(c, c->lo.state) + (size_t)seq_id * ST_WORDS, sizeof(st),
                       hipMemcpyDeviceToHost));
  if (s->prefilled && (st[ST_LEN] != s->len || st[ST_NPENDING] != s->n_pending))
    return fail(c, SPARK_ESTATE, "device state and host mirror disagree");
  if (len) *len = s->len;
  if (upper_valid) *upper_valid = s->len - s->n_pending;
  if (n_pending) *n_pending = s->n_pending;
  return SPARK_OK;
}

int spark_get_stats(spark_ctx *c, int32_t seq_id, spark_stats *out) {
  if (!c || !out) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  memset(out, 0, sizeof(*out));
  out->text_steps = s->text_steps;
  out->speech_full_steps = s->speech_full;
  out->speech_ee_steps = s->speech_ee;
  memcpy(out->flush_rows, s->flush_rows, sizeof(out->flush_rows));
  const double L = c->cfg.n_layers, e = c->cfg.exit_layer;
  out->text_ee_steps = s->text_ee;
  if (s->text_steps + s->text_ee)
    out->mean_text_depth = (s->text_steps * L + s->text_ee * e) / (double)(s->text_steps + s->text_ee);
  const int64_t ns = s->speech_full + s->speech_ee;
  if (ns) {
    out->mean_speech_depth = (s->speech_full * L + s->speech_ee * e) / (double)ns;
    out->speech_layer_saving = (1.0 - out->mean_speech_depth / L) * 100.0;
  }
  return SPARK_OK;
}

int spark_seq_close(spark_ctx *c, int32_t seq_id) {
  if (!c) return SPARK_EINVAL;
  Seq *s = find_seq(c, seq_id);
  if (!s) return fail(c, SPARK_ENOSEQ, "unknown sequence id %d", seq_id);
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int p : s->pages) c->free_pages.push_back(p);
  int zero[ST_WORDS] = {0};
  HIP_TRY(c, hipMemcpy(at<int>(c, c->lo.state) + (size_t)seq_id * ST_WORDS, zero, sizeof(zero),
                       hipMemcpyHostToDevice));
  *s = Seq();
  return SPARK_OK;
}

void spark_destroy(spark_ctx *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t ev : c->prof_ev) (void)hipEventDestroy(ev);
  if (c->static_scratch) {
    delete[] c->h_in;
    delete[] c->h_out;
    if (c->device >= 0 && c->device < MAX_DEVICES) static_scratch_busy[c->device] = false;
  } else {
    if (c->h_in) (void)hipHostFree(c->h_in);
    if (c->h_out) (void)hipHostFree(c->h_out);
  }
  delete c;
}

const char *spark_last_error(const spark_ctx *c) { return c ? c->err : "null context"; }

int spark_profile_select(spark_ctx *c, int32_t kernel_class) {
  if (!c || kernel_class < -1 || kernel_class >= SPARK_KC_COUNT) return SPARK_EINVAL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->prof_class = kernel_class;
  c->prof_used = 0;
  return SPARK_OK;
}

int spark_profile_read(spark_ctx *c, int64_t *n_launches, double *total_ms, double *empty_ms) {
  if (!c || !n_launches || !total_ms) return SPARK_EINVAL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  double tot = 0, empty = 0;
  for (size_t i = 0; i + 2 < c->prof_used; i += 3) {
    float ms = 0, ms0 = 0;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->prof_ev[i], c->prof_ev[i + 1]));
    HIP_TRY(c, hipEventElapsedTime(&ms0, c->prof_ev[i + 1], c->prof_ev[i + 2]));
    tot += ms;
    empty += ms0;
  }
  *n_launches = (int64_t)(c->prof_used / 3);
  *total_ms = tot;
  if (empty_ms) *empty_ms = empty;   // what the brackets themselves cost
  c->prof_used = 0;
  return SPARK_OK;
}

int spark_measure_read(spark_ctx *c, const void *buf, size_t bytes, int32_t reps, int32_t nontemporal,
                       double *gbps, uint32_t *checksum) {
  if (!c || !buf || !gbps || reps < 1) return SPARK_EINVAL;
  if (bytes < 16 || bytes % 16 || ((uintptr_t)buf & 15)) return fail(c, SPARK_EINVAL, "buffer must be 16-byte aligned and sized");
  // the wave sums go where the attention partials live between steps (at least 69 KB)
  const int blocks = c->n_cu * 8, words = blocks * (READ_THREADS / 64);
  const size_t part_bytes = c->lo.act - c->lo.part;
  if (sizeof(unsigned) * words > part_bytes) return fail(c, SPARK_ENOMEM, "scratch too small for the read kernel's sums");
  unsigned *sink = at<unsigned>(c, c->lo.part);
  const read_u32x4 *p = (const read_u32x4 *)buf;
  const size_t n16 = bytes / 16;
  hipEvent_t e0, e1;
  HIP_TRY(c, hipEventCreate(&e0));
  HIP_TRY(c, hipEventCreate(&e1));
  auto launch = [&]() {
    if (nontemporal) read_stream_k<true><<<blocks, READ_THREADS, 0, c->stream>>>(p, n16, sink);
    else read_stream_k<false><<<blocks, READ_THREADS, 0, c->stream>>>(p, n16, sink);
  };
  launch();   // untimed: code object, TLB
  int rc = SPARK_OK;
  float ms = 0.f;
  if (hipEventRecord(e0, c->stream) != hipSuccess) rc = SPARK_EHIP;
  for (int r = 0; r < reps && rc == SPARK_OK; ++r) launch();
  if (rc == SPARK_OK && (hipGetLastError() != hipSuccess || hipEventRecord(e1, c->stream) != hipSuccess ||
                         hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = SPARK_EHIP;
  if (rc == SPARK_OK && checksum) {
    std::vector<unsigned> h(words);
    if (hipMemcpy(h.data(), sink, sizeof(unsigned) * words, hipMemcpyDeviceToHost) != hipSuccess) rc = SPARK_EHIP;
    unsigned x = 0;
    for (unsigned v : h) x ^= v;
    *checksum = x;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != SPARK_OK) return fail(c, rc, "the read measurement failed");
  *gbps = (double)bytes * reps / ((double)ms * 1e-3) / 1e9;
  return SPARK_OK;
}

}  // extern "C"
