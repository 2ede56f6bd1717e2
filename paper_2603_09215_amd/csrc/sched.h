// SPAR-K schedule / dispatch on the device, embedding gather, token emission.
//
// The per-sequence decoding state lives in device memory, so consecutive steps can be enqueued
// without a round trip to the host: the dispatch kernel reads the state, decides each position's
// exit layer (Sec. IV-B.1) and builds the row lists of the step (Algorithm 1); the emit kernel
// turns the argmax keys into tokens and advances the state.
#pragma once
#include "device_common.h"

namespace spark {

// device-resident per-sequence state, 10 ints
enum { ST_LEN = 0, ST_G, ST_JSTREAM, ST_NPENDING, ST_OFFSET, ST_NEXT, ST_ACTIVE, ST_LASTFULL, ST_TEXTBUDGET, ST_PHASE, ST_WORDS };
// plan words
enum { PL_NLOWER = 0, PL_NUPPER, PL_NEE, PL_NFULL, PL_ERR, PL_WORDS = 8 };
enum { ERR_NAN = 1, ERR_INACTIVE = 2 };

struct SchedParams {
  int n_layers, exit_layer, period_k, phase, scope, n_text, n_speech;
  int rmax;  // hidden-state slots per sequence (pending rows + the current one)
  int text_period_k, text_phase;  // the same rule on text positions (Sec. V-C, row G10); <= 1: text is full depth
};

// The schedule as an integer function of the sequence counters.  Generated token g falls on slot
// (g + offset) mod (n_text + n_speech) of the interleave cycle; slots [0, n_text) are text.  A
// speech position has index j inside its chunk (scope 0) or among all speech positions (scope 1);
// it runs full depth iff j mod K == phase; e == L and K == 1 always run full depth.  Text runs
// full depth unless a text period is given: then the text position with index t (its slot inside
// the chunk, or the count of text positions emitted so far, g - j_stream) follows the same rule
// with (text_period_k, text_phase).
//
// The text of a response ends before its speech (Sec. IV-A: speech is 79.5 % / 81.2 % of the
// generated tokens, more than the 2/3 the interleave ratios alone give).  text_budget B > 0: once
// B text tokens have been emitted every position is speech, and the chunk then running goes on,
// so its index is the number of positions since the B-th text token.  That token's place in the
// stream follows from the cycle alone, which keeps the schedule a function of the counters.
__host__ __device__ inline int nth_text_position(const SchedParams &sp, int offset, int b /* 1-based */) {
  const int cyc = sp.n_text + sp.n_speech, off = offset % cyc;
  const int first = off < sp.n_text ? sp.n_text - off : 0;   // text slots left in the cycle entered
  if (b <= first) return b - 1;
  const int rest = b - first - 1;
  return (cyc - off) + (rest / sp.n_text) * cyc + rest % sp.n_text;
}

// speech_phase: the sequence's own phase on speech positions (sp.phase unless the caller moved it to
// line the sequence's full-depth steps up with those of the other sequences of its batch).
__host__ __device__ inline void schedule_decide(const SchedParams &sp, int g, int offset, int j_stream,
                                                int text_budget, int speech_phase, int &is_text, int &full) {
  const int cyc = sp.n_text + sp.n_speech;
  const int slot = (int)(((long long)g + offset) % cyc);
  const int texts = g - j_stream;                 // text positions so far
  const bool text_over = text_budget > 0 && texts >= text_budget;
  is_text = slot < sp.n_text && !text_over;
  const int period = is_text ? sp.text_period_k : sp.period_k;
  const int want = is_text ? sp.text_phase : speech_phase;
  int idx;
  if (is_text) idx = sp.scope == 0 ? slot : texts;
  else if (sp.scope != 0) idx = j_stream;
  else idx = text_over ? g - nth_text_position(sp, offset, text_budget) - 1 : slot - sp.n_text;
  full = sp.exit_layer == sp.n_layers || period <= 1 || idx % period == want;
}

constexpr int SCHED_THREADS = 256;  // >= max_batch

__global__ void __launch_bounds__(SCHED_THREADS)
sched_dispatch_k(SchedParams sp, int n, const int *__restrict__ seq_ids, const int *__restrict__ state,
                 RowDesc *lower, RowDesc *upper, RowDesc *ee, RowDesc *full_rows, int *plan,
                 int *step_flags, int *out_depth, unsigned long long *best) {
  __shared__ int s_m[SCHED_THREADS], s_full[SCHED_THREADS];
  __shared__ int s_uoff[SCHED_THREADS], s_hidx[SCHED_THREADS];
  const int i = threadIdx.x;
  int seq = 0, len = 0, npend = 0, is_text = 0, full = 0;
  if (i < n) {
    seq = seq_ids[i];
    const int *st = state + seq * ST_WORDS;
    len = st[ST_LEN];
    npend = st[ST_NPENDING];
    schedule_decide(sp, st[ST_G], st[ST_OFFSET], st[ST_JSTREAM], st[ST_TEXTBUDGET], st[ST_PHASE], is_text, full);
    lower[i] = RowDesc{seq * sp.rmax + npend, seq, len, i};
    out_depth[i] = full ? sp.n_layers : sp.exit_layer;
    step_flags[i] = full | (is_text << 1);
    best[i] = 0ull;
    s_m[i] = full ? npend + 1 : 0;
    s_full[i] = full;
    if (!st[ST_ACTIVE]) atomicOr(plan + PL_ERR, ERR_INACTIVE);
  }
  __syncthreads();
  if (i == 0) {
    int u = 0, ne = 0, nf = 0;
    for (int b = 0; b < n; ++b) {
      s_uoff[b] = u;
      u += s_m[b];
      s_hidx[b] = s_full[b] ? nf++ : ne++;
    }
    plan[PL_NLOWER] = n;
    plan[PL_NUPPER] = u;
    plan[PL_NEE] = ne;
    plan[PL_NFULL] = nf;
  }
  __syncthreads();
  if (i < n) {
    RowDesc cur = RowDesc{seq * sp.rmax + npend, seq, len, i};
    if (full) {
      // pending positions (oldest first) and the current one: contiguous positions len-npend..len
      for (int r = 0; r <= npend; ++r)
        upper[s_uoff[i] + r] = RowDesc{seq * sp.rmax + r, seq, len - npend + r, r == npend ? i : -1};
      full_rows[s_hidx[i]] = cur;
    } else {
      ee[s_hidx[i]] = cur;
    }
  }
}

// hidden[x_slot] = E[token]; token = the sequence's next input (decode) or tokens[r] (prefill)
template <typename WT>
__global__ void __launch_bounds__(256)
embed_rows_k(const RowDesc *__restrict__ rows, const int *__restrict__ state,
             const int *__restrict__ tokens, const WT *__restrict__ embed, int d, float *hidden) {
  const RowDesc rd = rows[blockIdx.x];
  const int tok = tokens ? tokens[blockIdx.x] : state[rd.seq * ST_WORDS + ST_NEXT];
  const WT *e = embed + (size_t)tok * d;
  float *h = hidden + (size_t)rd.x_slot * d;
  // 16 bytes per thread and trip, all trips' loads issued before the first store (a loop of
  // scalar loads pays a memory round trip per trip: fourteen of them for a 3584-wide row)
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int TRIPS = 4;
  if (d % VEC == 0 && d <= 256 * VEC * TRIPS) {
    uint4 v[TRIPS];
#pragma unroll
    for (int t = 0; t < TRIPS; ++t) {
      const int k = (t * 256 + threadIdx.x) * VEC;
      v[t] = *(const uint4 *)(e + (k < d ? k : 0));
    }
#pragma unroll
    for (int t = 0; t < TRIPS; ++t) {
      const int k = (t * 256 + threadIdx.x) * VEC;
      if (k < d) {
        float f[VEC];
        Elem<WT>::unpack(v[t], f);
#pragma unroll
        for (int i = 0; i < VEC; i += 4) *(float4 *)(h + k + i) = make_float4(f[i], f[i + 1], f[i + 2], f[i + 3]);
      }
    }
    return;
  }
  for (int k = threadIdx.x; k < d; k += 256) h[k] = Elem<WT>::widen(e[k]);
}

__global__ void __launch_bounds__(SCHED_THREADS)
emit_k(int n, const int *__restrict__ seq_ids, const int *__restrict__ forced,
       const int *__restrict__ step_flags, const unsigned long long *__restrict__ best, int *state,
       int *plan, int *out_tokens) {
  const int i = threadIdx.x;
  if (i >= n) return;
  const int seq = seq_ids[i];
  int *st = state + seq * ST_WORDS;
  const unsigned long long key = best[i];
  if ((uint32_t)(key >> 32) == 0xffffffffu || key == 0ull) atomicOr(plan + PL_ERR, ERR_NAN);
  const int tok = (int)(0xffffffffu - (uint32_t)(key & 0xffffffffull));
  const int full = step_flags[i] & 1, is_text = (step_flags[i] >> 1) & 1;
  out_tokens[i] = tok;
  const int f = forced ? forced[i] : -1;
  st[ST_LEN] += 1;
  st[ST_G] += 1;
  if (!is_text) st[ST_JSTREAM] += 1;
  st[ST_NPENDING] = full ? 0 : st[ST_NPENDING] + 1;
  st[ST_NEXT] = f >= 0 ? f : tok;
  st[ST_LASTFULL] = full;
}

// rope[pos][i] = (cos, sin)(pos * inv_freq[i]), angle formed in fp32, evaluated in fp64
__global__ void rope_table_k(const float *__restrict__ inv_freq, int half, int max_pos, float2 *rope) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= half * max_pos) return;
  int pos = idx / half, i = idx - pos * half;
  float ang = (float)pos * inv_freq[i];
  rope[idx] = make_float2((float)cos((double)ang), (float)sin((double)ang));
}

}  // namespace spark
