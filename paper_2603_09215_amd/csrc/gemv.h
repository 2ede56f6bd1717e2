// Weight-streaming projection kernel for a handful of activation rows (decode, flush).
//
// Small-batch decoding is bound by reading each layer's weights from HBM (Sec. IV-B.3, second
// paragraph), so the kernel is organised around the weight stream: every wave owns pairs of weight
// rows and walks them with 16-byte loads, 1 KiB per wave per instruction; the (few) activation
// rows sit in LDS as fp32 and are reused by every weight row; partial sums are combined with wave
// shuffles.  Up to MT activation rows share one pass over the weights, which is what makes the
// deferred completion of pending positions cost about one full-depth pass.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int GEMV_THREADS = 256;
constexpr int GEMV_WAVES = GEMV_THREADS / 64;
constexpr int GEMV_BIG_THREADS = 512;  // for launches whose activations fill the LDS of half a CU

// LDS position of activation element k (multiple of 4) of a row.  With 8 weights per lane and
// load, a lane needs x[8*lane .. 8*lane+8); storing the two float4 halves 256 floats apart makes
// consecutive lanes read consecutive 16-byte words (no bank conflicts).
template <int VEC> __device__ __forceinline__ int lds_pos(int k) {
  if (VEC == 8) return (k & ~511) + ((k >> 2) & 1) * 256 + ((k & 511) >> 3) * 4;
  return k;
}

// The last 512-element block of a staged row may be partial; lanes whose weights were masked to
// zero still multiply what lies there, so it must be finite: fill it with zeros.
template <int VEC, int NT> __device__ __forceinline__ void zero_tail(float *xrow, int klen) {
  const int end = (klen + 511) & ~511;
  for (int k = klen + threadIdx.x * 4; k < end; k += NT * 4)
    *(float4 *)(xrow + lds_pos<VEC>(k)) = make_float4(0.f, 0.f, 0.f, 0.f);
}

// The kernel hands the prologues its row descriptors with the rows beyond the pass already replaced
// by the last valid one, so rd[m] is read with the unrolled loops' constant m: an index computed
// at run time (even through a chain of selects, which the compiler turns back into an index) puts
// the array in scratch memory, a memory round trip per access.

// ------------------------------------------------------------------ prologues (fill LDS)

// rows come straight from a buffer: row r of the pass, or the row's hidden-state slot
struct ProPlain {
  const float *src;
  int stride;
  int indirect;  // 1: src row = x_slot of the row descriptor; 0: src row = pass row index
  // BATCH: loads a thread issues before it uses any.  A loop that loads, waits and stores per
  // iteration costs a memory round trip per iteration (18 of them for an MLP-width row); the
  // batch costs registers, so only the launches that have them to spare ask for more than one.
  template <int VEC, int MT, int BATCH, int NT>
  __device__ void stage(float *xs, int kc, const RowDesc *rd, int tile0, int n_valid, int k0,
                        int klen, float *red) const {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int mm = m < n_valid ? m : n_valid - 1;
      const int slot = indirect ? rd[m].x_slot : tile0 + mm;
      const float *row = src + (size_t)slot * stride + k0;
      float *xrow = xs + m * kc;
      for (int kb = threadIdx.x * 4; kb < klen; kb += NT * 4 * BATCH) {
        float4 v[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          const int k = kb + i * NT * 4;
          v[i] = *(const float4 *)(row + (k < klen ? k : 0));
        }
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          const int k = kb + i * NT * 4;
          if (k < klen) *(float4 *)(xrow + lds_pos<VEC>(k)) = v[i];
        }
      }
      zero_tail<VEC, NT>(xrow, klen);
    }
  }
};

// rows are RMSNorm(hidden[x_slot]; gamma): x / sqrt(mean x^2 + eps) * gamma  (whole row at once)
struct ProNorm {
  const float *hidden;
  const float *gamma;
  float eps;
  int d;
  int indirect;  // 1: row = x_slot of the row descriptor; 0: row = pass row index
  template <int VEC, int MT, int BATCH, int NT>
  __device__ void stage(float *xs, int kc, const RowDesc *rd, int tile0, int n_valid, int k0,
                        int klen, float *red) const {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int NI = 4096 / (NT * 4);   // 16-byte vectors per thread and row the register path holds: d <= 4096
    if (d <= NI * NT * 4) {
      // two rows at a time: their elements are requested before any is used (one memory round
      // trip per pair instead of two per row) and stay in registers between the two passes
      constexpr int RB = MT < 2 ? MT : 2;
      float4 g[NI];
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int k = threadIdx.x * 4 + i * NT * 4;
        g[i] = *(const float4 *)(gamma + (k < d ? k : 0));
      }
#pragma unroll
      for (int m0 = 0; m0 < MT; m0 += RB) {
        float4 v[RB][NI];
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          const int m = m0 + b < MT ? m0 + b : MT - 1;
          const int mm = m < n_valid ? m : n_valid - 1;
          const float *row = hidden + (size_t)(indirect ? rd[m].x_slot : tile0 + mm) * d;
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            const int k = threadIdx.x * 4 + i * NT * 4;
            v[b][i] = *(const float4 *)(row + (k < d ? k : 0));
          }
        }
        float ss[RB];
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          ss[b] = 0.f;
#pragma unroll
          for (int i = 0; i < NI; ++i)
            if (threadIdx.x * 4 + i * NT * 4 < d)
              ss[b] += v[b][i].x * v[b][i].x + v[b][i].y * v[b][i].y + v[b][i].z * v[b][i].z + v[b][i].w * v[b][i].w;
          ss[b] = wave_sum(ss[b]);
          if (lane == 0) red[wave * RB + b] = ss[b];
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          if (m0 + b < MT) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < (NT / 64); ++w) tot += red[w * RB + b];
            const float inv = 1.0f / sqrtf(tot / (float)d + eps);
            float *xrow = xs + (m0 + b) * kc;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
              const int k = threadIdx.x * 4 + i * NT * 4;
              if (k < d)
                *(float4 *)(xrow + lds_pos<VEC>(k)) =
                    make_float4(v[b][i].x * inv * g[i].x, v[b][i].y * inv * g[i].y, v[b][i].z * inv * g[i].z,
                                v[b][i].w * inv * g[i].w);
            }
            zero_tail<VEC, NT>(xrow, d);
          }
        }
        if (m0 + RB < MT) __syncthreads();   // `red` is reused by the next pair
      }
      return;
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int mm = m < n_valid ? m : n_valid - 1;
      const float *row = hidden + (size_t)(indirect ? rd[m].x_slot : tile0 + mm) * d;
      float ss = 0.f;
      for (int k = threadIdx.x * 4; k < d; k += NT * 4) {
        float4 v = *(const float4 *)(row + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      }
      ss = wave_sum(ss);
      if (lane == 0) red[wave * MT + m] = ss;
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int mm = m < n_valid ? m : n_valid - 1;
      const float *row = hidden + (size_t)(indirect ? rd[m].x_slot : tile0 + mm) * d;
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < (NT / 64); ++w) tot += red[w * MT + m];
      float inv = 1.0f / sqrtf(tot / (float)d + eps);
      for (int k = threadIdx.x * 4; k < d; k += NT * 4) {
        float4 v = *(const float4 *)(row + k);
        float4 g = *(const float4 *)(gamma + k);
        float4 o = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
        *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = o;
      }
      zero_tail<VEC, NT>(xs + m * kc, d);
    }
  }
};

// ------------------------------------------------------------------ epilogues
// Each wave task owns two weight rows; after the reduction lane m finishes activation row m.

struct NoState {};

// RMSNorm is linear in 1/rms: a projection of gamma (.) h can be scaled by 1/rms(h) afterwards.
// The launch that produces h (a residual projection's finishing step) then also writes the split
// gamma (.) h and adds the row's sum of squares, as a fixed-point integer so that the order of
// the additions does not matter, into one word per row; the next projection's epilogue reads it.
constexpr float SSQ_SCALE = 16777216.0f;   // 2^24: sums of squares up to 1e12 fit 64 bits
// words per row: the workgroups of the finishing launch add to word (workgroup % SSQ_WAYS) of the
// row, so that few atomics meet at one address (56 workgroups on one word took 5 us to drain)
constexpr int SSQ_WAYS = 8;
struct RowScale {
  const unsigned long long *ssq;   // [pass row][SSQ_WAYS] fixed-point sums of squares, nullptr: rows are normalised already
  float inv_d, eps;
  __device__ __forceinline__ float of(int r) const {
    if (!ssq) return 1.0f;
    unsigned long long w[SSQ_WAYS], tot = 0ull;
#pragma unroll
    for (int i = 0; i < SSQ_WAYS; ++i) w[i] = ssq[r * SSQ_WAYS + i];
#pragma unroll
    for (int i = 0; i < SSQ_WAYS; ++i) tot += w[i];
    return 1.0f / sqrtf((float)((double)tot * (1.0 / (double)SSQ_SCALE)) * inv_d + eps);
  }
};

// q, k, v projection + rotary embedding + KV-cache write.  Task t -> head t / (hd/2), pair index
// i = t % (hd/2): weight rows (head*hd + i) and (head*hd + i + hd/2), the two elements that the
// rotary embedding mixes.  Heads [0,nq) are queries, [nq,nq+nkv) keys, the rest values.
template <typename WT, bool DS = false> struct EpiQKV {
  typedef NoState State;
  const WT *wq, *wk, *wv;  // this layer
  int d, nq, nkv, hd, layer;
  float *qbuf;             // [pass row][nq*hd], rotated queries
  const float2 *rope;      // [pos][hd/2] (cos, sin)
  KVView kv;
  RowScale scale = RowScale{nullptr, 0.f, 0.f};
  __device__ void init(State &) const {}
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    int half = hd >> 1, head = task / half, i = task - head * half;
    const WT *base;
    int h = head;
    if (h < nq) base = wq;
    else if (h < nq + nkv) { base = wk; h -= nq; }
    else { base = wv; h -= nq + nkv; }
    r0 = base + (size_t)(h * hd + i) * d;
    r1 = r0 + (size_t)half * d;
  }
  __device__ void finish(int task, int r, const RowDesc &rd, float y0, float y1, State &) const {
    int half = hd >> 1, head = task / half, i = task - head * half;
    if (scale.ssq) { const float inv = scale.of(r); y0 *= inv; y1 *= inv; }
    if (head < nq + nkv) {
      float2 cs = rope[(size_t)rd.pos * half + i];
      float a = y0 * cs.x - y1 * cs.y, b = y1 * cs.x + y0 * cs.y;
      y0 = a; y1 = b;
    }
    if (head < nq) {
      float *q = qbuf + (size_t)r * nq * hd + head * hd + i;
      store_maybe_ds<DS>(q, y0);
      store_maybe_ds<DS>(q + half, y1);
    } else {
      int which = head < nq + nkv ? 0 : 1;
      int h = head - nq - which * nkv;
      WT *dst = (WT *)kv.pool + kv_elem_offset(kv, rd.seq, rd.pos, layer, which, h) + i;
      store_maybe_ds<DS>(dst, Elem<WT>::narrow(y0));
      store_maybe_ds<DS>(dst + half, Elem<WT>::narrow(y1));
    }
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};

// hidden[x_slot][i] += y  (attention output projection, MLP down projection)
template <typename WT, bool DS = false> struct EpiResidual {
  typedef NoState State;
  const WT *w;
  int n_in, n_out;
  float *hidden;
  int d;
  __device__ void init(State &) const {}
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    r0 = w + (size_t)(2 * task) * n_in;
    r1 = r0 + n_in;
  }
  __device__ void finish(int task, int r, const RowDesc &rd, float y0, float y1, State &) const {
    float *h = hidden + (size_t)rd.x_slot * d + 2 * task;
    float2 v = load2_maybe_ds<DS>(h);
    v.x += y0; v.y += y1;
    store2_maybe_ds<DS>(h, v);
  }
  // the same in two halves, for a caller that fetches the old value long before the sum is ready
  typedef float2 Old;
  __device__ float2 load_old(int task, const RowDesc &rd) const {
    return load2_maybe_ds<DS>(hidden + (size_t)rd.x_slot * d + 2 * task);
  }
  __device__ void finish_old(int task, int r, const RowDesc &rd, float y0, float y1, float2 old, State &) const {
    store2_maybe_ds<DS>(hidden + (size_t)rd.x_slot * d + 2 * task, make_float2(old.x + y0, old.y + y1));
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};
// hidden[x_slot][i] += y as above, and what the next projection needs of the new hidden state
// h: the three bf16 parts of gamma (.) h for pass row r, and h's sum of squares (see RowScale).
// For the finishing launch of a k-split projection, whose threads of one row are 32 lanes apart.
template <typename WT> struct EpiResidualNorm {
  struct State { float ssq; };
  const WT *w;
  int n_in, n_out;
  float *hidden;
  int d;
  const float *gamma;          // gain of the norm that follows
  SplitOut so;                 // where the split gamma (.) h goes
  unsigned long long *ssq;     // [pass row][SSQ_WAYS], zero before the launch
  __device__ void init(State &s) const { s.ssq = 0.f; }
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    r0 = w + (size_t)(2 * task) * n_in;
    r1 = r0 + n_in;
  }
  __device__ void finish(int task, int r, const RowDesc &rd, float y0, float y1, State &s) const {
    float *h = hidden + (size_t)rd.x_slot * d + 2 * task;
    float2 v = *(const float2 *)h;
    v.x += y0; v.y += y1;
    *(float2 *)h = v;
    s.ssq += v.x * v.x + v.y * v.y;
    const float2 g = *(const float2 *)(gamma + 2 * task);
    split_store2(so, r, 2 * task, v.x * g.x, v.y * g.y);
  }
  // the old value and the gains, requested together long before the sums are ready
  typedef float4 Old;
  __device__ float4 load_old(int task, const RowDesc &rd) const {
    const float2 v = *(const float2 *)(hidden + (size_t)rd.x_slot * d + 2 * task);
    const float2 g = *(const float2 *)(gamma + 2 * task);
    return make_float4(v.x, v.y, g.x, g.y);
  }
  __device__ void finish_old(int task, int r, const RowDesc &rd, float y0, float y1, float4 o, State &s) const {
    const float2 v = make_float2(o.x + y0, o.y + y1);
    *(float2 *)(hidden + (size_t)rd.x_slot * d + 2 * task) = v;
    s.ssq += v.x * v.x + v.y * v.y;
    split_store2(so, r, 2 * task, v.x * o.z, v.y * o.w);
  }
  // `sum`: the states of the threads that finished tasks of row r in this workgroup, added up
  __device__ void add_row_sum(int r, float sum) const {
    atomicAdd(ssq + r * SSQ_WAYS + (blockIdx.x % SSQ_WAYS), (unsigned long long)(sum * SSQ_SCALE + 0.5f));
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};
template <typename E> struct EpiHasRowSum { static constexpr bool value = false; };
template <typename WT> struct EpiHasRowSum<EpiResidualNorm<WT>> { static constexpr bool value = true; };

template <typename E> struct EpiHasLocalReduce { static constexpr bool value = false; };

template <typename E> struct EpiReadsOld { static constexpr bool value = false; };
template <typename WT, bool DS> struct EpiReadsOld<EpiResidual<WT, DS>> { static constexpr bool value = true; };
template <typename WT> struct EpiReadsOld<EpiResidualNorm<WT>> { static constexpr bool value = true; };

// act[r][i] = silu(Wg_i . n) * (Wu_i . n)
template <typename WT, bool DS = false> struct EpiSwiGLU {
  typedef NoState State;
  const WT *wg, *wu;
  int d, F;
  float *act;  // [pass row][F]
  __device__ void init(State &) const {}
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    r0 = wg + (size_t)task * d;
    r1 = wu + (size_t)task * d;
  }
  __device__ void finish(int task, int r, const RowDesc &, float y0, float y1, State &) const {
    float s = y0 / (1.0f + expf(-y0));
    store_maybe_ds<DS>(act + (size_t)r * F + task, s * y1);
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};

// the same, written as the three bf16 parts the down projection's MFMA kernel reads (no fp32 copy)
template <typename WT> struct EpiSwiGLUSplit {
  typedef NoState State;
  const WT *wg, *wu;
  int d, F;
  SplitOut so;
  RowScale scale = RowScale{nullptr, 0.f, 0.f};
  __device__ void init(State &) const {}
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    r0 = wg + (size_t)task * d;
    r1 = wu + (size_t)task * d;
  }
  __device__ void finish(int task, int r, const RowDesc &, float y0, float y1, State &) const {
    if (scale.ssq) { const float inv = scale.of(r); y0 *= inv; y1 *= inv; }
    float s = y0 / (1.0f + expf(-y0));
    split_store1(so, r, task, s * y1);
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};

// u[r][i] = h[i] + (A h)[i] + b[i]   (translator of the layer-specific head)
template <typename WT> struct EpiLensAffine {
  typedef NoState State;
  const WT *a;
  const float *b;
  const float *hidden;
  float *u;  // [pass row][d]
  int d;
  __device__ void init(State &) const {}
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    r0 = a + (size_t)(2 * task) * d;
    r1 = r0 + d;
  }
  __device__ void finish(int task, int r, const RowDesc &rd, float y0, float y1, State &) const {
    const float *h = hidden + (size_t)rd.x_slot * d + 2 * task;
    float2 o = make_float2(h[0] + y0 + b[2 * task], h[1] + y1 + b[2 * task + 1]);
    *(float2 *)(u + (size_t)r * d + 2 * task) = o;
  }
  __device__ void end(int, const RowDesc &, State &) const {}
};

// logits[out_idx][i] = y, and a running (max logit, lowest index) per activation row; one 64-bit
// atomic max per wave and row at the end makes the result independent of the order of arrival.
template <typename WT> struct EpiVocab {
  struct State { unsigned long long best; };
  const WT *w;
  int d, V;
  float *logits;               // [out_idx][V]
  unsigned long long *best;    // [out_idx]
  __device__ void init(State &s) const { s.best = 0ull; }
  __device__ void weight_rows(int task, const WT *&r0, const WT *&r1) const {
    int i1 = 2 * task + 1 < V ? 2 * task + 1 : 2 * task;
    r0 = w + (size_t)(2 * task) * d;
    r1 = w + (size_t)i1 * d;
  }
  __device__ void finish(int task, int r, const RowDesc &rd, float y0, float y1, State &s) const {
    float *lg = logits + (size_t)rd.out_idx * V;
    int i0 = 2 * task;
    lg[i0] = y0;
    unsigned long long k = argmax_key(y0, i0);
    if (k > s.best) s.best = k;
    if (i0 + 1 < V) {
      lg[i0 + 1] = y1;
      k = argmax_key(y1, i0 + 1);
      if (k > s.best) s.best = k;
    }
  }
  __device__ void end(int r, const RowDesc &rd, State &s) const {
    if (s.best) atomicMax(best + rd.out_idx, s.best);
  }
  // the same in two steps, for a caller that first combines the states of several threads that
  // serve one activation row in a word of LDS (zero = nothing yet)
  __device__ void reduce_local(const State &s, unsigned long long *lds_word) const {
    if (s.best) atomicMax(lds_word, s.best);
  }
  __device__ void end_reduced(const RowDesc &rd, unsigned long long key) const {
    atomicMax(best + rd.out_idx, key);
  }
};

template <typename WT> struct EpiHasLocalReduce<EpiVocab<WT>> { static constexpr bool value = true; };

// ------------------------------------------------------------------ the kernel

// 16-byte streaming load of weights: read once per step, so keep them out of the way of the
// activations and KV that live in L2 (non-temporal hint)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_weights16(const void *p) {
  u32x4_t t = __builtin_nontemporal_load((const u32x4_t *)p);
  return make_uint4(t.x, t.y, t.z, t.w);
}

constexpr int GEMV_U = 2;  // 16-byte loads per weight row and pipeline stage (many waves per CU)
constexpr int GEMV_D = 2;  // stages in the register ring (measured: 2 beats 3 when many waves share a CU)

// One pipeline stage of weights: U consecutive 1 KiB segments of both rows of a task.
template <int U> struct WStage {
  uint4 a[U], b[U];
};

// Issue the loads of elements [kb, kb + U*WSTEP) of a chunk of length klen (lanes beyond klen and
// waves without a task get zeros).
template <typename WT, int U>
__device__ __forceinline__ void issue_stage(WStage<U> &s, const WT *p0, const WT *p1, int kb, int klen,
                                            int lane, bool valid) {
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int WSTEP = 64 * VEC;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int k = kb + u * WSTEP + lane * VEC;
    if (valid && k < klen) {
      s.a[u] = load_weights16(p0 + k);
      s.b[u] = load_weights16(p1 + k);
    } else {
      s.a[u] = make_uint4(0, 0, 0, 0);
      s.b[u] = make_uint4(0, 0, 0, 0);
    }
  }
}

template <typename WT, int MT>
__device__ __forceinline__ void fma_block(const uint4 &a, const uint4 &b, const float *xs, int kc,
                                          int kb, int lane, float *acc0, float *acc1) {
  constexpr int VEC = Elem<WT>::VEC;
  float wa[VEC], wb[VEC];
  Elem<WT>::unpack(a, wa);
  Elem<WT>::unpack(b, wb);
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const float *xm = xs + m * kc + kb + lane * 4;
    float4 x0 = *(const float4 *)xm;
    acc0[m] += wa[0] * x0.x + wa[1] * x0.y + wa[2] * x0.z + wa[3] * x0.w;
    acc1[m] += wb[0] * x0.x + wb[1] * x0.y + wb[2] * x0.z + wb[3] * x0.w;
    if (VEC == 8) {
      float4 x1 = *(const float4 *)(xm + 256);
      acc0[m] += wa[4] * x1.x + wa[5] * x1.y + wa[6] * x1.z + wa[7] * x1.w;
      acc1[m] += wb[4] * x1.x + wb[5] * x1.y + wb[6] * x1.z + wb[7] * x1.w;
    }
  }
}

// Same loads without a branch around them: a lane beyond klen, or a wave without a task, reads the
// first 16 bytes of the row instead (a cache hit) and its products meet zeros in the staged
// activations (or are discarded).  With every load issued unconditionally the compiler knows how
// many are outstanding at each point and waits for exactly the stage it is about to use; a
// conditional load makes it wait for all of them, which empties the pipeline at every stage.
template <typename WT, int U>
__device__ __forceinline__ void issue_stage_nb(WStage<U> &s, const WT *p0, const WT *p1, int kb, int klen,
                                               int lane, bool valid) {
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int WSTEP = 64 * VEC;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int k = kb + u * WSTEP + lane * VEC;
    const int ko = (valid && k < klen) ? k : 0;
    s.a[u] = load_weights16(p0 + ko);
    s.b[u] = load_weights16(p1 + ko);
  }
}

// grid.x: blocks that share the weight rows; grid.y: tiles of MT activation rows.
// kc: activation elements of one row held in LDS at a time (multiple of 512).
// NT threads per workgroup.  Dynamic LDS: (MT*kc + (NT/64)*MT) floats.
//
// A wave walks its weights as one sequence of stages (U 16-byte loads per row and lane): for each
// of its tasks, for each LDS chunk of the input, for each group of the chunk.  D stages live in a
// ring of registers; a slot is refilled with the stage D ahead as soon as it has been consumed, so
// D-1 stages are in flight while one is multiplied, across chunk and task boundaries, and the
// first D stages are issued before the prologue touches the activations: the norm, the
// reductions and the epilogues all run under outstanding HBM requests.
template <typename WT, int MT, typename Pro, typename Epi, int U = GEMV_U, int D = GEMV_D, int NT = GEMV_THREADS>
__global__ void __launch_bounds__(NT)
gemv_rows_k(Pro pro, Epi epi, const RowDesc *__restrict__ rows, int m_rows, int n_in, int n_tasks,
            int kc) {
  extern __shared__ float4 smem4[];
  float *xs = (float *)smem4;          // [MT][kc] activations
  float *red = xs + MT * kc;           // [NT / 64][MT] partial sums of squares
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int WSTEP = 64 * VEC;
  constexpr int GSTEP = U * WSTEP;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tile0 = blockIdx.y * MT;
  const int n_valid = min(MT, m_rows - tile0);
  if (n_valid <= 0) return;
  RowDesc rd[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) rd[m] = rows[tile0 + (m < n_valid ? m : n_valid - 1)];

  const int n_chunks = (n_in + kc - 1) / kc;
  const int n_groups = (min(kc, n_in) + GSTEP - 1) / GSTEP;   // of a full chunk; a short last chunk masks
  const int n_waves = gridDim.x * (NT / 64), wave_global = blockIdx.x * (NT / 64) + wave;
  const int rounds = (n_tasks + n_waves - 1) / n_waves;       // same for every wave: the chunk staging synchronises the workgroup
  const int n_stages = rounds * n_chunks * n_groups;
  typename Epi::State st;
  epi.init(st);

  // issue cursor: runs D stages ahead of the consumption and past the last stage (no task: dummy loads)
  int ig = 0, ichunk = 0, itask = wave_global;
  bool ivalid = itask < n_tasks;
  const WT *ir0, *ir1;
  epi.weight_rows(ivalid ? itask : 0, ir0, ir1);
  auto issue = [&](WStage<U> &s) {
    const int k0 = ichunk * kc;
    issue_stage_nb<WT>(s, ir0 + k0, ir1 + k0, ig * GSTEP, min(kc, n_in - k0), lane, ivalid);
    if (++ig == n_groups) {
      ig = 0;
      if (++ichunk == n_chunks) {
        ichunk = 0;
        itask += n_waves;
        ivalid = itask < n_tasks;
        epi.weight_rows(ivalid ? itask : 0, ir0, ir1);
      }
    }
  };
  WStage<U> ring[D];
#pragma unroll
  for (int j = 0; j < D; ++j) issue(ring[j]);

  int g = 0, chunk = 0, task = wave_global;
  bool valid = task < n_tasks;
  float acc0[MT], acc1[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc0[m] = acc1[m] = 0.f;
  for (int f0 = 0; f0 < n_stages; f0 += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      if (f0 + j < n_stages) {
        const int k0 = chunk * kc, klen = min(kc, n_in - k0);
        if (g == 0 && (task == wave_global || n_chunks > 1)) {
          __syncthreads();
          pro.template stage<VEC, MT, (NT > GEMV_THREADS ? 4 : 1), NT>(xs, kc, rd, tile0, n_valid, k0, klen, red);
          __syncthreads();
        }
        if (valid) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int kb = g * GSTEP + u * WSTEP;
            if (kb < klen) fma_block<WT, MT>(ring[j].a[u], ring[j].b[u], xs, kc, kb, lane, acc0, acc1);
          }
        }
        if (++g == n_groups) {
          g = 0;
          if (++chunk == n_chunks) {   // the task is complete
            chunk = 0;
            if (valid) {
              float y0 = 0.f, y1 = 0.f;
              RowDesc mine = rd[0];
#pragma unroll
              for (int m = 0; m < MT; ++m) {
                float s0 = wave_sum(acc0[m]), s1 = wave_sum(acc1[m]);
                if (lane == m) { y0 = s0; y1 = s1; mine = rd[m]; }
                acc0[m] = acc1[m] = 0.f;
              }
              if (lane < n_valid) epi.finish(task, tile0 + lane, mine, y0, y1, st);
            }
            task += n_waves;
            valid = task < n_tasks;
          }
        }
      }
      issue(ring[j]);
    }
  }
  if constexpr (EpiHasLocalReduce<Epi>::value) {
    // a running state per wave and row (the heads' arg-max): the waves of the workgroup combine
    // theirs in LDS, where the activations are no longer needed, and one atomic per row and
    // workgroup goes to memory instead of one per wave (thousands of atomics on one address
    // drain one after the other)
    unsigned long long *s_best = (unsigned long long *)xs;
    __syncthreads();
    if (threadIdx.x < MT) s_best[threadIdx.x] = 0ull;
    __syncthreads();
    if (lane < n_valid) epi.reduce_local(st, s_best + lane);
    __syncthreads();
    if ((int)threadIdx.x < n_valid && s_best[threadIdx.x]) {
      RowDesc mine = rd[0];
#pragma unroll
      for (int m = 0; m < MT; ++m)
        if (lane == m) mine = rd[m];
      epi.end_reduced(mine, s_best[threadIdx.x]);
    }
  } else if (lane < n_valid) {
    RowDesc mine = rd[0];
#pragma unroll
    for (int m = 0; m < MT; ++m)
      if (lane == m) mine = rd[m];
    epi.end(tile0 + lane, mine, st);
  }
}

}  // namespace spark
