// Temperature / nucleus (top-p) sampling of the token from the logits of the head that ran
// (Sec. V-A "Models": Step-Audio-2 decodes with temperature 0.7 and top_p 0.9), as a replacement
// of the arg-max.  The definition is exact on integers so that a run is reproducible and can be
// checked against a plain CPU implementation of the same rule:
//   w_i = exp((l_i - max l) / T);  q_i = floor(w_i * 2^32 + 1/2), at most 2^32 - 1
//   order: larger q first, lower index first among equal q
//   nucleus: the shortest prefix of that order whose mass reaches ceil(top_p * sum q); M = its mass
//   x = floor(omega * M / 2^64) for the 64-bit random word omega of the step
//   token: the element of the prefix at which the running mass first exceeds x.
// Both questions have the form "the element at which the running mass of the order first reaches
// t", and the vocabulary is never sorted to answer them.
//
// Two launches, SAMPLE_CHUNK logits of one row per workgroup in both:
//   sample_mass_k  masses; every mass falls into one of 2048 classes (position of its leading one
//                  and the six bits below it, so a class spans 1/64 of its value); the row's mass
//                  per class is summed in memory.
//   sample_pick_k  every workgroup finds, from the class masses alone, the class c in which the
//                  nucleus ends and the few classes in which the draw can end (M is known to lie
//                  between the target and the mass through class c, which bounds x), and appends
//                  its members of those classes to the row's candidate list.  The workgroup that
//                  arrives last sorts the candidates in LDS and reads both answers off running
//                  sums inside one class each.  Should the candidates not fit (nearly equal
//                  logits), it falls back on a radix descent over the masses of the whole row:
//                  three digits whose buckets hold masses, slower and just as exact.
// Class masses, candidate count and arrival count are left at zero for the next step.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int SAMPLE_THREADS = 1024;
constexpr int SAMPLE_WAVES = SAMPLE_THREADS / 64;
constexpr int SAMPLE_CHUNK = 4096;   // logits per workgroup in the mass phase
constexpr int SAMPLE_BINS = 2048;    // mass classes, and buckets of the widest digit
constexpr int SAMPLE_CAP = 2048;     // candidates that the last workgroup sorts in LDS
static_assert(SAMPLE_BINS == 2 * SAMPLE_THREADS, "pick_digit gives every thread two buckets");
static_assert(SAMPLE_CHUNK % SAMPLE_THREADS == 0, "whole waves vote in hist_add");

typedef unsigned long long u64;

// class of a mass q > 0: 64 * (position of the leading one) + the six bits below it; grows with q
__device__ __forceinline__ unsigned mass_class(unsigned q) {
  const int e = 31 - __clz((int)q);
  const unsigned m = e >= 6 ? (q >> (e - 6)) & 63u : (q << (6 - e)) & 63u;
  return (unsigned)e * 64u + m;
}
// candidates are sorted as 64-bit keys: larger mass first, then the lower index
__device__ __forceinline__ u64 cand_key(unsigned q, int idx) {
  return ((u64)q << 32) | (u64)(0xffffffffu - (unsigned)idx);
}

// digit d (0 = most significant) of a mass: shift and bucket count
__device__ __forceinline__ int digit_shift(int d) { return d == 0 ? 21 : (d == 1 ? 10 : 0); }
__device__ __forceinline__ int digit_bins(int d) { return d == 2 ? 1024 : 2048; }

// Adds one mass per lane to a histogram in LDS.  Small masses share their upper digits, so most
// lanes of a wave usually want the same bucket and their atomics would queue up on one address:
// the lanes that agree with the first valid lane are summed in registers and added once.
// Called by whole waves.
__device__ __forceinline__ void hist_add(u64 *s_hist, bool valid, unsigned bucket, unsigned v) {
  const u64 active = __ballot(valid);
  if (!active) return;
  const int leader = __ffsll((long long)active) - 1;
  const unsigned b0 = __shfl(bucket, leader, 64);
  const bool same = valid && bucket == b0;
  if (__popcll(__ballot(same)) >= 8) {
    u64 sum = same ? v : 0u;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&s_hist[b0], sum);
    if (valid && !same) atomicAdd(&s_hist[bucket], (u64)v);
  } else if (valid) {
    atomicAdd(&s_hist[bucket], (u64)v);
  }
}

// Walks the buckets from the highest down: the bucket at which the running mass first reaches
// `remaining` (1 <= remaining <= sum of the buckets) and the mass of the buckets above it.
// Thread t holds the buckets at places 2t and 2t + 1 of that walk.
__device__ __forceinline__ unsigned pick_digit(const u64 *s_hist, int nbins, u64 remaining, u64 *s_wave,
                                               u64 *s_pick, u64 &before_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();                       // histogram complete, s_pick and s_wave no longer read
  if (threadIdx.x == 0) { s_pick[0] = 0; s_pick[1] = 0; }
  __syncthreads();
  const int b0 = nbins - 1 - 2 * (int)threadIdx.x, b1 = b0 - 1;
  const u64 h0 = b0 >= 0 ? s_hist[b0] : 0, h1 = b1 >= 0 ? s_hist[b1] : 0;
  u64 incl = h0 + h1;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const u64 up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  u64 before = incl - (h0 + h1);
  for (int w = 0; w < wave; ++w) before += s_wave[w];
  if (before < remaining && remaining <= before + h0) {
    s_pick[0] = (u64)b0;
    s_pick[1] = before;
  } else if (before + h0 < remaining && remaining <= before + h0 + h1) {
    s_pick[0] = (u64)b1;
    s_pick[1] = before + h0;
  }
  __syncthreads();
  before_out = s_pick[1];
  return (unsigned)s_pick[0];
}

// The slow, general way.  The element at which the running mass (larger q first, lower index
// first) first reaches `target`, 1 <= target <= total mass: returns its mass value K; above = mass
// of all elements with q > K; rank = how many elements with q == K the running mass needs
// (1-based).  Three passes over the row's masses by one workgroup.
__device__ __forceinline__ unsigned mass_descent(const unsigned *__restrict__ q, int V, u64 target, u64 *s_hist,
                                                 u64 *s_wave, u64 *s_pick, u64 &above, u64 &rank) {
  unsigned prefix = 0, mask = 0;
  u64 remaining = target, before;
  above = 0;
  for (int d = 0; d < 3; ++d) {
    const int shift = digit_shift(d), nbins = digit_bins(d);
    __syncthreads();
    for (int b = threadIdx.x; b < nbins; b += SAMPLE_THREADS) s_hist[b] = 0;
    __syncthreads();
    for (int base = 0; base < V; base += 4 * SAMPLE_THREADS) {   // (uniform trip count: whole waves vote)
      unsigned v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = base + j * SAMPLE_THREADS + threadIdx.x;
        v[j] = i < V ? q[i] : 0u;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        hist_add(s_hist, v[j] != 0 && (v[j] & mask) == prefix, (v[j] >> shift) & (unsigned)(nbins - 1), v[j]);
    }
    const unsigned digit = pick_digit(s_hist, nbins, remaining, s_wave, s_pick, before);
    prefix |= digit << shift;
    mask |= (unsigned)(nbins - 1) << shift;
    remaining -= before;
    above += before;
  }
  if (prefix == 0) prefix = 1;                 // (cannot happen: the target is at least 1)
  rank = (remaining + prefix - 1) / prefix;
  return prefix;
}

// largest logit of the row from the head's arg-max key; false if the key reports a NaN
__device__ __forceinline__ bool row_max(u64 head_key, float &mx) {
  const unsigned ok = (unsigned)(head_key >> 32);
  if (head_key == 0ull || ok == 0xffffffffu) return false;
  mx = __uint_as_float((ok & 0x80000000u) ? (ok & 0x7fffffffu) : ~ok);
  return true;
}

// grid (workgroups per row, rows); logits [row][V]; qbuf [row][V]; class_mass [row][SAMPLE_BINS],
// zero on entry; best [row]: the head's arg-max key (its upper half is the largest logit).  A NaN
// logit (the key says so) leaves everything as it is: the emit step reports it.
__global__ void __launch_bounds__(SAMPLE_THREADS)
sample_mass_k(const float *__restrict__ logits, int V, double temperature, unsigned *__restrict__ qbuf,
              u64 *__restrict__ class_mass, const u64 *__restrict__ best) {
  __shared__ u64 s_first[SAMPLE_BINS];
  const int row = blockIdx.y;
  const float *lg = logits + (size_t)row * V;
  unsigned *q = qbuf + (size_t)row * V;
  float mx;
  if (!row_max(best[row], mx)) return;
  for (int b = threadIdx.x; b < SAMPLE_BINS; b += SAMPLE_THREADS) s_first[b] = 0;
  __syncthreads();
  const int c0 = blockIdx.x * SAMPLE_CHUNK;
#pragma unroll
  for (int j = 0; j < SAMPLE_CHUNK / SAMPLE_THREADS; ++j) {
    const int i = c0 + j * SAMPLE_THREADS + threadIdx.x;
    unsigned v = 0;
    if (i < V) {
      // (in double, as the definition states it: the masses are integers that have to come out the
      // same wherever they are computed; 2^32 steps are finer than a float's exp resolves)
      const double w = exp(((double)lg[i] - (double)mx) / temperature);
      const double scaled = floor(w * 4294967296.0 + 0.5);
      v = scaled >= 4294967295.0 ? 4294967295u : (unsigned)scaled;
      q[i] = v;
    }
    hist_add(s_first, v != 0, v ? mass_class(v) : 0u, v);
  }
  __syncthreads();
  for (int b = threadIdx.x; b < SAMPLE_BINS; b += SAMPLE_THREADS)
    if (s_first[b])
      __hip_atomic_fetch_add(class_mass + (size_t)row * SAMPLE_BINS + b, s_first[b], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
}

// first index i of the sorted candidates s_keys[0..n) whose class is `cls` and whose running mass
// inside that class reaches t (1 <= t <= mass of the class): returns its key through s_pick[0] and
// that running mass through s_pick[1].  s_run[i] = sum of the masses of candidates 0..i.
__device__ __forceinline__ void class_walk(const u64 *s_keys, const u64 *s_run, int n, unsigned cls, u64 t,
                                           u64 *s_pick) {
  __syncthreads();
  // mass of the candidates in front of the class
  for (int i = threadIdx.x; i < n; i += SAMPLE_THREADS) {
    const unsigned qi = (unsigned)(s_keys[i] >> 32);
    if (qi != 0 && mass_class(qi) == cls && (i == 0 || mass_class((unsigned)(s_keys[i - 1] >> 32)) != cls))
      s_pick[2] = s_run[i] - qi;
  }
  __syncthreads();
  const u64 front = s_pick[2];
  for (int i = threadIdx.x; i < n; i += SAMPLE_THREADS) {
    const unsigned qi = (unsigned)(s_keys[i] >> 32);
    if (qi == 0 || mass_class(qi) != cls) continue;
    const u64 through = s_run[i] - front;
    if (through >= t && through - qi < t) {
      s_pick[0] = s_keys[i];
      s_pick[1] = through;
    }
  }
  __syncthreads();
}

// grid (workgroups per row, rows); omega [row]; cand [row][SAMPLE_CAP]; class_mass as
// sample_mass_k left it, zero on exit; cand_count [row] and arrive [row] zero on entry and exit;
// best [row]: the head's arg-max key on entry, the key of the drawn token on return.
__global__ void __launch_bounds__(SAMPLE_THREADS)
sample_pick_k(const float *__restrict__ logits, int V, double top_p, const u64 *__restrict__ omega,
              const unsigned *__restrict__ qbuf, u64 *__restrict__ class_mass, u64 *__restrict__ cand,
              unsigned *__restrict__ cand_count, unsigned *__restrict__ arrive, u64 *__restrict__ best) {
  __shared__ u64 s_first[SAMPLE_BINS], s_keys[SAMPLE_CAP], s_run[SAMPLE_CAP], s_wave[SAMPLE_WAVES], s_pick[3];
  __shared__ int s_cnt[SAMPLE_WAVES], s_n, s_slot, s_last;
  const int row = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *lg = logits + (size_t)row * V;
  const unsigned *q = qbuf + (size_t)row * V;
  u64 *row_mass = class_mass + (size_t)row * SAMPLE_BINS;
  u64 *row_cand = cand + (size_t)row * SAMPLE_CAP;
  float mx;
  if (!row_max(best[row], mx)) return;

  // ---- every workgroup: total, target, the classes that can matter
  u64 mine = 0;
  for (int b = threadIdx.x; b < SAMPLE_BINS; b += SAMPLE_THREADS) {
    const u64 h = row_mass[b];
    s_first[b] = h;
    mine += h;
  }
  if (threadIdx.x == 0) s_n = 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
  if (lane == 0) s_wave[wave] = mine;
  __syncthreads();
  u64 total = 0;
  for (int w = 0; w < SAMPLE_WAVES; ++w) total += s_wave[w];
  u64 target = (u64)ceil(top_p * (double)total);
  target = target < 1 ? 1 : (target > total ? total : target);
  const u64 word = omega[row];
  u64 above_cut, unused;
  const unsigned c_cut = pick_digit(s_first, SAMPLE_BINS, target, s_wave, s_pick, above_cut);
  // target <= M <= mass through class c_cut, and x = floor(word * M / 2^64) grows with M
  const u64 x_lo = __umul64hi(word, target), x_hi = __umul64hi(word, above_cut + s_first[c_cut]);
  const unsigned c_hi = pick_digit(s_first, SAMPLE_BINS, x_lo + 1, s_wave, s_pick, unused);
  const unsigned c_lo = pick_digit(s_first, SAMPLE_BINS, x_hi + 1, s_wave, s_pick, unused);

  // ---- this workgroup's candidates, then into the row's list
  const int c0 = blockIdx.x * SAMPLE_CHUNK;
#pragma unroll
  for (int j = 0; j < SAMPLE_CHUNK / SAMPLE_THREADS; ++j) {
    const int i = c0 + j * SAMPLE_THREADS + threadIdx.x;
    const unsigned v = i < V ? q[i] : 0u;
    if (v != 0) {
      const unsigned cls = mass_class(v);
      if (cls == c_cut || (cls >= c_lo && cls <= c_hi)) {
        const int at = atomicAdd(&s_n, 1);
        if (at < SAMPLE_CAP) s_keys[at] = cand_key(v, i);
      }
    }
  }
  __syncthreads();
  const int n_local = s_n;
  if (threadIdx.x == 0 && n_local > 0)
    s_slot = (int)__hip_atomic_fetch_add(cand_count + row, (unsigned)n_local, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (n_local > 0) {
    const int slot = s_slot;
    for (int j = threadIdx.x; j < n_local && j < SAMPLE_CAP; j += SAMPLE_THREADS)
      if (slot + j < SAMPLE_CAP)
        __hip_atomic_store(row_cand + slot + j, s_keys[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  wait_memory_ops();                     // candidates written before the count
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned prev = __hip_atomic_fetch_add(arrive + row, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = prev == gridDim.x - 1;
    if (s_last) {
      __hip_atomic_store(arrive + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_n = (int)__hip_atomic_load(cand_count + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(cand_count + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
  }
  __syncthreads();
  if (!s_last) return;

  // ---- the last workgroup of the row (every workgroup has read the class masses by now)
  for (int b = threadIdx.x; b < SAMPLE_BINS; b += SAMPLE_THREADS) row_mass[b] = 0;
  const int n = s_n;
  if (n <= SAMPLE_CAP) {
    // candidates into LDS, padded with zero keys (they sort last) to a power of two
    int np = 64;
    while (np < n) np <<= 1;
    for (int i = threadIdx.x; i < np; i += SAMPLE_THREADS)
      s_keys[i] = i < n ? __hip_atomic_load(row_cand + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
    // bitonic sort, largest key first
    for (int k = 2; k <= np; k <<= 1)
      for (int j = k >> 1; j > 0; j >>= 1) {
        __syncthreads();
        const int t = threadIdx.x;
        if (t < np / 2) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), p = i | j;
          const u64 a = s_keys[i], b = s_keys[p];
          const bool descending = (i & k) == 0;
          if ((a < b) == descending) { s_keys[i] = b; s_keys[p] = a; }
        }
      }
    __syncthreads();
    // running sums of the sorted masses: thread t holds candidates 2t and 2t + 1
    {
      const int i0 = 2 * threadIdx.x;
      const u64 q0 = i0 < np ? s_keys[i0] >> 32 : 0, q1 = i0 + 1 < np ? s_keys[i0 + 1] >> 32 : 0;
      u64 incl = q0 + q1;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const u64 up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
      }
      if (lane == 63) s_wave[wave] = incl;
      __syncthreads();
      u64 before = incl - (q0 + q1);
      for (int w = 0; w < wave; ++w) before += s_wave[w];
      if (i0 < np) s_run[i0] = before + q0;
      if (i0 + 1 < np) s_run[i0 + 1] = before + q0 + q1;
    }
    // the nucleus ends inside class c_cut; the draw ends inside the class that holds x + 1
    class_walk(s_keys, s_run, np, c_cut, target - above_cut, s_pick);
    const u64 nucleus_mass = above_cut + s_pick[1];
    const u64 x = __umul64hi(word, nucleus_mass);
    u64 above_tok;
    const unsigned c_tok = pick_digit(s_first, SAMPLE_BINS, x + 1, s_wave, s_pick, above_tok);
    class_walk(s_keys, s_run, np, c_tok, x + 1 - above_tok, s_pick);
    if (threadIdx.x == 0) {
      const int tok = (int)(0xffffffffu - (unsigned)(s_pick[0] & 0xffffffffull));
      best[row] = argmax_key(lg[tok], tok);
    }
    return;
  }

  // ---- too many candidates: radix descents over the whole row
  u64 above, rank;
  const unsigned k_cut = mass_descent(q, V, target, s_keys, s_wave, s_pick, above, rank);
  const u64 nucleus_mass = above + rank * k_cut;
  const u64 x = __umul64hi(word, nucleus_mass);
  const unsigned k_tok = mass_descent(q, V, x + 1, s_keys, s_wave, s_pick, above, rank);
  // the rank-th (by index) element with mass k_tok: every wave counts the matches in its own
  // stretch of indices; the wave whose stretch holds that element walks it once more
  const int seg = (((V + SAMPLE_WAVES - 1) / SAMPLE_WAVES) + 63) & ~63;
  const int w0 = wave * seg, w1 = min(V, w0 + seg);
  int cnt = 0;
  for (int base = w0; base < w1; base += 64) {
    const int i = base + lane;
    cnt += __popcll(__ballot(i < w1 && q[i] == k_tok));
  }
  if (lane == 0) s_cnt[wave] = cnt;
  __syncthreads();
  u64 seen = 0;
  for (int w = 0; w < wave; ++w) seen += (u64)s_cnt[w];
  if (seen < rank && rank <= seen + (u64)cnt) {
    int need = (int)(rank - seen);
    for (int base = w0; base < w1; base += 64) {
      const int i = base + lane;
      const bool hit = i < w1 && q[i] == k_tok;
      const u64 hits = __ballot(hit);
      const int c = __popcll(hits);
      if (need <= c) {
        if (hit && __popcll(hits & ((1ull << lane) - 1ull)) == need - 1) best[row] = argmax_key(lg[i], i);
        break;
      }
      need -= c;
    }
  }
}

}  // namespace spark
