// One persistent kernel for a run of transformer layers on up to four rows of one sequence
// (the new position of a decoding step; or the pending positions plus the new one on a full-depth
// step, Algorithm 1 line 8).
//
// The paper does not report wall-clock time because launching and dispatching one kernel per
// operation dominates a small-batch decoding loop (Sec. V-A "Metrics").  Here a run of layers is a
// single launch: one workgroup per CU stays resident, the five phases of a layer (q/k/v
// projection, attention, output projection, gate/up, down) are separated by grid-wide barriers
// built from device-scope atomics, and the activations that cross a barrier travel through
// device-scope stores and loads, so no cache is flushed or invalidated between phases.  Weights do
// not depend on activations: every wave issues the first loads of its next phase before it waits,
// which keeps HBM busy across the barrier and the activation staging of the next phase.
#pragma once
#include "attention.h"
#include "device_common.h"
#include "gemv.h"

namespace spark {

constexpr int PASS_THREADS = 512;
constexpr int PASS_WAVES = PASS_THREADS / 64;
constexpr int PASS_U = 4;  // 16-byte loads per weight row and pipeline stage (2 waves per SIMD: deeper than the stand-alone kernel)
typedef WStage<PASS_U> PStage;
constexpr unsigned PASS_SPIN_LIMIT = 1u << 22;  // polls before a barrier gives up (about a second)

// Barrier state in device memory: one arrival word per XCD (workgroups are dealt to the 8 XCDs
// round-robin), 128 bytes apart, and one global word counted by the last arrival of each XCD.
struct GridBarrier {
  unsigned *xcd_words;   // [8][32]
  unsigned *global_word;
  unsigned *error_word;  // set when a wait ran out of polls
};

// All workgroups of the grid meet here.  `round` counts barriers since the words were zeroed.
// Returns false (in every thread of the workgroup) if the wait gave up.
__device__ __forceinline__ bool grid_sync(const GridBarrier &gb, unsigned &round, int *s_flag) {
  ++round;
  wait_memory_ops();  // this wave's device-scope stores have completed
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned x = blockIdx.x & 7u;
    const unsigned members = (gridDim.x + 7u - x) >> 3;  // workgroups with blockIdx % 8 == x
    const unsigned groups = gridDim.x < 8u ? gridDim.x : 8u;
    unsigned prev = __hip_atomic_fetch_add(gb.xcd_words + x * 32, 1u, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    if (prev + 1 == round * members)
      __hip_atomic_fetch_add(gb.global_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned polls = 0;
    int ok = 1;
    while (__hip_atomic_load(gb.global_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
           round * groups) {
      __builtin_amdgcn_s_sleep(1);
      if (++polls > PASS_SPIN_LIMIT) {
        atomicOr(gb.error_word, 1u);
        ok = 0;
        break;
      }
    }
    if (__hip_atomic_load(gb.error_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) ok = 0;
    *s_flag = ok;
    // what other workgroups wrote through to memory is now visible to ordinary loads of this CU
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  __syncthreads();
  return *s_flag != 0;
}

// ------------------------------------------------------------------ activation staging (512 threads)

// xs[m][k] = src_row_m[k0 + k]; the rows were written through to memory by other workgroups and
// the barrier before this call dropped the stale cache lines, so ordinary 16-byte loads do
template <int VEC, int MT>
__device__ __forceinline__ void pass_stage_plain(float *xs, int kc, const float *src, int stride,
                                                 int n_valid, int k0, int klen) {
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int mm = m < n_valid ? m : n_valid - 1;
    const float *row = src + (size_t)mm * stride + k0;
    for (int k = threadIdx.x * 4; k < klen; k += PASS_THREADS * 4)
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = *(const float4 *)(row + k);
    const int end = (klen + 511) & ~511;
    for (int k = klen + threadIdx.x * 4; k < end; k += PASS_THREADS * 4)
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// xs[m][k] = RMSNorm(hidden[x_slot_m]; gamma)[k]; the whole row (d <= kc) is staged
template <int VEC, int MT>
__device__ __forceinline__ void pass_stage_norm(float *xs, int kc, const float *hidden,
                                                const RowDesc *rd, int n_valid, const float *gamma,
                                                float eps, int d, float *red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // raw row into LDS and the sum of squares on the way
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int mm = m < n_valid ? m : n_valid - 1;
    const float *row = hidden + (size_t)rd[mm].x_slot * d;
    float ss = 0.f;
    for (int k = threadIdx.x * 4; k < d; k += PASS_THREADS * 4) {
      const float4 v = *(const float4 *)(row + k);
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = v;
    }
    ss = wave_sum(ss);
    if (lane == 0) red[wave * MT + m] = ss;
  }
  __syncthreads();
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < PASS_WAVES; ++w) tot += red[w * MT + m];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    for (int k = threadIdx.x * 4; k < d; k += PASS_THREADS * 4) {   // same thread, same elements
      float4 *px = (float4 *)(xs + m * kc + lds_pos<VEC>(k));
      const float4 v = *px, g = *(const float4 *)(gamma + k);
      *px = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
    }
    const int end = (d + 511) & ~511;
    for (int k = d + threadIdx.x * 4; k < end; k += PASS_THREADS * 4)
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// ------------------------------------------------------------------ one projection phase

// Which activations a phase stages
enum { PASS_IN_NORM = 0, PASS_IN_PLAIN = 1 };

struct PhaseIn {
  int kind;
  const float *src;     // PLAIN: [row][stride]; NORM: hidden arena
  int stride;
  const float *gamma;
  float eps;
};

// Weight rows of the first stage a wave will need in a phase: primes `nxt`.
template <typename WT, typename Epi>
__device__ __forceinline__ void phase_prime(PStage &nxt, const Epi &epi, int n_in, int n_tasks, int kc,
                                            int wave_global, int lane) {
  const WT *r0, *r1;
  const bool valid = wave_global < n_tasks;
  epi.weight_rows(valid ? wave_global : 0, r0, r1);
  issue_stage<WT>(nxt, r0, r1, 0, min(kc, n_in), lane, valid);
}

// y = W x for the MT rows; `nxt` holds the already issued first stage on entry and the first
// stage of the following phase on exit (prime_next issues it at the point where this phase's
// pipeline would run dry).
template <typename WT, int MT, typename Epi, typename PrimeNext>
__device__ __forceinline__ void pass_gemv_phase(const PhaseIn &in, const Epi &epi, const RowDesc *rd,
                                                int n_valid, int n_in, int n_tasks, int kc, float *xs,
                                                float *red, PStage &nxt, const PrimeNext &prime_next,
                                                int n_waves, int wave_global, int lane) {
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int WSTEP = 64 * VEC;
  constexpr int GSTEP = PASS_U * WSTEP;
  const int n_chunks = (n_in + kc - 1) / kc;
  const int rounds = (n_tasks + n_waves - 1) / n_waves;
  typename Epi::State st;
  epi.init(st);
  const WT *r0, *r1;
  bool valid = wave_global < n_tasks;
  epi.weight_rows(valid ? wave_global : 0, r0, r1);

  for (int round = 0; round < rounds; ++round) {
    const int task = round * n_waves + wave_global;
    const int task_n = task + n_waves;
    const bool valid_n = round + 1 < rounds && task_n < n_tasks;
    const WT *r0n, *r1n;
    epi.weight_rows(valid_n ? task_n : 0, r0n, r1n);
    float acc0[MT], acc1[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc0[m] = acc1[m] = 0.f;

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
      const int k0 = chunk * kc, klen = min(kc, n_in - k0);
      if (round == 0 || n_chunks > 1) {
        __syncthreads();
        if (in.kind == PASS_IN_NORM)
          pass_stage_norm<VEC, MT>(xs, kc, in.src, rd, n_valid, in.gamma, in.eps, n_in, red);
        else
          pass_stage_plain<VEC, MT>(xs, kc, in.src, in.stride, n_valid, k0, klen);
        __syncthreads();
      }
      const int n_groups = (klen + GSTEP - 1) / GSTEP;
      for (int g = 0; g < n_groups; ++g) {
        const PStage cur = nxt;
        if (g + 1 < n_groups) {
          issue_stage<WT>(nxt, r0 + k0, r1 + k0, (g + 1) * GSTEP, klen, lane, valid);
        } else if (chunk + 1 < n_chunks) {
          issue_stage<WT>(nxt, r0 + k0 + kc, r1 + k0 + kc, 0, min(kc, n_in - k0 - kc), lane, valid);
        } else if (round + 1 < rounds) {
          issue_stage<WT>(nxt, r0n, r1n, 0, min(kc, n_in), lane, valid_n);
        } else {
          prime_next(nxt);
        }
        if (valid) {
#pragma unroll
          for (int u = 0; u < PASS_U; ++u) {
            const int kb = g * GSTEP + u * WSTEP;
            if (kb < klen) fma_block<WT, MT>(cur.a[u], cur.b[u], xs, kc, kb, lane, acc0, acc1);
          }
        }
      }
    }
    if (valid) {
      float y0 = 0.f, y1 = 0.f;
      RowDesc mine = rd[0];
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        float s0 = wave_sum(acc0[m]), s1 = wave_sum(acc1[m]);
        if (lane == m) { y0 = s0; y1 = s1; mine = rd[m]; }
      }
      if (lane < n_valid) epi.finish(task, lane, mine, y0, y1, st);
    }
    valid = valid_n;
    r0 = r0n;
    r1 = r1n;
  }
}

// ------------------------------------------------------------------ the kernel

template <typename WT> struct PassParams {
  // model
  int d, nq, nkv, hd, F;
  float eps;
  const WT *wq, *wk, *wv, *wo, *wg, *wu, *wd;   // layer 0 of each stacked tensor
  const float *attn_norm, *mlp_norm;
  int l0, l1;                                   // layers [l0, l1)
  // rows: consecutive positions of one sequence
  const RowDesc *rows;
  int m_rows;
  // buffers
  float *hidden, *qbuf, *attn_out, *act, *part;
  int *arrivals;
  const float2 *rope;
  KVView kv;
  int n_splits;
  float scale;
  // LDS split: activations of one chunk for the projections
  int kc_d, kc_q, kc_f;                         // chunk lengths for inputs of size d, nq*hd, F
  GridBarrier gb;
  unsigned round_base;                          // barriers passed since the words were zeroed
  unsigned long long *timeline;                 // debugging aid (nullable): 100 MHz clock of
                                                // workgroup 0 before and after every barrier
};

struct NoPrime {
  __device__ void operator()(PStage &) const {}
};

template <typename WT, int MT, int HD, int G>
__global__ void __launch_bounds__(PASS_THREADS)
spark_pass_k(PassParams<WT> p) {
  extern __shared__ float4 smem4[];
  float *lds = (float *)smem4;
  __shared__ int s_flag;
  __shared__ float red[PASS_WAVES * MT];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_waves = gridDim.x * PASS_WAVES, wave_global = blockIdx.x * PASS_WAVES + wave;
  const int n_valid = min(MT, p.m_rows);
  RowDesc rd[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) rd[m] = p.rows[m < n_valid ? m : n_valid - 1];
  unsigned round = p.round_base;
  int tl = 0;
  auto mark = [&]() {
    if (p.timeline && blockIdx.x == 0 && threadIdx.x == 0) p.timeline[tl] = wall_clock64();
    ++tl;
  };
  mark();

  const int d = p.d, qw = p.nq * HD, kvw = p.nkv * HD, F = p.F;
  const int t_qkv = (p.nq + 2 * p.nkv) * (HD / 2), t_o = d / 2, t_gu = F, t_dn = d / 2;

  auto epi_qkv = [&](int l) {
    EpiQKV<WT, true> e;
    e.wq = p.wq + (size_t)l * qw * d;
    e.wk = p.wk + (size_t)l * kvw * d;
    e.wv = p.wv + (size_t)l * kvw * d;
    e.d = d; e.nq = p.nq; e.nkv = p.nkv; e.hd = HD; e.layer = l;
    e.qbuf = p.qbuf; e.rope = p.rope; e.kv = p.kv;
    return e;
  };
  auto epi_o = [&](int l) {
    return EpiResidual<WT, true>{p.wo + (size_t)l * d * qw, qw, d, p.hidden, d};
  };
  auto epi_gu = [&](int l) {
    return EpiSwiGLU<WT, true>{p.wg + (size_t)l * F * d, p.wu + (size_t)l * F * d, d, F, p.act};
  };
  auto epi_dn = [&](int l) {
    return EpiResidual<WT, true>{p.wd + (size_t)l * d * F, F, d, p.hidden, d};
  };

  PStage nxt;
  phase_prime<WT>(nxt, epi_qkv(p.l0), d, t_qkv, p.kc_d, wave_global, lane);

  for (int l = p.l0; l < p.l1; ++l) {
    // ---- q, k, v projections (+ rotary embedding, query store, KV-cache write)
    {
      const auto e = epi_qkv(l);
      const auto en = epi_o(l);
      PhaseIn in{PASS_IN_NORM, p.hidden, d, p.attn_norm + (size_t)l * d, p.eps};
      pass_gemv_phase<WT, MT>(in, e, rd, n_valid, d, t_qkv, p.kc_d, lds, red, nxt,
                              [&](PStage &s) { phase_prime<WT>(s, en, qw, t_o, p.kc_q, wave_global, lane); },
                              n_waves, wave_global, lane);
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- attention: tasks (row, kv head, slice) dealt to the workgroups
    {
      const int per_row = p.nkv * p.n_splits;
      for (int t = blockIdx.x; t < n_valid * per_row; t += gridDim.x) {
        const int r = t / per_row, rem = t - r * per_row;
        const int hk = rem / p.n_splits, split = rem - hk * p.n_splits;
        RowDesc mine = rd[0];
#pragma unroll
        for (int m = 0; m < MT; ++m)
          if (m == r) mine = rd[m];
        if (split * ATTN_SLICE <= mine.pos) {
          __syncthreads();  // LDS of the previous task is free
          attn_task<WT, HD, G, PASS_THREADS, true>(mine, r, hk, split, p.qbuf, p.kv, l, p.nq,
                                                   p.n_splits, p.scale, p.part, p.arrivals,
                                                   p.attn_out, lds);
        }
      }
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- attention output projection, residual add
    {
      const auto e = epi_o(l);
      const auto en = epi_gu(l);
      PhaseIn in{PASS_IN_PLAIN, p.attn_out, qw, nullptr, 0.f};
      pass_gemv_phase<WT, MT>(in, e, rd, n_valid, qw, t_o, p.kc_q, lds, red, nxt,
                              [&](PStage &s) { phase_prime<WT>(s, en, d, t_gu, p.kc_d, wave_global, lane); },
                              n_waves, wave_global, lane);
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- gate and up projections, SiLU(gate) * up
    {
      const auto e = epi_gu(l);
      const auto en = epi_dn(l);
      PhaseIn in{PASS_IN_NORM, p.hidden, d, p.mlp_norm + (size_t)l * d, p.eps};
      pass_gemv_phase<WT, MT>(in, e, rd, n_valid, d, t_gu, p.kc_d, lds, red, nxt,
                              [&](PStage &s) { phase_prime<WT>(s, en, F, t_dn, p.kc_f, wave_global, lane); },
                              n_waves, wave_global, lane);
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- down projection, residual add
    {
      const auto e = epi_dn(l);
      PhaseIn in{PASS_IN_PLAIN, p.act, F, nullptr, 0.f};
      if (l + 1 < p.l1) {
        const auto en = epi_qkv(l + 1);
        pass_gemv_phase<WT, MT>(in, e, rd, n_valid, F, t_dn, p.kc_f, lds, red, nxt,
                                [&](PStage &s) { phase_prime<WT>(s, en, d, t_qkv, p.kc_d, wave_global, lane); },
                                n_waves, wave_global, lane);
        mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();
      } else {
        pass_gemv_phase<WT, MT>(in, e, rd, n_valid, F, t_dn, p.kc_f, lds, red, nxt, NoPrime(), n_waves,
                                wave_global, lane);
        mark();
      }
    }
  }
}

}  // namespace spark
