// One persistent kernel for a run of transformer layers on up to four rows of one sequence
// (the new position of a decoding step; or the pending positions plus the new one on a full-depth
// step, Algorithm 1 line 8).
//
// The paper does not report wall-clock time because launching and dispatching one kernel per
// operation dominates a small-batch decoding loop (Sec. V-A "Metrics").  Here a run of layers is a
// single launch: one workgroup per CU stays resident, the five phases of a layer (q/k/v
// projection, attention, output projection, gate/up, down) are separated by grid-wide barriers
// built from device-scope atomics, and the activations that cross a barrier travel through
// device-scope stores, so no cache is flushed between phases.  Weights do not depend on
// activations: every wave keeps a ring of PASS_D weight stages in flight and fills it with the
// first stages of its next phase while it finishes the current one, which keeps HBM busy across
// the barrier and the activation staging of the next phase.
#pragma once
#include "attention.h"
#include "device_common.h"
#include "gemv.h"

namespace spark {

constexpr int PASS_THREADS = 512;
constexpr int PASS_WAVES = PASS_THREADS / 64;
constexpr int PASS_U = 4;  // 16-byte loads per weight row and pipeline stage (2 waves per SIMD: deeper than the stand-alone kernel)
typedef WStage<PASS_U> PStage;
constexpr int PASS_D = 3;  // stages a wave keeps in flight (8 KB each with bf16 weights)
struct PRing {
  PStage s[PASS_D];
};
constexpr int PASS_MAX_ROUNDS = 16;  // rounds of tasks per wave and phase the result buffer holds
constexpr unsigned PASS_SPIN_LIMIT = 1u << 22;  // polls before a barrier gives up (about a second)

// Barrier state in device memory: one arrival word per XCD (workgroups are dealt to the 8 XCDs
// round-robin), 128 bytes apart, and one global word counted by the last arrival of each XCD.
// (Watching the eight XCD words directly, without the global word, was measured slower: 256
// workgroups polling eight addresses delay the arrivals.)
struct GridBarrier {
  unsigned *xcd_words;   // [8][32]
  unsigned *global_word;
  unsigned *error_word;  // set when a wait ran out of polls
};

// All workgroups of the grid meet here.  `round` counts barriers since the words were zeroed.
// Returns false (in every thread of the workgroup) if the wait gave up.
__device__ __forceinline__ bool grid_sync(const GridBarrier &gb, unsigned &round, int *s_flag) {
  ++round;
  // Every device-scope store of the phase was issued by wave 0 (projection epilogues) or has been
  // waited for by its own wave (attention); the other waves keep their prefetched weights in flight.
  if (threadIdx.x < 64) wait_memory_ops();
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
    while ((int)(__hip_atomic_load(gb.global_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                 round * groups) < 0) {
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
                                                 int n_valid, int k0, int klen, int tid) {
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int mm = m < n_valid ? m : n_valid - 1;
    const float *row = src + (size_t)mm * stride + k0;
    for (int k = tid * 4; k < klen; k += PASS_THREADS * 4)
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = *(const float4 *)(row + k);
    const int end = (klen + 511) & ~511;
    for (int k = klen + tid * 4; k < end; k += PASS_THREADS * 4)
      *(float4 *)(xs + m * kc + lds_pos<VEC>(k)) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// xs[m][k] = RMSNorm(hidden[x_slot_m]; gamma)[k]; the whole row (d <= kc) is staged
template <int VEC, int MT>
__device__ __forceinline__ void pass_stage_norm(float *xs, int kc, const float *hidden,
                                                const RowDesc *rd, int n_valid, const float *gamma,
                                                float eps, int d, float *red, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  // raw row into LDS and the sum of squares on the way
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const float *row = hidden + (size_t)rd[m].x_slot * d;   // rows beyond the pass repeat the last one
    float ss = 0.f;
    for (int k = tid * 4; k < d; k += PASS_THREADS * 4) {
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
    for (int k = tid * 4; k < d; k += PASS_THREADS * 4) {   // same thread, same elements
      float4 *px = (float4 *)(xs + m * kc + lds_pos<VEC>(k));
      const float4 v = *px, g = *(const float4 *)(gamma + k);
      *px = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
    }
    const int end = (d + 511) & ~511;
    for (int k = d + tid * 4; k < end; k += PASS_THREADS * 4)
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

// A wave walks the weights of a phase as a sequence of stages (PASS_U 16-byte loads per weight row
// and lane each): for every round of tasks, for every LDS chunk of the input, for every group of
// the chunk.  All waves of the grid have the same number of stages; the count is padded to a
// multiple of the ring depth so that a phase always starts at ring slot 0.
struct PhaseGeom {
  int n_in, n_tasks, kc, n_chunks, n_groups, rounds, n_real, n_pad;
};

template <typename WT>
__device__ __forceinline__ PhaseGeom make_geom(int n_in, int n_tasks, int kc, int n_waves) {
  constexpr int GSTEP = PASS_U * 64 * Elem<WT>::VEC;
  PhaseGeom g;
  g.n_in = n_in; g.n_tasks = n_tasks; g.kc = kc;
  g.n_chunks = (n_in + kc - 1) / kc;
  g.n_groups = (min(kc, n_in) + GSTEP - 1) / GSTEP;
  g.rounds = (n_tasks + n_waves - 1) / n_waves;
  g.n_real = g.rounds * g.n_chunks * g.n_groups;
  g.n_pad = (g.n_real + PASS_D - 1) / PASS_D * PASS_D;
  return g;
}

// Where a wave's stage sequence of a phase stands.  Past the last task the cursor has no valid
// task and its loads turn into cache hits on the first bytes of a row.
template <typename WT> struct StageCursor {
  const WT *r0, *r1;
  int g, chunk, task;
  bool valid;
};

template <typename WT, typename Epi>
__device__ __forceinline__ void cursor_begin(StageCursor<WT> &c, const Epi &epi, const PhaseGeom &pg,
                                             int wave_global) {
  c.g = 0; c.chunk = 0; c.task = wave_global;
  c.valid = c.task < pg.n_tasks;
  epi.weight_rows(c.valid ? c.task : 0, c.r0, c.r1);
}

template <typename WT, typename Epi>
__device__ __forceinline__ void cursor_advance(StageCursor<WT> &c, const Epi &epi, const PhaseGeom &pg,
                                               int n_waves) {
  if (++c.g == pg.n_groups) {
    c.g = 0;
    if (++c.chunk == pg.n_chunks) {
      c.chunk = 0;
      c.task += n_waves;
      c.valid = c.task < pg.n_tasks;
      epi.weight_rows(c.valid ? c.task : 0, c.r0, c.r1);
    }
  }
}

// the loads of the cursor's stage, issued without a branch (see issue_stage_nb)
template <typename WT>
__device__ __forceinline__ void cursor_load(PStage &s, const StageCursor<WT> &c, const PhaseGeom &pg,
                                            int lane, bool enable) {
  constexpr int GSTEP = PASS_U * 64 * Elem<WT>::VEC;
  const int k0 = c.chunk * pg.kc;
  issue_stage_nb<WT>(s, c.r0 + k0, c.r1 + k0, c.g * GSTEP, min(pg.kc, pg.n_in - k0), lane,
                     c.valid && enable);
}

// The first PASS_D stages of a phase, issued before the barrier in front of it.  Wave 0 holds back
// all but one (its thread 0 polls the barrier, and a poll returns only after the loads the wave
// issued before it); the phase issues the rest when it starts.
template <typename WT, typename Epi>
__device__ __forceinline__ void prime_ring(PRing &ring, const Epi &epi, const PhaseGeom &pg, bool enable,
                                           int n_waves, int wave_global, int lane, int wave) {
  StageCursor<WT> c;
  cursor_begin(c, epi, pg, wave_global);
#pragma unroll
  for (int j = 0; j < PASS_D; ++j) {
    cursor_load(ring.s[j], c, pg, lane, enable && (wave != 0 || j == 0));
    cursor_advance(c, epi, pg, n_waves);
  }
}

// y = W x for the MT rows.  On entry the ring holds stages 0..PASS_D-1 of this phase (wave 0: stage
// 0); while the last PASS_D stages are consumed the slots are refilled with the first stages of
// the following phase (prime_next), so they are in flight across the epilogue, the barrier and the
// next activation staging.  Results go to LDS and wave 0 alone runs the epilogues after the last
// stage: only that wave then has stores to wait for before the workgroup arrives at the barrier
// (a wave cannot wait for its stores without also waiting for every load it has in flight).
template <typename WT, int MT, typename Epi, typename EpiNext>
__device__ __forceinline__ void pass_gemv_phase(const PhaseIn &in, const Epi &epi, const PhaseGeom &pg,
                                                const EpiNext &epi_next, const PhaseGeom &pg_next,
                                                bool prime_next, const RowDesc *rd, int n_valid,
                                                float *xs, float *red, float *yres, PRing &ring,
                                                int n_waves, int wave_global, int tid_in) {
  constexpr int VEC = Elem<WT>::VEC;
  constexpr int WSTEP = 64 * VEC;
  constexpr int GSTEP = PASS_U * WSTEP;
  // per-lane addresses are recomputed in every phase instead of being kept in registers across all
  // of them: the ring needs the registers
  int tid = tid_in;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;

  // wave 0 runs the epilogues; an epilogue that adds to what is in memory fetches the old values
  // now (they were written at least one barrier ago), not at the end of the phase
  const int per_wave = pg.rounds * MT;
  float2 old = make_float2(0.f, 0.f);
  if constexpr (EpiReadsOld<Epi>::value) {
    if (wave == 0 && lane < PASS_WAVES * per_wave) {
      const int w = lane / per_wave, rem = lane - w * per_wave;
      const int rnd = rem / MT, m = rem - rnd * MT;
      const int task = rnd * n_waves + blockIdx.x * PASS_WAVES + w;
      if (task < pg.n_tasks && m < n_valid) {
        const RowDesc mine = rd[m];
        old = epi.load_old(task, mine);
      }
    }
  }

  StageCursor<WT> ic;
  cursor_begin(ic, epi, pg, wave_global);
  if (wave == 0) {   // the stages this wave held back before the barrier
    StageCursor<WT> lc = ic;
#pragma unroll
    for (int j = 1; j < PASS_D; ++j) {
      cursor_advance(lc, epi, pg, n_waves);
      cursor_load(ring.s[j], lc, pg, lane, true);
    }
  }
#pragma unroll
  for (int j = 0; j < PASS_D; ++j) cursor_advance(ic, epi, pg, n_waves);   // ic: stage PASS_D

  int g = 0, chunk = 0, round = 0;
  bool valid = wave_global < pg.n_tasks;
  float acc0[MT], acc1[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc0[m] = acc1[m] = 0.f;
  auto consume = [&](const PStage &slot) {
    const int k0 = chunk * pg.kc, klen = min(pg.kc, pg.n_in - k0);
    if (g == 0 && (round == 0 || pg.n_chunks > 1)) {
      __syncthreads();
      if (in.kind == PASS_IN_NORM)
        pass_stage_norm<VEC, MT>(xs, pg.kc, in.src, rd, n_valid, in.gamma, in.eps, pg.n_in, red, tid);
      else
        pass_stage_plain<VEC, MT>(xs, pg.kc, in.src, in.stride, n_valid, k0, klen, tid);
      __syncthreads();
    }
    if (valid) {
#pragma unroll
      for (int u = 0; u < PASS_U; ++u) {
        const int kb = g * GSTEP + u * WSTEP;
        if (kb < klen) fma_block<WT, MT>(slot.a[u], slot.b[u], xs, pg.kc, kb, lane, acc0, acc1);
      }
    }
    if (++g == pg.n_groups) {
      g = 0;
      if (++chunk == pg.n_chunks) {   // the task is complete
        chunk = 0;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const float s0 = wave_sum(acc0[m]), s1 = wave_sum(acc1[m]);
          if (lane == 0) {
            float *y = yres + ((wave * PASS_MAX_ROUNDS + round) * MT + m) * 2;
            y[0] = s0; y[1] = s1;
          }
          acc0[m] = acc1[m] = 0.f;
        }
        ++round;
        valid = round * n_waves + wave_global < pg.n_tasks;
      }
    }
  };

  int f0 = 0;
  for (; f0 + PASS_D < pg.n_pad; f0 += PASS_D) {
#pragma unroll
    for (int j = 0; j < PASS_D; ++j) {
      if (f0 + j < pg.n_real) consume(ring.s[j]);
      cursor_load(ring.s[j], ic, pg, lane, true);
      cursor_advance(ic, epi, pg, n_waves);
    }
  }
  {   // the last PASS_D stages; their slots take the first stages of the following phase
    StageCursor<WT> nc;
    cursor_begin(nc, epi_next, pg_next, wave_global);
#pragma unroll
    for (int j = 0; j < PASS_D; ++j) {
      if (f0 + j < pg.n_real) consume(ring.s[j]);
      cursor_load(ring.s[j], nc, pg_next, lane, prime_next && (wave != 0 || j == 0));
      cursor_advance(nc, epi_next, pg_next, n_waves);
    }
  }
  __syncthreads();
  if (wave == 0) {
    typename Epi::State st;
    epi.init(st);
    for (int i = lane; i < PASS_WAVES * per_wave; i += 64) {
      const int w = i / per_wave, rem = i - w * per_wave;
      const int rnd = rem / MT, m = rem - rnd * MT;
      const int task = rnd * n_waves + blockIdx.x * PASS_WAVES + w;
      if (task < pg.n_tasks && m < n_valid) {
        const RowDesc mine = rd[m];
        const float *y = yres + ((w * PASS_MAX_ROUNDS + rnd) * MT + m) * 2;
        if constexpr (EpiReadsOld<Epi>::value) {
          if (i == lane) epi.finish_old(task, mine, y[0], y[1], old);
          else epi.finish(task, m, mine, y[0], y[1], st);
        } else {
          epi.finish(task, m, mine, y[0], y[1], st);
        }
      }
    }
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

template <typename WT, int MT, int HD, int G>
__global__ void __launch_bounds__(PASS_THREADS)
spark_pass_k(PassParams<WT> p) {
  extern __shared__ float4 smem4[];
  float *lds = (float *)smem4;
  __shared__ int s_flag;
  __shared__ float red[PASS_WAVES * MT];
  __shared__ float yres[PASS_WAVES * PASS_MAX_ROUNDS * MT * 2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_waves = gridDim.x * PASS_WAVES, wave_global = blockIdx.x * PASS_WAVES + wave;
  const int n_valid = min(MT, p.m_rows);
  // the row descriptors live in LDS: several places pick one by an index known only at run time,
  // which in registers would send the array to scratch memory
  __shared__ RowDesc rd[MT];
  if (tid < MT) rd[tid] = p.rows[tid < n_valid ? tid : n_valid - 1];
  __syncthreads();
  unsigned round = p.round_base;
  int tl = 0;
  auto mark = [&]() {
    if (p.timeline && blockIdx.x == 0 && threadIdx.x == 0) p.timeline[tl] = wall_clock64();
    ++tl;
  };
  mark();

  const int d = p.d, qw = p.nq * HD, kvw = p.nkv * HD, F = p.F;
  const PhaseGeom g_qkv = make_geom<WT>(d, (p.nq + 2 * p.nkv) * (HD / 2), p.kc_d, n_waves);
  const PhaseGeom g_o = make_geom<WT>(qw, d / 2, p.kc_q, n_waves);
  const PhaseGeom g_gu = make_geom<WT>(d, F, p.kc_d, n_waves);
  const PhaseGeom g_dn = make_geom<WT>(F, d / 2, p.kc_f, n_waves);

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

  PRing ring;
  prime_ring<WT>(ring, epi_qkv(p.l0), g_qkv, true, n_waves, wave_global, lane, wave);

  for (int l = p.l0; l < p.l1; ++l) {
    // ---- q, k, v projections (+ rotary embedding, query store, KV-cache write); nothing is
    // prefetched across the attention phase, which needs the registers
    {
      PhaseIn in{PASS_IN_NORM, p.hidden, d, p.attn_norm + (size_t)l * d, p.eps};
      pass_gemv_phase<WT, MT>(in, epi_qkv(l), g_qkv, epi_o(l), g_o, false, rd, n_valid, lds, red,
                              yres, ring, n_waves, wave_global, tid);
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
        const RowDesc mine = rd[r];
        if (split * ATTN_SLICE <= mine.pos) {
          __syncthreads();  // LDS of the previous task is free
          attn_task<WT, HD, G, PASS_THREADS, true>(mine, r, hk, hk * G, G, split, p.qbuf, p.kv, l,
                                                   p.nq, p.n_splits, p.scale, p.part,
                                                   p.arrivals + r * p.nkv + hk, p.attn_out, SplitOut{nullptr, 0, 0, 0}, lds);
        }
      }
    }
    // the output projection's first weights fly during the barrier
    prime_ring<WT>(ring, epi_o(l), g_o, true, n_waves, wave_global, lane, wave);
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- attention output projection, residual add
    {
      PhaseIn in{PASS_IN_PLAIN, p.attn_out, qw, nullptr, 0.f};
      pass_gemv_phase<WT, MT>(in, epi_o(l), g_o, epi_gu(l), g_gu, true, rd, n_valid, lds, red, yres,
                              ring, n_waves, wave_global, tid);
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- gate and up projections, SiLU(gate) * up
    {
      PhaseIn in{PASS_IN_NORM, p.hidden, d, p.mlp_norm + (size_t)l * d, p.eps};
      pass_gemv_phase<WT, MT>(in, epi_gu(l), g_gu, epi_dn(l), g_dn, true, rd, n_valid, lds, red, yres,
                              ring, n_waves, wave_global, tid);
    }
    mark();
    if (!grid_sync(p.gb, round, &s_flag)) return;
    mark();

    // ---- down projection, residual add
    {
      PhaseIn in{PASS_IN_PLAIN, p.act, F, nullptr, 0.f};
      const bool more = l + 1 < p.l1;
      pass_gemv_phase<WT, MT>(in, epi_dn(l), g_dn, epi_qkv(more ? l + 1 : l), g_qkv, more, rd, n_valid,
                              lds, red, yres, ring, n_waves, wave_global, tid);
      mark();
      if (more) {
        if (!grid_sync(p.gb, round, &s_flag)) return;
        mark();
      }
    }
  }
}

}  // namespace spark
