// Grouped-query attention of a few query rows over the paged KV cache (decode, flush, prefill
// chunks).  Row r attends cache entries 0..pos_r of its own sequence; since the projection step
// has already written K/V of every row of the pass, this is causal inside a batch of pending
// positions as well (the "length-K causal mask" of Sec. IV-B.3).
//
// Few KV heads cannot fill 256 CUs, so the context is cut into slices of 64 tokens: one task per
// (slice, kv head, row) produces an unnormalised partial (max, sum, weighted values) for all the
// query heads of the group, and the workgroup that finishes last for a (row, kv head) merges the
// slices (arrival counter, device-scope accesses), so no second launch is needed.  Inside a task a
// token's key (and value) vector is spread over LPT consecutive lanes, 16 bytes each, so a wave
// reads 64/LPT whole rows per instruction; all K and V loads of the slice are issued before any
// use.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int ATTN_THREADS = 256;
constexpr int ATTN_SLICE = 64;      // tokens per task
constexpr int ATTN_MAX_GROUP = 16;  // query heads per KV head
static_assert(ATTN_SLICE == 64, "the softmax step maps one token to one lane of a wave");

// Synchronise the NT threads that execute a task: a workgroup barrier, or, when a single wave runs
// the task inside a larger workgroup, only the memory ordering (a wave is in lockstep already).
template <int NT> __device__ __forceinline__ void task_sync() {
  if (NT == 64) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
  } else {
    __syncthreads();
  }
}

// floats of LDS one task needs with NT threads: scores, softmax statistics, per-wave sums
template <int HD, int G, int NT> constexpr int attn_lds_floats() {
  return G * ATTN_SLICE + G * 2 + (NT / 64) * G * HD + 4;
}

// partial layout: part[((r*nq + hq)*n_splits + split)*(HD+4)] = {o[HD], m, l, pad, pad}
//
// One task, executed by all NT threads of a workgroup: query heads hq0 .. hq0 + g_count - 1
// (g_count <= G, all sharing KV head hk) of row r over one slice; `cnt` counts the slices of this
// (row, group of heads) that are done.  DS: the queries were written, and the output will be
// read, by other workgroups of the same kernel (device-scope accesses).
template <typename KT, int HD, int G, int NT, bool DS>
__device__ __forceinline__ void attn_task(const RowDesc &rd, int r, int hk, int hq0, int g_count,
                                          int split, const float *__restrict__ qbuf, const KVView &kv,
                                          int layer, int nq, int n_splits, float scale,
                                          float *__restrict__ part, int *__restrict__ cnt,
                                          float *__restrict__ out, const SplitOut &so, float *lds) {
  constexpr int VEC = Elem<KT>::VEC;
  constexpr int LPT = HD / VEC;                   // lanes per token
  constexpr int TPI = NT / LPT;                   // tokens per iteration of the workgroup
  constexpr int ITERS = (ATTN_SLICE + TPI - 1) / TPI;
  constexpr int WAVES = NT / 64;
  constexpr int PS = HD + 4;
  float *sc = lds;                                // [G][ATTN_SLICE] scores, then probabilities
  float *ml = sc + G * ATTN_SLICE;                // [G][2]
  float *ored = ml + G * 2;                       // [WAVES][G][HD]
  int *s_last = (int *)(lds + attn_lds_floats<HD, G, NT>() - 4);

  const int ctx = rd.pos + 1;
  const int t0 = split * ATTN_SLICE;
  const int n_tok = min(ATTN_SLICE, ctx - t0);
  const int tid = threadIdx.x % NT, lane = tid & 63, wave = tid >> 6;
  const int tg = tid / LPT, dc = tid % LPT;       // token slot in an iteration, 16-byte chunk of the row

  // issue every K and V load of the slice
  uint4 kraw[ITERS], vraw[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int t = it * TPI + tg;
    if (t < n_tok) {
      const KT *kp = (const KT *)kv.pool + kv_elem_offset(kv, rd.seq, t0 + t, layer, 0, hk) + dc * VEC;
      const KT *vp = (const KT *)kv.pool + kv_elem_offset(kv, rd.seq, t0 + t, layer, 1, hk) + dc * VEC;
      kraw[it] = *(const uint4 *)kp;
      vraw[it] = *(const uint4 *)vp;
    } else {
      kraw[it] = make_uint4(0, 0, 0, 0);
      vraw[it] = make_uint4(0, 0, 0, 0);
    }
  }

  // this lane's chunk of every query head of the group, pre-scaled
  float q[G][VEC];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float *qp = qbuf + (size_t)r * nq * HD + (hq0 + min(g, g_count - 1)) * HD + dc * VEC;
#pragma unroll
    for (int e = 0; e < VEC; e += 2) {
      float2 v = load2_maybe_ds<DS>(qp + e);
      q[g][e] = v.x * scale; q[g][e + 1] = v.y * scale;
    }
  }

  // scores
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int t = it * TPI + tg;
    float kf[VEC];
    Elem<KT>::unpack(kraw[it], kf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += q[g][e] * kf[e];
#pragma unroll
      for (int o = LPT / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (dc == 0 && t < ATTN_SLICE) sc[g * ATTN_SLICE + t] = t < n_tok ? s : -INFINITY;
    }
  }
  task_sync<NT>();

  // softmax statistics of the slice, one wave per query head at a time (lane = token)
  for (int g = wave; g < g_count; g += WAVES) {
    float s = sc[g * ATTN_SLICE + lane];
    float mx = wave_max(s);
    float p = lane < n_tok ? expf(s - mx) : 0.f;
    sc[g * ATTN_SLICE + lane] = p;
    float sum = wave_sum(p);
    if (lane == 0) { ml[g * 2] = mx; ml[g * 2 + 1] = sum; }
  }
  task_sync<NT>();

  // weighted values: acc[g][e] over this thread's tokens, then over the token slots of the wave
  float acc[G][VEC];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[g][e] = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int t = it * TPI + tg;
    if (t < ATTN_SLICE) {
      float vf[VEC];
      Elem<KT>::unpack(vraw[it], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = sc[g * ATTN_SLICE + t];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[g][e] += p * vf[e];
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      float a = acc[g][e];
#pragma unroll
      for (int o = LPT; o < 64; o <<= 1) a += __shfl_xor(a, o, 64);
      if (lane < LPT) ored[(wave * G + g) * HD + dc * VEC + e] = a;
    }
  task_sync<NT>();
  for (int i = tid; i < g_count * HD; i += NT) {
    const int g = i / HD, c = i - g * HD;
    float o = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) o += ored[(w * G + g) * HD + c];
    store_device_scope(part + ((size_t)(r * nq + hq0 + g) * n_splits + split) * PS + c, o);
  }
  if (tid < g_count * 2) {
    const int g = tid >> 1, w = tid & 1;
    store_device_scope(part + ((size_t)(r * nq + hq0 + g) * n_splits + split) * PS + HD + w,
                       ml[g * 2 + w]);
  }

  // The workgroup that arrives last for this (row, kv head) merges the slices:
  // out = sum_s exp(m_s - M) o_s / sum_s exp(m_s - M) l_s.
  // Partials are written through to memory (device-scope stores) and counted with a device-scope
  // atomic; the merging workgroup drops its stale cache lines once and then reads them normally.
  const int used = (rd.pos + ATTN_SLICE) / ATTN_SLICE;   // slices that intersect the context
  wait_memory_ops();                                      // partials written before the count
  task_sync<NT>();
  if (tid == 0) {
    const int prev = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_last = prev == used - 1;
    if (*s_last) {
      __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next layer
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // one cache invalidate for the workgroup
    }
  }
  task_sync<NT>();
  if (!*s_last) return;

  // every thread merges four output elements of one head over all slices in one pass (running
  // maximum, rescaled sums), eight slices' loads in flight at a time
  for (int i = tid; i < g_count * (HD / 4); i += NT) {
    const int g = i / (HD / 4), c = (i - g * (HD / 4)) * 4;
    const float *p = part + (size_t)(r * nq + hq0 + g) * n_splits * PS;
    float M = -INFINITY, L = 0.f;
    float4 acc4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < used; s0 += 8) {
      float2 ml8[8];
      float4 o8[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int sl = min(s0 + k, used - 1);
        ml8[k] = *(const float2 *)(p + (size_t)sl * PS + HD);
        o8[k] = *(const float4 *)(p + (size_t)sl * PS + c);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (s0 + k < used) {
          const float Mn = fmaxf(M, ml8[k].x);
          const float so = expf(M - Mn), sn = expf(ml8[k].x - Mn);   // exp(-inf) = 0 on the first slice
          acc4.x = acc4.x * so + o8[k].x * sn; acc4.y = acc4.y * so + o8[k].y * sn;
          acc4.z = acc4.z * so + o8[k].z * sn; acc4.w = acc4.w * so + o8[k].w * sn;
          L = L * so + ml8[k].y * sn;
          M = Mn;
        }
      }
    }
    const float inv = 1.0f / L;
    float *dst = out + (size_t)r * nq * HD + (hq0 + g) * HD + c;
    store2_maybe_ds<DS>(dst, make_float2(acc4.x * inv, acc4.y * inv));
    store2_maybe_ds<DS>(dst + 2, make_float2(acc4.z * inv, acc4.w * inv));
    // for the MFMA output projection: the same values as three bf16 parts
    if (so.xs)
      split_store4(so, r, (hq0 + g) * HD + c, make_float4(acc4.x * inv, acc4.y * inv, acc4.z * inv, acc4.w * inv));
  }
  if (DS) wait_memory_ops();   // the caller's next barrier arrival does not wait for these stores
}

// stand-alone launch: one workgroup per (slice, group of G query heads, row).  A KV head's `group`
// query heads are dealt to ceil(group / G) workgroups: with few rows and few KV heads that is what
// gives the chip enough workgroups, at the price of reading the slice's K and V once per group.
template <typename KT, int HD, int G>
__global__ void __launch_bounds__(ATTN_THREADS)
attn_rows_k(const RowDesc *__restrict__ rows, const float *__restrict__ qbuf, KVView kv,
            int layer, int nq, int group, int n_splits, float scale, float *__restrict__ part,
            int *__restrict__ arrivals, float *__restrict__ out, SplitOut so) {
  __shared__ float lds[attn_lds_floats<HD, G, ATTN_THREADS>()];
  const int n_groups = (group + G - 1) / G;
  const int split = blockIdx.x, hk = blockIdx.y / n_groups, gi = blockIdx.y - hk * n_groups, r = blockIdx.z;
  const RowDesc rd = rows[r];
  if (split * ATTN_SLICE > rd.pos) return;        // slice beyond the row's context
  attn_task<KT, HD, G, ATTN_THREADS, false>(rd, r, hk, hk * group + gi * G, min(G, group - gi * G), split,
                                            qbuf, kv, layer, nq, n_splits, scale, part,
                                            arrivals + r * gridDim.y + blockIdx.y, out, so, lds);
}

}  // namespace spark
