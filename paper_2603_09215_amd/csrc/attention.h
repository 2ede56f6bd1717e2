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
// Second half of a task, executed by all NT threads that produced the partial of one slice for
// query heads hq0 .. hq0 + g_count - 1 of row r: count the slice as done; the workgroup that
// arrives last for this (row, group of heads) merges the slices,
// out = sum_s exp(m_s - M) o_s / sum_s exp(m_s - M) l_s.
template <int HD, int NT, bool DS>
__device__ __forceinline__ void attn_merge(const RowDesc &rd, int r, int hq0, int g_count, int nq,
                                           int n_splits, int slice_tokens, const float *__restrict__ part,
                                           int *__restrict__ cnt, float *__restrict__ out,
                                           const SplitOut &so, int *s_last) {
  constexpr int PS = HD + 4;
  const int tid = threadIdx.x % NT;
  // Partials are written through to memory (device-scope stores) and counted with a device-scope
  // atomic; the merging workgroup drops its stale cache lines once and then reads them normally.
  const int used = rd.pos / slice_tokens + 1;   // slices that intersect the context
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
  attn_merge<HD, NT, DS>(rd, r, hq0, g_count, nq, n_splits, ATTN_SLICE, part, cnt, out, so, s_last);
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

// ------------------------------------------------------------------ the same task on the MFMA units
//
// bf16 cache, head_dim 128, up to 16 query heads per KV head, one workgroup (4 waves) per
// (slice, KV head or half of its query heads, row); a slice is one or several 64-token pieces,
// taken one after the other.  Per piece, v_mfma_f32_16x16x32_bf16 twice:
//   scores   S^T[token][head] = K[token][:] . Q[head][:]   wave w takes tokens 16w .. 16w+15; the K
//            rows go from memory straight into the A operand (lane l: token l%16, eight
//            consecutive elements at 8*(l/16) of each 32-wide step), the scaled queries, split into
//            three bf16 parts that add up to the fp32 value (once per workgroup, handed to the
//            waves through LDS), are the B operand;
//   values   O[head][hd] = P[head][token] . V[token][hd]   wave w takes hd 32w .. 32w+31 over all
//            64 tokens; P (two bf16 parts) crosses the waves through LDS in A-operand order, V is
//            staged in LDS as it lies in the cache (token-major) and gathered column-wise, the
//            only transposition the operation needs.
// The partial it leaves and the merge are those of the vector task.
typedef __attribute__((ext_vector_type(8))) __bf16 attn_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float attn_f32x4_t;
typedef unsigned int attn_u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int attn_u32x2_t __attribute__((ext_vector_type(2)));

constexpr int AM_VPITCH = 130;   // bf16 elements per V row in LDS: 65 dwords, so the four token groups of a gather hit different banks
constexpr int AM_PPITCH = 72;    // tokens per P row in LDS (16-byte aligned rows)
constexpr int AM_QPITCH = 136;   // elements per Q row in LDS (16-byte aligned rows, 4 dwords of skew)

__device__ __forceinline__ unsigned pack_bf16(bf16_t lo, bf16_t hi) { return (unsigned)lo | ((unsigned)hi << 16); }

// loads of one 64-token piece: V as the workgroup stages it, K as this wave's A operand
struct AttnPiece {
  attn_u32x4_t v[4];
  attn_bf16x8_t k[4];
};

template <int HD>
__device__ __forceinline__ void attn_piece_load(AttnPiece &pc, const KVView &kv, const bf16_t *pool, int seq,
                                                int layer, int hk, int t0, int n_tok, bool one_page,
                                                int tid, int wave, int col, int quad) {
  // tokens beyond the context read token t0 instead (it exists) and are masked later.  With pages
  // of a multiple of 64 tokens the piece lies inside one page: one address for the workgroup.
  const size_t piece_k = one_page ? kv_elem_offset(kv, seq, t0, layer, 0, hk) : 0;
  const size_t piece_v = one_page ? kv_elem_offset(kv, seq, t0, layer, 1, hk) : 0;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int t = it * 16 + (tid >> 4), tt = t < n_tok ? t : 0;
    const size_t o = one_page ? piece_v + (size_t)tt * HD : kv_elem_offset(kv, seq, t0 + tt, layer, 1, hk);
    pc.v[it] = *(const attn_u32x4_t *)(pool + o + (tid & 15) * 8);
  }
  const int t = 16 * wave + col, tt = t < n_tok ? t : 0;
  const size_t o = one_page ? piece_k + (size_t)tt * HD : kv_elem_offset(kv, seq, t0 + tt, layer, 0, hk);
  const bf16_t *kp = pool + o + quad * 8;
#pragma unroll
  for (int s = 0; s < 4; ++s) pc.k[s] = __builtin_bit_cast(attn_bf16x8_t, *(const attn_u32x4_t *)(kp + 32 * s));
}

// `pieces` 64-token pieces per workgroup (slice = 64 * pieces tokens): a workgroup's life is mostly
// dependent round trips (row descriptor, page table, K/V, partial, arrival), so with many rows it
// pays to put several pieces behind one such chain; the pieces are folded with a running maximum.
template <int HD>
__global__ void __launch_bounds__(ATTN_THREADS)
attn_rows_mfma_k(const RowDesc *__restrict__ rows, const float *__restrict__ qbuf, KVView kv, int layer,
                 int nq, int kv_group, int heads_per_wg, int n_splits, int pieces, float scale,
                 float *__restrict__ part, int *__restrict__ arrivals, float *__restrict__ out, SplitOut so) {
  static_assert(HD == 128, "four 32-wide steps per key row, four waves of 32 value columns");
  constexpr int PS = HD + 4;
  __shared__ __align__(16) bf16_t s_v[ATTN_SLICE * AM_VPITCH];
  __shared__ __align__(16) bf16_t s_p[2 * 16 * AM_PPITCH];
  __shared__ __align__(16) bf16_t s_q[3 * 16 * AM_QPITCH];
  __shared__ float s_max[4 * 16], s_sum[4 * 16], s_alpha[16];
  __shared__ int s_last;
  // blockIdx.y = (KV head, part of its query heads): with few rows and few KV heads the query
  // heads of a KV head are dealt to several workgroups, which shortens each one's merge
  const int wg_per_kv = (kv_group + heads_per_wg - 1) / heads_per_wg;
  const int split = blockIdx.x, hk = blockIdx.y / wg_per_kv, r = blockIdx.z;
  const int h_first = (blockIdx.y - hk * wg_per_kv) * heads_per_wg;
  const int group = min(heads_per_wg, kv_group - h_first);   // query heads of this workgroup
  const RowDesc rd = rows[r];
  const int span = ATTN_SLICE * pieces;
  if (split * span > rd.pos) return;              // slice beyond the row's context
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, quad = lane >> 4;    // operand column / row, and which eight of a 32-wide step
  const int hq0 = hk * kv_group + h_first;
  const bf16_t *pool = (const bf16_t *)kv.pool;
  const bool one_page = (kv.page_tokens & (ATTN_SLICE - 1)) == 0;
  const int n_pieces = min(pieces, (rd.pos - split * span) / ATTN_SLICE + 1);   // pieces the context reaches

  AttnPiece cur;
  attn_piece_load<HD>(cur, kv, pool, rd.seq, layer, hk, split * span, min(ATTN_SLICE, rd.pos + 1 - split * span),
                      one_page, tid, wave, col, quad);

  // the scaled queries as three bf16 parts that add up to the fp32 value (each part keeps the
  // upper 8 significant bits of what the parts before it left: truncation, exact remainders):
  // split once by the workgroup, eight elements per thread, and handed to the waves through LDS
  {
    const int h = tid >> 4, e0 = (tid & 15) * 8;
    attn_u32x4_t ph = {0u, 0u, 0u, 0u}, pm = ph, pl = ph;
    if (h < group) {
      const float *qp = qbuf + ((size_t)r * nq + hq0 + h) * HD + e0;
      const float4 q0 = *(const float4 *)qp, q1 = *(const float4 *)(qp + 4);
      const float qf[8] = {q0.x * scale, q0.y * scale, q0.z * scale, q0.w * scale,
                           q1.x * scale, q1.y * scale, q1.z * scale, q1.w * scale};
      unsigned hi[8], mi[8], lo[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        hi[e] = __float_as_uint(qf[e]) & 0xffff0000u;
        const float r1 = qf[e] - __uint_as_float(hi[e]);
        mi[e] = __float_as_uint(r1) & 0xffff0000u;
        lo[e] = __float_as_uint(r1 - __uint_as_float(mi[e]));   // at most 8 significant bits are left
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        ph[e] = (hi[2 * e] >> 16) | hi[2 * e + 1];
        pm[e] = (mi[2 * e] >> 16) | mi[2 * e + 1];
        pl[e] = (lo[2 * e] >> 16) | (lo[2 * e + 1] & 0xffff0000u);
      }
    }
    *(attn_u32x4_t *)(s_q + (0 * 16 + h) * AM_QPITCH + e0) = ph;
    *(attn_u32x4_t *)(s_q + (1 * 16 + h) * AM_QPITCH + e0) = pm;
    *(attn_u32x4_t *)(s_q + (2 * 16 + h) * AM_QPITCH + e0) = pl;
  }

  // running state.  Score layout: lane = (head col, tokens 4*quad + i of the wave's 16);
  // output layout: lane = (hd 32*wave + 16*t + col, heads 4*quad + i).
  float run_max = -INFINITY, run_sum = 0.f;       // of head `col`; the sum is this wave's share
  attn_f32x4_t oacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

  for (int j = 0; j < n_pieces; ++j) {
    const int t0 = split * span + j * ATTN_SLICE;
    const int n_tok = min(ATTN_SLICE, rd.pos + 1 - t0);
    if (j > 0) __syncthreads();                   // the last piece's V and P have been consumed
    // V into LDS as it lies in the cache (4-byte stores: the row pitch is an odd number of dwords)
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      unsigned *dst = (unsigned *)(s_v + (it * 16 + (tid >> 4)) * AM_VPITCH + (tid & 15) * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e) dst[e] = cur.v[it][e];
    }
    attn_bf16x8_t ka[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) ka[s] = cur.k[s];
    if (j + 1 < n_pieces)                          // the next piece's loads fly during this one's arithmetic
      attn_piece_load<HD>(cur, kv, pool, rd.seq, layer, hk, t0 + ATTN_SLICE,
                          min(ATTN_SLICE, rd.pos + 1 - t0 - ATTN_SLICE), one_page, tid, wave, col, quad);
    __syncthreads();

    // scores of this wave's 16 tokens
    attn_f32x4_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int p = 0; p < 3; ++p) {
        const attn_bf16x8_t qb = __builtin_bit_cast(
            attn_bf16x8_t, *(const attn_u32x4_t *)(s_q + (p * 16 + col) * AM_QPITCH + 32 * s + 8 * quad));
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[s], qb, sc, 0, 0, 0);
      }
    const int tok0 = 16 * wave + 4 * quad;
    float mw = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (tok0 + i >= n_tok) sc[i] = -INFINITY;
      mw = fmaxf(mw, sc[i]);
    }
    mw = fmaxf(mw, __shfl_xor(mw, 16, 64));
    mw = fmaxf(mw, __shfl_xor(mw, 32, 64));
    if (quad == 0) s_max[wave * 16 + col] = mw;
    __syncthreads();
    const float piece_max = fmaxf(fmaxf(s_max[col], s_max[16 + col]), fmaxf(s_max[32 + col], s_max[48 + col]));
    const float new_max = fmaxf(run_max, piece_max);   // finite: token 0 of every piece is real
    const float alpha = expf(run_max - new_max);       // exp(-inf) = 0 on the first piece
    run_max = new_max;
    float pr[4], lw = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pr[i] = tok0 + i < n_tok ? expf(sc[i] - new_max) : 0.f;
      lw += pr[i];
    }
    lw += __shfl_xor(lw, 16, 64);
    lw += __shfl_xor(lw, 32, 64);
    run_sum = run_sum * alpha + lw;
    if (wave == 0 && quad == 0) s_alpha[col] = alpha;
    {
      // probabilities as two bf16 parts (16 significant bits)
      unsigned h[4], l[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        h[i] = __float_as_uint(pr[i]) & 0xffff0000u;
        l[i] = __float_as_uint(pr[i] - __uint_as_float(h[i])) & 0xffff0000u;
      }
      attn_u32x2_t ph = {(h[0] >> 16) | h[1], (h[2] >> 16) | h[3]};
      attn_u32x2_t pl = {(l[0] >> 16) | l[1], (l[2] >> 16) | l[3]};
      *(attn_u32x2_t *)(s_p + col * AM_PPITCH + tok0) = ph;
      *(attn_u32x2_t *)(s_p + 16 * AM_PPITCH + col * AM_PPITCH + tok0) = pl;
    }
    __syncthreads();

    // weighted values on top of the rescaled sums of the earlier pieces
    if (j > 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a = s_alpha[4 * quad + i];
        oacc[0][i] *= a;
        oacc[1][i] *= a;
      }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const attn_bf16x8_t pa0 = __builtin_bit_cast(
          attn_bf16x8_t, *(const attn_u32x4_t *)(s_p + col * AM_PPITCH + 32 * ks + 8 * quad));
      const attn_bf16x8_t pa1 = __builtin_bit_cast(
          attn_bf16x8_t, *(const attn_u32x4_t *)(s_p + 16 * AM_PPITCH + col * AM_PPITCH + 32 * ks + 8 * quad));
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16_t *vcol = s_v + (32 * ks + 8 * quad) * AM_VPITCH + 32 * wave + 16 * t + col;
        attn_u32x4_t vb;
#pragma unroll
        for (int e = 0; e < 4; ++e) vb[e] = pack_bf16(vcol[(2 * e) * AM_VPITCH], vcol[(2 * e + 1) * AM_VPITCH]);
        const attn_bf16x8_t b = __builtin_bit_cast(attn_bf16x8_t, vb);
        oacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa0, b, oacc[t], 0, 0, 0);
        oacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa1, b, oacc[t], 0, 0, 0);
      }
    }
  }

  // the slice's partial: weighted values, maximum, sum over the waves
  if (quad == 0) { s_sum[wave * 16 + col] = run_sum; s_max[col] = run_max; }
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = 4 * quad + i;
      if (g < group)
        store_device_scope(part + ((size_t)(r * nq + hq0 + g) * n_splits + split) * PS + 32 * wave + 16 * t + col,
                           oacc[t][i]);
    }
  __syncthreads();
  if (tid < group * 2) {
    const int g = tid >> 1;
    const float v = (tid & 1) ? s_sum[g] + s_sum[16 + g] + s_sum[32 + g] + s_sum[48 + g] : s_max[g];
    store_device_scope(part + ((size_t)(r * nq + hq0 + g) * n_splits + split) * PS + HD + (tid & 1), v);
  }
  attn_merge<HD, ATTN_THREADS, false>(rd, r, hq0, group, nq, n_splits, span, part,
                                      arrivals + r * gridDim.y + blockIdx.y, out, so, &s_last);
}

}  // namespace spark
