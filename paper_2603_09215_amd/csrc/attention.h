// Grouped-query attention of a few query rows over the paged KV cache (decode, flush, prefill
// chunks).  Row r attends cache entries 0..pos_r of its own sequence; since the projection kernel
// has already written K/V of every row of the pass, this is causal inside a batch of pending
// positions as well (the "length-K causal mask" of Sec. IV-B.3).
//
// Few KV heads cannot fill 256 CUs, so the context is cut into slices: one block per
// (slice, kv head, row) produces an unnormalised partial (max, sum, weighted values) for all the
// query heads of the group, and a second kernel merges the slices.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int ATTN_THREADS = 256;
constexpr int ATTN_MAX_GROUP = 16;  // query heads per KV head

// partial layout: part[((r*nq + hq)*n_splits + split)*(hd+2)] = {o[hd], m, l}
template <typename KT, int HD>
__global__ void __launch_bounds__(ATTN_THREADS)
attn_partial_k(const RowDesc *__restrict__ rows, const float *__restrict__ qbuf, KVView kv,
               int layer, int nq, int group, int slice, int n_splits, float scale,
               float *__restrict__ part) {
  extern __shared__ float4 smem4[];
  float *qs = (float *)smem4;           // [group][HD]
  float *sc = qs + group * HD;          // [group][slice]
  float *ml = sc + group * slice;       // [group][2]
  float *ored = ml + group * 2;         // [ATTN_THREADS/ (HD/2)][group][HD] partial outputs

  const int split = blockIdx.x, hk = blockIdx.y, r = blockIdx.z;
  const RowDesc rd = rows[r];
  const int ctx = rd.pos + 1;
  const int t0 = split * slice, t1 = min(ctx, t0 + slice);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hq0 = hk * group;

  if (t0 >= ctx) {  // empty slice: neutral element of the merge
    for (int i = tid; i < group * (HD + 2); i += ATTN_THREADS) {
      int g = i / (HD + 2), c = i - g * (HD + 2);
      float *p = part + ((size_t)(r * nq + hq0 + g) * n_splits + split) * (HD + 2);
      p[c] = c == HD ? -INFINITY : 0.f;
    }
    return;
  }
  const int n_tok = t1 - t0;

  for (int i = tid; i < group * HD; i += ATTN_THREADS)
    qs[i] = qbuf[(size_t)r * nq * HD + hq0 * HD + i] * scale;
  __syncthreads();

  // scores: one token per thread, the whole key row in registers 16 bytes at a time
  constexpr int VEC = Elem<KT>::VEC;
  for (int t = tid; t < slice; t += ATTN_THREADS) {
    if (t < n_tok) {
      const KT *kp = (const KT *)kv.pool + kv_elem_offset(kv, rd.seq, t0 + t, layer, 0, hk);
      float s[ATTN_MAX_GROUP];
#pragma unroll
      for (int g = 0; g < ATTN_MAX_GROUP; ++g) s[g] = 0.f;
#pragma unroll 4
      for (int c = 0; c < HD; c += VEC) {
        uint4 raw = *(const uint4 *)(kp + c);
        float kf[VEC];
        Elem<KT>::unpack(raw, kf);
#pragma unroll
        for (int g = 0; g < ATTN_MAX_GROUP; ++g) {
          if (g < group) {
            const float *q = qs + g * HD + c;
#pragma unroll
            for (int e = 0; e < VEC; ++e) s[g] += q[e] * kf[e];
          }
        }
      }
#pragma unroll
      for (int g = 0; g < ATTN_MAX_GROUP; ++g)
        if (g < group) sc[g * slice + t] = s[g];
    } else {
      for (int g = 0; g < group; ++g) sc[g * slice + t] = -INFINITY;
    }
  }
  __syncthreads();

  // per query head: max, exp, sum over the slice (one wave per head at a time)
  for (int g = wave; g < group; g += ATTN_THREADS / 64) {
    float mx = -INFINITY;
    for (int t = lane; t < slice; t += 64) mx = fmaxf(mx, sc[g * slice + t]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int t = lane; t < slice; t += 64) {
      float p = t < n_tok ? expf(sc[g * slice + t] - mx) : 0.f;
      sc[g * slice + t] = p;
      sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) { ml[g * 2] = mx; ml[g * 2 + 1] = sum; }
  }
  __syncthreads();

  // weighted values: thread owns two adjacent dims of one token stripe
  constexpr int DT = HD / 2;                 // threads per token
  constexpr int STRIPES = ATTN_THREADS / DT; // tokens in flight
  const int dpair = tid % DT, stripe = tid / DT;
  float o0[ATTN_MAX_GROUP], o1[ATTN_MAX_GROUP];
#pragma unroll
  for (int g = 0; g < ATTN_MAX_GROUP; ++g) o0[g] = o1[g] = 0.f;
  for (int t = stripe; t < n_tok; t += STRIPES) {
    const KT *vp = (const KT *)kv.pool + kv_elem_offset(kv, rd.seq, t0 + t, layer, 1, hk) + 2 * dpair;
    float v0 = Elem<KT>::widen(vp[0]), v1 = Elem<KT>::widen(vp[1]);
#pragma unroll
    for (int g = 0; g < ATTN_MAX_GROUP; ++g) {
      if (g < group) {
        float p = sc[g * slice + t];
        o0[g] += p * v0;
        o1[g] += p * v1;
      }
    }
  }
#pragma unroll
  for (int g = 0; g < ATTN_MAX_GROUP; ++g) {
    if (g < group) {
      ored[(stripe * group + g) * HD + 2 * dpair] = o0[g];
      ored[(stripe * group + g) * HD + 2 * dpair + 1] = o1[g];
    }
  }
  __syncthreads();
  for (int i = tid; i < group * HD; i += ATTN_THREADS) {
    int g = i / HD, c = i - g * HD;
    float o = 0.f;
#pragma unroll
    for (int s = 0; s < STRIPES; ++s) o += ored[(s * group + g) * HD + c];
    part[((size_t)(r * nq + hq0 + g) * n_splits + split) * (HD + 2) + c] = o;
  }
  if (tid < group * 2) {
    int g = tid >> 1, w = tid & 1;
    part[((size_t)(r * nq + hq0 + g) * n_splits + split) * (HD + 2) + HD + w] = ml[g * 2 + w];
  }
}

inline size_t attn_partial_lds_bytes(int group, int hd, int slice) {
  int stripes = ATTN_THREADS / (hd / 2);
  return sizeof(float) * ((size_t)group * hd + (size_t)group * slice + group * 2 +
                          (size_t)stripes * group * hd);
}

// out[r][hq*HD + c] = sum_s exp(m_s - M) o_s[c] / sum_s exp(m_s - M) l_s
template <int HD>
__global__ void __launch_bounds__(HD)
attn_merge_k(const float *__restrict__ part, int nq, int n_splits, float *__restrict__ out) {
  const int hq = blockIdx.x, r = blockIdx.y, c = threadIdx.x;
  const float *p = part + (size_t)(r * nq + hq) * n_splits * (HD + 2);
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, p[s * (HD + 2) + HD]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    float m = p[s * (HD + 2) + HD];
    if (m == -INFINITY) continue;
    float w = expf(m - M);
    num += w * p[s * (HD + 2) + c];
    den += w * p[s * (HD + 2) + HD + 1];
  }
  out[(size_t)r * nq * HD + hq * HD + c] = num / den;
}

}  // namespace spark
