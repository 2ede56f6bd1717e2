// Projections for 16..128 activation rows at once (prompt chunks, batched decoding) on the MFMA
// units.  With that many rows a projection is a real dense contraction: every weight element is
// used 32..128 times, so the vector kernel that serves a handful of rows would be ALU-bound.
//
// Weights are bf16.  Activations are fp32; each is split into three bf16 parts (x = hi + mid + lo
// exactly, 3 x 8 mantissa bits) and all three go through the MFMA, which keeps the result at fp32
// accuracy instead of rounding the activations to 8 bits of mantissa.  (Two parts leave 2^-17
// relative error per element; re-rounded to bf16 in the KV cache that is enough to double the
// deviation from the oracle, so the third part is kept.)
//
// v_mfma_f32_32x32x16_bf16: A is 32 weight rows x 16 k, B is 16 k x 32 activation rows; lane l
// supplies 8 consecutive k of row (l % 32), k-block (l / 32); of the 16 results in a lane,
// register r belongs to weight row (r/4)*8 + (l/32)*4 + r%4 and activation row l % 32.
//
// A workgroup owns 128 "tasks" (the same pairs of weight rows the vector kernel uses, so the
// epilogues are shared: rotary pairs, gate/up pairs, adjacent rows), 32 per wave, and all rows of
// one 32..128-row tile.  The k range may be split over blockIdx.y; partial sums then go to a
// buffer and a second kernel finishes them, which is what fills 256 CUs when a matrix has only a
// few thousand rows.
#pragma once
#include "device_common.h"
#include "gemv.h"

namespace spark {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int MG_THREADS = 256;
constexpr int MG_WAVES = 4;
constexpr int MG_KC = 64;              // k per LDS chunk (4 MFMA steps of 16)
constexpr int MG_ROWPAD = MG_KC + 8;   // bf16 per staged activation row (16-byte skew per row)
constexpr int MG_TASKS_PER_WAVE = 32;
constexpr int MG_TASKS_PER_BLOCK = MG_WAVES * MG_TASKS_PER_WAVE;

// ------------------------------------------------------------------ activation preparation

// xs[part][r][k] = the three bf16 parts of x_r[k], x_r = src row (plain) or
// RMSNorm(hidden[x_slot_r]; gamma); part p starts at xs + p * part_stride
__global__ void __launch_bounds__(256)
prep_rows_k(const RowDesc *__restrict__ rows, const float *__restrict__ src, int stride, int indirect,
            const float *__restrict__ gamma, float eps, int n, bf16_t *__restrict__ xs,
            size_t part_stride) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const float *row = src + (size_t)(indirect ? rows[r].x_slot : r) * stride;
  float inv = 1.0f;
  if (gamma) {
    float ss = 0.f;
    for (int k = threadIdx.x * 4; k < n; k += 1024) {
      const float4 v = *(const float4 *)(row + k);
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)n + eps);
  }
  for (int k = threadIdx.x * 4; k < n; k += 1024) {
    float4 v = *(const float4 *)(row + k);
    if (gamma) {
      const float4 g = *(const float4 *)(gamma + k);
      v = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
    }
    const float f[4] = {v.x, v.y, v.z, v.w};
    bf16_t h[4], mid[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h[e] = f32_to_bf16(f[e]);
      const float rem = f[e] - bf16_to_f32(h[e]);      // exact
      mid[e] = f32_to_bf16(rem);
      l[e] = f32_to_bf16(rem - bf16_to_f32(mid[e]));   // exact remainder has at most 8 bits left
    }
    bf16_t *dst = xs + (size_t)r * n + k;
    *(uint2 *)dst = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    *(uint2 *)(dst + part_stride) = make_uint2(mid[0] | ((uint32_t)mid[1] << 16), mid[2] | ((uint32_t)mid[3] << 16));
    *(uint2 *)(dst + 2 * part_stride) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
  }
}

// ------------------------------------------------------------------ the contraction

// grid.x: blocks of 128 tasks; grid.y: k splits; grid.z: tiles of 32*MTILES activation rows.
// SPLIT: write partial sums part[split][task][2][m_pad] instead of running the epilogue.
template <int MTILES, typename Epi, bool SPLIT>
__global__ void __launch_bounds__(MG_THREADS)
mfma_rows_k(Epi epi, const RowDesc *__restrict__ rows, int m_rows, const bf16_t *__restrict__ xs,
            size_t part_stride, int n_in, int n_tasks, int chunks_per_split,
            float *__restrict__ part, int m_pad) {
  constexpr int MROWS = 32 * MTILES;
  __shared__ __attribute__((aligned(16))) bf16_t s_x[3][MROWS * MG_ROWPAD];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = blockIdx.z * MROWS;
  const int task0 = blockIdx.x * MG_TASKS_PER_BLOCK + wave * MG_TASKS_PER_WAVE;
  const int my_task = task0 + (lane & 31);
  const int n_chunks = (n_in + MG_KC - 1) / MG_KC;
  const int c_begin = blockIdx.y * chunks_per_split;
  const int c_end = min(n_chunks, c_begin + chunks_per_split);

  const bf16_t *r0, *r1;
  epi.weight_rows(my_task < n_tasks ? my_task : 0, r0, r1);
  const int koff = (lane >> 5) * 8;   // this lane's k-block inside an MFMA step

  f32x16_t acc0[MTILES], acc1[MTILES];
#pragma unroll
  for (int c = 0; c < MTILES; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[c][r] = acc1[c][r] = 0.f;

  // weights of one chunk: 4 MFMA steps x 2 tiles, 16 bytes each; n_in is a multiple of 8, a
  // chunk's tail beyond n_in reads as zero
  uint4 wa[MG_KC / 16], wb[MG_KC / 16];
  auto load_chunk = [&](int chunk) {
#pragma unroll
    for (int s = 0; s < MG_KC / 16; ++s) {
      const int k = chunk * MG_KC + s * 16 + koff;
      if (k < n_in) {
        wa[s] = load_weights16(r0 + k);
        wb[s] = load_weights16(r1 + k);
      } else {
        wa[s] = make_uint4(0, 0, 0, 0);
        wb[s] = make_uint4(0, 0, 0, 0);
      }
    }
  };

  if (c_begin < c_end) load_chunk(c_begin);
  for (int chunk = c_begin; chunk < c_end; ++chunk) {
    uint4 ca[MG_KC / 16], cb[MG_KC / 16];
#pragma unroll
    for (int s = 0; s < MG_KC / 16; ++s) { ca[s] = wa[s]; cb[s] = wb[s]; }
    __syncthreads();   // the previous chunk's activations are no longer read
    // stage activations of this chunk: MROWS rows x 64 k, hi and lo, 16 bytes per thread and step
    for (int v = threadIdx.x; v < MROWS * (MG_KC / 8); v += MG_THREADS) {
      const int m = v / (MG_KC / 8), kv = (v - m * (MG_KC / 8)) * 8;
      const int k = chunk * MG_KC + kv;
      uint4 x3[3] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
      if (row0 + m < m_rows && k < n_in) {
        const bf16_t *src = xs + (size_t)(row0 + m) * n_in + k;
#pragma unroll
        for (int p = 0; p < 3; ++p) x3[p] = *(const uint4 *)(src + p * part_stride);
      }
#pragma unroll
      for (int p = 0; p < 3; ++p) *(uint4 *)(s_x[p] + m * MG_ROWPAD + kv) = x3[p];
    }
    if (chunk + 1 < c_end) load_chunk(chunk + 1);   // next chunk's weights fly during the MFMAs
    __syncthreads();
#pragma unroll
    for (int s = 0; s < MG_KC / 16; ++s) {
      const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, ca[s]);
      const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, cb[s]);
#pragma unroll
      for (int c = 0; c < MTILES; ++c) {
        const int off = (c * 32 + (lane & 31)) * MG_ROWPAD + s * 16 + koff;
        // smallest part first, so that the large terms are added last
#pragma unroll
        for (int p = 2; p >= 0; --p) {
          const bf16x8_t b = __builtin_bit_cast(bf16x8_t, *(const uint4 *)(s_x[p] + off));
          acc0[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc0[c], 0, 0, 0);
          acc1[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc1[c], 0, 0, 0);
        }
      }
    }
  }

  // results: register r <-> task (r/4)*8 + (lane/32)*4 + r%4 of this wave, activation row lane%32
  typename Epi::State st;
  epi.init(st);
#pragma unroll
  for (int c = 0; c < MTILES; ++c) {
    const int m = row0 + c * 32 + (lane & 31);
    const bool m_ok = m < m_rows;
    RowDesc rd = rows[m_ok ? m : 0];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int task = task0 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      if (task < n_tasks) {
        if (SPLIT) {
          float *p = part + (((size_t)blockIdx.y * n_tasks + task) * 2) * m_pad + m;
          if (m < m_pad) { p[0] = acc0[c][r]; p[m_pad] = acc1[c][r]; }
        } else if (m_ok) {
          epi.finish(task, m, rd, acc0[c][r], acc1[c][r], st);
        }
      }
    }
    if (!SPLIT && MTILES == 1 && m_ok) epi.end(m, rd, st);
  }
}

// sums the k-split partials and runs the epilogue: one thread per (task, activation row)
template <typename Epi>
__global__ void __launch_bounds__(256)
mfma_finish_k(Epi epi, const RowDesc *__restrict__ rows, int m_rows, int n_tasks, int n_split,
              const float *__restrict__ part, int m_pad) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int task = idx / m_pad, m = idx - task * m_pad;
  if (task >= n_tasks || m >= m_rows) return;
  float y0 = 0.f, y1 = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float *p = part + (((size_t)s * n_tasks + task) * 2) * m_pad + m;
    y0 += p[0];
    y1 += p[m_pad];
  }
  typename Epi::State st;
  epi.init(st);
  epi.finish(task, m, rows[m], y0, y1, st);
}

}  // namespace spark
