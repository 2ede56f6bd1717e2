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
// Two kernels run the contraction: mfma_tiled_k (further down) takes its weights from a copy in
// MFMA operand order that the context wrote when it was created, and is the one a context with
// such a copy runs; mfma_rows_k, described next, takes them from the caller's row-major tensors.
//
// A workgroup of eight waves owns 256 "tasks" (the same pairs of weight rows the vector kernel
// uses, so the epilogues are shared: rotary pairs, gate/up pairs, adjacent rows), 32 per wave, and
// all rows of one tile of 32 or 64 activation rows; more rows are further tiles (grid.z), whose
// workgroups read the same weights at about the same time.  The k range may be split over
// blockIdx.y; partial sums then go to a buffer and a second kernel finishes them, which is what
// fills 256 CUs when a matrix has only a few thousand rows.
//
// HBM delivers its bandwidth only to loads that cover whole 128-byte lines of a row in one
// instruction (measured: 6.3 TB/s, against 2.6 TB/s when a wave instruction takes 32 bytes from
// each of 32 rows, which is what loading straight into the A-operand layout does).  So a wave
// loads its 64 weight rows eight lanes per row, 128 bytes per row and instruction, and turns the
// result into the A-operand layout through a private piece of LDS: written as (row, 16-byte
// segment), read back as (lane % 32 = row, lane / 32 = segment of the MFMA step).
#pragma once
#include <type_traits>
#include "device_common.h"
#include "gemv.h"

namespace spark {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int MG_THREADS = 512;
constexpr int MG_WAVES = 8;
constexpr int MG_KC = 64;              // k per chunk: one 128-byte line of a weight row, 4 MFMA steps
constexpr int MG_ROWPAD = MG_KC + 8;   // bf16 per staged row (a 16-byte skew per row keeps the operand reads conflict-free)
constexpr int MG_TASKS_PER_WAVE = 32;
constexpr int MG_TASKS_PER_BLOCK = MG_WAVES * MG_TASKS_PER_WAVE;
constexpr int MG_MAX_MTILES = 2;       // activation rows per workgroup: 32 or 64
// bf16 parts of an activation that meet the weights: all three, so that every product is the
// exact product of the fp32 activation and the bf16 weight, as in the vector kernel.  (Two parts,
// 16 significant bits, would cut the MFMA and LDS work by a third at an error of 2^-17 per
// product; tried: the 1e-5 perturbations change which cache entries round up or down to bf16,
// and at the 40-layer shape that moved a logit by 0.022, past the 0.02 the parity tests allow.)
constexpr int MG_PARTS = 3;
// weight chunks a wave has in registers, on their way from HBM
constexpr int MG_W_DEPTH = 2;
// dynamic LDS of mfma_rows_k: per wave 64 padded weight rows of one chunk; two buffers of three
// parts of 32*MTILES padded activation rows
constexpr size_t mg_lds_bytes(int mtiles, int waves = MG_WAVES) {
  return sizeof(bf16_t) * (waves * 64 * MG_ROWPAD + 2 * MG_PARTS * 32 * mtiles * MG_ROWPAD);
}

// ------------------------------------------------------------------ activation preparation

// xs[part][r][k] = the three bf16 parts of x_r[k], x_r = src row (plain) or
// RMSNorm(hidden[x_slot_r]; gamma); rows are n_pad apart (n rounded up to the chunk of the
// contraction) and zero beyond n; part p starts at xs + p * part_stride
__global__ void __launch_bounds__(256)
prep_rows_k(const RowDesc *__restrict__ rows, const float *__restrict__ src, int stride, int indirect,
            const float *__restrict__ gamma, float eps, int n, int n_pad, bf16_t *__restrict__ xs,
            size_t part_stride) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const float *row = src + (size_t)(indirect ? rows[r].x_slot : r) * stride;
  if (gamma && n <= 4096) {
    // the row and the gains in registers: every load is issued before the first is used (one
    // memory round trip instead of one per loop trip of two passes)
    constexpr int NI = 4;
    float4 v[NI], g[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int k = threadIdx.x * 4 + i * 1024;
      v[i] = *(const float4 *)(row + (k < n ? k : 0));
      g[i] = *(const float4 *)(gamma + (k < n ? k : 0));
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i)
      if (threadIdx.x * 4 + i * 1024 < n) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)n + eps);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int k = threadIdx.x * 4 + i * 1024;
      if (k < n) {
        const float f[4] = {v[i].x * inv * g[i].x, v[i].y * inv * g[i].y, v[i].z * inv * g[i].z, v[i].w * inv * g[i].w};
        bf16_t h[4], mid[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split3_bf16(f[e], h[e], mid[e], l[e]);
        bf16_t *dst = xs + (size_t)r * n_pad + k;
        *(uint2 *)dst = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
        *(uint2 *)(dst + part_stride) = make_uint2(mid[0] | ((uint32_t)mid[1] << 16), mid[2] | ((uint32_t)mid[3] << 16));
        *(uint2 *)(dst + 2 * part_stride) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
      }
    }
    for (int k = n + threadIdx.x * 4; k < n_pad; k += 1024) {
      bf16_t *dst = xs + (size_t)r * n_pad + k;
      *(uint2 *)dst = make_uint2(0, 0);
      *(uint2 *)(dst + part_stride) = make_uint2(0, 0);
      *(uint2 *)(dst + 2 * part_stride) = make_uint2(0, 0);
    }
    return;
  }
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
    for (int e = 0; e < 4; ++e) split3_bf16(f[e], h[e], mid[e], l[e]);
    bf16_t *dst = xs + (size_t)r * n_pad + k;
    *(uint2 *)dst = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    *(uint2 *)(dst + part_stride) = make_uint2(mid[0] | ((uint32_t)mid[1] << 16), mid[2] | ((uint32_t)mid[3] << 16));
    *(uint2 *)(dst + 2 * part_stride) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
  }
  for (int k = n + threadIdx.x * 4; k < n_pad; k += 1024) {
    bf16_t *dst = xs + (size_t)r * n_pad + k;
    *(uint2 *)dst = make_uint2(0, 0);
    *(uint2 *)(dst + part_stride) = make_uint2(0, 0);
    *(uint2 *)(dst + 2 * part_stride) = make_uint2(0, 0);
  }
}

// ------------------------------------------------------------------ the contraction

// A workgroup takes one tile of 256 (or 128) tasks, one k range and one tile of 32*MTILES activation rows.
// SPLIT: write partial sums part[split][task][2][m_pad] instead of running the epilogue.
//
// The loop over 64-wide chunks of k is software-pipelined.  Weights: a wave has MG_W_DEPTH chunks
// of its 64 rows on their way in registers; the oldest is written to the wave's LDS piece, read
// back as A operands and its registers are reloaded with the chunk MG_W_DEPTH ahead (LDS
// operations of one wave execute in order, so the piece needs no barrier).  Activations: two LDS
// buffers shared by the workgroup; while the MFMAs read one, the next chunk (loaded into
// registers one iteration earlier) is written to the other and the chunk after that is requested:
// one workgroup barrier per chunk and no load whose latency is exposed.  All loads are
// unconditional (rows, tasks and chunks past the end are clamped to valid addresses and their
// products skipped or discarded), which lets the compiler wait for exactly the loads a step needs;
// loads return in issue order, so inside an iteration the activation loads are issued before the
// weight loads and the order of the steps is pinned.
// WAVES: 8, or 4 for matrices of few rows, whose launches then have twice as many workgroups
template <int MTILES, typename Epi, bool SPLIT, int WAVES = MG_WAVES>
__global__ void __launch_bounds__(64 * WAVES)
mfma_rows_k(Epi epi, const RowDesc *__restrict__ rows, int m_rows, const bf16_t *__restrict__ xs,
            size_t part_stride, int n_in, int n_tasks, int chunks_per_split,
            float *__restrict__ part, int m_pad, int n_task_tiles, int n_splits, int n_row_tiles,
            int xcd_groups) {
  static_assert(MTILES <= MG_MAX_MTILES, "accumulators and LDS are sized for 64 rows");
  // Workgroup -> (task tile, k range, row tile).  Consecutive workgroup ids go to consecutive
  // XCDs, each with its own L2: the row tiles of one (task tile, k range) read the same weights,
  // so they get ids 8 apart (same XCD, launched together) and the weights cross HBM once for them.
  // Ids are dealt in groups of 8 * n_row_tiles: 8 tiles, one per XCD, times their row tiles.
  // (xcd_groups: chosen by the launch; measured to pay for few, long k ranges: gate/up of a prompt
  // pass 191 -> 169 us, while down with its many short ranges lost, 101 -> 116 us.)
  int bx, by, bz;
  if (!xcd_groups) {   // task tiles fastest, then k ranges, then row tiles
    const int tiles = n_task_tiles * n_splits;
    bz = blockIdx.x / tiles;
    const int tile = blockIdx.x - bz * tiles;
    if (bz >= n_row_tiles) return;
    by = tile / n_task_tiles;
    bx = tile - by * n_task_tiles;
  } else {
    const int per_group = 8 * n_row_tiles;
    const int group = blockIdx.x / per_group, r = blockIdx.x - group * per_group;
    const int tile = group * 8 + (r & 7);
    if (tile >= n_task_tiles * n_splits) return;
    bz = r >> 3;
    by = tile / n_task_tiles;
    bx = tile - by * n_task_tiles;
  }
  constexpr int MROWS = 32 * MTILES;
  constexpr int WD = MG_W_DEPTH;
  constexpr int XPOS = MROWS * (MG_KC / 8);                  // 16-byte vectors of one part of a chunk
  constexpr int XV = (XPOS + (64 * WAVES) - 1) / (64 * WAVES);   // of them per thread
  // Every thread stages XV vectors, wrapping around when the workgroup has more threads than a
  // chunk has vectors (32 rows in an eight-wave workgroup: two threads then write the same data to
  // the same place).  A store under a condition would take its load with it: the compiler sinks a
  // load whose only use is conditional into that branch, next to the store, and the wave then
  // waits out the whole memory latency once per chunk instead of having the data a chunk ahead.
  static_assert(XPOS % (64 * WAVES) == 0 || (64 * WAVES) % XPOS == 0, "the staging wraps evenly");
  constexpr int PART_ELEMS = MROWS * MG_ROWPAD;
  constexpr int WI = 8;                                      // load instructions per chunk: 8 rows x 128 bytes each
  extern __shared__ uint4 mg_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16_t *s_w = (bf16_t *)mg_smem + wave * 64 * MG_ROWPAD;             // this wave's [64][MG_ROWPAD]
  bf16_t *s_x = (bf16_t *)mg_smem + WAVES * 64 * MG_ROWPAD;         // [2][3][MROWS * MG_ROWPAD]
  const int row0 = bz * MROWS;
  const int task0 = bx * (WAVES * MG_TASKS_PER_WAVE) + wave * MG_TASKS_PER_WAVE;
  const int n_chunks = (n_in + MG_KC - 1) / MG_KC;   // the last one may be short: activations are zero-padded
  const int x_stride = n_chunks * MG_KC;
  const int c_begin = by * chunks_per_split;
  const int c_end = min(n_chunks, c_begin + chunks_per_split);
  // the rows' sums of squares that this projection's finishing launch will add up start at zero
  if constexpr (EpiHasRowSum<Epi>::value)
    if (blockIdx.x == 0)
      for (int i = threadIdx.x; i < m_rows * SSQ_WAYS; i += 64 * WAVES) epi.ssq[i] = 0ull;
  if (c_begin >= c_end) return;

  // Load instruction i covers the wave's rows 8i..8i+7 (rows 0..31: first weight row of tasks
  // task0.., rows 32..63: their second weight row); this lane takes segment lane % 8 of row
  // 8i + lane / 8.
  const bf16_t *wrow[WI];
#pragma unroll
  for (int i = 0; i < WI; ++i) {
    const int q = 8 * i + (lane >> 3);
    const int task = task0 + (q & 31);
    const bf16_t *a, *b;
    epi.weight_rows(task < n_tasks ? task : 0, a, b);
    wrow[i] = q < 32 ? a : b;
  }
  const int w_seg = (lane & 7) * 8;   // this lane's k inside a chunk
  const int w_dst = (lane >> 3) * MG_ROWPAD + (lane & 7) * 8;          // + 8 i rows
  const int koff = (lane >> 5) * 8;                                    // this lane's k-block inside an MFMA step
  const int a_off = (lane & 31) * MG_ROWPAD + koff;                    // + 32 rows for the second tile, + 16 s

  f32x16_t acc0[MTILES], acc1[MTILES];
#pragma unroll
  for (int c = 0; c < MTILES; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[c][r] = acc1[c][r] = 0.f;

  u32x4_t wr[WD][WI];   // (a native vector type: arrays of it are kept in registers)
  // this thread's vectors of the three parts of a chunk's activations: xr[i][p]
  int x_src[XV], x_dst[XV];
#pragma unroll
  for (int i = 0; i < XV; ++i) {
    const int pos = ((int)threadIdx.x + i * (64 * WAVES)) % XPOS;
    const int m = pos / (MG_KC / 8), kv = (pos - m * (MG_KC / 8)) * 8;
    x_src[i] = min(row0 + m, m_rows - 1) * x_stride + kv;    // rows past the end repeat the last one
    x_dst[i] = m * MG_ROWPAD + kv;
  }
  u32x4_t xr[XV][MG_PARTS];

  {
    const int k_ = c_begin * MG_KC;
#pragma unroll
    for (int i = 0; i < XV; ++i) {
#pragma unroll
      for (int p = 0; p < MG_PARTS; ++p) xr[i][p] = *(const u32x4_t *)(xs + p * part_stride + x_src[i] + k_);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
#pragma unroll
      for (int p = 0; p < MG_PARTS; ++p) *(u32x4_t *)(s_x + p * PART_ELEMS + x_dst[i]) = xr[i][p];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  {
    const int k_ = min(c_begin + 1, c_end - 1) * MG_KC;
#pragma unroll
    for (int i = 0; i < XV; ++i) {
#pragma unroll
      for (int p = 0; p < MG_PARTS; ++p) xr[i][p] = *(const u32x4_t *)(xs + p * part_stride + x_src[i] + k_);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < WD; ++j) {
    int k_ = min(c_begin + j, c_end - 1) * MG_KC + w_seg;
    k_ = k_ < n_in ? k_ : 0;   // past the row's end: any finite weights, they meet zero activations
#pragma unroll
    for (int i = 0; i < WI; ++i) wr[j][i] = __builtin_nontemporal_load((const u32x4_t *)(wrow[i] + k_));
  }
  __syncthreads();

  for (int base = c_begin; base < c_end; base += WD) {
#pragma unroll
    for (int j = 0; j < WD; ++j) {
      const int chunk = base + j;
      const int buf = j & 1;   // WD is even, so a chunk's buffer is its slot's parity
      // weights of this chunk into the wave's LDS piece (the MFMAs of the previous chunk have
      // issued their reads of it: one wave's LDS operations stay in order)
#pragma unroll
      for (int i = 0; i < WI; ++i) *(u32x4_t *)(s_w + 8 * i * MG_ROWPAD + w_dst) = wr[j][i];
      __builtin_amdgcn_sched_barrier(0);
      // activations of chunk + 1, requested one iteration ago, into the other buffer
      {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
#pragma unroll
          for (int p = 0; p < MG_PARTS; ++p)
            *(u32x4_t *)(s_x + ((buf ^ 1) * MG_PARTS + p) * PART_ELEMS + x_dst[i]) = xr[i][p];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        const int k_ = min(chunk + 2, c_end - 1) * MG_KC;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
#pragma unroll
          for (int p = 0; p < MG_PARTS; ++p) xr[i][p] = *(const u32x4_t *)(xs + p * part_stride + x_src[i] + k_);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        int k_ = min(chunk + WD, c_end - 1) * MG_KC + w_seg;
        k_ = k_ < n_in ? k_ : 0;
#pragma unroll
        for (int i = 0; i < WI; ++i) wr[j][i] = __builtin_nontemporal_load((const u32x4_t *)(wrow[i] + k_));
      }
      __builtin_amdgcn_sched_barrier(0);
      if (chunk < c_end) {
        const bf16_t *xb = s_x + buf * MG_PARTS * PART_ELEMS + a_off;
#pragma unroll
        for (int s = 0; s < MG_KC / 16; ++s) {
          const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, *(const u32x4_t *)(s_w + a_off + s * 16));
          const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, *(const u32x4_t *)(s_w + 32 * MG_ROWPAD + a_off + s * 16));
          // smallest part first, so that the large terms are added last; consecutive MFMAs go to
          // different accumulators
#pragma unroll
          for (int p = MG_PARTS - 1; p >= 0; --p) {
#pragma unroll
            for (int c = 0; c < MTILES; ++c) {
              const bf16x8_t b = __builtin_bit_cast(
                  bf16x8_t, *(const u32x4_t *)(xb + p * PART_ELEMS + c * 32 * MG_ROWPAD + s * 16));
              acc0[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc0[c], 0, 0, 0);
              acc1[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc1[c], 0, 0, 0);
            }
          }
        }
      }
      __syncthreads();
    }
  }

  // results: register r <-> task (r/4)*8 + (lane/32)*4 + r%4 of this wave, activation row lane%32
  if constexpr (!SPLIT && std::is_same<typename Epi::State, NoState>::value) {
    // The epilogue runs here, and what it writes runs along the tasks (consecutive elements of a
    // row of the hidden state, of q, of the cache, of the split activations), while a lane's
    // registers hold 16 tasks of ONE row: stored as they lie, every store instruction would put
    // 64 single elements into 64 different rows (measured on the gate/up projection of a prompt
    // pass: 178 -> 163 us).  So each 32 x 32 tile is turned in the wave's own piece of LDS (free
    // now; the wave's LDS operations execute in order, no barrier) and the epilogue is called with
    // the tasks across the lanes: 32 consecutive elements per half-wave.
    float *s_t = (float *)s_w;   // [2][32 tasks][33]
    NoState st;
    const int tl = lane & 31, rh = (lane >> 5) * 16;
#pragma unroll
    for (int c = 0; c < MTILES; ++c) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        s_t[t * 33 + (lane & 31)] = acc0[c][r];
        s_t[32 * 33 + t * 33 + (lane & 31)] = acc1[c][r];
      }
      const int task = task0 + tl;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int m = row0 + c * 32 + rh + i;
        const float y0 = s_t[tl * 33 + rh + i], y1 = s_t[32 * 33 + tl * 33 + rh + i];
        if (task < n_tasks && m < m_rows) epi.finish(task, m, rows[m], y0, y1, st);
      }
    }
    return;
  }
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
          float *p = part + (((size_t)by * n_tasks + task) * 2) * m_pad + m;
          if (m < m_pad) { p[0] = acc0[c][r]; p[m_pad] = acc1[c][r]; }
        } else if (m_ok) {
          epi.finish(task, m, rd, acc0[c][r], acc1[c][r], st);
        }
      }
    }
    if (!SPLIT && MTILES == 1 && m_ok) epi.end(m, rd, st);
  }
}

// ------------------------------------------------------------------ the contraction on tiled weights
//
// A context that owns enough memory keeps a second copy of every bf16 projection matrix in the
// order the MFMA consumes it: for each block of 32 tasks, for each of its two weight rows per
// task, for each 64-wide chunk of k, one 4 KiB tile [step 0..3][lane 0..63][8 elements], lane l of
// step s holding row l % 32, elements 64 c + 16 s + 8 (l / 32) .. + 7.  A wave then loads a whole
// A operand with one fully coalesced instruction (64 lanes x 16 bytes, consecutive) straight into
// registers: the weights never touch LDS, which leaves LDS to the activations, and a wave can hold
// four A tiles (64 tasks), so that every B operand it reads from LDS feeds four MFMAs instead of
// two.  tile_weights_k writes the copy once, when the context is created, from the same
// weight_rows() of the epilogue that the kernels use.
constexpr int TG_WAVES = 4;
constexpr int TG_TILE = 32 * MG_KC;   // elements of one A tile of one chunk

constexpr size_t tg_tiled_elems(int n_tasks, int n_in) {
  return (size_t)((n_tasks + 31) / 32) * 2 * ((n_in + MG_KC - 1) / MG_KC) * TG_TILE;
}

template <typename Epi>
__global__ void __launch_bounds__(256)
tile_weights_k(Epi epi, int n_tasks, int n_in, int n_chunks, bf16_t *__restrict__ dst) {
  const int c = blockIdx.x, tbw = blockIdx.y, tb = tbw >> 1, which = tbw & 1;
  const int s = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int task = tb * 32 + (lane & 31);
  const int k = c * MG_KC + s * 16 + (lane >> 5) * 8;
  u32x4_t v = {0u, 0u, 0u, 0u};   // beyond the matrix: zeros
  if (task < n_tasks && k < n_in) {
    const bf16_t *a, *b;
    epi.weight_rows(task, a, b);
    v = *(const u32x4_t *)((which ? b : a) + k);
  }
  *(u32x4_t *)(dst + ((size_t)tbw * n_chunks + c) * TG_TILE + s * 512 + lane * 8) = v;
}

// dynamic LDS of mfma_tiled_k: two buffers of three parts of 32*MTILES padded activation rows, or
// the four waves' pieces for turning the result tiles, whichever is larger
constexpr size_t tg_lds_bytes(int mtiles) {
  const size_t x = sizeof(bf16_t) * 2 * MG_PARTS * 32 * mtiles * MG_ROWPAD;
  const size_t t = sizeof(float) * TG_WAVES * 2 * 32 * 33;
  return x > t ? x : t;
}

// A workgroup of four waves takes 128 * TB tasks (wave w: TB blocks of 32 tasks, 2 * TB A tiles),
// one k range and one tile of 32 * MTILES activation rows; grid and arguments as mfma_rows_k.
// SPLIT, or an epilogue without a running state.
//
// The loop over the chunks is written group by group in the order it is to execute, and every
// group ends with a scheduling barrier: a group is the 2 * TB MFMAs that share one B operand, the
// LDS read of a B operand of the NEXT step, and at most a few of the chunk's other operations (a
// weight load, an activation load, an LDS write of the staging), which issue while the MFMAs
// execute.  Left to itself the compiler puts each LDS read next to its use and the loads at the
// end of the chunk, and the MFMA pipe then idles half the time (measured on the gate/up projection
// of a 192-row prompt pass: 174 us; in this order 133 us; the same loop without any memory
// operation 110 us).
template <int MTILES, int TB, typename Epi, bool SPLIT>
__global__ void __launch_bounds__(64 * TG_WAVES)
mfma_tiled_k(Epi epi, const bf16_t *__restrict__ tiled, const RowDesc *__restrict__ rows, int m_rows,
             const bf16_t *__restrict__ xs, size_t part_stride, int n_in, int n_tasks, int chunks_per_split,
             float *__restrict__ part, int m_pad, int n_task_tiles, int n_splits, int n_row_tiles,
             int xcd_groups) {
  static_assert(SPLIT || std::is_same<typename Epi::State, NoState>::value, "a running state needs the finishing launch");
  static_assert(MTILES <= MG_MAX_MTILES && (TB == 1 || TB == 2), "accumulators are sized for 64 rows x 64 tasks");
  int bx, by, bz;   // workgroup -> (task tile, k range, row tile), as in mfma_rows_k
  if (!xcd_groups) {
    const int tiles = n_task_tiles * n_splits;
    bz = blockIdx.x / tiles;
    const int tile = blockIdx.x - bz * tiles;
    if (bz >= n_row_tiles) return;
    by = tile / n_task_tiles;
    bx = tile - by * n_task_tiles;
  } else {
    const int per_group = 8 * n_row_tiles;
    const int group = blockIdx.x / per_group, r = blockIdx.x - group * per_group;
    const int tile = group * 8 + (r & 7);
    if (tile >= n_task_tiles * n_splits) return;
    bz = r >> 3;
    by = tile / n_task_tiles;
    bx = tile - by * n_task_tiles;
  }
  constexpr int MROWS = 32 * MTILES;
  constexpr int NT = 64 * TG_WAVES;
  constexpr int XPOS = MROWS * (MG_KC / 8);
  constexpr int XV = XPOS / NT;
  static_assert(XPOS % NT == 0, "every thread stages the same number of vectors");
  constexpr int PART_ELEMS = MROWS * MG_ROWPAD;
  constexpr int STEPS = MG_KC / 16;
  constexpr int QT = 2 * TB;                        // A tiles per wave
  constexpr int NB = MG_PARTS * MTILES;             // B operands (and groups of QT MFMAs) per step
  constexpr int NX = XV * MG_PARTS;                 // activation vectors a thread stages per chunk
  static_assert(NX == NB, "one staging operation per group");
  constexpr int PER = (QT + NB - 1) / NB;           // weight loads per group
  constexpr int BUF_ELEMS = MG_PARTS * PART_ELEMS;
  extern __shared__ uint4 tg_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16_t *s_x = (bf16_t *)tg_smem;                  // [2][3][MROWS * MG_ROWPAD]
  const int row0 = bz * MROWS;
  const int n_chunks = (n_in + MG_KC - 1) / MG_KC;
  const int x_stride = n_chunks * MG_KC;
  const int c_begin = by * chunks_per_split;
  const int c_end = min(n_chunks, c_begin + chunks_per_split);
  if constexpr (EpiHasRowSum<Epi>::value)
    if (blockIdx.x == 0)
      for (int i = threadIdx.x; i < m_rows * SSQ_WAYS; i += NT) epi.ssq[i] = 0ull;
  if (c_begin >= c_end) return;
  const int n_tb = (n_tasks + 31) / 32;
  const int tb0 = (bx * TG_WAVES + wave) * TB;       // this wave's first block of 32 tasks

  const bf16_t *abase[QT];   // A tile q: block tb0 + q / 2, weight row q % 2 of its tasks (blocks past the end: the last one)
#pragma unroll
  for (int q = 0; q < QT; ++q)
    abase[q] = tiled + ((size_t)(min(tb0 + (q >> 1), n_tb - 1) * 2 + (q & 1)) * n_chunks) * TG_TILE + lane * 8;
  const int a_off = (lane & 31) * MG_ROWPAD + (lane >> 5) * 8;

  f32x16_t acc[QT][MTILES];
#pragma unroll
  for (int q = 0; q < QT; ++q)
#pragma unroll
    for (int c = 0; c < MTILES; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[q][c][r] = 0.f;

  int x_src[XV], x_dst[XV];
#pragma unroll
  for (int i = 0; i < XV; ++i) {
    const int pos = (int)threadIdx.x + i * NT;
    const int m = pos / (MG_KC / 8), kv = (pos - m * (MG_KC / 8)) * 8;
    x_src[i] = min(row0 + m, m_rows - 1) * x_stride + kv;    // rows past the end repeat the last one
    x_dst[i] = m * MG_ROWPAD + kv;
  }
  u32x4_t xr[XV][MG_PARTS];
  // chunks of weights in registers, slot = chunk % RING: three for 64-row tiles, whose one wave per
  // SIMD has nothing else to cover a late load with (prompt pass 29.6 -> 28.6 ms, passes of 33..64
  // rows in a batch of 32: 5.23 -> 5.17 ms per step); 32-row tiles keep two workgroups on a CU with
  // a ring of two, and lose with three (4.44 -> 4.61 ms per step)
  constexpr int RING = MTILES == 2 ? 3 : 2;
  u32x4_t wr[RING][QT][STEPS];
  const u32x4_t zero4 = {0u, 0u, 0u, 0u};

  // all loads are unconditional (chunks past the range are clamped to its last one) so that the
  // compiler waits for exactly the loads a step needs; a chunk past the range is staged as zeros
  auto load_x1 = [&](int n, int chunk) {
    const int k_ = min(chunk, c_end - 1) * MG_KC;
    xr[n / MG_PARTS][n % MG_PARTS] = *(const u32x4_t *)(xs + (n % MG_PARTS) * part_stride + x_src[n / MG_PARTS] + k_);
  };
  auto store_x1 = [&](int n, int buf, bool real) {
    *(u32x4_t *)(s_x + buf * BUF_ELEMS + (n % MG_PARTS) * PART_ELEMS + x_dst[n / MG_PARTS]) =
        real ? xr[n / MG_PARTS][n % MG_PARTS] : zero4;
  };
  // B operand i of step s of a buffer: parts from the smallest to the largest (the large terms
  // are added last), row tiles inside
  auto load_b1 = [&](int i, int buf, int s) -> u32x4_t {
    const int p = MG_PARTS - 1 - i / MTILES, c = i % MTILES;
    return *(const u32x4_t *)(s_x + buf * BUF_ELEMS + p * PART_ELEMS + c * 32 * MG_ROWPAD + s * 16 + a_off);
  };
  auto load_a1 = [&](int slot, int q, int s, int chunk) {
    wr[slot][q][s] = __builtin_nontemporal_load(
        (const u32x4_t *)(abase[q] + (size_t)min(chunk, c_end - 1) * TG_TILE + s * 512));
  };

#pragma unroll
  for (int n = 0; n < NX; ++n) load_x1(n, c_begin);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int n = 0; n < NX; ++n) store_x1(n, 0, true);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int n = 0; n < NX; ++n) load_x1(n, c_begin + 1);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < RING; ++j)
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
#pragma unroll
      for (int q = 0; q < QT; ++q) load_a1(j, q, s, c_begin + j);
  __syncthreads();
  u32x4_t bcur[NB], bnext[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) bcur[i] = zero4;

  // Region k (one barrier each) works on chunk i = c_begin + k, whose weights sit in ring slot
  // k % RING and whose activations in LDS buffer k % 2:
  //   step 3 of chunk i - 1 (its B operands were fetched before the last barrier; zeros in region 0),
  //   steps 0..2 of chunk i, while the B operands of the step after each are fetched,
  //   the staging of chunk i + 1 into the other buffer, the loads of the activations of chunk i + 2,
  //   and the reloads of the weight registers whose step has just been finished with (chunks
  //   i + RING - 1 and i + RING).
  // Every read of a buffer lies in the region of its chunk, every write to it in the regions next
  // to that one, so the one barrier per region separates them; the MFMAs run on across it.
  // A number of chunks that is not a multiple of RING is filled up with regions on zeros.
  const int n_regions = (c_end - c_begin + RING - 1) / RING * RING;
  int buf = 0;   // LDS buffer of the region's chunk
  for (int k0 = 0; k0 < n_regions; k0 += RING) {
#pragma unroll
    for (int j = 0; j < RING; ++j) {
      const int chunk = c_begin + k0 + j;
      const int jp = (j + RING - 1) % RING;
#pragma unroll
      for (int t = 0; t < STEPS; ++t) {
        // t = 0: step 3 of the previous chunk; t = 1..3: steps 0..2 of this one
        const int slot = t == 0 ? jp : j, s = t == 0 ? STEPS - 1 : t - 1;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int c = i % MTILES;
#pragma unroll
          for (int q = 0; q < QT; ++q)
            acc[q][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wr[slot][q][s]),
                                                                __builtin_bit_cast(bf16x8_t, bcur[i]), acc[q][c], 0, 0, 0);
          bnext[i] = load_b1(i, buf, t);   // operands of step t of this chunk (t = 0 follows the last barrier)
#pragma unroll
          for (int e = 0; e < PER; ++e) {
            const int q = i * PER + e;
            if (q < QT) {
              if (t == 0) load_a1(jp, q, STEPS - 2, chunk + RING - 1);        // step 2 of chunk i - 1 -> chunk i - 1 + RING
              else if (t == 1) load_a1(jp, q, STEPS - 1, chunk + RING - 1);   // step 3 of chunk i - 1 likewise
              else load_a1(j, q, t - 2, chunk + RING);                 // steps 0, 1 of chunk i -> chunk i + RING
            }
          }
          if (t == 1) store_x1(i, buf ^ 1, chunk + 1 < c_end);
          if (t == 2) load_x1(i, chunk + 2);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) bcur[i] = bnext[i];
      }
      __syncthreads();
      buf ^= 1;
    }
  }
  // step 3 of the last chunk
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int q = 0; q < QT; ++q)
      acc[q][i % MTILES] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wr[RING - 1][q][STEPS - 1]),
                                                                   __builtin_bit_cast(bf16x8_t, bcur[i]), acc[q][i % MTILES], 0, 0, 0);

  // register r of acc[2 jb + which][c] <-> weight row `which` of task (tb0 + jb) * 32 + (r/4)*8 + (lane/32)*4 + r%4,
  // activation row lane % 32 of row tile c
  if constexpr (SPLIT) {
#pragma unroll
    for (int jb = 0; jb < TB; ++jb)
#pragma unroll
      for (int c = 0; c < MTILES; ++c) {
        const int m = row0 + c * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int task = (tb0 + jb) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          if (task < n_tasks && m < m_pad) {
            float *p = part + (((size_t)by * n_tasks + task) * 2) * m_pad + m;
            p[0] = acc[2 * jb][c][r];
            p[m_pad] = acc[2 * jb + 1][c][r];
          }
        }
      }
  } else {
    // the epilogue's stores run along the tasks: each 32 x 32 tile is turned in the wave's piece of
    // LDS (the buffers are free once every wave has left the loop)
    __syncthreads();
    float *s_t = (float *)tg_smem + wave * 2 * 32 * 33;
    NoState st;
    const int tl = lane & 31, rh = (lane >> 5) * 16;
#pragma unroll
    for (int jb = 0; jb < TB; ++jb) {
#pragma unroll
      for (int c = 0; c < MTILES; ++c) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int t = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          s_t[t * 33 + (lane & 31)] = acc[2 * jb][c][r];
          s_t[32 * 33 + t * 33 + (lane & 31)] = acc[2 * jb + 1][c][r];
        }
        const int task = (tb0 + jb) * 32 + tl;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int m = row0 + c * 32 + rh + i;
          const float y0 = s_t[tl * 33 + rh + i], y1 = s_t[32 * 33 + tl * 33 + rh + i];
          if (task < n_tasks && m < m_rows) epi.finish(task, m, rows[m], y0, y1, st);
        }
      }
    }
  }
}

// The partial sums of one (task, row) over the k ranges, added in the order of the ranges.  All
// loads are issued before the first is used: a loop that loads and adds pays a memory round trip
// per trip, and a projection with few tiles has up to MG_MAX_SPLIT ranges.
constexpr int MG_MAX_SPLIT = 32;
// MAXS: the most ranges this instance adds (8 or MG_MAX_SPLIT): the loads live in 2 * MAXS
// registers, and a finishing launch with hundreds of workgroups wants two of them on a CU
template <int MAXS>
__device__ __forceinline__ void sum_splits(const float *__restrict__ part, int n_split, int n_tasks, int task,
                                           int m_pad, int m, float &y0, float &y1) {
  const size_t stride = (size_t)n_tasks * 2 * m_pad;
  const float *p = part + ((size_t)task * 2) * m_pad + m;
  float a[MAXS], b[MAXS];
#pragma unroll
  for (int i = 0; i < MAXS; ++i) { const int s = i < n_split ? i : 0; a[i] = p[s * stride]; b[i] = p[s * stride + m_pad]; }
#pragma unroll
  for (int i = 0; i < MAXS; ++i) if (i < n_split) { y0 += a[i]; y1 += b[i]; }
}

// sums the k-split partials and runs the epilogue: one thread per activation row and group of
// `tasks_per_thread` consecutive tasks, for epilogues that keep a running state worth reducing
// before it goes to memory (the arg-max of the vocabulary heads).  The running states of a
// workgroup's threads that serve the same activation row are combined in LDS (64-bit maximum), so
// that one atomic per row and workgroup reaches memory; with that the groups can be small (eight
// tasks: every thread issues all loads of a k range at once and the launch has thousands of
// waves; with 64 tasks per thread a head of 158 497 rows was 620 waves that each walked 32 dependent
// round trips, 59 us).
template <typename Epi>
__global__ void __launch_bounds__(256)
mfma_finish_k(Epi epi, const RowDesc *__restrict__ rows, int m_rows, int n_tasks, int n_split,
              const float *__restrict__ part, int m_pad, int tasks_per_thread) {
  __shared__ unsigned long long s_best[256];   // per activation row of this workgroup (m_pad <= 256)
  s_best[threadIdx.x] = 0ull;
  __syncthreads();
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int group = idx / m_pad, m = idx - group * m_pad;
  const int t_begin = group * tasks_per_thread;
  if (t_begin < n_tasks && m < m_rows) {
    const int t_end = min(n_tasks, t_begin + tasks_per_thread);
    typename Epi::State st;
    epi.init(st);
    const RowDesc rd = rows[m];
    // eight tasks at a time: the loads of their partial sums of one k range are issued together
    // (a thread that takes its tasks one by one pays a round trip per task and range); every task's
    // ranges are still added in their order
    constexpr int G = 8;
    const size_t stride = (size_t)n_tasks * 2 * m_pad;
    for (int task = t_begin; task < t_end; task += G) {
      float y0[G], y1[G];
#pragma unroll
      for (int i = 0; i < G; ++i) y0[i] = y1[i] = 0.f;
      for (int s = 0; s < n_split; ++s) {
        float a[G], b[G];
#pragma unroll
        for (int i = 0; i < G; ++i) {
          const float *p = part + s * stride + ((size_t)min(task + i, t_end - 1) * 2) * m_pad + m;
          a[i] = p[0];
          b[i] = p[m_pad];
        }
#pragma unroll
        for (int i = 0; i < G; ++i) { y0[i] += a[i]; y1[i] += b[i]; }
      }
#pragma unroll
      for (int i = 0; i < G; ++i)
        if (task + i < t_end) epi.finish(task + i, m, rd, y0[i], y1[i], st);
    }
    epi.reduce_local(st, s_best + m);
  }
  __syncthreads();
  if ((int)threadIdx.x < m_rows && s_best[threadIdx.x]) epi.end_reduced(rows[threadIdx.x], s_best[threadIdx.x]);
}

// The same for epilogues without a running state, with the stores in mind: a workgroup of 1024
// threads takes 32 tasks x 32 activation rows, one pair per thread.  It sums the k ranges with the
// rows fastest across threads (the order in which the partials lie), turns the tile in LDS, and
// runs the epilogue with the tasks fastest, so that what the epilogue writes (consecutive
// elements of a row of the hidden state, of q, of the cache, of the split activations) leaves a
// wave as whole segments instead of single words 7 KB apart.  grid (tasks / 32, m_pad / 32).
template <typename Epi, int MAXS>
__global__ void __launch_bounds__(1024)
mfma_finish_tile_k(Epi epi, const RowDesc *__restrict__ rows, int m_rows, int n_tasks, int n_split,
                   const float *__restrict__ part, int m_pad) {
  __shared__ float s_y[2][32][33];
  const int task0 = blockIdx.x * 32, row0 = blockIdx.y * 32;
  // what the epilogue will need besides the sums is requested first: the row's descriptor, and
  // through it the old value of a residual projection; both round trips run under the loads of
  // the partial sums
  const int tl = threadIdx.x & 31, ml = threadIdx.x >> 5, task = task0 + tl, m = row0 + ml;
  const bool live = task < n_tasks && m < m_rows;
  const RowDesc rd = rows[m < m_rows ? m : 0];
  auto old = [&]() {
    if constexpr (EpiReadsOld<Epi>::value) return epi.load_old(live ? task : 0, rd);
    else return 0;
  }();
  {
    const int ml_ = threadIdx.x & 31, tl_ = threadIdx.x >> 5, task_ = min(task0 + tl_, n_tasks - 1);
    float y0 = 0.f, y1 = 0.f;
    if (row0 + ml_ < m_pad) sum_splits<MAXS>(part, n_split, n_tasks, task_, m_pad, row0 + ml_, y0, y1);
    s_y[0][tl_][ml_] = y0;
    s_y[1][tl_][ml_] = y1;
  }
  __syncthreads();
  typename Epi::State st;
  epi.init(st);
  if (live) {
    if constexpr (EpiReadsOld<Epi>::value) epi.finish_old(task, m, rd, s_y[0][tl][ml], s_y[1][tl][ml], old, st);
    else epi.finish(task, m, rd, s_y[0][tl][ml], s_y[1][tl][ml], st);
  }
  if constexpr (EpiHasRowSum<Epi>::value) {
    // the 32 threads of a row are half a wave: their states are added with shuffles (a fixed
    // order), and one of them hands the sum on
    float sum = st.ssq;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (tl == 0 && m < m_rows) epi.add_row_sum(m, sum);
  } else {
    if (live) epi.end(m, rd, st);
  }
}

}  // namespace spark
