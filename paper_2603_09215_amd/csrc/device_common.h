// Shared device-side types and helpers of the SPAR-K HIP library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spark {

typedef uint16_t bf16_t;  // bf16 bit pattern

// One activation row of a pass through a range of layers.
struct RowDesc {
  int x_slot;   // row of the hidden-state arena that holds this row's residual stream
  int seq;      // sequence slot (selects the page table)
  int pos;      // absolute position in the sequence (RoPE angle, KV slot, causal limit)
  int out_idx;  // row of per-step outputs (logits, argmax) this row reports to, or -1
};

// Paged KV cache: pool[page][layer][k|v][kv_head][token_in_page][head_dim]
struct KVView {
  void *pool;
  const int *page_table;  // [seq][max_pages] -> physical page
  int max_pages;
  int n_layers, n_kv_heads, page_tokens, head_dim;
};

__device__ __forceinline__ size_t kv_elem_offset(const KVView &kv, int seq, int pos, int layer,
                                                 int which, int head) {
  int page = kv.page_table[seq * kv.max_pages + pos / kv.page_tokens];
  size_t o = (size_t)page * kv.n_layers + layer;
  o = (o * 2 + which) * kv.n_kv_heads + head;
  o = o * kv.page_tokens + pos % kv.page_tokens;
  return o * kv.head_dim;
}

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VEC = 4;  // elements per 16-byte load
  __device__ static __forceinline__ float widen(float v) { return v; }
  __device__ static __forceinline__ float narrow(float v) { return v; }
  __device__ static __forceinline__ void unpack(const uint4 &r, float *f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
template <> struct Elem<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static __forceinline__ float widen(bf16_t v) { return bf16_to_f32(v); }
  __device__ static __forceinline__ bf16_t narrow(float v) { return f32_to_bf16(v); }
  __device__ static __forceinline__ void unpack(const uint4 &r, float *f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

// x = hi + mid + lo exactly, each part a bf16 (3 x 8 mantissa bits cover the 24 of an fp32): the
// form in which activations meet bf16 weights on the MFMA units without losing fp32 accuracy
__device__ __forceinline__ void split3_bf16(float x, bf16_t &hi, bf16_t &mid, bf16_t &lo) {
  hi = f32_to_bf16(x);
  const float rem = x - bf16_to_f32(hi);      // exact
  mid = f32_to_bf16(rem);
  lo = f32_to_bf16(rem - bf16_to_f32(mid));   // the exact remainder has at most 8 bits left
}

// Where the three parts of pass row r's activations go for the MFMA kernels: part p of element k at
// xs[p * part_stride + r * row_stride + k]; rows are zero beyond the `width` real elements.
struct SplitOut {
  bf16_t *xs;            // nullptr: not wanted
  size_t part_stride;
  int row_stride, width;
};

// four consecutive elements k..k+3 (k a multiple of 4) of row r; the thread that writes the row's
// last elements also clears its padding
__device__ __forceinline__ void split_store4(const SplitOut &so, int r, int k, float4 v) {
  const float f[4] = {v.x, v.y, v.z, v.w};
  bf16_t h[4], m[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) split3_bf16(f[e], h[e], m[e], l[e]);
  bf16_t *dst = so.xs + (size_t)r * so.row_stride + k;
  *(uint2 *)dst = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
  *(uint2 *)(dst + so.part_stride) = make_uint2(m[0] | ((uint32_t)m[1] << 16), m[2] | ((uint32_t)m[3] << 16));
  *(uint2 *)(dst + 2 * so.part_stride) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
  if (k + 4 >= so.width)
    for (int z = so.width; z < so.row_stride; z += 4)
#pragma unroll
      for (int p = 0; p < 3; ++p)
        *(uint2 *)(so.xs + p * so.part_stride + (size_t)r * so.row_stride + z) = make_uint2(0, 0);
}

// two consecutive elements k, k+1 (k even) of row r
__device__ __forceinline__ void split_store2(const SplitOut &so, int r, int k, float v0, float v1) {
  bf16_t h0, m0, l0, h1, m1, l1;
  split3_bf16(v0, h0, m0, l0);
  split3_bf16(v1, h1, m1, l1);
  bf16_t *dst = so.xs + (size_t)r * so.row_stride + k;
  *(uint32_t *)dst = h0 | ((uint32_t)h1 << 16);
  *(uint32_t *)(dst + so.part_stride) = m0 | ((uint32_t)m1 << 16);
  *(uint32_t *)(dst + 2 * so.part_stride) = l0 | ((uint32_t)l1 << 16);
  if (k + 2 >= so.width)
    for (int z = so.width; z < so.row_stride; z += 2)
#pragma unroll
      for (int p = 0; p < 3; ++p) *(uint32_t *)(so.xs + p * so.part_stride + (size_t)r * so.row_stride + z) = 0u;
}

// one element
__device__ __forceinline__ void split_store1(const SplitOut &so, int r, int k, float v) {
  bf16_t h, m, l;
  split3_bf16(v, h, m, l);
  bf16_t *dst = so.xs + (size_t)r * so.row_stride + k;
  dst[0] = h;
  dst[so.part_stride] = m;
  dst[2 * so.part_stride] = l;
  if (k + 1 >= so.width)
    for (int z = so.width; z < so.row_stride; ++z)
#pragma unroll
      for (int p = 0; p < 3; ++p) so.xs[p * so.part_stride + (size_t)r * so.row_stride + z] = 0;
}

// Data handed from one workgroup to another inside a kernel goes through device-scope relaxed
// atomic accesses: they are served at the level where all XCDs agree, so neither side has to
// flush or invalidate a whole L2 (each of the 8 XCDs has its own).
__device__ __forceinline__ void store_device_scope(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_scope(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_device_scope2(const float *p) {   // p 8-byte aligned
  unsigned long long v = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}
__device__ __forceinline__ void store_device_scope2(float *p, float2 v) {
  unsigned long long u = (unsigned long long)__float_as_uint(v.x) |
                         ((unsigned long long)__float_as_uint(v.y) << 32);
  __hip_atomic_store((unsigned long long *)p, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_device_scope(bf16_t *p, bf16_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// DS selects device-scope (cross-workgroup, same kernel) or ordinary accesses at compile time
template <bool DS, typename T> __device__ __forceinline__ void store_maybe_ds(T *p, T v) {
  if (DS) store_device_scope(p, v); else *p = v;
}
template <bool DS> __device__ __forceinline__ float2 load2_maybe_ds(const float *p) {
  if (DS) return load_device_scope2(p);
  return *(const float2 *)p;
}
template <bool DS> __device__ __forceinline__ void store2_maybe_ds(float *p, float2 v) {
  if (DS) store_device_scope2(p, v); else *(float2 *)p = v;
}
// wait until every memory operation this wave has issued is complete
__device__ __forceinline__ void wait_memory_ops() { __builtin_amdgcn_s_waitcnt(0); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Order-preserving map float -> uint32 (larger float => larger key; every NaN above +inf).
__device__ __forceinline__ uint32_t float_order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0xffffffffu;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
// 64-bit argmax key: larger logit wins, then the lower index.
__device__ __forceinline__ unsigned long long argmax_key(float logit, int idx) {
  return ((unsigned long long)float_order_key(logit) << 32) | (uint32_t)(0xffffffffu - (uint32_t)idx);
}

}  // namespace spark
