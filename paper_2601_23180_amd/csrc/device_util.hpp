// Small device helpers shared by the kernel translation units.
#pragma once

#include "internal.hpp"

namespace ts {

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // round-to-nearest-even

// Activation operands.  fp32 models keep one fp32 panel.  bf16 models keep every matmul / attention
// operand as TWO bf16 panels, hi = round(v) and lo = round(v - hi) (hi + lo carries ~16 significant
// bits), `panel` elements apart; the matrix cores multiply both by the bf16 weights and accumulate
// in fp32.  No activation is ever rounded to 8 significant bits, so the pass is a smooth function
// of its inputs and reproducible to ~1e-5 against an unrounded reference.
__device__ __forceinline__ void store_act(float *base, size_t panel, size_t idx, float v) {
  (void)panel;
  base[idx] = v;
}
__device__ __forceinline__ void store_act(bf16 *base, size_t panel, size_t idx, float v) {
  const bf16 hi = (bf16)v;
  base[idx] = hi;
  base[panel + idx] = (bf16)(v - (float)hi);
}

// Sum over a 64-lane wavefront, fixed butterfly order (deterministic).
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

// Sum over a workgroup of NW wavefronts; every thread gets the result. `red` >= NW floats of LDS.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += red[i];
  return t;
}

// Running (largest, its column, second largest, sum of exp relative to the largest) of a set of
// logits.  Among equal maxima the lowest column wins, in push order and in any merge order.
struct Top2 {
  float l1, l2, s;
  int idx;
};
__device__ __forceinline__ Top2 top2_empty() {
  Top2 t;
  t.l1 = -INFINITY; t.l2 = -INFINITY; t.s = 0.f; t.idx = 0x7fffffff;
  return t;
}
__device__ __forceinline__ Top2 top2_merge(const Top2 &a, const Top2 &b) {
  if (b.l1 == -INFINITY) return a;
  if (a.l1 == -INFINITY) return b;
  Top2 r;
  if (b.l1 > a.l1 || (b.l1 == a.l1 && b.idx < a.idx)) {
    r.l1 = b.l1; r.idx = b.idx;
    r.l2 = fmaxf(a.l1, b.l2);
    r.s = a.s * expf(a.l1 - b.l1) + b.s;
  } else {
    r.l1 = a.l1; r.idx = a.idx;
    r.l2 = fmaxf(b.l1, a.l2);
    r.s = a.s + b.s * expf(b.l1 - a.l1);
  }
  return r;
}
__device__ __forceinline__ void top2_push(Top2 &t, float v, int col) {
  // columns arrive in ascending order
  if (v > t.l1) {
    t.s = (t.l1 == -INFINITY) ? 1.f : t.s * expf(t.l1 - v) + 1.f;
    t.l2 = t.l1; t.l1 = v; t.idx = col;
  } else if (v != -INFINITY) {
    t.s += expf(v - t.l1);
    t.l2 = fmaxf(t.l2, v);
  }
}
__device__ __forceinline__ Top2 top2_shfl_xor(const Top2 &t, int o) {
  Top2 r;
  r.l1 = __shfl_xor(t.l1, o, 64);
  r.l2 = __shfl_xor(t.l2, o, 64);
  r.s = __shfl_xor(t.s, o, 64);
  r.idx = __shfl_xor(t.idx, o, 64);
  return r;
}

}  // namespace ts
