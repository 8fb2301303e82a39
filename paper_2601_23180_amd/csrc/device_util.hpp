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

// Operand layout of a matmul activation [rows_pad = 32 * MB, K] (bf16 hi part + bf16 lo part):
// the order in which the matrix cores consume it.  For every 64-deep k block `blk`, MFMA step j,
// 32-row block mb and part p (0 = hi, 1 = lo), one contiguous 1 KB fragment holds the 64 lanes'
// 16-byte A operands: lane (ln, g) = row 32 mb + ln, k = 64 blk + 32 g + 8 j + 0..7.  A consumer
// copies whole fragments global -> LDS with fully contiguous loads and reads them back with one
// conflict-free 16-byte LDS read per lane; producers scatter their outputs into this order once.
// Returns the element offset of (row r, reduction index k, part p).
__device__ __forceinline__ size_t ol_offset(int r, int k, int part, int mb_count) {
  const int blk = k >> 6, g = (k >> 5) & 1, j = (k >> 3) & 3, e = k & 7;
  const int mb = r >> 5, ln = r & 31;
  return ((((size_t)blk * 4 + j) * mb_count + mb) * 2 + part) * 512 + (g * 32 + ln) * 8 + e;
}

// Data handed from one workgroup to another INSIDE a kernel (split-K partial tiles, per-tile
// sums) is written and read with agent-scope relaxed atomics: on gfx950 these are ordinary
// stores / loads that write through, respectively bypass, the per-XCD L2, so they are coherent
// across the chip without the L2 write-back + invalidate a full __threadfence() costs (measured:
// two fences per workgroup added ~100 us to a 10 us kernel).  publish_then_count() then makes the
// stores complete before the tile counter is bumped.
__device__ __forceinline__ void st_agent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 8- and 16-byte forms: a vector is moved as 64-bit agent-scope pieces (the widest scalar the
// atomic builtins take), so each piece still writes through / bypasses the per-XCD L2.
__device__ __forceinline__ void st_agent_u64(void *p, uint64_t v) {
  __hip_atomic_store((uint64_t *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_agent_u64(const void *p) {
  return __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x4 ld_agent_f32x4(const float *p) {
  union { uint64_t u[2]; f32x4 v; } t;
  t.u[0] = ld_agent_u64(p);
  t.u[1] = ld_agent_u64(p + 2);
  return t.v;
}
// Stores of a kernel's results.  WT = false: plain stores (the end of the kernel makes them
// visible).  WT = true: write-through, for results that another workgroup of the SAME launch reads
// after a device-side barrier.
template <bool WT>
__device__ __forceinline__ void store_f32x4(float *p, f32x4 v) {
  if constexpr (WT) {
    union { uint64_t u[2]; f32x4 v; } t;
    t.v = v;
    st_agent_u64(p, t.u[0]);
    st_agent_u64(p + 2, t.u[1]);
  } else {
    *(f32x4 *)p = v;
  }
}
template <bool WT>
__device__ __forceinline__ void store_bf16x4(bf16 *p, bf16x4 v) {
  if constexpr (WT) {
    union { uint64_t u; bf16x4 v; } t;
    t.v = v;
    st_agent_u64(p, t.u);
  } else {
    *(bf16x4 *)p = v;
  }
}
template <bool WT>
__device__ __forceinline__ void store_f32(float *p, float v) {
  if constexpr (WT) st_agent(p, v);
  else *p = v;
}

// Device-side barrier between the phases of one launch (every workgroup of the grid is resident:
// the host checks that before it chooses such a kernel).  bar_arrive: called by every thread after
// its write-through stores; the stores are acknowledged before the counter moves.  bar_wait:
// thread 0 polls until `expect` workgroups have arrived, for at most `limit` ticks of the 100 MHz
// wall clock; on expiry it raises the sticky abort word (later waits return at once) and bit 2 of
// the status word, and the kernel carries on to its normal end with meaningless results.
constexpr int kStatusWaitExpired = 4;
__device__ __forceinline__ void bar_arrive(int32_t *counter) {
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void bar_wait(const int32_t *counter, int expect, unsigned long long limit,
                                         int32_t *abort_word, int32_t *status, int naps = 1) {
  if (threadIdx.x == 0) {
    const unsigned long long t0 = wall_clock64();
    if (__hip_atomic_load(abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
      while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < expect) {
        for (int i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(8);
        if (wall_clock64() - t0 > limit) {
          __hip_atomic_store(abort_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          atomicOr(status, kStatusWaitExpired);
          break;
        }
      }
    }
  }
  __syncthreads();
}

// Called by every thread of the workgroup after its st_agent stores.  Returns (to all threads)
// whether this workgroup was the `expected`-th, i.e. last, to arrive; the counter is reset by the
// last arriver so that it is zero again for the next launch.
__device__ __forceinline__ bool publish_then_count(int32_t *counter, int expected, int *s_flag) {
  __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0): this thread's write-through stores are acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == expected - 1);
    if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_flag = last;
  }
  __syncthreads();
  return *s_flag != 0;
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
// t = sum of exp(l - l1) * (l - l1) rides along for the entropy: with d = l - l1 and s = sum e^d,
// p = e^d / s and H = -sum p ln p = ln s - t / s.
struct Top2 {
  float l1, l2, s, t;
  int idx;
};
__device__ __forceinline__ Top2 top2_empty() {
  Top2 t;
  t.l1 = -INFINITY; t.l2 = -INFINITY; t.s = 0.f; t.t = 0.f; t.idx = 0x7fffffff;
  return t;
}
__device__ __forceinline__ Top2 top2_merge(const Top2 &a, const Top2 &b) {
  if (b.l1 == -INFINITY) return a;
  if (a.l1 == -INFINITY) return b;
  Top2 r;
  if (b.l1 > a.l1 || (b.l1 == a.l1 && b.idx < a.idx)) {
    const float d = a.l1 - b.l1, e = expf(d);     // a's terms move down by d <= 0
    r.l1 = b.l1; r.idx = b.idx;
    r.l2 = fmaxf(a.l1, b.l2);
    r.s = a.s * e + b.s;
    r.t = (a.t + a.s * d) * e + b.t;
  } else {
    const float d = b.l1 - a.l1, e = expf(d);
    r.l1 = a.l1; r.idx = a.idx;
    r.l2 = fmaxf(b.l1, a.l2);
    r.s = a.s + b.s * e;
    r.t = a.t + (b.t + b.s * d) * e;
  }
  return r;
}
__device__ __forceinline__ void top2_push(Top2 &t, float v, int col) {
  // columns arrive in ascending order
  if (v > t.l1) {
    if (t.l1 == -INFINITY) {
      t.s = 1.f; t.t = 0.f;
    } else {
      const float d = t.l1 - v, e = expf(d);
      t.t = (t.t + t.s * d) * e;                 // the new maximum itself adds e^0 * 0
      t.s = t.s * e + 1.f;
    }
    t.l2 = t.l1; t.l1 = v; t.idx = col;
  } else if (v != -INFINITY) {
    const float d = v - t.l1, e = expf(d);
    t.s += e;
    t.t += e * d;
    t.l2 = fmaxf(t.l2, v);
  }
}
__device__ __forceinline__ Top2 top2_shfl_xor(const Top2 &t, int o) {
  Top2 r;
  r.l1 = __shfl_xor(t.l1, o, 64);
  r.l2 = __shfl_xor(t.l2, o, 64);
  r.s = __shfl_xor(t.s, o, 64);
  r.t = __shfl_xor(t.t, o, 64);
  r.idx = __shfl_xor(t.idx, o, 64);
  return r;
}

}  // namespace ts
