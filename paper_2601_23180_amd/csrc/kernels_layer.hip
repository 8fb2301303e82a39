// One launch for the matmuls between two attention calls: O projection (+ residual), gate + up
// (+ SwiGLU), down projection (+ residual) and the NEXT layer's QKV projection (+ rotary
// embedding, KV append), as phases of one resident grid with a device-side barrier between them.
//
// Why: at 60 rows every one of these matmuls is a 30 - 200 MB weight stream of 5 - 35 us, and as
// separate launches each pays a launch gap, an empty pipeline at its start and an idle memory
// system during its tail (split reduction, epilogue, hand-over): measured, about 45 % of a layer.
// Here a workgroup issues the loads of its NEXT phase's first DEPTH weight chunks as soon as it has
// arrived at the barrier, so HBM keeps streaming weights while the last workgroups of the phase
// reduce their tiles, while the barrier settles and while the next activation panel is fetched.
//
// The phases are the matmul of kernels_gemm.hip (same packed weights, same operand layout, same
// MFMA schedule, same epilogues) restricted to its fast path: every workgroup's k range is a whole
// number of DEPTH chunks.  Work item of workgroup g in a phase: tile g % n_tiles, split
// g / n_tiles (idle if g >= n_tiles * n_splits); a fixed function of g, so results do not depend
// on scheduling.
//
// Memory rules inside one launch (there is no cache invalidation between phases):
//   * everything a later phase reads is written through to memory (agent-scope stores) and the
//     writer's stores are acknowledged before it arrives at the barrier;
//   * a buffer is read with plain loads only if no workgroup has touched it earlier in this
//     launch, which the host guarantees by alternating buffers (residual stream x_a -> x_b -> x_a,
//     operand panels h_b for gate/up and h_a for QKV, sums of squares likewise);
//   * every phase has its own split-K partial region (written through, read once with plain
//     loads by the workgroup that combines the tile); the tile counters are shared and go through
//     agent-scope atomics only.
// The barrier waits are bounded (bar_wait): a grid that is not fully resident cannot hang.
#include "gemm_epilogue.hpp"

namespace ts {

namespace {

struct Item {
  bool has;
  int tile, split, k_begin, n_chunks, rot;
  const bf16 *wrow;   // this wavefront's packed run at k_begin, lane offset included
};

// This wavefront's packed sub-tile for (tile, split) of matmul `a` — as in k_gemm_bf16.
template <int KC>
__device__ __forceinline__ Item item_of(const GemmArgs &a, int epi, int wg, int wave, int lane) {
  Item it;
  const int n_items = a.n_tiles * a.n_splits;
  it.has = wg < n_items;
  const int g = it.has ? wg : 0;
  it.tile = g % a.n_tiles;
  it.split = g / a.n_tiles;
  it.k_begin = it.split * a.k_per_split;
  it.n_chunks = a.k_per_split / KC;
  it.rot = (int)(((unsigned)it.tile * 11u + (unsigned)it.split * 5u) % (unsigned)it.n_chunks);
  int sidx, sub;
  if (epi == EPI_SWIGLU) {
    sidx = wave >> 1;
    sub = 2 * it.tile + (wave & 1);
  } else {
    const int n0 = it.tile * kGemmTileN + wave * 32;
    sidx = 0;
    if (a.n_seg > 1 && n0 >= a.seg[1].col0) sidx = 1;
    if (a.n_seg > 2 && n0 >= a.seg[2].col0) sidx = 2;
    const int col0 = sidx == 0 ? a.seg[0].col0 : (sidx == 1 ? a.seg[1].col0 : a.seg[2].col0);
    sub = (n0 - col0) >> 5;
  }
  const bf16 *wseg = (const bf16 *)(sidx == 0 ? a.seg[0].w : (sidx == 1 ? a.seg[1].w : a.seg[2].w));
  const int seg_rows = sidx == 0 ? a.seg[0].n_rows : (sidx == 1 ? a.seg[1].n_rows : a.seg[2].n_rows);
  sub = min(max(sub, 0), ((seg_rows + 31) >> 5) - 1);   // idle wavefronts of a ragged last tile stay in bounds
  it.wrow = wseg + ((size_t)sub * (a.k >> 6) + (it.k_begin >> 6)) * 2048 + lane * 8;
  return it;
}

// block of 64 reduction indices starting at k (relative to the run's first index)
__device__ __forceinline__ const bf16 *wrow_block(const bf16 *wrow, int k) { return wrow + (size_t)(k >> 6) * 2048; }

template <int N>
struct IntC {
  static constexpr int value = N;
};

}  // namespace

template <int MB, int KC, int DEPTH, int NPH>
__global__ __launch_bounds__(256) void k_layer_bf16(LayerArgs la) {
  constexpr int KB = KC / 64;
  constexpr int FRAGS = KB * 4 * MB * 2;
  constexpr int BUF = FRAGS * 1024;
  constexpr int XV = FRAGS / 4;
  constexpr int EPI_BYTES = MB * 32 * (kGemmTileN + 4) * 4;
  constexpr int LDS_BYTES = 2 * BUF > EPI_BYTES ? 2 * BUF : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];
  __shared__ int s_last;
  __shared__ float s_rs[kMaxRows];
  __shared__ float s_rsp[4 * kMaxRows];

  const int tid = threadIdx.x, lane = tid & 63;
  // scalar: what is selected by it (this wavefront's weight segment) is then fetched with scalar
  // loads from the kernel arguments, not with a vector load that the first weight request waits for
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x, n_wg = gridDim.x;
  auto stamp = [&](int slot) {
    if (la.stamps != nullptr && wg == la.stamp_wg && tid == 0) la.stamps[slot] = wall_clock64();
  };
  stamp(0);

  bf16x8 w[DEPTH][KB][4];
  // the first DEPTH chunks of an item's weight run into the ring (chunk d -> set d)
  auto ring_fill = [&](const Item &it) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int cc = d + it.rot, c = cc >= it.n_chunks ? cc - it.n_chunks : cc;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const bf16 *p = wrow_block(it.wrow, c * KC + kb * 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) w[d][kb][j] = __builtin_nontemporal_load((const bf16x8 *)(p + 512 * j));
      }
    }
  };

  // One phase: the matmul `a` with epilogue EPI for item `it` (ring already requested), then the
  // arrival at this phase's barrier.  `first`: the inputs come from an earlier launch, no wait.
  auto run_phase = [&](auto epi_c, const GemmArgs &a, const Item &it, int p) {
    constexpr int EPI = decltype(epi_c)::value;
    if (p > 0) bar_wait(la.bar + (p - 1), n_wg, la.spin_limit, la.abort_word, la.status, la.poll_naps);
    stamp(1 + 3 * p);
    if (it.has) {
      const int n_chunks = it.n_chunks, rot = it.rot;
      auto rc = [&](int c) { const int cc = c + rot; return cc >= n_chunks ? cc - n_chunks : cc; };
      const bf16 *xg = (const bf16 *)a.x + ((size_t)(it.k_begin >> 6) * 4 * MB * 2 + wave * XV) * 512 + lane * 8;
      float rs_in[(MB + 1) / 2][8];
      rstd_load<256, MB>(a, rs_in);
      f32x16 acc[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;
      typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
      // two register stages: the panel chunk requested at the start of chunk c is chunk c + 3 and is
      // written to LDS two chunks later, so a wait for it leaves two chunks of younger loads in flight
      u32x4 xr[2][XV];
      auto load_w_block = [&](int set, int c, int kb) {
        const bf16 *p = wrow_block(it.wrow, rc(c) * KC + kb * 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) w[set][kb][j] = __builtin_nontemporal_load((const bf16x8 *)(p + 512 * j));
      };
      auto load_x_at = [&](int stage, int c) {
        const bf16 *src = xg + (size_t)rc(c) * FRAGS * 512;
#pragma unroll
        for (int i = 0; i < XV; ++i) xr[stage][i] = *(const u32x4 *)(src + i * 512);
      };
      auto store_x = [&](int buf) {    // register stage buf -> LDS stage buf (chunk parity)
        unsigned char *dst = lds + buf * BUF + (wave * XV) * 1024 + lane * 16;
#pragma unroll
        for (int i = 0; i < XV; ++i) *(u32x4 *)(dst + i * 1024) = xr[buf][i];
      };
      bf16x8 xf[2][2 * MB];
      auto read_frags = [&](int slot, int t, int buf) {
        const unsigned char *xp = lds + buf * BUF + (size_t)(t * MB * 2) * 1024 + lane * 16;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          xf[slot][2 * mb] = *(const bf16x8 *)(xp + (mb * 2) * 1024);
          xf[slot][2 * mb + 1] = *(const bf16x8 *)(xp + (mb * 2 + 1) * 1024);
        }
      };
      auto compute_chunk = [&](int set, int buf, int c_next, bool loadw) {
        constexpr int T = 4 * KB;
        read_frags(0, 0, buf);
        read_frags(1, 1, buf);
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const int kb = t >> 2, j = t & 3;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[t & 1][2 * mb], w[set][kb][j], acc[mb], 0, 0, 0);
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[t & 1][2 * mb + 1], w[set][kb][j], acc[mb], 0, 0, 0);
          if (t + 2 < T) read_frags(t & 1, t + 2, buf);
          if (j == 3 && loadw) load_w_block(set, c_next, kb);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      load_x_at(0, 0);
      load_x_at(1, 1);
      __builtin_amdgcn_sched_barrier(0);
      store_x(0);
      load_x_at(0, 2);                                  // n_chunks >= DEPTH >= 4
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      // The first group of DEPTH chunks is peeled off the loop: its loads were requested long ago and
      // in another order than the loop's own, and the wait counts at a loop head are the merge of
      // both ways in — unpeeled, every wait of the steady state would be as strict as the first.
      int c0 = 0;
      if (n_chunks > DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
          store_x((d + 1) & 1);
          load_x_at((d + 1) & 1, d + 3);                // n_chunks >= 2 * DEPTH here
          __builtin_amdgcn_sched_barrier(0);
          compute_chunk(d, d & 1, d + DEPTH, true);
          __syncthreads();
        }
        for (c0 = DEPTH; c0 + DEPTH < n_chunks; c0 += DEPTH) {
#pragma unroll
          for (int d = 0; d < DEPTH; ++d) {
            store_x((d + 1) & 1);
            load_x_at((d + 1) & 1, min(c0 + d + 3, n_chunks - 1));
            __builtin_amdgcn_sched_barrier(0);
            compute_chunk(d, d & 1, c0 + d + DEPTH, true);
            __syncthreads();
          }
        }
      }
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        if (d + 1 < DEPTH) store_x((d + 1) & 1);
        if (d + 3 < DEPTH) load_x_at((d + 1) & 1, c0 + d + 3);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(d, d & 1, 0, false);
        if (d + 1 < DEPTH) __syncthreads();
      }
      stamp(2 + 3 * p);
      rstd_finish<256, MB>(a, rs_in, s_rsp, s_rs);
      __syncthreads();
      gemm_epilogue<MB, EPI, 4, 1, MB, true>(a, reinterpret_cast<f32x16(&)[1][MB]>(acc), lds, &s_last, s_rs, it.tile,
                                             it.split);
    }
    bar_arrive(la.bar + p);
    stamp(3 + 3 * p);
  };

  // Phase order: O projection, gate + up, down projection, next layer's QKV.
  const Item i0 = item_of<KC>(la.ph[0], EPI_RESID, wg, wave, lane);
  if (i0.has) ring_fill(i0);
  const Item i1 = item_of<KC>(la.ph[1], EPI_SWIGLU, wg, wave, lane);
  run_phase(IntC<EPI_RESID>{}, la.ph[0], i0, 0);
  if (i1.has) ring_fill(i1);
  const Item i2 = item_of<KC>(la.ph[2], EPI_RESID, wg, wave, lane);
  run_phase(IntC<EPI_SWIGLU>{}, la.ph[1], i1, 1);
  if (i2.has) ring_fill(i2);
  if constexpr (NPH == 4) {
    const Item i3 = item_of<KC>(la.ph[3], EPI_QKV, wg, wave, lane);
    run_phase(IntC<EPI_RESID>{}, la.ph[2], i2, 2);
    if (i3.has) ring_fill(i3);
    run_phase(IntC<EPI_QKV>{}, la.ph[3], i3, 3);
  } else {
    run_phase(IntC<EPI_RESID>{}, la.ph[2], i2, 2);
  }
}

template <int NPH>
static bool dispatch_layer(hipStream_t st, const LayerArgs &la, int grid, bool query_only, int *max_grid) {
  const GemmArgs &a = la.ph[0];
  // every phase's k range must be a whole number of DEPTH chunks of KC
  auto fits = [&](int kc, int depth) {
    for (int p = 0; p < NPH; ++p) {
      const GemmArgs &g = la.ph[p];
      if (g.k_per_split % (depth * kc) != 0 || g.k % g.k_per_split != 0 || g.k_per_split * g.n_splits != g.k) return false;
    }
    return true;
  };
#define TS_LAYER(MB_, KC_, DEPTH_)                                                                      \
  do {                                                                                                  \
    if (!fits(KC_, DEPTH_)) return false;                                                               \
    auto kern = k_layer_bf16<MB_, KC_, DEPTH_, NPH>;                                                    \
    if (max_grid) {                                                                                     \
      int nb = 0, dev = 0, cus = 0;                                                                     \
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 256, 0) != hipSuccess) return false;  \
      if (hipGetDevice(&dev) != hipSuccess ||                                                           \
          hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)        \
        return false;                                                                                   \
      *max_grid = nb * cus;                                                                             \
    }                                                                                                   \
    if (!query_only) hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, la);                        \
    return true;                                                                                        \
  } while (0)
  // two ring depths per row count: `deep` (8 chunks, 256 KB of weights in flight per workgroup at up
  // to 64 rows) where every k range is a multiple of it, else 4 chunks
  const bool deep = la.ring_depth == 8;
  switch (a.rows_pad) {
    case 32:
      if (deep) TS_LAYER(1, 128, 8);
      TS_LAYER(1, 128, 4);
    case 64:
      if (deep) TS_LAYER(2, 128, 8);
      TS_LAYER(2, 128, 4);
    case 128:
      if (deep) TS_LAYER(4, 64, 8);
      TS_LAYER(4, 64, 4);
    default: return false;   // 256-row panels: the ring does not fit next to the accumulators
  }
#undef TS_LAYER
}

// Largest grid of the layer kernel for this row count that is resident all at once on the current
// device (0: no such kernel for these shapes).  Makes HIP occupancy queries: not for the hot path.
int layer_kernel_max_grid(const LayerArgs &la) {
  int g = 0;
  const bool ok = la.n_phases == 4 ? dispatch_layer<4>(nullptr, la, 0, true, &g) : dispatch_layer<3>(nullptr, la, 0, true, &g);
  return ok ? g : 0;
}

bool launch_layer_bf16(hipStream_t st, const LayerArgs &la, int grid) {
  return la.n_phases == 4 ? dispatch_layer<4>(st, la, grid, false, nullptr) : dispatch_layer<3>(st, la, grid, false, nullptr);
}

}  // namespace ts
