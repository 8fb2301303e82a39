// Weight-streaming small-M matmul on the matrix cores (bf16 in, fp32 accumulate).
//
//   out[split][r][n] = sum_{k in split} X[r][k] * W[n][k]        r < rows_pad <= 256
//
// At these row counts the product is bound by streaming W from HBM once, so the layout serves
// the W stream: every wavefront owns 32 output columns (= 32 rows of W) and pulls them straight
// from global memory into registers, 64 contiguous bytes per lane per 64-deep k block (each W
// row is consumed in whole 128-byte lines); W never passes through LDS and is never re-read.
// The small activation panel X is what all four wavefronts share: it is staged through LDS in
// chunks of KC reduction elements, double buffered, with a 16-byte row pad that makes the
// 16-byte operand reads conflict free.  X arrives as two bf16 panels, hi and lo (hi + lo carries
// ~16 significant bits of the fp32 activation); each W fragment is multiplied by both, so no
// activation is rounded to bf16 precision and W is still read exactly once.  MFMA 32x32x16: A = X fragment (row = activation row),
// B = W fragment (column = output column), so accumulator register e of lane (ln, g) holds
// out[8*(e/4) + 4*g + e%4][ln] and a half wavefront stores 128 contiguous bytes per row.
// The k index inside a 64 block is permuted (lane half g owns k = 32g + 8j + 0..7 at MFMA step
// j) identically for both operands, which is what lets a lane read 64 contiguous bytes.
//
// Work is split over (column tile of 128, k split); the splits are summed in ascending order by
// the consumer kernels, so results do not depend on scheduling.
//
// HEAD variant (LM head): instead of storing logits, every workgroup reduces its 128 columns to
// per-row (largest logit, its column, second largest, sum of exp relative to the largest) —
// the probabilities are never materialised.
#include "device_util.hpp"

namespace ts {

template <int MB, int KC, bool HEAD>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmArgs a, HeadStats hs, float *dbg) {
  constexpr int KB = KC / 64;                 // 64-deep k blocks per chunk
  constexpr int STRIDE = KC * 2 + 16;         // LDS bytes per activation row
  constexpr int PANEL = MB * 32 * STRIDE;     // one operand panel (hi or lo) of one stage
  constexpr int BUF = 2 * PANEL;
  constexpr int XV = MB * 32 * (KC / 8) / 256;  // 16-byte vectors per thread per chunk, per panel
  constexpr int TILE_LD = 132;                // floats per row of the HEAD logits tile
  static_assert(!HEAD || 2 * BUF >= 32 * TILE_LD * 4, "logits tile must fit the staging LDS");
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, g = lane >> 5;
  const int tile = blockIdx.x, split = blockIdx.y;
  const int k_begin = split * a.k_per_split;
  const int klen = min(a.k, k_begin + a.k_per_split) - k_begin;
  const int n_chunks = (klen + KC - 1) / KC;

  // ---- this wavefront's 32 output columns and the W rows behind them
  const int n0 = tile * kGemmTileN + wave * 32;
  const bool active = n0 < a.n_total;
  int sidx = 0;
  if (a.n_seg > 1 && n0 >= a.seg[1].col0) sidx = 1;
  if (a.n_seg > 2 && n0 >= a.seg[2].col0) sidx = 2;
  const bf16 *wseg = (const bf16 *)(sidx == 0 ? a.seg[0].w : (sidx == 1 ? a.seg[1].w : a.seg[2].w));
  const int seg_rows = sidx == 0 ? a.seg[0].n_rows : (sidx == 1 ? a.seg[1].n_rows : a.seg[2].n_rows);
  const int seg_col0 = sidx == 0 ? a.seg[0].col0 : (sidx == 1 ? a.seg[1].col0 : a.seg[2].col0);
  const int nloc = n0 - seg_col0 + ln;
  const bool n_ok = active && nloc < seg_rows;
  const bf16 *wrow = wseg + (size_t)min(max(nloc, 0), seg_rows - 1) * a.k + k_begin + 32 * g;
  const bf16 *xg = (const bf16 *)a.x + k_begin;

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;

  bf16x8 w0[KB][4], w1[KB][4];
  uint4 xr[2][XV];

  auto load_w = [&](bf16x8 (&w)[KB][4], int c) {
    if (!active) return;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
      if (c * KC + kb * 64 < klen) {
#pragma unroll
        for (int j = 0; j < 4; ++j) w[kb][j] = *(const bf16x8 *)(wrow + c * KC + kb * 64 + 8 * j);
      }
  };
  auto load_x = [&](int c) {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int v = tid + 256 * i;
      const int row = v / (KC / 8), col = c * KC + (v % (KC / 8)) * 8;
      const bf16 *src = xg + (size_t)row * a.k + col;
      xr[0][i] = (col < klen) ? *(const uint4 *)src : make_uint4(0, 0, 0, 0);
      xr[1][i] = (col < klen) ? *(const uint4 *)(src + a.x_panel) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int v = tid + 256 * i;
      const int row = v / (KC / 8), cv = v % (KC / 8);
      *(uint4 *)(lds + buf * BUF + row * STRIDE + cv * 16) = xr[0][i];
      *(uint4 *)(lds + buf * BUF + PANEL + row * STRIDE + cv * 16) = xr[1][i];
    }
  };
  auto compute = [&](const bf16x8 (&w)[KB][4], int c, int buf) {
    if (!active) return;
    const unsigned char *xb = lds + buf * BUF + ln * STRIDE + 64 * g;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
      if (c * KC + kb * 64 < klen) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            const unsigned char *xp = xb + mb * 32 * STRIDE + kb * 128 + j * 16;
            const bf16x8 xhi = *(const bf16x8 *)xp;
            const bf16x8 xlo = *(const bf16x8 *)(xp + PANEL);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xhi, w[kb][j], acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xlo, w[kb][j], acc[mb], 0, 0, 0);
          }
      }
  };
  auto step = [&](const bf16x8 (&wc)[KB][4], bf16x8 (&wn)[KB][4], int c) {
    const bool more = c + 1 < n_chunks;
    if (more) {
      load_w(wn, c + 1);
      load_x(c + 1);
    }
    compute(wc, c, c & 1);
    if (more) store_x((c + 1) & 1);
    __syncthreads();
  };

  load_w(w0, 0);
  load_x(0);
  store_x(0);
  __syncthreads();
  for (int c = 0; c < n_chunks; c += 2) {
    step(w0, w1, c);
    if (c + 1 < n_chunks) step(w1, w0, c + 1);
  }

  if (!HEAD) {
    if (!n_ok) return;
    float *o = a.out + (size_t)split * a.rows_pad * a.n_total + n0 + ln;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = mb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        if (r < a.rows) o[(size_t)r * a.n_total] = acc[mb][e];
      }
    return;
  }

  // ---- HEAD: per row, reduce this tile's 128 logits to (l1, column, l2, sum exp)
  float *tl = (float *)lds;
  const int srow = tid >> 3, part = tid & 7;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 16; ++e)
      tl[(8 * (e >> 2) + 4 * g + (e & 3)) * TILE_LD + wave * 32 + ln] = acc[mb][e];
    __syncthreads();
    const int r = mb * 32 + srow;
    Top2 t = top2_empty();
    const int cbase = tile * kGemmTileN + part * 16;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const float v = tl[srow * TILE_LD + part * 16 + c];
      if (cbase + c < a.n_total) {
        top2_push(t, v, cbase + c);
        if (dbg != nullptr && r < a.rows) dbg[(size_t)r * a.n_total + cbase + c] = v;
      }
    }
    t = top2_merge(t, top2_shfl_xor(t, 1));
    t = top2_merge(t, top2_shfl_xor(t, 2));
    t = top2_merge(t, top2_shfl_xor(t, 4));
    if (part == 0 && r < a.rows) {
      const size_t o = (size_t)r * hs.n_tiles + tile;
      hs.l1[o] = t.l1; hs.l2[o] = t.l2; hs.sumexp[o] = t.s; hs.idx[o] = t.idx;
    }
  }
}

template <bool HEAD>
static void dispatch(hipStream_t st, const GemmArgs &a, const HeadStats &hs, float *dbg) {
  const int tiles = (a.n_total + kGemmTileN - 1) / kGemmTileN;
  dim3 grid(tiles, a.n_splits), block(256);
  switch (a.rows_pad) {
    case 32: hipLaunchKernelGGL((k_gemm_bf16<1, 256, HEAD>), grid, block, 0, st, a, hs, dbg); break;
    case 64: hipLaunchKernelGGL((k_gemm_bf16<2, 128, HEAD>), grid, block, 0, st, a, hs, dbg); break;
    case 128: hipLaunchKernelGGL((k_gemm_bf16<4, 64, HEAD>), grid, block, 0, st, a, hs, dbg); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<8, 64, HEAD>), grid, block, 0, st, a, hs, dbg); break;
  }
}

void launch_gemm_bf16(hipStream_t st, const GemmArgs &a) {
  HeadStats none = {};
  dispatch<false>(st, a, none, nullptr);
}

void launch_lmhead_bf16(hipStream_t st, const GemmArgs &a, const HeadStats &hs, float *debug_logits) {
  dispatch<true>(st, a, hs, debug_logits);
}

}  // namespace ts
