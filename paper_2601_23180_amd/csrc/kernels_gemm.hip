// Weight-streaming small-M matmul on the matrix cores (bf16 in, fp32 accumulate).
//
//   out[split][r][n] = sum_{k in split} X[r][k] * W[n][k]        r < rows_pad <= 256
//
// At these row counts the product is bound by streaming W from HBM once, so the layout serves
// the W stream.  W is read from the PACKED copy made once by k_pack_weights: for every 32-row
// sub-tile s and 64-deep k block kb, one contiguous 4 KB block holding the four MFMA B-operand
// fragments of that (s, kb) in lane order.  A wavefront owns one sub-tile (32 output columns) and
// pulls its blocks straight from global memory into registers — every load instruction reads
// 1 KB contiguous (8 whole 128-byte lines), a sub-tile's k range is one contiguous run, W never
// passes through LDS and is never re-read.  (Reading row-major W with the same operand layout
// touches 32 rows x 32 bytes per instruction and reaches ~75 % of the contiguous rate.)
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

// RAGGED: some k split is not a whole number of KC chunks (odd shapes only; the model shapes this
// is tuned for never need it).  The fast variant has no bounds logic at all in the stream.
template <int MB, int KC, bool HEAD, bool RAGGED>
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
  // packed sub-tile of this wavefront (clamped to the segment's last one: always valid memory;
  // rows past the segment's end are zero in the packed copy)
  const int n_sub_seg = (seg_rows + 31) >> 5;
  const int sub = min(max((n0 - seg_col0) >> 5, 0), n_sub_seg - 1);
  const bf16 *wrow = wseg + ((size_t)sub * (a.k >> 6) + (k_begin >> 6)) * 2048 + lane * 8;
  const bf16 *xg = (const bf16 *)a.x + k_begin;

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;

  // The streaming loop is kept free of branches around loads: a load behind a branch makes the
  // wait-count analysis assume it may not have been issued, which turns every wait into "drain
  // everything" and serialises the stream.
  //
  // Fast variant (every k split is a whole, even number of KC chunks), per chunk c:
  //   1. X registers (chunk c+1, fetched during chunk c-1) -> LDS stage (c+1)&1
  //   2. issue the X loads of chunk c+2
  //   3. per 64-deep block: 4 x MB x 2 MFMAs on W set c&1, then refill that block of the set
  //      with chunk c+2 — so a W load has two chunks of compute to arrive
  //   4. workgroup barrier
  // sched_barrier pins the load issue points; the compiler would otherwise sink every load to
  // just before its first use and expose the whole memory latency once per chunk.
  bf16x8 w[2][KB][4];
  uint4 xr[2][XV];

  auto load_w_block = [&](int set, int c, int kb) {   // W rows of this wavefront, block kb of chunk c
    const int k = c * KC + kb * 64;
    const bf16 *p = wrow + (size_t)((!RAGGED || k < klen) ? (k >> 6) : 0) * 2048;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[set][kb][j] = *(const bf16x8 *)(p + 512 * j);
  };
  auto load_x = [&](int c) {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const int v = tid + 256 * i;
      const int row = v / (KC / 8), col = c * KC + (v % (KC / 8)) * 8;
      const bool ok = !RAGGED || col < klen;
      const bf16 *src = xg + (size_t)row * a.k + (ok ? col : 0);
      const uint4 hi = *(const uint4 *)src;
      const uint4 lo = *(const uint4 *)(src + a.x_panel);
      xr[0][i] = ok ? hi : make_uint4(0, 0, 0, 0);
      xr[1][i] = ok ? lo : make_uint4(0, 0, 0, 0);
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
  auto mfma_block = [&](int set, int kb, int buf) {
    const unsigned char *xb = lds + buf * BUF + ln * STRIDE + 64 * g + kb * 128;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const unsigned char *xp = xb + mb * 32 * STRIDE + j * 16;
        const bf16x8 xhi = *(const bf16x8 *)xp;
        const bf16x8 xlo = *(const bf16x8 *)(xp + PANEL);
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xhi, w[set][kb][j], acc[mb], 0, 0, 0);
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xlo, w[set][kb][j], acc[mb], 0, 0, 0);
      }
  };

  if (RAGGED) {
    // simple one-chunk-ahead loop with bounds logic (odd shapes only)
    load_x(0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) load_w_block(0, 0, kb);
    store_x(0);
    __syncthreads();
    for (int c = 0; c + 1 < n_chunks; ++c) {
      load_x(c + 1);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        mfma_block(0, kb, c & 1);
        load_w_block(0, c + 1, kb);
      }
      store_x((c + 1) & 1);
      __syncthreads();
    }
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) mfma_block(0, kb, (n_chunks - 1) & 1);
  } else {
    // n_chunks is even and >= 2.  The prologue issues its loads in the order the steady state
    // does (X of a chunk before the W refill of the same step), so the wait counts merged at the
    // loop head are the steady-state ones.
    load_x(0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) load_w_block(0, 0, kb);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0);
    load_x(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) load_w_block(1, 1, kb);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    // chunk pair (c, c+1) with c even: set 0 serves chunk c, set 1 serves chunk c+1
    for (int c = 0; c + 2 < n_chunks; c += 2) {
      store_x(1);            // chunk c+1
      load_x(c + 2);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        mfma_block(0, kb, 0);
        load_w_block(0, c + 2, kb);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
      store_x(0);            // chunk c+2
      load_x(c + 3);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        mfma_block(1, kb, 1);
        load_w_block(1, c + 3, kb);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
    }
    // last pair: nothing left to fetch
    store_x(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) mfma_block(0, kb, 0);
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) mfma_block(1, kb, 1);
  }

  if (!HEAD) {
    if (!n_ok) return;   // clamped duplicate columns and idle wavefronts computed on valid memory
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

// One-time repack of a row-major [n_rows, k] bf16 matrix into the layout above.  One thread per
// 16-byte piece of the output: piece (s, kb, j, lane) = W[32 s + (lane & 31)][64 kb + 32 (lane >> 5) + 8 j .. + 8].
__global__ __launch_bounds__(256) void k_pack_weights(const bf16 *w, int n_rows, int k, uint4 *out,
                                                      size_t n_pieces) {
  const size_t p = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= n_pieces) return;
  const int lane = (int)(p & 63), j = (int)((p >> 6) & 3);
  const size_t blk = p >> 8;
  const int kblocks = k >> 6;
  const int kb = (int)(blk % kblocks);
  const int s = (int)(blk / kblocks);
  const int row = 32 * s + (lane & 31);
  const int col = 64 * kb + 32 * (lane >> 5) + 8 * j;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < n_rows) v = *(const uint4 *)(w + (size_t)row * k + col);
  out[p] = v;
}

size_t packed_weight_bytes(int n_rows, int k) { return (size_t)((n_rows + 31) / 32) * (k / 64) * 4096; }

void launch_pack_weights(hipStream_t st, const void *w, int n_rows, int k, void *out) {
  const size_t n_pieces = packed_weight_bytes(n_rows, k) / 16;
  hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)((n_pieces + 255) / 256)), dim3(256), 0, st,
                     (const bf16 *)w, n_rows, k, (uint4 *)out, n_pieces);
}

template <bool HEAD>
static void dispatch(hipStream_t st, const GemmArgs &a, const HeadStats &hs, float *dbg) {
  const int tiles = (a.n_total + kGemmTileN - 1) / kGemmTileN;
  dim3 grid(tiles, a.n_splits), block(256);
#define TS_LAUNCH(MB_, KC_)                                                                         \
  do {                                                                                              \
    if (a.k_per_split % (2 * KC_) == 0 && a.k % (2 * KC_) == 0)                                     \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, HEAD, false>), grid, block, 0, st, a, hs, dbg);     \
    else                                                                                            \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, HEAD, true>), grid, block, 0, st, a, hs, dbg);      \
  } while (0)
  switch (a.rows_pad) {
    case 32: TS_LAUNCH(1, 256); break;
    case 64: TS_LAUNCH(2, 128); break;
    case 128: TS_LAUNCH(4, 64); break;
    default: TS_LAUNCH(8, 64); break;
  }
#undef TS_LAUNCH
}

void launch_gemm_bf16(hipStream_t st, const GemmArgs &a) {
  HeadStats none = {};
  dispatch<false>(st, a, none, nullptr);
}

void launch_lmhead_bf16(hipStream_t st, const GemmArgs &a, const HeadStats &hs, float *debug_logits) {
  dispatch<true>(st, a, hs, debug_logits);
}

}  // namespace ts
