// Weight-streaming small-M matmul on the matrix cores (bf16 weights, fp32 accumulate) with the
// surrounding element-wise work fused in.
//
//   y[r][n] = row_scale[r] * sum_k X[r][k] * W[n][k]        r < rows_pad <= 256
//
// At these row counts the product is bound by streaming W from HBM once, so the layout serves
// the W stream.  W is read from the PACKED copy made once by k_pack_weights: for every 32-row
// sub-tile s and 64-deep k block kb, one contiguous 4 KB block holding the four MFMA B-operand
// fragments of that (s, kb) in lane order.  A wavefront owns one sub-tile (32 output columns) and
// pulls its blocks straight from global memory into registers — every load instruction reads
// 1 KB contiguous (8 whole 128-byte lines), a sub-tile's k range is one contiguous run, W never
// passes through LDS and is never re-read.  (Reading row-major W with the same operand layout
// touches 32 rows x 32 bytes per instruction and reaches ~75 % of the contiguous rate.)
//
// The activation panel X (at most 256 rows) is what the four wavefronts of a workgroup share.
// It arrives as two bf16 panels, a high part and a low part (hi = round(v), lo = round(v - hi),
// written once by whichever kernel produced the activation — splitting it here would repeat the
// conversion in every one of the hundreds of workgroups and costs more issue slots than the
// MFMAs).  Each W fragment is multiplied by both parts, so the activations keep ~16 significant
// bits, the pass is a smooth function of its inputs, and W is still read exactly once.  X is
// staged through LDS in chunks of KC reduction elements, double buffered, rows padded by 16
// bytes so that the 16-byte operand reads are conflict free.
// RMSNorm is fused around the matmul: the producer stores x * w_norm (the per-column weight) as
// the operand panels, and the per-row 1/rms (row_scale) multiplies the reduced sums here.
//
// MFMA 32x32x16: A = X fragment (row = activation row), B = W fragment (column = output
// column), so accumulator register e of lane (ln, g) holds y[8*(e/4) + 4*g + e%4][ln].  The k
// index inside a 64 block is permuted (lane half g owns k = 32g + 8j + 0..7 at MFMA step j)
// identically for both operands.
//
// Work = (tile of 128 output columns) x (k split).  Every workgroup stores its fp32 partial tile;
// the LAST workgroup to finish a tile (an atomic counter per tile) sums the splits in ascending
// order — so the result does not depend on scheduling — and applies the tile's epilogue:
//   QKV    rotary embedding, fp32 q/k/v for the attention kernels, bf16 K and V^T cache append
//   RESID  residual add into the fp32 stream, operand panels (x * next norm weight, hi/lo) for
//          the next matmul, per-row sum of squares; the last TILE turns the sums into 1/rms
//   SWIGLU SiLU(gate) * up as operand panels (a tile holds 64 gate columns and the matching 64
//          up columns)
//   HEAD   (LM head, no k split) per-row (largest logit, its column, second largest, sum of exp)
//          of the tile's 128 logits — the probabilities are never materialised.
#include "device_util.hpp"

namespace ts {

template <int MB, int KC, int EPI, bool RAGGED>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmArgs a) {
  constexpr int KB = KC / 64;                 // 64-deep k blocks per chunk
  constexpr int STRIDE = KC * 2 + 16;         // LDS bytes per activation row (one panel)
  constexpr int PANEL = MB * 32 * STRIDE;     // one operand panel (hi or lo) of one stage
  constexpr int BUF = 2 * PANEL;
  constexpr int XV = MB * 32 * (KC / 8) / 256;  // 16-byte vectors per thread per chunk, per panel
  constexpr int ROWS_PER_PASS = 256 / (KC / 8); // rows covered by one vector index step
  constexpr int TILE_LD = 132;                // floats per row of the HEAD logits tile
  static_assert(2 * BUF >= 32 * TILE_LD * 4, "logits tile must fit the staging LDS");
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, g = lane >> 5;
  const int tile = blockIdx.x, split = blockIdx.y;
  const int k_begin = split * a.k_per_split;
  const int klen = min(a.k, k_begin + a.k_per_split) - k_begin;
  const int n_chunks = (klen + KC - 1) / KC;

  // ---- this wavefront's packed sub-tile.  Plain tiles: 4 consecutive sub-tiles of the
  // concatenated segments.  SWIGLU tiles: waves 0,1 -> gate sub-tiles 2t, 2t+1; waves 2,3 -> the
  // same sub-tiles of the up projection.
  int sidx, sub;
  if (EPI == EPI_SWIGLU) {
    sidx = wave >> 1;
    sub = 2 * tile + (wave & 1);
  } else {
    const int n0 = tile * kGemmTileN + wave * 32;
    sidx = 0;
    if (a.n_seg > 1 && n0 >= a.seg[1].col0) sidx = 1;
    if (a.n_seg > 2 && n0 >= a.seg[2].col0) sidx = 2;
    const int col0 = sidx == 0 ? a.seg[0].col0 : (sidx == 1 ? a.seg[1].col0 : a.seg[2].col0);
    sub = (n0 - col0) >> 5;
  }
  const bf16 *wseg = (const bf16 *)(sidx == 0 ? a.seg[0].w : (sidx == 1 ? a.seg[1].w : a.seg[2].w));
  const int seg_rows = sidx == 0 ? a.seg[0].n_rows : (sidx == 1 ? a.seg[1].n_rows : a.seg[2].n_rows);
  // clamped to the segment's last sub-tile: always valid memory (idle wavefronts of a ragged last
  // tile compute on it and their columns are never stored)
  sub = min(max(sub, 0), ((seg_rows + 31) >> 5) - 1);
  const bf16 *wrow = wseg + ((size_t)sub * (a.k >> 6) + (k_begin >> 6)) * 2048 + lane * 8;

  // ---- X staging: thread copies 16-byte column c8 of rows r0 + ROWS_PER_PASS * i, both panels
  const int c8 = tid % (KC / 8), r0 = tid / (KC / 8);
  const bf16 *xg = (const bf16 *)a.x + (size_t)r0 * a.k + k_begin + c8 * 8;

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

  auto load_w_block = [&](int set, int c, int kb) {
    const int k = c * KC + kb * 64;
    const bf16 *p = wrow + (size_t)((!RAGGED || k < klen) ? (k >> 6) : 0) * 2048;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[set][kb][j] = *(const bf16x8 *)(p + 512 * j);
  };
  auto load_x = [&](int c) {
    const bool ok = !RAGGED || (c * KC + c8 * 8 < klen);
    const int off = ok ? c * KC : 0;
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      const bf16 *src = xg + (size_t)(ROWS_PER_PASS * i) * a.k + off;
      uint4 hi = *(const uint4 *)src;
      uint4 lo = *(const uint4 *)(src + a.x_panel);
      if (RAGGED && !ok) { hi = make_uint4(0, 0, 0, 0); lo = make_uint4(0, 0, 0, 0); }
      xr[0][i] = hi;
      xr[1][i] = lo;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      unsigned char *dst = lds + buf * BUF + (r0 + ROWS_PER_PASS * i) * STRIDE + c8 * 16;
      *(uint4 *)dst = xr[0][i];
      *(uint4 *)(dst + PANEL) = xr[1][i];
    }
  };
  // One chunk of MFMAs, software pipelined: step t = (k block, j) needs four A fragments
  // (row block 0/1 x hi/lo); they are read from LDS two steps ahead into a 2-slot register ring,
  // so the LDS latency hides behind the previous step's four MFMAs.  After the last step of a k
  // block, that block of the W set is refilled from chunk `c_next` (if LOADW).
  bf16x8 xf[2][2 * MB];
  auto read_frags = [&](int slot, int t, int buf) {
    const int kb = t >> 2, j = t & 3;
    const unsigned char *xp = lds + buf * BUF + ln * STRIDE + 64 * g + kb * 128 + j * 16;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      xf[slot][2 * mb] = *(const bf16x8 *)(xp + mb * 32 * STRIDE);
      xf[slot][2 * mb + 1] = *(const bf16x8 *)(xp + mb * 32 * STRIDE + PANEL);
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
      for (int mb = 0; mb < MB; ++mb) {
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[t & 1][2 * mb], w[set][kb][j], acc[mb], 0, 0, 0);
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[t & 1][2 * mb + 1], w[set][kb][j], acc[mb], 0, 0, 0);
      }
      if (t + 2 < T) read_frags(t & 1, t + 2, buf);
      if (j == 3 && loadw) load_w_block(set, c_next, kb);
      __builtin_amdgcn_sched_barrier(0);
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
      compute_chunk(0, c & 1, c + 1, true);
      store_x((c + 1) & 1);
      __syncthreads();
    }
    compute_chunk(0, (n_chunks - 1) & 1, 0, false);
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
      compute_chunk(0, 0, c + 2, true);
      __syncthreads();
      store_x(0);            // chunk c+2
      load_x(c + 3);
      __builtin_amdgcn_sched_barrier(0);
      compute_chunk(1, 1, c + 3, true);
      __syncthreads();
    }
    // last pair: nothing left to fetch
    store_x(1);
    __builtin_amdgcn_sched_barrier(0);
    compute_chunk(0, 0, 0, false);
    __syncthreads();
    compute_chunk(1, 1, 0, false);
  }

  if (EPI == EPI_HEAD) {
    // ---- per row, reduce this tile's 128 logits to (l1, column, l2, sum exp)
    float *tl = (float *)lds;
    const int srow = tid >> 3, part = tid & 7;
    // (row_scale is applied when the tile is read back: the scan thread owns one row)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 16; ++e)
        tl[(8 * (e >> 2) + 4 * g + (e & 3)) * TILE_LD + wave * 32 + ln] = acc[mb][e];
      __syncthreads();
      const int r = mb * 32 + srow;
      const float rsc = (a.row_scale != nullptr && r < a.rows) ? a.row_scale[r] : 1.0f;
      Top2 t = top2_empty();
      const int cbase = tile * kGemmTileN + part * 16;
#pragma unroll
      for (int c = 0; c < 16; ++c) {
        const float v = tl[srow * TILE_LD + part * 16 + c] * rsc;
        if (cbase + c < a.n_total) {
          top2_push(t, v, cbase + c);
          if (a.debug_logits != nullptr && r < a.rows) a.debug_logits[(size_t)r * a.n_total + cbase + c] = v;
        }
      }
      t = top2_merge(t, top2_shfl_xor(t, 1));
      t = top2_merge(t, top2_shfl_xor(t, 2));
      t = top2_merge(t, top2_shfl_xor(t, 4));
      if (part == 0 && r < a.rows) {
        const size_t o = (size_t)r * a.hs.n_tiles + tile;
        a.hs.l1[o] = t.l1; a.hs.l2[o] = t.l2; a.hs.sumexp[o] = t.s; a.hs.idx[o] = t.idx;
      }
    }
    return;
  }

  // ---- store the partial tile: part[split][tile][row][128]
  const size_t tile_elems = (size_t)a.rows_pad * kGemmTileN;
  {
    float *o = a.part + ((size_t)split * a.n_tiles + tile) * tile_elems + wave * 32 + ln;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = mb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        if (r < a.rows) st_agent(o + (size_t)r * kGemmTileN, acc[mb][e]);
      }
  }
  // ---- the last workgroup of this tile reduces the splits and runs the epilogue
  if (!publish_then_count(&a.counters[tile], a.n_splits, &s_last)) return;
  // The partial tiles were written through to memory (st_agent) and nobody on this chip has read
  // these lines before, so plain vector loads see them.
  const float *p0 = a.part + (size_t)tile * tile_elems;
  const size_t split_stride = (size_t)a.n_tiles * tile_elems;
  auto reduced4 = [&](int r, int c) {   // 4 consecutive columns, splits summed in ascending order
    const float *p = p0 + (size_t)r * kGemmTileN + c;
    f32x4 v = *(const f32x4 *)p;
    for (int s = 1; s < a.n_splits; ++s) v += *(const f32x4 *)(p + (size_t)s * split_stride);
    return v;
  };

  if (EPI == EPI_QKV) {
    // a tile is one head (d = 128) or two heads (d = 64); thread = (row, 4 rotation pairs)
    const int d = a.head_dim, half = d >> 1;
    const int n_q = a.n_q_heads, n_kv = a.n_kv_heads;
    const int quads = kGemmTileN / 8;                       // 4-pair groups per row
    for (int t = tid; t < a.rows * quads; t += 256) {
      const int r = t / quads, qi = t - r * quads;
      const int hl = (qi * 4) / half, j = qi * 4 - hl * half;   // head within the tile, first pair
      const int c_lo = hl * d + j;                          // tile-local column of the low elements
      const int col = tile * kGemmTileN + c_lo;             // global column
      if (col >= a.n_total) continue;
      const int hh = col / d;                               // global head index (q heads, k heads, v heads)
      const float rsc = a.row_scale[r];
      f32x4 lo = reduced4(r, c_lo) * rsc, hi = reduced4(r, c_lo + half) * rsc;
      const int b = r / a.n_nodes, node = r - b * a.n_nodes;
      const int slot = a.ctx.v[b] + node;
      if (hh < n_q + n_kv) {
        const f32x4 c = *(const f32x4 *)(a.cos_t + r * half + j), sn = *(const f32x4 *)(a.sin_t + r * half + j);
        const f32x4 rl = lo * c - hi * sn, rh = hi * c + lo * sn;
        lo = rl; hi = rh;
      }
      *(f32x4 *)(a.qkv_f32 + (size_t)r * a.n_total + col) = lo;
      *(f32x4 *)(a.qkv_f32 + (size_t)r * a.n_total + col + half) = hi;
      if (hh >= n_q && hh < n_q + n_kv) {
        bf16 *kc = (bf16 *)a.k_cache + (((size_t)b * n_kv + (hh - n_q)) * a.capacity + slot) * d;
        bf16x4 l4, h4;
#pragma unroll
        for (int e = 0; e < 4; ++e) { l4[e] = (bf16)lo[e]; h4[e] = (bf16)hi[e]; }
        *(bf16x4 *)(kc + j) = l4;
        *(bf16x4 *)(kc + j + half) = h4;
      } else if (hh >= n_q + n_kv) {
        bf16 *vc = (bf16 *)a.v_cache + ((size_t)b * n_kv + (hh - n_q - n_kv)) * d * a.capacity;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          vc[(size_t)(j + e) * a.capacity + slot] = (bf16)lo[e];
          vc[(size_t)(j + e + half) * a.capacity + slot] = (bf16)hi[e];
        }
      }
    }
    return;
  }

  if (EPI == EPI_SWIGLU) {
    // columns [0, 64) of the tile are gate, [64, 128) the matching up columns
    for (int t = tid; t < a.rows * 16; t += 256) {
      const int r = t >> 4, f = (t & 15) * 4;
      const int feat = tile * 64 + f;
      if (feat >= a.ffn) continue;
      const float rsc = a.row_scale[r];
      const f32x4 gt = reduced4(r, f) * rsc, up = reduced4(r, 64 + f) * rsc;
      bf16x4 hi, lo;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float o = gt[e] / (1.0f + expf(-gt[e])) * up[e];
        hi[e] = (bf16)o;
        lo[e] = (bf16)(o - (float)hi[e]);
      }
      bf16 *dst = (bf16 *)a.act_out + (size_t)r * a.ffn + feat;
      *(bf16x4 *)dst = hi;
      *(bf16x4 *)(dst + a.out_panel) = lo;
    }
    return;
  }

  // ---- EPI_RESID: x += y; per-row sum of squares of the new x over this tile's columns.
  // A half wavefront (32 lanes x 4 columns) covers one row of the tile.
  {
    float *ssp = a.ss_part + (size_t)tile * a.rows_pad;
    const int c = ln * 4, col = tile * kGemmTileN + c;
    for (int r = wave * 2 + g; r < a.rows_pad; r += 8) {
      float ss = 0.f;
      if (r < a.rows && col < a.n_total) {
        float *xp = a.x_resid + (size_t)r * a.n_total + col;
        const f32x4 v = *(const f32x4 *)xp + reduced4(r, c);
        *(f32x4 *)xp = v;
        ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        // operand of the next matmul: x * (next RMSNorm weight), as bf16 hi + lo
        const bf16x4 nw = *(const bf16x4 *)((const bf16 *)a.next_norm_w + col);
        bf16x4 hi, lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float o = v[e] * (float)nw[e];
          hi[e] = (bf16)o;
          lo[e] = (bf16)(o - (float)hi[e]);
        }
        bf16 *dst = (bf16 *)a.xw_out + (size_t)r * a.n_total + col;
        *(bf16x4 *)dst = hi;
        *(bf16x4 *)(dst + a.out_panel) = lo;
      }
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
      if (ln == 0 && r < a.rows) st_agent(ssp + r, ss);
    }
    if (!publish_then_count(&a.counters[a.n_tiles], a.n_tiles, &s_last)) return;
    // last tile of the launch: 1/rms of every row for the next matmul's prologue
    for (int r = tid; r < a.rows; r += 256) {
      float ss = 0.f;
      for (int t = 0; t < a.n_tiles; ++t) ss += ld_agent(a.ss_part + (size_t)t * a.rows_pad + r);
      a.rstd_out[r] = 1.0f / sqrtf(ss / (float)a.n_total + a.eps);
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

template <int EPI>
static void dispatch(hipStream_t st, const GemmArgs &a) {
  dim3 grid(a.n_tiles, a.n_splits), block(256);
#define TS_LAUNCH(MB_, KC_)                                                                   \
  do {                                                                                        \
    if (a.k_per_split % (2 * KC_) == 0 && a.k % (2 * KC_) == 0)                               \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, EPI, false>), grid, block, 0, st, a);         \
    else                                                                                      \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, EPI, true>), grid, block, 0, st, a);          \
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
  switch (a.epi) {
    case EPI_QKV: dispatch<EPI_QKV>(st, a); break;
    case EPI_RESID: dispatch<EPI_RESID>(st, a); break;
    case EPI_SWIGLU: dispatch<EPI_SWIGLU>(st, a); break;
    default: dispatch<EPI_HEAD>(st, a); break;
  }
}

}  // namespace ts
