// Weight-streaming small-M matmul on the matrix cores (bf16 weights, fp32 accumulate) with the
// surrounding element-wise work fused in.
//
//   y[r][n] = rstd[r] * sum_k X[r][k] * W[n][k]        r < rows_pad <= 256
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
// stored in the operand layout (device_util.hpp: 1 KB fragments in consumption order), staged
// through LDS in chunks of KC reduction elements, double buffered, by plain contiguous copies;
// the 16-byte operand reads are conflict free.
// RMSNorm is fused around the matmul: the producer stores x * w_norm (the per-column weight) as
// the operand panels, and the per-row 1/rms multiplies the reduced sums in the epilogue here.
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
//          the next matmul, per-row sum of squares of the tile (the consumer turns the tile sums
//          into 1/rms — a second chip-wide counter here costs more than re-adding 32 numbers)
//   SWIGLU SiLU(gate) * up as operand panels (a tile holds 64 gate columns and the matching 64
//          up columns)
//   HEAD   (LM head, no k split) per-row (largest logit, its column, second largest, sum of exp)
//          of the tile's 128 logits — the probabilities are never materialised.
#include "gemm_epilogue.hpp"

namespace ts {

template <int MB, int KC, int EPI, bool RAGGED, int DEPTH>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmArgs a) {
  constexpr int KB = KC / 64;                 // 64-deep k blocks per chunk
  constexpr int FRAGS = KB * 4 * MB * 2;      // 1 KB operand fragments per chunk (operand layout)
  constexpr int BUF = FRAGS * 1024;           // one LDS stage
  constexpr int XV = FRAGS / 4;               // fragments (16 bytes per lane) per wavefront per chunk
  constexpr int EPI_BYTES = MB * 32 * (kGemmTileN + 4) * 4;   // the epilogue's fp32 tile reuses the stages
  constexpr int LDS_BYTES = 2 * BUF > EPI_BYTES ? 2 * BUF : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];
  __shared__ int s_last;
  __shared__ float s_rs[kMaxRows];   // 1/rms of the rows of the matmul's input
  __shared__ float s_rsp[4 * kMaxRows];

  const int tid = threadIdx.x, lane = tid & 63;
  // scalar: what is selected by it (this wavefront's weight segment) is then fetched with scalar
  // loads from the kernel arguments, not with a vector load that the first weight request waits for
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, g = lane >> 5;
  const int tile = blockIdx.x, split = blockIdx.y;
  const int k_begin = split * a.k_per_split;
  const int klen = min(a.k, k_begin + a.k_per_split) - k_begin;
  const int n_chunks = (klen + KC - 1) / KC;
  // Workgroups that run side by side start at different depths of their k range (and wrap
  // around), so that they do not all walk the memory channels in lockstep.  The order of the
  // additions is still a fixed function of (tile, split).
  const int rot = RAGGED ? 0 : (int)((blockIdx.x * 11u + blockIdx.y * 5u) % (unsigned)n_chunks);
  auto rc = [&](int c) { const int cc = c + rot; return cc >= n_chunks ? cc - n_chunks : cc; };

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

  // ---- X staging: the chunk is a contiguous run of FRAGS fragments in operand layout; this
  // wavefront copies fragments wave*XV .. wave*XV + XV-1, 16 bytes per lane each
  const bf16 *xg = (const bf16 *)a.x + ((size_t)(k_begin >> 6) * 4 * MB * 2 + wave * XV) * 512 + lane * 8;

  // 1/rms of every row of the matmul's INPUT (used by the epilogue): the loads go out here, ahead
  // of the stream, and are consumed after it.
  float rs_in[(MB + 1) / 2][8];
  rstd_load<256, MB>(a, rs_in);

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mb][e] = 0.f;

  // The streaming loop is kept free of branches around loads: a load behind a branch makes the
  // wait-count analysis assume it may not have been issued, which turns every wait into "drain
  // everything" and serialises the stream.
  //
  // Fast variant (every k split is a whole multiple of DEPTH chunks of KC), per chunk c:
  //   1. X registers (chunk c+1, fetched during chunk c-1) -> LDS stage (c+1)&1
  //   2. issue the X loads of chunk c+2
  //   3. per 64-deep block: 4 x MB x 2 MFMAs on W set c % DEPTH, then refill that block of the
  //      set with chunk c+DEPTH — a W load has DEPTH chunks of compute to arrive, and a wavefront
  //      keeps about DEPTH * KC/64 * 4 KB in flight.  (HBM latency under load is several
  //      microseconds; at 8 wavefronts per CU it takes this much to keep the stream full.)
  //   4. workgroup barrier
  // sched_barrier pins the load issue points; the compiler would otherwise sink every load to
  // just before its first use and expose the whole memory latency once per chunk.
  bf16x8 w[DEPTH][KB][4];
  uint4 xr[XV];

  auto load_w_block = [&](int set, int c, int kb) {
    const int k = rc(c) * KC + kb * 64;
    const bf16 *p = wrow + (size_t)((!RAGGED || k < klen) ? (k >> 6) : 0) * 2048;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[set][kb][j] = __builtin_nontemporal_load((const bf16x8 *)(p + 512 * j));
  };
  auto load_x = [&](int c) {
    const bool ok = !RAGGED || (c * KC < klen);
    const bf16 *src = xg + (size_t)(ok ? rc(c) : 0) * FRAGS * 512;
#pragma unroll
    for (int i = 0; i < XV; ++i) {
      uint4 v = *(const uint4 *)(src + i * 512);
      if (RAGGED) {
        // fragment (wave*XV + i) belongs to k block kb of the chunk; blocks past the split are zero
        const int kb = (wave * XV + i) / (4 * MB * 2);
        if (!ok || c * KC + kb * 64 >= klen) v = make_uint4(0, 0, 0, 0);
      }
      xr[i] = v;
    }
  };
  auto store_x = [&](int buf) {
    unsigned char *dst = lds + buf * BUF + (wave * XV) * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < XV; ++i) *(uint4 *)(dst + i * 1024) = xr[i];
  };
  // One chunk of MFMAs, software pipelined: step t = (k block, j) needs four A fragments
  // (row block 0/1 x hi/lo); they are read from LDS two steps ahead into a 2-slot register ring,
  // so the LDS latency hides behind the previous step's four MFMAs.  After the last step of a k
  // block, that block of the W set is refilled from chunk `c_next` (if LOADW).
  bf16x8 xf[2][2 * MB];
  auto read_frags = [&](int slot, int t, int buf) {
    const unsigned char *xp = lds + buf * BUF + (size_t)(t * MB * 2) * 1024 + lane * 16;   // t = kb*4 + j
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
      // high parts of every row block, then the low parts: a matrix instruction that adds to the
      // result of the one just before it would have to wait for it
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
    // n_chunks is a multiple of DEPTH (DEPTH even).  The prologue issues its loads in the order
    // the steady state does (X of a chunk before the W refill of the same step), so the wait
    // counts merged at the loop head are the steady-state ones.
    load_x(0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) load_w_block(0, 0, kb);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0);
    load_x(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 1; d < DEPTH; ++d)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) load_w_block(d, d, kb);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    int c0 = 0;
    for (; c0 + DEPTH < n_chunks; c0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        store_x((d + 1) & 1);                       // chunk c0+d+1
        load_x(min(c0 + d + 2, n_chunks - 1));      // clamped, never a branch
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(d, d & 1, c0 + d + DEPTH, true);
        __syncthreads();
      }
    }
    // last DEPTH chunks: nothing left to fetch from W
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (d + 1 < DEPTH) store_x((d + 1) & 1);
      if (d + 2 < DEPTH) load_x(c0 + d + 2);
      __builtin_amdgcn_sched_barrier(0);
      compute_chunk(d, d & 1, 0, false);
      if (d + 1 < DEPTH) __syncthreads();
    }
  }

  rstd_finish<256, MB>(a, rs_in, s_rsp, s_rs);
  __syncthreads();   // every wavefront is done reading the last X stage
  gemm_epilogue<MB, EPI, 4>(a, reinterpret_cast<f32x16(&)[1][MB]>(acc), lds, &s_last, s_rs, tile, split);
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
  // (the 4-deep W ring does not fit the register file next to the accumulators of 256 rows)
#define TS_LAUNCH(MB_, KC_)                                                                   \
  do {                                                                                        \
    bool deep = false;                                                                        \
    if constexpr (MB_ < 8) {                                                                  \
      deep = a.k_per_split % (4 * KC_) == 0 && a.k % (4 * KC_) == 0;                          \
      if (deep) hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, EPI, false, 4>), grid, block, 0, st, a); \
    }                                                                                         \
    if (deep) break;                                                                          \
    if (a.k_per_split % (2 * KC_) == 0 && a.k % (2 * KC_) == 0)                               \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, EPI, false, 2>), grid, block, 0, st, a);      \
    else                                                                                      \
      hipLaunchKernelGGL((k_gemm_bf16<MB_, KC_, EPI, true, 1>), grid, block, 0, st, a);       \
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
    case EPI_PLAIN: dispatch<EPI_PLAIN>(st, a); break;
    default: dispatch<EPI_HEAD>(st, a); break;
  }
}

}  // namespace ts
