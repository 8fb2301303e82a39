// Epilogue of the weight-streaming matmul kernel (see kernels_gemm.hip), written for any number
// of wavefronts per workgroup and of 32-column sub-tiles per wavefront.
#pragma once

#include "device_util.hpp"

namespace ts {

// 1/rms of every row of a matmul's INPUT, from the per-tile sums of squares its producer left.
// rstd_load only ISSUES loads (wavefront q of the workgroup takes tiles q, q+Q, ...; a lane takes
// rows lane, lane+64, ...) and is called before the weight stream starts, so that nothing waits
// for them; rstd_finish, called after the stream, adds them up (plus any tiles beyond the first
// 8*Q, which only very wide models have) and combines the wavefronts' sums through LDS.  The
// order of the additions is fixed, so the result does not depend on scheduling.
template <int NT, int MB>
__device__ __forceinline__ void rstd_load(const GemmArgs &a, float (&x)[(MB + 1) / 2][8]) {
  constexpr int Q = NT / 64, RI = (MB + 1) / 2;
  const int q = threadIdx.x >> 6, r0 = threadIdx.x & 63;
  if (a.ss_in == nullptr) return;
#pragma unroll
  for (int i = 0; i < RI; ++i) {
    const int r = min(r0 + 64 * i, a.rows_pad - 1);
#pragma unroll
    for (int u = 0; u < 8; ++u) x[i][u] = a.ss_in[(size_t)min(q + Q * u, a.ss_tiles - 1) * a.rows_pad + r];
  }
}

// s_rsp: NT/64 * kMaxRows floats of LDS.  The caller synchronises the workgroup before s_rs is read.
template <int NT, int MB>
__device__ __forceinline__ void rstd_finish(const GemmArgs &a, const float (&x)[(MB + 1) / 2][8], float *s_rsp,
                                            float *s_rs) {
  constexpr int Q = NT / 64, RI = (MB + 1) / 2;
  const int q = threadIdx.x >> 6, r0 = threadIdx.x & 63;
  if (a.ss_in != nullptr) {
#pragma unroll
    for (int i = 0; i < RI; ++i) {
      float v = 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) v += (q + Q * u < a.ss_tiles) ? x[i][u] : 0.f;
      const int r = min(r0 + 64 * i, a.rows_pad - 1);
      for (int t = q + Q * 8; t < a.ss_tiles; t += Q) v += a.ss_in[(size_t)t * a.rows_pad + r];
      s_rsp[q * kMaxRows + r0 + 64 * i] = v;
    }
  }
  __syncthreads();
  for (int r = threadIdx.x; r < a.rows; r += NT) {
    float ss = 0.f;
#pragma unroll
    for (int qq = 0; qq < Q; ++qq) ss += s_rsp[qq * kMaxRows + r];
    s_rs[r] = a.ss_in != nullptr ? 1.0f / sqrtf(ss / (float)a.k + a.eps) : 1.0f;
  }
}

template <int N>
struct SplitGroup {
  static constexpr int value = N;
};

// Epilogue of one (tile, split).  A wavefront owns NB adjacent 32-column sub-tiles of the tile:
// acc[nb][mb][e] of lane (ln, g) of wavefront `wave` holds
//   y[mb*32 + 8*(e/4) + 4*g + e%4][(wave*NB + nb)*32 + ln].
// The reduced fp32 tile goes through LDS in groups of MG 32-row blocks (MG = MB when the whole
// tile fits).  lds: at least MG*32*(TN+4)*4 bytes, free for reuse (every wavefront has passed a
// barrier after its last operand read).  s_rs: 1/rms per input row.
// WT: the results that a later PHASE of the same launch reads (residual stream, operand panels,
// sums of squares) are written through to memory; false for a kernel whose consumer is a later launch.
template <int MB, int EPI, int NW, int NB = 1, int MG = MB, bool WT = false>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, f32x16 (&acc)[NB][MB], unsigned char *lds,
                                              int *s_last, const float *s_rs, int tile, int split) {
  constexpr int TN = NW * NB * 32, NT = NW * 64;
  static_assert(MB % MG == 0, "row groups must tile the rows");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, g = lane >> 5;
  if (EPI == EPI_HEAD) {
    // ---- per row, reduce this tile's TN logits to (l1, column, l2, sum exp)
    float *tl = (float *)lds;
    constexpr int PARTS = TN / 16;        // threads scanning one row, 16 columns each
    constexpr int RP = NT / PARTS;        // rows per scan pass
    const int srow = tid / PARTS, part = tid % PARTS;
    // (row_scale is applied when the tile is read back: the scan thread owns one row)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      __syncthreads();
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          tl[(8 * (e >> 2) + 4 * g + (e & 3)) * (TN + 4) + (wave * NB + nb) * 32 + ln] = acc[nb][mb][e];
      __syncthreads();
#pragma unroll
      for (int rp = 0; rp < 32; rp += RP) {
        const int lr = rp + srow, r = mb * 32 + lr;
        const float rsc = (a.ss_in != nullptr && r < a.rows) ? s_rs[r] : 1.0f;
        Top2 t = top2_empty();
        const int cbase = tile * TN + part * 16;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          const float v = tl[lr * (TN + 4) + part * 16 + c] * rsc;
          if (cbase + c < a.n_total) {
            top2_push(t, v, cbase + c);
            if (a.debug_logits != nullptr && r < a.rows) a.debug_logits[(size_t)r * a.n_total + cbase + c] = v;
          }
        }
#pragma unroll
        for (int o = 1; o < PARTS; o <<= 1) t = top2_merge(t, top2_shfl_xor(t, o));
        if (part == 0 && r < a.rows) {
          const size_t o = (size_t)r * a.hs.n_tiles + tile;
          a.hs.l1[o] = t.l1; a.hs.l2[o] = t.l2; a.hs.sumexp[o] = t.s; a.hs.ent[o] = t.t; a.hs.idx[o] = t.idx;
        }
      }
    }
    return;
  }

  // ---- hand the tile to the epilogue, as an fp32 tile in LDS.  One split: straight from the
  // accumulators.  Several splits: write-through partial tiles part[split][tile][row][TN] + a
  // counter per tile; only the last workgroup to arrive goes on.
  constexpr int EPI_LD = TN + 4;       // floats per row of the LDS tile
  float *tl = (float *)lds;
  const bool single = a.n_splits == 1;
  const size_t tile_elems = (size_t)a.rows_pad * TN;
  __syncthreads();   // every wavefront is done reading the last X stage
  if (!single) {
    float *o = a.part + ((size_t)split * a.n_tiles + tile) * tile_elems + wave * NB * 32 + ln;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = mb * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
          if (r < a.rows) st_agent(o + (size_t)r * TN + nb * 32, acc[nb][mb][e]);
        }
    if (!publish_then_count(&a.counters[tile], a.n_splits, s_last)) return;
  }

  // Loads of the epilogue that do not depend on the reduced tile (rotary tables; residual rows and
  // the next norm weight).  Issued together with the loads of the partial tiles: a memory round
  // trip costs more than everything else the epilogue does, so they must not follow each other.
  constexpr int QKV_PASSES = MG * 32 * (TN / 8) / NT;
  constexpr int RES_LPR = TN / 4, RES_RPP = NT / RES_LPR, RES_PASSES = MG * 32 / RES_RPP;
  constexpr int RES_UB = RES_PASSES < 8 ? RES_PASSES : 8;
  f32x4 pre_a[EPI == EPI_QKV ? QKV_PASSES : (EPI == EPI_RESID ? RES_UB : 1)];
  f32x4 pre_b[EPI == EPI_QKV ? QKV_PASSES : 1];
  bf16x4 pre_nw;

#pragma unroll 1
  for (int g0 = 0; g0 < MB; g0 += MG) {
    const int row0 = g0 * 32;          // first row of this group
    if (g0 > 0) __syncthreads();       // the previous group's LDS tile has been consumed
    // -- loads that do not depend on the tile
    if constexpr (EPI == EPI_QKV) {
      const int half = a.head_dim >> 1;
#pragma unroll
      for (int u = 0; u < QKV_PASSES; ++u) {
        const int t = tid + u * NT, r = min(row0 + t / (TN / 8), a.rows - 1), qi = t % (TN / 8);
        const int j = qi * 4 - ((qi * 4) / half) * half;
        pre_a[u] = *(const f32x4 *)(a.cos_t + r * half + j);
        pre_b[u] = *(const f32x4 *)(a.sin_t + r * half + j);
      }
    } else if constexpr (EPI == EPI_RESID) {
      const int col = tile * TN + (tid % RES_LPR) * 4, colc = col < a.n_total ? col : 0;
      pre_nw = *(const bf16x4 *)((const bf16 *)a.next_norm_w + colc);
#pragma unroll
      for (int u = 0; u < RES_UB; ++u)
        pre_a[u] = *(const f32x4 *)(a.x_resid + (size_t)min(row0 + tid / RES_LPR + u * RES_RPP, a.rows - 1) * a.n_total + colc);
    }
    // -- the reduced tile of this row group into LDS
    if (single) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          if (mb >= g0 && mb < g0 + MG) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
              tl[((mb - g0) * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * EPI_LD + (wave * NB + nb) * 32 + ln] = acc[nb][mb][e];
          }
    } else {
      // Last workgroup of the tile: sum the splits, in ascending order.  The partial tiles were
      // written through to memory (st_agent) by workgroups anywhere on the chip and are read here
      // with plain vector loads, which may be served by this XCD's L2.  That is correct because a
      // line of the partial buffer cannot be in this L2 from before it was written: every launch
      // starts with the invalidation of the L2s that makes a kernel see its predecessors' results
      // at all on this multi-XCD chip, and inside one launch a partial line is read only here, by
      // the one workgroup that combines its tile, after the counter says all of it is written (a
      // launch that runs several matmuls gives each its own partial region for the same reason).
      // Agent-scope loads would not need that argument, but they exist only up to 8 bytes and,
      // measured, cost 0.15 ms per pass here.
      // Every load of up to SG splits (UB vectors each) is in flight before the first addition: the
      // reduction then costs one or two memory round trips, not one per pair of splits — it is the
      // longest link of the serial chain that ends a matmul.
      constexpr int PER = MG * 32 * (TN / 4) / NT;   // 4-column vectors per thread
      constexpr int UB = PER < 4 ? PER : 4;
      const float *p0 = a.part + (size_t)tile * tile_elems + (size_t)row0 * TN + (size_t)tid * 4;
      const size_t split_stride = (size_t)a.n_tiles * tile_elems;
      auto reduce_groups = [&](auto sg_c) {
        constexpr int SG = decltype(sg_c)::value;
#pragma unroll 1
        for (int ub = 0; ub < PER; ub += UB) {
          f32x4 sum[UB];
#pragma unroll 1
          for (int s0 = 0; s0 < a.n_splits; s0 += SG) {
            f32x4 v[SG][UB];
#pragma unroll
            for (int q = 0; q < SG; ++q) {
              const float *ps = p0 + (size_t)min(s0 + q, a.n_splits - 1) * split_stride;
#pragma unroll
              for (int u = 0; u < UB; ++u) v[q][u] = *(const f32x4 *)(ps + (size_t)(ub + u) * NT * 4);
            }
#pragma unroll
            for (int q = 0; q < SG; ++q)
#pragma unroll
              for (int u = 0; u < UB; ++u) {
                if (s0 + q == 0) sum[u] = v[q][u];
                else if (s0 + q < a.n_splits) sum[u] += v[q][u];
              }
          }
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int idx = tid + (ub + u) * NT, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            *(f32x4 *)(tl + r * EPI_LD + c) = sum[u];
          }
        }
      };
      // the group size is the number of splits itself where that is small: no load is wasted on a
      // clamped duplicate (a 256-row partial tile is 128 KB per split)
      if constexpr (MG * 32 >= 256) {
        // 256-row tiles: the workgroup is out of registers here (rotary tables or residual rows are
        // held across the reduction), so two splits of 8 vectors at a time
        constexpr int UB8 = PER < 8 ? PER : 8;
#pragma unroll 1
        for (int ub = 0; ub < PER; ub += UB8) {
          f32x4 sum[UB8];
#pragma unroll
          for (int u = 0; u < UB8; ++u) sum[u] = *(const f32x4 *)(p0 + (size_t)(ub + u) * NT * 4);
          for (int s = 1; s < a.n_splits; s += 2) {
            const bool two = s + 1 < a.n_splits;
            const float *pa = p0 + (size_t)s * split_stride, *pb = pa + (two ? split_stride : 0);
            f32x4 va[UB8], vb[UB8];
#pragma unroll
            for (int u = 0; u < UB8; ++u) {
              va[u] = *(const f32x4 *)(pa + (size_t)(ub + u) * NT * 4);
              vb[u] = *(const f32x4 *)(pb + (size_t)(ub + u) * NT * 4);
            }
#pragma unroll
            for (int u = 0; u < UB8; ++u) {
              sum[u] += va[u];
              if (two) sum[u] += vb[u];
            }
          }
#pragma unroll
          for (int u = 0; u < UB8; ++u) {
            const int idx = tid + (ub + u) * NT, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            *(f32x4 *)(tl + r * EPI_LD + c) = sum[u];
          }
        }
      } else
      switch (a.n_splits) {
        case 2: reduce_groups(SplitGroup<2>{}); break;
        case 3: reduce_groups(SplitGroup<3>{}); break;
        case 4: reduce_groups(SplitGroup<4>{}); break;
        case 5: reduce_groups(SplitGroup<5>{}); break;
        case 6: reduce_groups(SplitGroup<6>{}); break;
        case 7: reduce_groups(SplitGroup<7>{}); break;
        default: reduce_groups(SplitGroup<8>{}); break;
      }
    }
    __syncthreads();
    auto reduced4 = [&](int lr, int c) {   // 4 consecutive columns of row (row0 + lr) of the reduced tile
      return *(const f32x4 *)(tl + lr * EPI_LD + c);
    };

    if constexpr (EPI == EPI_QKV) {
      // a tile holds whole heads; thread = (row, 4 rotation pairs)
      const int d = a.head_dim, half = d >> 1;
      const int n_q = a.n_q_heads, n_kv = a.n_kv_heads;
      const bool paged = a.kv.page_table != nullptr;          // uniform: the contiguous cache's addresses stay plain arithmetic
      constexpr int quads = TN / 8;                           // 4-pair groups per row
#pragma unroll
      for (int u = 0; u < QKV_PASSES; ++u) {
        const int t = tid + u * NT;
        const int lr = t / quads, qi = t - lr * quads, r = row0 + lr;
        const int hl = (qi * 4) / half, j = qi * 4 - hl * half;   // head within the tile, first pair
        const int c_lo = hl * d + j;                          // tile-local column of the low elements
        const int col = tile * TN + c_lo;                     // global column
        const bool live = r < a.rows && col < a.n_total;
        const int hh = col / d;                               // global head index (q heads, k heads, v heads)
        const float rsc = live ? s_rs[r] : 0.f;
        f32x4 lo = reduced4(lr, c_lo) * rsc, hi = reduced4(lr, c_lo + half) * rsc;
        if (a.q_norm_w != nullptr) {
          // RMSNorm of a query / key head over its d features: the half / 4 consecutive lanes that hold
          // the head add their sums of squares (every lane takes part: no early exit above)
          float ss = lo[0] * lo[0] + lo[1] * lo[1] + lo[2] * lo[2] + lo[3] * lo[3] + hi[0] * hi[0] + hi[1] * hi[1] +
                     hi[2] * hi[2] + hi[3] * hi[3];
          for (int o = 1; o < half / 4; o <<= 1) ss += __shfl_xor(ss, o, 64);
          if (live && hh < n_q + n_kv) {
            const float rn = 1.0f / sqrtf(ss / (float)d + a.eps);
            const bf16 *nw = (const bf16 *)(hh < n_q ? a.q_norm_w : a.k_norm_w);
            const bf16x4 wl = *(const bf16x4 *)(nw + j), wh = *(const bf16x4 *)(nw + j + half);
#pragma unroll
            for (int e = 0; e < 4; ++e) { lo[e] *= rn * (float)wl[e]; hi[e] *= rn * (float)wh[e]; }
          }
        }
        if (!live) continue;
        const int b = r / a.n_nodes, node = r - b * a.n_nodes;
        const int slot = a.ctx.v[b] + node;
        if (hh < n_q + n_kv) {
          const f32x4 rl = lo * pre_a[u] - hi * pre_b[u], rh = hi * pre_a[u] + lo * pre_b[u];
          lo = rl; hi = rh;
        }
        *(f32x4 *)(a.qkv_f32 + (size_t)r * a.n_total + col) = lo;
        *(f32x4 *)(a.qkv_f32 + (size_t)r * a.n_total + col + half) = hi;
        if (hh < n_q) {
          // matrix-core operand of the context attention: q * log2(e) / sqrt(d) as bf16 hi + lo, so
          // that the scores come out of the MFMA ready for exp2
          const float qs = 1.44269504088896f / sqrtf((float)d);
          bf16x4 lh, ll, hh4, hl4;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float ql_ = lo[e] * qs, qh_ = hi[e] * qs;
            lh[e] = (bf16)ql_; ll[e] = (bf16)(ql_ - (float)lh[e]);
            hh4[e] = (bf16)qh_; hl4[e] = (bf16)(qh_ - (float)hh4[e]);
          }
          bf16 *qo = (bf16 *)a.q_out + (size_t)r * n_q * d + col;
          *(bf16x4 *)qo = lh;
          *(bf16x4 *)(qo + a.q_panel) = ll;
          *(bf16x4 *)(qo + half) = hh4;
          *(bf16x4 *)(qo + half + a.q_panel) = hl4;
        }
        if (hh >= n_q && hh < n_q + n_kv) {
          bf16 *kc = (bf16 *)a.k_cache + (paged ? a.kv.k_row(b, hh - n_q, slot)
                                               : (((size_t)b * n_kv + (hh - n_q)) * a.kv.capacity + slot) * d);
          bf16x4 l4, h4;
#pragma unroll
          for (int e = 0; e < 4; ++e) { l4[e] = (bf16)lo[e]; h4[e] = (bf16)hi[e]; }
          *(bf16x4 *)(kc + j) = l4;
          *(bf16x4 *)(kc + j + half) = h4;
        } else if (hh >= n_q + n_kv) {
          bf16 *vc = (bf16 *)a.v_cache + (paged ? a.kv.v_col(b, hh - n_q - n_kv, slot)
                                               : ((size_t)b * n_kv + (hh - n_q - n_kv)) * d * a.kv.capacity + slot);
          const size_t vs = paged ? (size_t)kKvPage : (size_t)a.kv.capacity;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            vc[(size_t)(j + e) * vs] = (bf16)lo[e];
            vc[(size_t)(j + e + half) * vs] = (bf16)hi[e];
          }
        }
      }
    } else if constexpr (EPI == EPI_SWIGLU) {
      // columns [0, TN/2) of the tile are gate, [TN/2, TN) the matching up columns
      constexpr int FQ = TN / 8;   // float4 groups of features per row (TN/2 gate + TN/2 up columns)
      for (int t = tid; t < MG * 32 * FQ; t += NT) {
        const int lr = t / FQ, f = (t % FQ) * 4, r = row0 + lr;
        const int feat = tile * (TN / 2) + f;
        if (r >= a.rows || feat >= a.ffn) continue;
        const float rsc = s_rs[r];
        const f32x4 gt = reduced4(lr, f) * rsc, up = reduced4(lr, TN / 2 + f) * rsc;
        bf16x4 hi, lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float o = gt[e] / (1.0f + expf(-gt[e])) * up[e];
          hi[e] = (bf16)o;
          lo[e] = (bf16)(o - (float)hi[e]);
        }
        bf16 *dst = (bf16 *)a.act_out;   // operand layout of the down projection (K = ffn)
        store_bf16x4<WT>(dst + ol_offset(r, feat, 0, MB), hi);
        store_bf16x4<WT>(dst + ol_offset(r, feat, 1, MB), lo);
      }
    } else if constexpr (EPI == EPI_PLAIN) {
      // ---- y = (x W^T) / rms + bias, written as it is (the adapter on the exported features)
      constexpr int Q4 = TN / 4;
      for (int t = tid; t < MG * 32 * Q4; t += NT) {
        const int lr = t / Q4, c = (t % Q4) * 4, r = row0 + lr, col = tile * TN + c;
        if (r >= a.rows || col >= a.n_total) continue;
        f32x4 v = reduced4(lr, c) * s_rs[r];
        if (a.bias != nullptr) v += *(const f32x4 *)(a.bias + col);
        *(f32x4 *)(a.out + (size_t)r * a.n_total + col) = v;
      }
    } else {
      // ---- EPI_RESID: x += y; per-row sum of squares of the new x over this tile's columns.
      // TN/4 consecutive lanes (4 columns each) cover one row of the tile.
      constexpr int LPR = RES_LPR, RPP = RES_RPP;   // lanes per row, rows per pass
      constexpr int PASSES = RES_PASSES, UB = RES_UB;
      float *ssp = a.ss_part + (size_t)tile * a.rows_pad;
      const int c = (tid % LPR) * 4, col = tile * TN + c, r0 = tid / LPR;
      const bool col_ok = col < a.n_total;
      const int colc = col_ok ? col : 0;
      const bf16x4 nw = pre_nw;
#pragma unroll 1
      for (int ub = 0; ub < PASSES; ub += UB) {
        // the residual rows of UB passes at once (the first UB were fetched before the reduction)
        f32x4 xv[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) xv[u] = pre_a[u];
        if (ub > 0) {
#pragma unroll
          for (int u = 0; u < UB; ++u)
            xv[u] = *(const f32x4 *)(a.x_resid + (size_t)min(row0 + r0 + (ub + u) * RPP, a.rows - 1) * a.n_total + colc);
        }
        float ss[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int lr = r0 + (ub + u) * RPP, r = row0 + lr;
          ss[u] = 0.f;
          if (r < a.rows && col_ok) {
            const f32x4 v = xv[u] + reduced4(lr, c);
            store_f32x4<WT>(a.x_resid_out + (size_t)r * a.n_total + col, v);
            ss[u] = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
            // operand of the next matmul: x * (next RMSNorm weight), as bf16 hi + lo
            bf16x4 hi, lo;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float o = v[e] * (float)nw[e];
              hi[e] = (bf16)o;
              lo[e] = (bf16)(o - (float)hi[e]);
            }
            bf16 *dst = (bf16 *)a.xw_out;   // operand layout of the next matmul (K = hidden)
            store_bf16x4<WT>(dst + ol_offset(r, col, 0, MB), hi);
            store_bf16x4<WT>(dst + ol_offset(r, col, 1, MB), lo);
          }
        }
        // the UB row sums are reduced side by side, so the exchanges of one hide behind the others'
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1)
#pragma unroll
          for (int u = 0; u < UB; ++u) ss[u] += __shfl_xor(ss[u], o, 64);
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int r = row0 + r0 + (ub + u) * RPP;
          if (tid % LPR == 0 && r < a.rows) store_f32<WT>(ssp + r, ss[u]);   // read by the next matmul
        }
      }
    }
  }
}

}  // namespace ts
