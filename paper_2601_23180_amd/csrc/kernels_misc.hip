// Small kernels of the verification pass: set-up, rotary table, embedding (+ first RMSNorm
// statistic), vocabulary statistics reduction and the routing decision; plus the plain fp32
// pipeline (matmul, rotary + KV append, residual + RMSNorm, SiLU*up as separate simple kernels)
// that serves fp32 models, where reference precision matters and speed does not.
#include "device_util.hpp"

namespace ts {

// ------------------------------------------------------------------ set-up
// Also clears `zero[0 .. n_zero)`: the tile counters of the split-K matmuls and the barrier
// counters / abort word of the layer kernels, which must be zero when the pass starts.
__global__ void k_setup(NodeTable tab, int rows, int n_nodes, AncMask *anc, int32_t *parent, int32_t *status,
                        int32_t *zero, int n_zero) {
  const int i = threadIdx.x;
  if (i < rows) {
    // root path of node i: walk up the parents (validated on the host: parent < node, root = -1)
    const int base = (i / n_nodes) * n_nodes;
    AncMask m;
    m.lo = m.hi = 0ull;
    for (int j = i - base, guard = 0; j >= 0 && guard < kMaxNodes; ++guard) {
      m.set(j);
      j = tab.parent[base + j];
    }
    anc[i] = m;
    parent[i] = tab.parent[i];
  }
  if (i == 0 && status != nullptr) *status = 0;
  for (int j = i; j < n_zero; j += kMaxRows) zero[j] = 0;
}

void launch_setup(hipStream_t st, const NodeTable &tab, int rows, int n_nodes, AncMask *anc, int32_t *parent,
                  int32_t *status, int32_t *zero, int n_zero) {
  hipLaunchKernelGGL(k_setup, dim3(1), dim3(kMaxRows), 0, st, tab, rows, n_nodes, anc, parent, status, zero, n_zero);
}

__global__ void k_wait_probe(int32_t *counter, int expect, unsigned long long limit, int32_t *abort_word,
                             int32_t *status) {
  bar_wait(counter, expect, limit, abort_word, status);
}

void launch_wait_probe(hipStream_t st, int32_t *counter, int expect, unsigned long long limit,
                       int32_t *abort_word, int32_t *status) {
  hipLaunchKernelGGL(k_wait_probe, dim3(1), dim3(64), 0, st, counter, expect, limit, abort_word, status);
}

// angle[r][j] = position_r * base^(-2j/d), evaluated in fp64 so that large positions keep
// their phase; the table holds fp32 cos / sin.
__global__ void k_rope_table(const int32_t *positions, int head_dim, float base, float *cos_t,
                             float *sin_t) {
  const int r = blockIdx.x, j = threadIdx.x;
  const int half = head_dim >> 1;
  if (j >= half) return;
  const double inv = pow((double)base, -2.0 * (double)j / (double)head_dim);
  const double ang = (double)positions[r] * inv;
  cos_t[r * half + j] = (float)cos(ang);
  sin_t[r * half + j] = (float)sin(ang);
}

void launch_rope_table(hipStream_t st, const int32_t *positions, int rows, int head_dim, float base,
                       float *cos_t, float *sin_t) {
  hipLaunchKernelGGL(k_rope_table, dim3(rows), dim3(head_dim / 2), 0, st, positions, head_dim, base,
                     cos_t, sin_t);
}

// ------------------------------------------------------------------ embedding + first RMSNorm
// x[r] = E[token_r] (fp32 residual stream).  fp32 models: h[r] = x * rstd * w.  bf16 models: the
// first matmul's operand panels h = x * w as bf16 hi + lo, and the row's sum of squares (that
// matmul's epilogue turns it into 1/rms).
template <typename AT>
__global__ __launch_bounds__(256) void k_embed_norm(const int32_t *tokens, const AT *embed,
                                                    const AT *norm_w, int hidden, int vocab, float eps,
                                                    float *x, void *h, size_t h_panel, float *ss_out,
                                                    int32_t *status) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  int tok = tokens[r];
  if (tok < 0 || tok >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, 1);
    tok = 0;
  }
  const AT *e = embed + (size_t)tok * hidden;
  float *xr = x + (size_t)r * hidden;
  if constexpr (sizeof(AT) == 2) {
    // bf16 models (hidden is a multiple of 64): 8 elements = one 16-byte vector per step; a run of
    // 8 reduction indices is contiguous in the operand layout as well
    constexpr int MAXV = 4;                         // vectors per thread held in registers (hidden <= 8192)
    const int nv = hidden / 8;
    bf16x8 ev[MAXV], wv[MAXV];
#pragma unroll
    for (int u = 0; u < MAXV; ++u) {
      const int v = min((int)threadIdx.x + 256 * u, nv - 1);
      ev[u] = *(const bf16x8 *)(e + 8 * v);
      wv[u] = *(const bf16x8 *)(norm_w + 8 * v);
    }
    float ss = 0.f;
    for (int v0 = 0; v0 < nv; v0 += 256 * MAXV) {
#pragma unroll
      for (int u = 0; u < MAXV; ++u) {
        const int v = v0 + (int)threadIdx.x + 256 * u;
        if (v >= nv) continue;
        bf16x8 evv = ev[u], wvv = wv[u];
        if (v0 > 0) { evv = *(const bf16x8 *)(e + 8 * v); wvv = *(const bf16x8 *)(norm_w + 8 * v); }   // very wide models
        f32x4 x0, x1;
        bf16x8 hi, lo;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float xv = (float)evv[k];
          (k < 4 ? x0 : x1)[k & 3] = xv;
          ss += xv * xv;
          const float hv = xv * (float)wvv[k];
          hi[k] = (bf16)hv;
          lo[k] = (bf16)(hv - (float)hi[k]);
        }
        *(f32x4 *)(xr + 8 * v) = x0;
        *(f32x4 *)(xr + 8 * v + 4) = x1;
        bf16 *hp = (bf16 *)h;   // operand layout; h_panel carries the number of 32-row blocks
        *(bf16x8 *)(hp + ol_offset(r, 8 * v, 0, (int)h_panel)) = hi;
        *(bf16x8 *)(hp + ol_offset(r, 8 * v, 1, (int)h_panel)) = lo;
      }
    }
    ss = block_sum<4>(ss, red);
    if (threadIdx.x == 0) ss_out[r] = ss;
    (void)eps;
  } else {
    float ss = 0.f;
    for (int i = threadIdx.x; i < hidden; i += 256) {
      const float v = to_f32(e[i]);
      xr[i] = v;
      ss += v * v;
    }
    ss = block_sum<4>(ss, red);
    const float rstd = 1.0f / sqrtf(ss / (float)hidden + eps);
    float *hp = (float *)h + (size_t)r * hidden;
    for (int i = threadIdx.x; i < hidden; i += 256) hp[i] = to_f32(e[i]) * rstd * to_f32(norm_w[i]);
    (void)h_panel; (void)ss_out;
  }
}

void launch_embed_norm(hipStream_t st, int dtype, const int32_t *tokens, const void *embed,
                       const void *norm_w, int rows, int hidden, int vocab, float eps, float *x,
                       void *h, size_t h_panel, float *ss_out, int32_t *status) {
  if (dtype == TRISPEC_F32)
    hipLaunchKernelGGL(k_embed_norm<float>, dim3(rows), dim3(256), 0, st, tokens, (const float *)embed,
                       (const float *)norm_w, hidden, vocab, eps, x, h, h_panel, (float *)nullptr, status);
  else
    hipLaunchKernelGGL(k_embed_norm<bf16>, dim3(rows), dim3(256), 0, st, tokens, (const bf16 *)embed,
                       (const bf16 *)norm_w, hidden, vocab, eps, x, h, h_panel, ss_out, status);
}

__global__ void k_zero_counters(int32_t *counters, int n_counters) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_counters) counters[i] = 0;
}

void launch_zero_counters(hipStream_t st, int32_t *counters, int n_counters) {
  hipLaunchKernelGGL(k_zero_counters, dim3((n_counters + 255) / 256), dim3(256), 0, st, counters, n_counters);
}

// Sum of the split-K partials of one output element, ascending split order.
__device__ __forceinline__ float sum_splits(const float *part, int n_splits, size_t slice, size_t off) {
  float v = part[off];
  for (int s = 1; s < n_splits; ++s) v += part[(size_t)s * slice + off];
  return v;
}

// ------------------------------------------------------------------ fp32 pipeline: QKV epilogue
// One workgroup per (row, head): rotary embedding of q and k heads (pair (j, j + d/2)), q to the
// attention operand buffer, k and v to cache slot ctx_len + node (v transposed).
__global__ void k_qkv_epilogue_f32(const float *part, int n_splits, int rows_pad, int n_q_heads,
                                   int n_kv_heads, int head_dim, const float *cos_t, const float *sin_t,
                                   int n_nodes, CtxLens ctx, KvMap kvm, float *q_out, float *k_cache,
                                   float *v_cache, const float *q_norm_w, const float *k_norm_w, float eps) {
  __shared__ float s_sq[64];
  const int r = blockIdx.x, hh = blockIdx.y, j = threadIdx.x;   // head_dim / 2 threads
  const int half = head_dim >> 1;
  const int n_total = (n_q_heads + 2 * n_kv_heads) * head_dim;
  const size_t slice = (size_t)rows_pad * n_total;
  const size_t off = (size_t)r * n_total + (size_t)hh * head_dim + j;
  float a = sum_splits(part, n_splits, slice, off);
  float b = sum_splits(part, n_splits, slice, off + half);
  if (q_norm_w != nullptr && hh < n_q_heads + n_kv_heads) {   // RMSNorm over the head (uniform branch)
    s_sq[j] = a * a + b * b;
    __syncthreads();
    float ss = 0.f;
    for (int i = 0; i < half; ++i) ss += s_sq[i];           // ascending: the same order in every thread
    const float rn = 1.0f / sqrtf(ss / (float)head_dim + eps);
    const float *nw = hh < n_q_heads ? q_norm_w : k_norm_w;
    a *= rn * nw[j];
    b *= rn * nw[j + half];
  }
  const int bidx = r / n_nodes, node = r - bidx * n_nodes;
  const int slot = ctx.v[bidx] + node;
  if (hh < n_q_heads + n_kv_heads) {
    const float c = cos_t[r * half + j], s = sin_t[r * half + j];
    const float ra = a * c - b * s;
    const float rb = b * c + a * s;
    a = ra; b = rb;
  }
  if (hh < n_q_heads) {
    float *q = q_out + (size_t)r * n_q_heads * head_dim + (size_t)hh * head_dim;
    q[j] = a;
    q[j + half] = b;
  } else if (hh < n_q_heads + n_kv_heads) {
    const int kvh = hh - n_q_heads;
    float *k = k_cache + kvm.k_row(bidx, kvh, slot);
    k[j] = a;
    k[j + half] = b;
  } else {
    const int kvh = hh - n_q_heads - n_kv_heads;
    float *v = v_cache + kvm.v_col(bidx, kvh, slot);
    v[(size_t)j * kvm.v_stride()] = a;
    v[(size_t)(j + half) * kvm.v_stride()] = b;
  }
}

void launch_qkv_epilogue(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                         int rows_pad, int n_q_heads, int n_kv_heads, int head_dim,
                         const float *cos_t, const float *sin_t, int n_nodes, CtxLens ctx,
                         const KvMap &kvm, void *q_out, void *k_cache, void *v_cache, const float *q_norm_w,
                         const float *k_norm_w, float eps) {
  (void)dtype;
  dim3 grid(rows, n_q_heads + 2 * n_kv_heads), block(head_dim / 2);
  hipLaunchKernelGGL(k_qkv_epilogue_f32, grid, block, 0, st, part, n_splits, rows_pad, n_q_heads,
                     n_kv_heads, head_dim, cos_t, sin_t, n_nodes, ctx, kvm, (float *)q_out,
                     (float *)k_cache, (float *)v_cache, q_norm_w, k_norm_w, eps);
}

// ------------------------------------------------------------------ fp32 pipeline: residual + RMSNorm
// x[r] += y[r]; h[r] = x[r] * rstd * w.  One workgroup per row.
__global__ __launch_bounds__(256) void k_reduce_residual_norm_f32(const float *part, int n_splits,
                                                                  int rows_pad, int hidden,
                                                                  const float *norm_w, float eps, float *x,
                                                                  float *h) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const size_t slice = (size_t)rows_pad * hidden;
  float *xr = x + (size_t)r * hidden;
  float ss = 0.f;
  for (int i = threadIdx.x; i < hidden; i += 256) {
    const float v = xr[i] + sum_splits(part, n_splits, slice, (size_t)r * hidden + i);
    xr[i] = v;
    ss += v * v;
  }
  ss = block_sum<4>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)hidden + eps);
  for (int i = threadIdx.x; i < hidden; i += 256) h[(size_t)r * hidden + i] = xr[i] * rstd * norm_w[i];
}

void launch_reduce_residual_norm(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                                 int rows_pad, int hidden, const void *norm_w, float eps, float *x,
                                 void *h) {
  (void)dtype;
  hipLaunchKernelGGL(k_reduce_residual_norm_f32, dim3(rows), dim3(256), 0, st, part, n_splits, rows_pad,
                     hidden, (const float *)norm_w, eps, x, (float *)h);
}

// ------------------------------------------------------------------ fp32 pipeline: SiLU(gate) * up
// columns [0, F) of y are the gate projection, [F, 2F) the up projection.
__global__ __launch_bounds__(256) void k_reduce_swiglu_f32(const float *part, int n_splits, int rows_pad,
                                                           int ffn, float *act) {
  const int r = blockIdx.y;
  const int f = blockIdx.x * 256 + threadIdx.x;
  if (f >= ffn) return;
  const size_t slice = (size_t)rows_pad * 2 * ffn;
  const size_t off = (size_t)r * 2 * ffn + f;
  const float g = sum_splits(part, n_splits, slice, off);
  const float u = sum_splits(part, n_splits, slice, off + ffn);
  const float silu = g / (1.0f + expf(-g));
  act[(size_t)r * ffn + f] = silu * u;
}

void launch_reduce_swiglu(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                          int rows_pad, int ffn, void *act) {
  (void)dtype;
  dim3 grid((ffn + 255) / 256, rows);
  hipLaunchKernelGGL(k_reduce_swiglu_f32, grid, dim3(256), 0, st, part, n_splits, rows_pad, ffn, (float *)act);
}

// ------------------------------------------------------------------ fp32 reference-precision matmul
// One wavefront per (output column, group of 8 rows); lanes stride the reduction.
__global__ __launch_bounds__(64) void k_gemm_f32(GemmArgs a) {
  const int col = blockIdx.x;
  const int r0 = blockIdx.y * 8;
  int s = 0;
  while (s + 1 < a.n_seg && col >= a.seg[s + 1].col0) ++s;
  const float *w = (const float *)a.seg[s].w + (size_t)(col - a.seg[s].col0) * a.k;
  const float *x = (const float *)a.x;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int k = threadIdx.x; k < a.k; k += 64) {
    const float wv = w[k];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (r0 + j < a.rows) acc[j] += x[(size_t)(r0 + j) * a.k + k] * wv;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float v = wave_sum(acc[j]);
    if (threadIdx.x == 0 && r0 + j < a.rows)
      a.out[(size_t)(r0 + j) * a.n_total + col] = v + (a.bias != nullptr ? a.bias[col] : 0.f);
  }
}

void launch_gemm_f32(hipStream_t st, const GemmArgs &a) {
  hipLaunchKernelGGL(k_gemm_f32, dim3(a.n_total, (a.rows + 7) / 8), dim3(64), 0, st, a);
}

// ------------------------------------------------------------------ vocabulary statistics
// fp32 models: scan a row of materialised logits.  One workgroup per row, 256 threads, each
// scanning a contiguous slab in ascending order.
__global__ __launch_bounds__(256) void k_stats_from_logits(const float *logits, int vocab, HeadStats hs) {
  __shared__ Top2 sm[4];
  const int r = blockIdx.x;
  const float *row = logits + (size_t)r * vocab;
  const int per = (vocab + 255) / 256;
  const int lo = threadIdx.x * per, hi = min(vocab, lo + per);
  Top2 t = top2_empty();
  for (int c = lo; c < hi; ++c) top2_push(t, row[c], c);
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) t = top2_merge(t, top2_shfl_xor(t, o));
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    Top2 a = sm[0];
    for (int w = 1; w < 4; ++w) a = top2_merge(a, sm[w]);
    hs.l1[r] = a.l1; hs.l2[r] = a.l2; hs.sumexp[r] = a.s; hs.ent[r] = a.t; hs.idx[r] = a.idx;
  }
}

void launch_stats_from_logits(hipStream_t st, const float *logits, int rows, int vocab,
                              const HeadStats &hs) {
  hipLaunchKernelGGL(k_stats_from_logits, dim3(rows), dim3(256), 0, st, logits, vocab, hs);
}

// Merge the per-tile statistics of every row: one workgroup of 16 wavefronts per row, threads
// stride the tiles (every load of a thread is requested before the first merge), then a fixed
// butterfly per wavefront and the wavefronts in ascending order.
constexpr int kStatsThreads = 1024;
__global__ __launch_bounds__(kStatsThreads) void k_stats_reduce(HeadStats hs, float *node_l1, float *node_l2,
                                                                float *node_sum, float *node_ent, int32_t *node_idx) {
  __shared__ Top2 s_w[kStatsThreads / 64];
  const int r = blockIdx.x, tid = threadIdx.x;
  Top2 t = top2_empty();
  for (int i0 = tid; i0 < hs.n_tiles; i0 += 4 * kStatsThreads) {
    Top2 b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kStatsThreads;
      const size_t o = (size_t)r * hs.n_tiles + min(i, hs.n_tiles - 1);
      b[u].l1 = hs.l1[o]; b[u].l2 = hs.l2[o]; b[u].s = hs.sumexp[o]; b[u].t = hs.ent[o]; b[u].idx = hs.idx[o];
      if (i >= hs.n_tiles) b[u] = top2_empty();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) t = top2_merge(t, b[u]);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) t = top2_merge(t, top2_shfl_xor(t, o));
  if ((tid & 63) == 0) s_w[tid >> 6] = t;
  __syncthreads();
  if (tid == 0) {
    t = s_w[0];
    for (int w = 1; w < kStatsThreads / 64; ++w) t = top2_merge(t, s_w[w]);
    node_l1[r] = t.l1; node_l2[r] = t.l2; node_sum[r] = t.s; node_ent[r] = t.t; node_idx[r] = t.idx;
  }
}

void launch_stats_reduce(hipStream_t st, const HeadStats &hs, int rows, float *node_l1, float *node_l2,
                         float *node_sum, float *node_ent, int32_t *node_idx) {
  hipLaunchKernelGGL(k_stats_reduce, dim3(rows), dim3(kStatsThreads), 0, st, hs, node_l1, node_l2, node_sum,
                     node_ent, node_idx);
}

// One workgroup per node: count the vocabulary entries that precede the node's token in its
// parent's row of logits (exact integer sum: any order gives the same count).
__global__ __launch_bounds__(256) void k_draft_ranks(const float *logits, const int32_t *tokens, NodeTable tab,
                                                     int n_nodes, int vocab, int32_t *ranks) {
  __shared__ int red[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  const int b = r / n_nodes, par = tab.parent[r], x = tokens[r];
  if (par < 0 || x < 0 || x >= vocab) {   // uniform over the workgroup
    if (tid == 0) ranks[r] = -1;
    return;
  }
  const float *row = logits + (size_t)(b * n_nodes + par) * vocab;
  const float lx = row[x];
  int n = 0;
  for (int c = tid; c < vocab; c += 256) {
    const float v = row[c];
    n += (v > lx) || (v == lx && c < x);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
  if ((tid & 63) == 0) red[tid >> 6] = n;
  __syncthreads();
  if (tid == 0) ranks[r] = red[0] + red[1] + red[2] + red[3];
}

void launch_draft_ranks(hipStream_t st, const float *logits, const int32_t *tokens, const NodeTable &tab,
                        int batch, int n_nodes, int vocab, int32_t *ranks) {
  hipLaunchKernelGGL(k_draft_ranks, dim3(batch * n_nodes), dim3(256), 0, st, logits, tokens, tab, n_nodes, vocab, ranks);
}

// ------------------------------------------------------------------ decision
// One workgroup per sequence.  Threads fill the per-node outputs; thread 0 then walks the tree:
// at the current node test the trust predicate first (tau_a = tau_m is an escalation), then
// follow the lowest-numbered child whose draft token equals the verifier's argmax.
__global__ __launch_bounds__(kMaxNodes) void k_decide(DecideArgs a) {
  __shared__ float s_conf[kMaxNodes], s_margin[kMaxNodes], s_ent[kMaxNodes];
  __shared__ int s_arg[kMaxNodes], s_tok[kMaxNodes], s_par[kMaxNodes], s_rank[kMaxNodes];
  const int b = blockIdx.x, i = threadIdx.x, M = a.n_nodes;
  if (i < M) {
    const int r = b * M + i;
    const float s = a.node_sum[r];
    const float conf = 1.0f / s;                                   // exp(l1 - l1) / sum
    const float p2 = expf(a.node_l2[r] - a.node_l1[r]) / s;        // 0 when there is no second entry
    s_conf[i] = conf;
    s_margin[i] = conf - p2;
    s_ent[i] = logf(s) - a.node_ent[r] / s;                        // ln sum e^d - sum e^d d / sum e^d
    s_rank[i] = a.draft_ranks != nullptr ? a.draft_ranks[r] : -1;
    s_arg[i] = a.node_idx[r];
    s_tok[i] = a.tokens[r];
    s_par[i] = a.parent[r];
    if (a.out.argmax) a.out.argmax[r] = s_arg[i];
    if (a.out.confidence) a.out.confidence[r] = conf;
    if (a.out.margin) a.out.margin[r] = s_margin[i];
    if (a.out.entropy) a.out.entropy[r] = s_ent[i];
  }
  if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE + i] = -1;
  __syncthreads();
  if (i != 0) return;
  int cur = a.n_forced - 1, acc = 0, token = -1, esc = 0;
  if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE] = cur;
  const bool relaxed = a.accept_top_k > 1 && a.draft_ranks != nullptr;
  for (int step = 0; step <= M; ++step) {
    // trusted: statistic on the right side of the threshold (a NaN statistic is never trusted)
    const bool trusted = a.criterion == TRISPEC_CRIT_ENTROPY
                             ? (s_ent[cur] <= a.threshold)
                             : ((a.criterion == TRISPEC_CRIT_MARGIN ? s_margin[cur] : s_conf[cur]) >= a.threshold);
    if (!trusted) { esc = 1; token = -1; break; }
    const int t = s_arg[cur];
    int nxt = -1;
    for (int c = cur + 1; c < M; ++c)
      if (s_par[c] == cur && (relaxed ? (s_rank[c] >= 0 && s_rank[c] < a.accept_top_k) : s_tok[c] == t)) { nxt = c; break; }
    if (nxt < 0) { token = t; break; }
    cur = nxt;
    ++acc;
    if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE + acc] = cur;
  }
  if (b == 0 && a.out.status) *a.out.status = *a.status_src;
  if (a.out.accepted_len) a.out.accepted_len[b] = acc;
  if (a.out.token) a.out.token[b] = token;
  if (a.out.escalate) a.out.escalate[b] = esc;
}

void launch_decide(hipStream_t st, const DecideArgs &a) {
  hipLaunchKernelGGL(k_decide, dim3(a.batch), dim3(kMaxNodes), 0, st, a);
}

// Plain streaming copy: grid-stride over blocks of 4 x 256 16-byte vectors, four independent
// loads in flight per thread before the stores.
__global__ __launch_bounds__(256) void k_copy_probe(uint4 *dst_, const uint4 *src_, size_t n) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  u32x4 *dst = (u32x4 *)dst_;
  const u32x4 *src = (const u32x4 *)src_;
  const size_t stride = (size_t)gridDim.x * 1024;
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  for (; i + 768 < n; i += stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256);
    const u32x4 c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + 256);
    __builtin_nontemporal_store(c, dst + i + 512);
    __builtin_nontemporal_store(d, dst + i + 768);
  }
  for (; i < n; i += 256) dst[i] = src[i];   // ragged end of the last block
}

void launch_copy_probe(hipStream_t st, void *dst, const void *src, size_t bytes) {
  const size_t n = bytes / 16;
  size_t blocks = (n + 1023) / 1024;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_copy_probe, dim3((unsigned)blocks), dim3(256), 0, st, (uint4 *)dst, (const uint4 *)src, n);
}

// Feature export: the final-norm output of every row in fp32.  One workgroup per row.
template <typename T>
__global__ __launch_bounds__(256) void k_export_hidden(const float *x, const T *w, const float *ss, int ss_tiles,
                                                        int rows_pad, int hidden, float eps, float *out) {
  const int r = blockIdx.x;
  float rstd = 1.f;
  if (ss != nullptr) {
    float s = 0.f;
    for (int t = 0; t < ss_tiles; ++t) s += ss[(size_t)t * rows_pad + r];   // ascending tile order
    rstd = 1.0f / sqrtf(s / (float)hidden + eps);
  }
  for (int c = threadIdx.x; c < hidden; c += 256) {
    const float v = x[(size_t)r * hidden + c];
    out[(size_t)r * hidden + c] = (ss != nullptr) ? v * rstd * to_f32(w[c]) : v;
  }
}

void launch_export_hidden(hipStream_t st, int dtype, const float *x, const void *norm_w, const float *ss,
                          int ss_tiles, int rows, int rows_pad, int hidden, float eps, float *out) {
  if (dtype == TRISPEC_F32)
    hipLaunchKernelGGL(k_export_hidden<float>, dim3(rows), dim3(256), 0, st, x, (const float *)norm_w, ss,
                       ss_tiles, rows_pad, hidden, eps, out);
  else
    hipLaunchKernelGGL(k_export_hidden<bf16>, dim3(rows), dim3(256), 0, st, x, (const bf16 *)norm_w, ss,
                       ss_tiles, rows_pad, hidden, eps, out);
}

// Commit of a verified path: per (kv head, sequence, layer) the K rows and the V^T columns of the
// path's nodes move from slot ctx + node[i] to slot ctx + i.  node[i] >= i, so a destination may
// be another row's source: everything is read into registers, then a barrier, then written.
template <typename T>
__global__ __launch_bounds__(256) void k_kv_commit(T *k_cache, T *v_cache, size_t layer_elems, KvMap kvm,
                                                    CommitTable t) {
  const int h = blockIdx.x, b = blockIdx.y, l = blockIdx.z, tid = threadIdx.x;
  const int n = t.n[b], ctx = t.ctx[b], d = kvm.d;
  if (n == 0) return;   // uniform over the workgroup
  T *kc = k_cache + (size_t)l * layer_elems;   // this layer; rows and columns through the slot map
  T *vc = v_cache + (size_t)l * layer_elems;
  const size_t vs = kvm.v_stride();
  constexpr int VEC = 16 / sizeof(T);                       // elements per 16-byte vector
  constexpr int MAXV = kMaxNodes * 128 / VEC / 256;         // vectors per thread at d = 128
  constexpr int MAXE = kMaxNodes * 128 / 256;               // V^T elements per thread at d = 128
  const int vec_per_row = d / VEC;
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
  u32x4 kv[MAXV];
  T ve[MAXE];
#pragma unroll
  for (int u = 0; u < MAXV; ++u) {
    const int idx = tid + 256 * u, i = idx / vec_per_row, c = idx - i * vec_per_row;
    if (i < n) kv[u] = *(const u32x4 *)(kc + kvm.k_row(b, h, ctx + t.node[b][i]) + c * VEC);
  }
#pragma unroll
  for (int u = 0; u < MAXE; ++u) {
    const int idx = tid + 256 * u, f = idx / kMaxNodes, i = idx - f * kMaxNodes;   // 64 consecutive threads: one feature
    if (f < d && i < n) ve[u] = vc[kvm.v_col(b, h, ctx + t.node[b][i]) + (size_t)f * vs];
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < MAXV; ++u) {
    const int idx = tid + 256 * u, i = idx / vec_per_row, c = idx - i * vec_per_row;
    if (i < n) *(u32x4 *)(kc + kvm.k_row(b, h, ctx + i) + c * VEC) = kv[u];
  }
#pragma unroll
  for (int u = 0; u < MAXE; ++u) {
    const int idx = tid + 256 * u, f = idx / kMaxNodes, i = idx - f * kMaxNodes;
    if (f < d && i < n) vc[kvm.v_col(b, h, ctx + i) + (size_t)f * vs] = ve[u];
  }
}

void launch_kv_commit(hipStream_t st, int dtype, void *k_cache, void *v_cache, int n_layers, size_t layer_elems,
                      int batch, const KvMap &kvm, const CommitTable &t) {
  dim3 grid(kvm.n_kv, batch, n_layers);
  if (dtype == TRISPEC_F32)
    hipLaunchKernelGGL(k_kv_commit<float>, grid, dim3(256), 0, st, (float *)k_cache, (float *)v_cache, layer_elems,
                       kvm, t);
  else
    hipLaunchKernelGGL(k_kv_commit<bf16>, grid, dim3(256), 0, st, (bf16 *)k_cache, (bf16 *)v_cache, layer_elems,
                       kvm, t);
}

}  // namespace ts
