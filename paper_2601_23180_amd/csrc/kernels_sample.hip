// Sampling (temperature > 0) form of the decision on a draft chain (paper Sec. 2.1 acceptance
// min(1, p_v / p_d) and residual resampling; Sec. 3.2 Eq. 6 - Eq. 9 and the routing).
// Four small kernels over logits that are already in memory:
//   k_sample_chunkstats per chain node and 4096-token chunk: max / second max / argmax of the logits
//                      and the chunk's share of the partition sum Z = sum exp((l - max) / T)
//   k_sample_walk      per sequence: merges the chunks of every node, the two probabilities Eq. 6
//                      compares, trust predicate, Bernoulli acceptance, routing; picks the node
//                      whose distribution yields the next token
//   k_sample_chunksum  per sequence and 4096-token chunk: mass of that node's tempered distribution
//                      and of max(0, p_v - p_d)
//   k_sample_pick      per sequence: the chunk, then the token, whose cumulative mass first exceeds
//                      u * total (inverse CDF in ascending token order)
// Loads are coalesced; all sums run in a fixed order, so results do not depend on scheduling.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "internal.hpp"

namespace ts {

namespace {

constexpr int kStatThreads = 1024;
constexpr int kDrawThreads = 1024;
constexpr int kPerThread = 4;                           // consecutive tokens per thread inside a chunk
constexpr int kChunk = kDrawThreads * kPerThread;       // tokens per chunk (== kSampleChunk)
static_assert(kChunk == kSampleChunk, "chunk size is part of the scratch layout");

// max / second max / lowest argmax of one thread's slab, then of the workgroup
struct Max2 {
  float l1, l2;
  int idx;
};
__device__ __forceinline__ Max2 max2_merge(const Max2 &a, const Max2 &b) {
  Max2 r;
  if (b.l1 > a.l1 || (b.l1 == a.l1 && b.idx < a.idx)) {
    r.l1 = b.l1; r.idx = b.idx; r.l2 = fmaxf(a.l1, b.l2);
  } else {
    r.l1 = a.l1; r.idx = a.idx; r.l2 = fmaxf(b.l1, a.l2);
  }
  return r;
}

}  // namespace

// Fixed-order sum of one double per thread over the workgroup (inclusive scan over the lanes of a
// wave, then the waves in ascending order).  Returns this thread's exclusive prefix, *total to all.
template <int NT>
__device__ __forceinline__ double block_scan(double v, double *s_w, double *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double inc = v;
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(inc, o, 64);
    if (lane >= o) inc += up;
  }
  __syncthreads();              // s_w may still be read from an earlier call
  if (lane == 63) s_w[wave] = inc;
  __syncthreads();
  double base = 0.0, tot = 0.0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const double t = s_w[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  return base + inc - v;
}

// grid (chunks, rows): max / second max / lowest argmax of one chunk of a row, and the chunk's
// partition sum relative to ITS maximum, sum exp((l - max_chunk) / T)
__global__ __launch_bounds__(kStatThreads) void k_sample_chunkstats(SampleArgs a) {
  __shared__ Max2 s_m[kStatThreads / 64];
  __shared__ double s_w[kStatThreads / 64];
  const int chunk = blockIdx.x, r = blockIdx.y, tid = threadIdx.x, V = a.vocab;
  // status word of the whole call: cleared by the first kernel, bits are OR-ed in by the later ones
  if (chunk == 0 && r == 0 && tid == 0 && a.out.status) *a.out.status = 0;
  const float *row = a.logits + (size_t)r * V;
  const int c0 = chunk * kChunk + tid * kPerThread;
  float v[kPerThread];
  Max2 m;
  m.l1 = -INFINITY; m.l2 = -INFINITY; m.idx = 0x7fffffff;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {       // ascending: the lowest index of equal maxima stays
    v[e] = (c0 + e < V) ? row[c0 + e] : -INFINITY;
    if (v[e] > m.l1) { m.l2 = m.l1; m.l1 = v[e]; m.idx = c0 + e; }
    else m.l2 = fmaxf(m.l2, v[e]);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    Max2 b;
    b.l1 = __shfl_xor(m.l1, o, 64); b.l2 = __shfl_xor(m.l2, o, 64); b.idx = __shfl_xor(m.idx, o, 64);
    m = max2_merge(m, b);
  }
  if ((tid & 63) == 0) s_m[tid >> 6] = m;
  __syncthreads();
  m = s_m[0];
#pragma unroll
  for (int w = 1; w < kStatThreads / 64; ++w) m = max2_merge(m, s_m[w]);
  double z = 0.0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e)
    if (c0 + e < V) z += (double)expf((v[e] - m.l1) * a.inv_temp);
  double zt;
  (void)block_scan<kStatThreads>(z, s_w, &zt);
  if (tid != 0) return;
  const size_t o = (size_t)r * a.n_chunks + chunk;
  a.cs_l1[o] = m.l1; a.cs_l2[o] = m.l2; a.cs_idx[o] = m.idx; a.cs_z[o] = zt;
}

__global__ __launch_bounds__(64) void k_sample_walk(SampleArgs a) {
  __shared__ float s_conf[kMaxNodes], s_margin[kMaxNodes];
  __shared__ float s_pv[kMaxNodes], s_q[kMaxNodes];
  const int b = blockIdx.x, i = threadIdx.x, M = a.n_nodes, V = a.vocab;
  int bad = 0;
  for (int n = 0; n < M; ++n) {
    // merge node n's chunk statistics: lanes stride the chunks, then a fixed butterfly
    const size_t o = (size_t)(b * M + n) * a.n_chunks;
    Max2 m;
    m.l1 = -INFINITY; m.l2 = -INFINITY; m.idx = 0x7fffffff;
    for (int c = i; c < a.n_chunks; c += 64) {
      Max2 t;
      t.l1 = a.cs_l1[o + c]; t.l2 = a.cs_l2[o + c]; t.idx = a.cs_idx[o + c];
      m = max2_merge(m, t);
    }
#pragma unroll
    for (int w = 1; w < 64; w <<= 1) {
      Max2 t;
      t.l1 = __shfl_xor(m.l1, w, 64); t.l2 = __shfl_xor(m.l2, w, 64); t.idx = __shfl_xor(m.idx, w, 64);
      m = max2_merge(m, t);
    }
    double z = 0.0;
    for (int c = i; c < a.n_chunks; c += 64)
      z += a.cs_z[o + c] * (double)expf((a.cs_l1[o + c] - m.l1) * a.inv_temp);
#pragma unroll
    for (int w = 1; w < 64; w <<= 1) z += __shfl_xor(z, w, 64);
    if (i == n) {   // lane n keeps node n
      const int r = b * M + n;
      a.row_l1[r] = m.l1; a.row_l2[r] = m.l2; a.row_idx[r] = m.idx; a.row_z[r] = z;
      // Eq. 6 operands of the NEXT chain node's token, judged by this node's distribution
      float pv = 0.f, q = 1.f;
      if (n + 1 < M) {
        const int x = a.tokens[r + 1];
        if (x >= 0 && x < V) {
          pv = (float)((double)expf((a.logits[(size_t)r * V + x] - m.l1) * a.inv_temp) / z);
          q = a.p_draft[((size_t)b * (M - 1) + n) * V + x];
        } else {
          pv = -1.f;   // token id outside the vocabulary: never accepted, reported in the status word
          bad = 1;
        }
      }
      s_pv[n] = pv; s_q[n] = q;
    }
  }
  bad = __syncthreads_or(bad);
  if (i == 0) {
    a.seq_bad[b] = bad;
    if (bad && a.out.status) atomicOr(a.out.status, 1);
  }
  if (i < M) {
    const int r = b * M + i;
    const double z = a.row_z[r];
    const float conf = (float)(1.0 / z);
    const float p2 = (float)((double)expf((a.row_l2[r] - a.row_l1[r]) * a.inv_temp) / z);   // 0 for a one-token vocabulary
    s_conf[i] = conf;
    s_margin[i] = conf - p2;
    if (a.out.argmax) a.out.argmax[r] = a.row_idx[r];
    if (a.out.confidence) a.out.confidence[r] = conf;
    if (a.out.margin) a.out.margin[r] = s_margin[i];
  }
  if (a.out.path)
    for (int j = i; j < TRISPEC_PATH_STRIDE; j += 64) a.out.path[b * TRISPEC_PATH_STRIDE + j] = -1;
  __syncthreads();
  if (i != 0) return;
  int cur = a.n_forced - 1, acc = 0, esc = 0, row = -1, mode = 0;   // mode: 0 none, 1 direct, 2 residual
  if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE] = cur;
  for (int step = 0; step <= M; ++step) {
    const float stat = (a.criterion == TRISPEC_CRIT_MARGIN) ? s_margin[cur] : s_conf[cur];
    if (!(stat >= a.threshold)) { esc = 1; break; }
    if (cur + 1 >= M) { row = cur; mode = 1; break; }          // every draft token accepted
    const int r = b * M + cur;
    if (a.u_accept[r + 1] * s_q[cur] < s_pv[cur]) {           // u < min(1, p_v(x) / p_d(x))
      ++cur; ++acc;
      if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE + acc] = cur;
      continue;
    }
    row = cur;
    mode = (a.resample == TRISPEC_RESAMPLE_RESIDUAL) ? 2 : 1;
    break;
  }
  a.sel_row[b] = row;
  a.sel_mode[b] = mode;
  if (a.out.accepted_len) a.out.accepted_len[b] = acc;
  if (a.out.escalate) a.out.escalate[b] = esc;
  if (a.out.token && mode == 0) a.out.token[b] = -1;
}

// The draw.  The vocabulary is cut into chunks of kChunk tokens; inside a chunk thread t owns the
// kPerThread consecutive tokens from kPerThread * t.  chunk_masses() evaluates them and scans the
// workgroup in token order — the same instructions in k_sample_chunksum (every chunk in parallel:
// its total) and in k_sample_pick (the one chunk that holds the target), so the two agree bit
// for bit.  kind 0: tempered p_v; kind 1: max(0, p_v - p_d).
struct DrawRow {
  const float *logits, *q;
  float l1, inv_temp;
  double z;
  int vocab;
};
__device__ __forceinline__ double chunk_masses(const DrawRow &d, int chunk, int kind, float (&mv)[kPerThread],
                                               double *s_w, double *total) {
  const int c0 = chunk * kChunk + threadIdx.x * kPerThread;
  double part = 0.0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int c = c0 + e;
    float v = 0.f;
    if (c < d.vocab) {
      v = (float)((double)expf((d.logits[c] - d.l1) * d.inv_temp) / d.z);
      if (kind == 1) v = fmaxf(0.f, v - d.q[c]);
    }
    mv[e] = v;
    part += (double)v;
  }
  return block_scan<kDrawThreads>(part, s_w, total);
}
__device__ __forceinline__ bool draw_row(const SampleArgs &a, int b, DrawRow *d) {
  const int mode = a.sel_mode[b];
  if (mode == 0) return false;
  const int node = a.sel_row[b], r = b * a.n_nodes + node;
  d->logits = a.logits + (size_t)r * a.vocab;
  d->q = (mode == 2) ? a.p_draft + ((size_t)b * (a.n_nodes - 1) + node) * a.vocab : nullptr;
  d->l1 = a.row_l1[r];
  d->inv_temp = a.inv_temp;
  d->z = a.row_z[r];
  d->vocab = a.vocab;
  return true;
}

// grid (chunks, batch): chunk totals of the tempered distribution and, for a residual draw, of the residual
__global__ __launch_bounds__(kDrawThreads) void k_sample_chunksum(SampleArgs a) {
  __shared__ double s_w[kDrawThreads / 64];
  const int chunk = blockIdx.x, b = blockIdx.y;
  DrawRow d;
  if (!a.out.token || !draw_row(a, b, &d)) return;   // uniform over the workgroup
  float mv[kPerThread];
  double total;
  (void)chunk_masses(d, chunk, 0, mv, s_w, &total);
  if (threadIdx.x == 0) a.chunk_sum[((size_t)b * 2 + 0) * a.n_chunks + chunk] = total;
  if (d.q != nullptr) {
    (void)chunk_masses(d, chunk, 1, mv, s_w, &total);
    if (threadIdx.x == 0) a.chunk_sum[((size_t)b * 2 + 1) * a.n_chunks + chunk] = total;
  }
}

// grid (batch): scan the chunk totals in ascending order, find the chunk that holds u * total, and
// inside it the token
__global__ __launch_bounds__(kDrawThreads) void k_sample_pick(SampleArgs a) {
  __shared__ double s_w[kDrawThreads / 64];
  __shared__ double s_begin[kDrawThreads];
  __shared__ double s_target;
  __shared__ int s_chunk, s_kind, s_tok, s_last;
  const int b = blockIdx.x, tid = threadIdx.x;
  DrawRow d;
  if (!a.out.token || !draw_row(a, b, &d)) return;   // uniform over the workgroup
  // chunk totals in ascending order: thread c holds chunk c (at most kDrawThreads chunks)
  int kind = (d.q != nullptr) ? 1 : 0;
  double cs = 0.0, cbegin = 0.0, ctotal = 0.0;
  for (;;) {
    cs = (tid < a.n_chunks) ? a.chunk_sum[((size_t)b * 2 + kind) * a.n_chunks + tid] : 0.0;
    cbegin = block_scan<kDrawThreads>(cs, s_w, &ctotal);
    if (ctotal > 0.0 || kind == 0) break;
    kind = 0;   // a residual without mass (the draft row dominates the verifier's): draw from p_v
  }
  const double ctarget = (double)a.u_sample[b] * ctotal;
  if (tid == 0) s_chunk = -1;
  __syncthreads();
  if (cs > 0.0 && cbegin <= ctarget) atomicMax(&s_chunk, tid);   // the last chunk with mass that begins at or below the target
  __syncthreads();
  if (tid == s_chunk) { s_target = ctarget - cbegin; s_kind = kind; }
  __syncthreads();
  if (s_chunk < 0) {
    // No chunk qualifies: the total or the target is NaN (a NaN or infinite logit, draft
    // probability or uniform) or there is no mass at all.  No draw is possible; the node's argmax
    // is returned and bit 1 of the status word says so.  (Uniform over the workgroup.)
    if (tid == 0) {
      a.out.token[b] = a.row_idx[b * a.n_nodes + a.sel_row[b]];
      if (a.out.status) atomicOr(a.out.status, 2);
    }
    return;
  }
  const int chunk = s_chunk;
  kind = s_kind;
  const double target = s_target;
  float mv[kPerThread];
  double total;
  const double begin = chunk_masses(d, chunk, kind, mv, s_w, &total);
  // Thread t owns [begin_t, begin_{t+1}); the owner is the LAST thread whose begin does not exceed
  // the target, which exists whatever the rounding of the scan (begin_0 = 0 <= target).  Should
  // rounding ever make two threads qualify, the lower token wins; a thread that finds no token of
  // its own beyond the target falls back to the chunk's last token with mass.
  s_begin[tid] = begin;
  int my_last = -1;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e)
    if (mv[e] > 0.f) my_last = tid * kPerThread + e;
  if (tid == 0) { s_tok = 0x7fffffff; s_last = -1; }
  __syncthreads();
  if (my_last >= 0) atomicMax(&s_last, my_last);
  __syncthreads();
  const bool owner = begin <= target && (tid == kDrawThreads - 1 || target < s_begin[tid + 1]);
  if (owner) {
    double run = begin;
    int pick = -1;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      run += (double)mv[e];
      if (pick < 0 && mv[e] > 0.f && run > target) pick = tid * kPerThread + e;
    }
    if (pick < 0) pick = (my_last >= 0) ? my_last : s_last;
    atomicMin(&s_tok, pick);
  }
  __syncthreads();
  if (tid == 0) a.out.token[b] = chunk * kChunk + s_tok;
}

void launch_sample_decide(hipStream_t st, const SampleArgs &a) {
  hipLaunchKernelGGL(k_sample_chunkstats, dim3(a.n_chunks, a.batch * a.n_nodes), dim3(kStatThreads), 0, st, a);
  hipLaunchKernelGGL(k_sample_walk, dim3(a.batch), dim3(64), 0, st, a);
  hipLaunchKernelGGL(k_sample_chunksum, dim3(a.n_chunks, a.batch), dim3(kDrawThreads), 0, st, a);
  hipLaunchKernelGGL(k_sample_pick, dim3(a.batch), dim3(kDrawThreads), 0, st, a);
}

}  // namespace ts
