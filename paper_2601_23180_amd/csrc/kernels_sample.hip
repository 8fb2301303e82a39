// Sampling (temperature > 0) form of the decision on a draft chain (paper Sec. 2.1 acceptance
// min(1, p_v / p_d) and residual resampling; Sec. 3.2 Eq. 6 - Eq. 9 and the routing).
// Three small kernels over logits that are already in memory:
//   k_sample_rowstats  per chain node: max / second max / argmax of the logits, the partition sum
//                      Z = sum exp((l - max) / T), and the two probabilities Eq. 6 compares
//   k_sample_walk      per sequence: trust predicate, Bernoulli acceptance, routing; picks the
//                      node whose distribution yields the next token
//   k_sample_token     per sequence: one inverse-CDF draw from that node's tempered distribution
//                      or from max(0, p_v - p_d)
// All sums run in a fixed order (per-thread slabs in ascending token order, then ascending
// thread order), so results do not depend on scheduling.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "internal.hpp"

namespace ts {

namespace {

constexpr int kStatThreads = 256;
constexpr int kDrawThreads = 1024;

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

__global__ __launch_bounds__(kStatThreads) void k_sample_rowstats(SampleArgs a) {
  __shared__ Max2 s_m[kStatThreads / 64];
  __shared__ double s_z[kStatThreads / 64];
  const int r = blockIdx.x, tid = threadIdx.x, V = a.vocab;
  const float *row = a.logits + (size_t)r * V;
  const int per = (V + kStatThreads - 1) / kStatThreads;
  const int lo = min(V, tid * per), hi = min(V, lo + per);
  Max2 m;
  m.l1 = -INFINITY; m.l2 = -INFINITY; m.idx = 0x7fffffff;
  for (int c = lo; c < hi; ++c) {
    const float v = row[c];
    if (v > m.l1) { m.l2 = m.l1; m.l1 = v; m.idx = c; }
    else m.l2 = fmaxf(m.l2, v);
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
  // partition sum at temperature T, slabs in ascending order
  double z = 0.0;
  for (int c = lo; c < hi; ++c) z += (double)expf((row[c] - m.l1) * a.inv_temp);
  // fixed order: inclusive scan over the lanes of a wave, then the waves in ascending order
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(z, o, 64);
    if ((tid & 63) >= o) z += up;
  }
  if ((tid & 63) == 63) s_z[tid >> 6] = z;
  __syncthreads();
  if (tid != 0) return;
  double zt = 0.0;
#pragma unroll
  for (int w = 0; w < kStatThreads / 64; ++w) zt += s_z[w];
  a.row_l1[r] = m.l1;
  a.row_l2[r] = m.l2;
  a.row_idx[r] = m.idx;
  a.row_z[r] = zt;
  // Eq. 6 operands of the NEXT chain node's token, judged by this node's distribution
  const int b = r / a.n_nodes, node = r - b * a.n_nodes;
  float pv = 0.f, q = 1.f;
  if (node + 1 < a.n_nodes) {
    const int x = a.tokens[r + 1];
    if (x >= 0 && x < V) {
      pv = (float)((double)expf((row[x] - m.l1) * a.inv_temp) / zt);
      q = a.p_draft[((size_t)b * (a.n_nodes - 1) + node) * V + x];
    } else {
      pv = -1.f;   // token id outside the vocabulary: never accepted, reported in the status word
    }
  }
  a.row_pv[r] = pv;
  a.row_q[r] = q;
}

__global__ __launch_bounds__(64) void k_sample_walk(SampleArgs a) {
  __shared__ float s_conf[kMaxNodes], s_margin[kMaxNodes];
  const int b = blockIdx.x, i = threadIdx.x, M = a.n_nodes;
  if (b == 0 && a.out.status) {   // status word of the whole call
    int bad = 0;
    for (int r = i; r < a.batch * M; r += 64) bad |= (a.row_pv[r] < 0.f);
    bad = __syncthreads_or(bad);
    if (i == 0) *a.out.status = bad ? 1 : 0;
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
  if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE + i] = -1;
  __syncthreads();
  if (i != 0) return;
  int cur = a.n_forced - 1, acc = 0, esc = 0, row = -1, mode = 0;   // mode: 0 none, 1 direct, 2 residual
  if (a.out.path) a.out.path[b * TRISPEC_PATH_STRIDE] = cur;
  for (int step = 0; step <= M; ++step) {
    const float stat = (a.criterion == TRISPEC_CRIT_MARGIN) ? s_margin[cur] : s_conf[cur];
    if (!(stat >= a.threshold)) { esc = 1; break; }
    if (cur + 1 >= M) { row = cur; mode = 1; break; }          // every draft token accepted
    const int r = b * M + cur;
    if (a.u_accept[r + 1] * a.row_q[r] < a.row_pv[r]) {       // u < min(1, p_v(x) / p_d(x))
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

__global__ __launch_bounds__(kDrawThreads) void k_sample_token(SampleArgs a) {
  __shared__ double s_part[kDrawThreads];
  __shared__ double s_total;
  const int b = blockIdx.x, tid = threadIdx.x, V = a.vocab;
  int mode = a.sel_mode[b];
  if (mode == 0 || !a.out.token) return;   // uniform over the workgroup
  const int node = a.sel_row[b], r = b * a.n_nodes + node;
  const float *row = a.logits + (size_t)r * V;
  const float *q = (mode == 2) ? a.p_draft + ((size_t)b * (a.n_nodes - 1) + node) * V : nullptr;
  const float l1 = a.row_l1[r];
  const double z = a.row_z[r];
  const int per = (V + kDrawThreads - 1) / kDrawThreads;
  const int lo = min(V, tid * per), hi = min(V, lo + per);
  auto mass = [&](int c) -> float {
    const float p = (float)((double)expf((row[c] - l1) * a.inv_temp) / z);
    return (mode == 2) ? fmaxf(0.f, p - q[c]) : p;
  };
  for (int attempt = 0; attempt < 2; ++attempt) {
    double part = 0.0;
    for (int c = lo; c < hi; ++c) part += (double)mass(c);
    s_part[tid] = part;
    __syncthreads();
    if (tid == 0) {   // exclusive prefix over the slabs, ascending
      double run = 0.0;
      for (int t = 0; t < kDrawThreads; ++t) {
        const double p = s_part[t];
        s_part[t] = run;
        run += p;
      }
      s_total = run;
    }
    __syncthreads();
    const double total = s_total;
    if (total > 0.0) {
      const double target = (double)a.u_sample[b] * total;
      const double begin = s_part[tid];
      if (part > 0.0 && begin <= target && target < begin + part) {   // exactly one slab owns the target
        double c_run = begin;
        int pick = -1, last = -1;
        for (int c = lo; c < hi; ++c) {
          const float mv = mass(c);
          if (mv > 0.f) last = c;
          c_run += (double)mv;
          if (c_run > target) { pick = c; break; }
        }
        a.out.token[b] = pick >= 0 ? pick : last;
      }
      return;
    }
    // a residual without mass (the draft row equals or dominates the verifier's): draw from p_v
    mode = 1;
    __syncthreads();
  }
}

void launch_sample_decide(hipStream_t st, const SampleArgs &a) {
  hipLaunchKernelGGL(k_sample_rowstats, dim3(a.batch * a.n_nodes), dim3(kStatThreads), 0, st, a);
  hipLaunchKernelGGL(k_sample_walk, dim3(a.batch), dim3(64), 0, st, a);
  hipLaunchKernelGGL(k_sample_token, dim3(a.batch), dim3(kDrawThreads), 0, st, a);
}

}  // namespace ts
