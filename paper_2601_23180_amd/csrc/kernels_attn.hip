// Tree-masked grouped-query attention of the draft nodes over (context cache + draft nodes).
//
// Node i of sequence b attends to cache slots [0, ctx_len_b) and to every draft node j on its
// root path (bit j of anc[i]).  K is cached [slot][d]; V is cached transposed [d][slot] so that
// both products read matrix-core operands with 16-byte loads.
//
// bf16 path, two parts.  (1) Context: one workgroup per (context split, kv head, sequence) streams
// the cached K/V — no mask is needed there, every context key is visible to every node.
// (2) Draft nodes: at most 64 keys, of which a node sees only its ancestors; the merge kernel
// evaluates them in fp32 straight from this pass's unrounded q/k/v projections (the cache gets
// bf16 copies for later rounds, but the pass itself never reads them back) and folds them in as
// one more softmax partial.
// A merge kernel combines the splits in ascending order.
#include "device_util.hpp"

namespace ts {

// ------------------------------------------------------------------ fp32 path (small models)
// One wavefront per (row, query head).  Scores of all allowed keys go to LDS, then a plain
// two-pass softmax and the value sum with one lane per output feature.
constexpr int kAttnF32MaxKeys = 12288;

__global__ __launch_bounds__(64) void k_attn_f32(AttnArgs a) {
  extern __shared__ float sc[];
  const int r = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  const int d = a.head_dim, group = a.n_q_heads / a.n_kv_heads, kvh = head / group;
  const int b = r / a.n_nodes, node = r - b * a.n_nodes;
  const int ctx = a.ctx.v[b];
  const int n_keys = ctx + a.n_nodes;
  const AncMask mask = a.anc[r];
  const float *q = (const float *)a.q + (size_t)r * a.n_q_heads * d + (size_t)head * d;
  const float *kc = (const float *)a.k_cache, *vc = (const float *)a.v_cache;   // slots through a.kv
  const float scale = 1.0f / sqrtf((float)d);
  float mx = -INFINITY;
  for (int k = lane; k < n_keys; k += 64) {
    const bool ok = (k < ctx) || mask.has(k - ctx);
    float s = -INFINITY;
    if (ok) {
      const float *kr = kc + a.kv.k_row(b, kvh, k);
      float acc = 0.f;
      for (int j = 0; j < d; ++j) acc += q[j] * kr[j];
      s = acc * scale;
    }
    sc[k] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int k = lane; k < n_keys; k += 64) {
    const float p = (sc[k] == -INFINITY) ? 0.f : expf(sc[k] - mx);
    sc[k] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  float *o = (float *)a.out + (size_t)r * a.n_q_heads * d + (size_t)head * d;
  for (int j = lane; j < d; j += 64) {
    const size_t vj = (size_t)j * a.kv.v_stride();
    float acc = 0.f;
    for (int k = 0; k < n_keys; ++k) acc += sc[k] * vc[a.kv.v_col(b, kvh, k) + vj];
    o[j] = acc / sum;
  }
}

void launch_attn_f32(hipStream_t st, const AttnArgs &a) {
  int max_keys = 0;
  for (int b = 0; b < a.batch; ++b) max_keys = max(max_keys, a.ctx.v[b] + a.n_nodes);
  hipLaunchKernelGGL(k_attn_f32, dim3(a.batch * a.n_nodes, a.n_q_heads), dim3(64),
                     (size_t)max_keys * sizeof(float), st, a);
}

// ------------------------------------------------------------------ bf16 path
// KT = keys per LDS tile
template <int D, int KT>
struct AttnLds {
  static constexpr int kStrideK = D * 2 + 16;     // bytes per key row of the K tile
  static constexpr int kStrideV = KT * 2 + 8;     // bytes per feature row of the V^T tile
  static constexpr int kBytesK = KT * kStrideK;
  static constexpr int kBytesV = D * kStrideV;
  static constexpr int kBuf = kBytesK + kBytesV;  // one stage
};

// NW waves, each owning RBW blocks of 32 query rows: a workgroup covers 32 * NW * RBW rows.
// <KT 128, NW 4>: one workgroup per CU.  <KT 64, NW 8>: 256 rows share every staged K/V tile
// (trees of more than 128 rows read the cache once, not twice) and two waves per SIMD overlap
// one another's softmax arithmetic and matrix work.
// PAGED: the cache is in pages of kKvPage slots (a multiple of KT, and every split starts at a
// multiple of KT, so a tile never straddles two pages): one scalar page lookup per tile.
template <int D, int RBW, int KT, int NW, bool PAGED>
__global__ __launch_bounds__(64 * NW) void k_attn_bf16(AttnArgs a) {
  using L = AttnLds<D, KT>;
  constexpr int NT = 64 * NW;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * L::kBuf];
  const int split = blockIdx.x, kvh = blockIdx.y;
  const int b = blockIdx.z / a.n_row_groups, rg = blockIdx.z - b * a.n_row_groups;   // sequence, group of query rows
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: branches on it are wave-uniform
  const int ln = lane & 31, g = lane >> 5;
  const int M = a.n_nodes, group = a.n_q_heads / a.n_kv_heads;
  const int p_rows = group * M;
  const int ctx = a.ctx.v[b];
  const int n_keys = ctx;            // context only; the draft nodes are handled by the merge kernel
  const int k_begin = split * a.keys_per_split;
  const int k_end = min(n_keys, k_begin + a.keys_per_split);
  const size_t part_base = ((size_t)b * a.n_kv_heads + kvh) * a.n_splits + split;

  // ---- this lane's query rows
  int prow[RBW];
#pragma unroll
  for (int i = 0; i < RBW; ++i) prow[i] = (rg * NW * RBW + wave + NW * i) * 32 + ln;

  if (k_begin >= k_end) {   // empty split: neutral partial
#pragma unroll
    for (int i = 0; i < RBW; ++i)
      if (prow[i] < p_rows && g == 0) {
        a.part_m[part_base * p_rows + prow[i]] = -INFINITY;
        a.part_l[part_base * p_rows + prow[i]] = 0.f;
      }
    return;
  }

  static_assert(kKvPage % KT == 0, "a tile must not straddle pages");
  const int cap = PAGED ? kKvPage : a.kv.capacity;   // slots behind kc / vc, and the V^T row stride
  const bf16 *kc0 = (const bf16 *)a.k_cache, *vc0 = (const bf16 *)a.v_cache;
  if (!PAGED) {
    kc0 += ((size_t)b * a.n_kv_heads + kvh) * a.kv.capacity * D;
    vc0 += ((size_t)b * a.n_kv_heads + kvh) * D * a.kv.capacity;
  }

  // ---- tile staging: K tile = KT rows of D*2 bytes (16-byte vectors), V^T tile = D rows of KT*2 bytes
  constexpr int KV_PER_T = KT * D * 2 / 16 / NT;   // 16-byte vectors per thread, each of K and V^T
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  u32x4 kreg[KV_PER_T], vreg[KV_PER_T];
  // load_tile only ISSUES loads — anything that looked at a loaded value here would make the
  // compiler wait for each load in turn; the slots past the context are zeroed in store_tile.
  auto load_tile = [&](int k0g) {
    // contiguous: k0 counts from the sequence's first slot; paged: from the first slot of the tile's page
    const bf16 *kc = kc0, *vc = vc0;
    int k0 = k0g;
    if (PAGED) {
      const int page = a.kv.page_of(b, k0g);
      kc += ((size_t)page * a.n_kv_heads + kvh) * kKvPage * D;
      vc += ((size_t)page * a.n_kv_heads + kvh) * D * kKvPage;
      k0 = k0g % kKvPage;
    }
#pragma unroll
    for (int i = 0; i < KV_PER_T; ++i) {
      const int v = tid + NT * i;
      {  // K: vector v -> key v / (D/8), 16-byte column v % (D/8)
        const int key = v / (D / 8), c = v % (D / 8);
        // rows past the context hold no token (their scores are masked); clamped into the cache
        kreg[i] = *(const u32x4 *)(kc + (size_t)min(k0 + key, cap - 1) * D + c * 8);
      }
      {  // V^T: vector v -> feature v / (KT/8), 8 keys starting at (v % (KT/8)) * 8
        const int f = v / (KT / 8), c = v % (KT / 8);
        vreg[i] = *(const u32x4 *)(vc + (size_t)f * cap + min(k0 + c * 8, cap - 8));
      }
    }
  };
  auto store_tile = [&](int buf, int k0) {
    unsigned char *base = lds + buf * L::kBuf;
    const bool ragged = k0 + KT > n_keys;   // uniform over the workgroup: the context ends inside this tile
#pragma unroll
    for (int i = 0; i < KV_PER_T; ++i) {
      const int v = tid + NT * i;
      {
        const int key = v / (D / 8), c = v % (D / 8);
        *(u32x4 *)(base + key * L::kStrideK + c * 16) = kreg[i];
      }
      {
        const int f = v / (KT / 8), c = v % (KT / 8);
        u32x4 t = vreg[i];
        if (ragged) {   // zero the values of slots that hold no token (two keys per 32-bit word)
          const int left = n_keys - (k0 + c * 8);   // keys of this vector inside the context
          auto keep = [&](uint32_t x, int e0) {
            return x & ((e0 < left ? 0x0000ffffu : 0u) | (e0 + 1 < left ? 0xffff0000u : 0u));
          };
          t = u32x4{keep(t.x, 0), keep(t.y, 2), keep(t.z, 4), keep(t.w, 6)};
        }
        u32x2 *dst = (u32x2 *)(base + L::kBytesK + f * L::kStrideV + c * 16);
        dst[0] = u32x2{t.x, t.y};
        dst[1] = u32x2{t.z, t.w};
      }
    }
  };

  // ---- running state per row block: one query row per lane (both lane halves hold the same row)
  float m_run[RBW], l_run[RBW];
  f32x16 oacc[RBW][D / 32];
#pragma unroll
  for (int i = 0; i < RBW; ++i) {
    m_run[i] = -INFINITY;
    l_run[i] = 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[i][db][e] = 0.f;
  }

  const int n_tiles = (k_end - k_begin + KT - 1) / KT;
  load_tile(k_begin);
  // The query rows (as many bytes per workgroup as a tile) are requested after the first tile,
  // whose wait then does not include them, and without a branch (a row past the end reads the
  // last row: every lane's row is independent and such lanes store nothing).
  // rotated query as bf16 high part + bf16 low part (written by the QKV epilogue)
  bf16x8 qf[RBW][D / 16], ql[RBW][D / 16];
#pragma unroll
  for (int i = 0; i < RBW; ++i) {
    const int pc = min(prow[i], p_rows - 1);
    const int al = pc / M, node = pc - al * M;
    const int r = b * M + node;
    const bf16 *q = (const bf16 *)a.q + (size_t)r * a.n_q_heads * D + (size_t)(kvh * group + al) * D;
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
      qf[i][t] = *(const bf16x8 *)(q + 16 * t + 8 * g);
      ql[i][t] = *(const bf16x8 *)(q + a.q_panel + 16 * t + 8 * g);
    }
  }
  store_tile(0, k_begin);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int k0 = k_begin + t * KT;
    const int buf = t & 1;
    if (t + 1 < n_tiles) load_tile(k0 + KT);
    const unsigned char *kb = lds + buf * L::kBuf;
    const unsigned char *vb = kb + L::kBytesK;
    const bool need_mask = (k0 + KT > k_end);   // ragged end of the context or of this split

#pragma unroll
    for (int i = 0; i < RBW; ++i) {
      if ((rg * NW * RBW + wave + NW * i) * 32 >= p_rows) continue;   // wave-uniform
      // S^T[key][row] for the 32-key sub-tiles.  Consecutive matrix instructions go to different
      // accumulators: one that adds to the result of the instruction before it has to wait for it.
      f32x16 s[KT / 32];
#pragma unroll
      for (int ks = 0; ks < KT / 32; ++ks)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[ks][e] = 0.f;
#pragma unroll
      for (int tt = 0; tt < D / 16; ++tt) {
        bf16x8 kf[KT / 32];
#pragma unroll
        for (int ks = 0; ks < KT / 32; ++ks)
          kf[ks] = *(const bf16x8 *)(kb + (ks * 32 + ln) * L::kStrideK + (16 * tt + 8 * g) * 2);
#pragma unroll
        for (int ks = 0; ks < KT / 32; ++ks)
          s[ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[i][tt], s[ks], 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < KT / 32; ++ks)
          s[ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], ql[i][tt], s[ks], 0, 0, 0);
      }
      // mask (only the tile in which the context or the split ends: a scalar branch), tile max;
      // the scores arrive scaled: q was pre-multiplied by log2(e) / sqrt(d).  The vector ALU, not
      // the matrix cores, sets the pace of a tile step, so every instruction saved here counts.
      if (need_mask) {
#pragma unroll
        for (int ks = 0; ks < KT / 32; ++ks)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = k0 + ks * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
            s[ks][e] = (key < k_end) ? s[ks][e] : -INFINITY;
          }
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int ks = 0; ks < KT / 32; ++ks)
#pragma unroll
        for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[ks][e]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run[i], tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[i] - m_safe);   // exp2(-inf) = 0 on the first tile
      m_run[i] = m_new;
      float psum = 0.f;
      bf16x8 phi[KT / 16], plo[KT / 16];
#pragma unroll
      for (int ks = 0; ks < KT / 32; ++ks)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(s[ks][e] - m_safe);   // exp2(-inf) = 0 for masked keys
          psum += p;
          const bf16 hi = (bf16)p;
          const bf16 lo = (bf16)(p - (float)hi);
          phi[ks * 2 + (e >> 3)][e & 7] = hi;
          plo[ks * 2 + (e >> 3)][e & 7] = lo;
        }
      l_run[i] = l_run[i] * alpha + psum;
      // O^T[feature][row] = alpha * O^T + V^T P^T, the feature blocks interleaved for the same reason
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // the running maximum of some row moved
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[i][db][e] *= alpha;
      }
#pragma unroll
      for (int u = 0; u < KT / 16; ++u) {
        bf16x8 vf[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
          // key slots of lane half g at step u: 16u + 4g + {0..3} and 16u + 8 + 4g + {0..3}
          const unsigned char *vp = vb + (db * 32 + ln) * L::kStrideV + (16 * u + 4 * g) * 2;
          const u32x2 v0 = *(const u32x2 *)vp;
          const u32x2 v1 = *(const u32x2 *)(vp + 16);
          const u32x4 vv = u32x4{v0.x, v0.y, v1.x, v1.y};
          vf[db] = *(const bf16x8 *)&vv;
        }
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
          oacc[i][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], phi[u], oacc[i][db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
          oacc[i][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], plo[u], oacc[i][db], 0, 0, 0);
      }
    }
    if (t + 1 < n_tiles) store_tile(buf ^ 1, k0 + KT);
    __syncthreads();
  }

  // ---- write the split's partial: O[row][feature] unnormalised, m, l
#pragma unroll
  for (int i = 0; i < RBW; ++i) {
    const int p = prow[i];
    if (p >= p_rows) continue;
    const float l_tot = l_run[i] + __shfl_xor(l_run[i], 32, 64);
    if (g == 0) {
      a.part_m[part_base * p_rows + p] = m_run[i] * 0.693147180559945f;   // back to natural-log units
      a.part_l[part_base * p_rows + p] = l_tot;
    }
    float *o = a.part_o + (part_base * p_rows + p) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 v;
        v[0] = oacc[i][db][4 * q4 + 0]; v[1] = oacc[i][db][4 * q4 + 1];
        v[2] = oacc[i][db][4 * q4 + 2]; v[3] = oacc[i][db][4 * q4 + 3];
        *(f32x4 *)(o + db * 32 + 8 * q4 + 4 * g) = v;
      }
  }
}

// Combine the context splits of one (row, kv head) — all `group` query heads that share the kv
// head — in ascending split order, with the draft-node part: for every ancestor-or-self j of the
// node, score = q . k_j / sqrt(d) and value v_j, all taken in fp32 from this pass's projections
// (a.qkv: [row][(nq + 2 nkv) * d], q and k already rotated).
// Memory round trips, not arithmetic, set this kernel's time: the ancestor mask (one word, quick
// to arrive) is fetched alone, then everything else — query rows, the first 16 split partials,
// the ancestors' keys and the first ancestors' values — in ONE round trip.  Block = group * d / 2 threads, two adjacent output features each;
// the ancestor list (at most 64 nodes) is scored by (slot x quarter of the features) threads.
constexpr int kMergePreV = 8;    // ancestors whose values are fetched ahead of the scores
// e^x through the hardware exp2 (about 1e-7 |x| relative error; the arguments here are <= 0)
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

template <int D>
__global__ __launch_bounds__(512) void k_attn_merge(AttnArgs a) {
  __shared__ float s_q[kMaxGroup][D];
  __shared__ float s_sc[kMaxGroup][kMaxNodes];
  __shared__ int s_anc[kMaxNodes];
  const int r = blockIdx.x, kvh = blockIdx.y, tid = threadIdx.x, nt = blockDim.x;
  const int M = a.n_nodes, group = a.n_q_heads / a.n_kv_heads;
  const int b = r / M, node = r - b * M;
  const int p_rows = group * M;
  const size_t base = ((size_t)b * a.n_kv_heads + kvh) * a.n_splits;
  const int n_total = (a.n_q_heads + 2 * a.n_kv_heads) * D;
  const bool active = tid < group * D / 2;
  const int al = active ? tid / (D / 2) : 0, f = active ? (tid - al * (D / 2)) * 2 : 0;   // head, first feature
  const int p = al * M + node;

  // ---- the ancestor list first: one word per workgroup arrives quickly, and every address of
  // the second group of loads depends on it
  const AncMask mask = a.anc[r];           // bit j: node j is on the root path of this node (self included)
  const int n_anc = mask.count();          // >= 1
  for (int j = tid; j < kMaxNodes; j += nt)
    if (mask.has(j)) s_anc[mask.rank(j)] = j;
  __syncthreads();

  // ---- one round trip for everything else: the query rows, the
  // first 16 split partials of this thread's outputs, the values of the first ancestors and the
  // keys of the first batch of ancestors
  const float2 q2 = *(const float2 *)(a.qkv + (size_t)r * n_total + (size_t)(kvh * group + al) * D + f);
  float pm[16], pl[16];
  float2 po[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const size_t idx = (base + min(i, a.n_splits - 1)) * p_rows + p;
    pm[i] = a.part_m[idx];
    pl[i] = a.part_l[idx];
    po[i] = *(const float2 *)(a.part_o + idx * D + f);
  }
  const float *vbase = a.qkv + (size_t)(a.n_q_heads + a.n_kv_heads + kvh) * D + f;
  float2 vpre[kMergePreV];
#pragma unroll
  for (int i = 0; i < kMergePreV; ++i)
    vpre[i] = *(const float2 *)(vbase + (size_t)(b * M + s_anc[min(i, n_anc - 1)]) * n_total);
  const int qq = tid & 3;
  f32x4 kv4[D / 16];
  {
    const int j = s_anc[min(tid >> 2, n_anc - 1)];
    const float *kp = a.qkv + (size_t)(b * M + j) * n_total + (size_t)(a.n_q_heads + kvh) * D + qq * (D / 4);
#pragma unroll
    for (int i = 0; i < D / 16; ++i) kv4[i] = *(const f32x4 *)(kp + 4 * i);
  }
  if (active) { s_q[al][f] = q2.x; s_q[al][f + 1] = q2.y; }
  __syncthreads();

  // ---- scores of the ancestors: (slot x quarter of the features) threads, nt / 4 slots per batch
  const float scale = 1.0f / sqrtf((float)D);
  for (int s0 = 0; s0 < n_anc; s0 += nt / 4) {
    const int slot = s0 + (tid >> 2);
    if (s0 > 0) {   // later batches (deep paths on small workgroups) fetch their keys here
      const int j = s_anc[min(slot, n_anc - 1)];
      const float *kp = a.qkv + (size_t)(b * M + j) * n_total + (size_t)(a.n_q_heads + kvh) * D + qq * (D / 4);
#pragma unroll
      for (int i = 0; i < D / 16; ++i) kv4[i] = *(const f32x4 *)(kp + 4 * i);
    }
    for (int h = 0; h < group; ++h) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < D / 16; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc += kv4[i][e] * s_q[h][qq * (D / 4) + 4 * i + e];
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      if (qq == 0 && slot < n_anc) s_sc[h][slot] = acc * scale;
    }
  }
  __syncthreads();
  if (!active) return;

  float m_tot = -INFINITY;
  for (int i = 0; i < n_anc; ++i) m_tot = fmaxf(m_tot, s_sc[al][i]);
#pragma unroll
  for (int i = 0; i < 16; ++i) m_tot = fmaxf(m_tot, (i < a.n_splits) ? pm[i] : -INFINITY);
  for (int s0 = 16; s0 < a.n_splits; s0 += 16) {   // long contexts only
    float t[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) t[i] = (s0 + i < a.n_splits) ? a.part_m[(base + s0 + i) * p_rows + p] : -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) m_tot = fmaxf(m_tot, t[i]);
  }
  float num0 = 0.f, num1 = 0.f, den = 0.f;
  for (int s0 = 0; s0 < a.n_splits; s0 += 16) {    // ascending split order
    if (s0 > 0) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const size_t idx = (base + min(s0 + i, a.n_splits - 1)) * p_rows + p;
        pm[i] = a.part_m[idx];
        pl[i] = a.part_l[idx];
        po[i] = *(const float2 *)(a.part_o + idx * D + f);
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (s0 + i >= a.n_splits || pm[i] == -INFINITY) continue;   // empty split: its o / l were never written
      const float w = fast_exp(pm[i] - m_tot);
      num0 += po[i].x * w;
      num1 += po[i].y * w;
      den += pl[i] * w;
    }
  }
#pragma unroll
  for (int i = 0; i < kMergePreV; ++i)
    if (i < n_anc) {
      const float w = fast_exp(s_sc[al][i] - m_tot);
      num0 += w * vpre[i].x;
      num1 += w * vpre[i].y;
      den += w;
    }
  for (int i0 = kMergePreV; i0 < n_anc; i0 += 4) {
    float2 vv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      vv[i] = *(const float2 *)(vbase + (size_t)(b * M + s_anc[min(i0 + i, n_anc - 1)]) * n_total);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i0 + i < n_anc) {
        const float w = fast_exp(s_sc[al][i0 + i] - m_tot);
        num0 += w * vv[i].x;
        num1 += w * vv[i].y;
        den += w;
      }
  }
  const float o0 = num0 / den, o1 = num1 / den;
  const bf16 h0 = (bf16)o0, h1 = (bf16)o1;
  bf16 *dst = (bf16 *)a.out;   // operand layout of the O projection; out_panel = number of 32-row blocks
  const int kk = (kvh * group + al) * D + f;   // even: both features sit in the same 8-element run
  bf16 *d0 = dst + ol_offset(r, kk, 0, (int)a.out_panel), *d1 = dst + ol_offset(r, kk, 1, (int)a.out_panel);
  d0[0] = h0; d0[1] = h1;
  d1[0] = (bf16)(o0 - (float)h0); d1[1] = (bf16)(o1 - (float)h1);
}

template <int D>
static void launch_attn_bf16_d(hipStream_t st, const AttnArgs &a) {
  dim3 grid(a.n_splits, a.n_kv_heads, a.batch * a.n_row_groups);
  if (a.kv.page_table) {
    if (a.rows_per_wg == 256) hipLaunchKernelGGL((k_attn_bf16<D, 1, 64, 8, true>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((k_attn_bf16<D, 1, 128, 4, true>), grid, dim3(256), 0, st, a);
  } else {
    if (a.rows_per_wg == 256) hipLaunchKernelGGL((k_attn_bf16<D, 1, 64, 8, false>), grid, dim3(512), 0, st, a);
    else hipLaunchKernelGGL((k_attn_bf16<D, 1, 128, 4, false>), grid, dim3(256), 0, st, a);
  }
  const int group = a.n_q_heads / a.n_kv_heads;
  const int merge_threads = group * D / 2 < 64 ? 64 : group * D / 2;   // <= 512 (group <= 8, d <= 128)
  hipLaunchKernelGGL(k_attn_merge<D>, dim3(a.batch * a.n_nodes, a.n_kv_heads), dim3(merge_threads), 0, st, a);
}

void launch_attn_bf16(hipStream_t st, const AttnArgs &a) {
  if (a.head_dim == 128) launch_attn_bf16_d<128>(st, a);
  else launch_attn_bf16_d<64>(st, a);
}

}  // namespace ts
