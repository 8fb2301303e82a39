// Host side of the C ABI: validation, workspace carve-up, launch sequence of one pass.
// No allocation, no synchronisation and no HIP call other than kernel launches on the hot path.
#include <math.h>
#include <cmath>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "internal.hpp"
#include "host_objects.hpp"

using namespace ts;

namespace {

// Records an event pair around one launch when a timer of this class is attached.
struct TimedLaunch {
  trispec_timer *t;
  hipStream_t st;
  bool on;
  TimedLaunch(trispec_timer *timer, int cls, hipStream_t s, double bytes) : t(timer), st(s), on(false) {
    if (t && t->kernel_class == cls && t->count < t->capacity) {
      on = true;
      t->bytes += bytes;
      (void)hipEventRecord(t->start[t->count], st);
    }
  }
  ~TimedLaunch() {
    if (on) {
      (void)hipEventRecord(t->stop[t->count], st);
      ++t->count;
    }
  }
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == TRISPEC_F32 ? 4 : 2; }

int rows_pad_for(int rows) {
  if (rows <= 32) return 32;
  if (rows <= 64) return 64;
  if (rows <= 128) return 128;
  return 256;
}

// Workspace regions, in order.  Offsets are a pure function of (model, batch, n_nodes).
struct Layout {
  size_t anc, parent, status, cos_t, sin_t, x, x2, h, h2, q, qkv_f32, attn_out, act, part, counters, ss_part, attn_o, attn_m, attn_l, head_l1, head_l2, head_sum, head_ent, head_idx, node_l1, node_l2, node_sum,
      node_ent, node_idx, logits, total;
  int rows_max, rows_pad_max, head_tiles, max_tiles;
  // `counters` holds, in this order: max_tiles + 1 tile counters of the split-K matmuls, kLayerPhases
  // barrier counters per layer, the abort word — n_zero ints that the set-up kernel clears
  int bar_index, abort_index, n_zero;
  size_t part_phase;   // floats per partial region of one phase of the layer kernel
};

// Decomposition of one bf16 matmul into (128-column tile, k split) workgroups: about kTargetWgs
// workgroups in all (two fit on a CU), every k split a whole number of 256-deep steps (512 when
// long enough) when the reduction allows it, and at least 512 deep.
struct SplitPlan {
  int tile_n, n_tiles, n_splits, k_per_split;
};
constexpr int kTargetWgs = 192;   // swept 128 .. 384 at the 8B shape: 192 - 224 is the flat optimum
constexpr int kLayerMaxGrid = 256;   // workgroups of the layer kernel (one per CU)
constexpr int kLayerSplitCap = 8;    // k splits of one matmul inside the layer kernel
// Longest wait at a device-side barrier, in ticks of the 100 MHz wall clock (2 s: three orders of
// magnitude above a whole pass).  trispec_debug_set_spin_limit changes it (tests of the expiry path).
unsigned long long g_spin_limit = 200000000ull;

SplitPlan plan_gemm(int epi, int n_cols, int k, int rows_pad) {
  (void)rows_pad;
  SplitPlan p;
  p.tile_n = kGemmTileN;
  // SWIGLU: n_cols = 2 * ffn, a tile holds tile_n/2 gate columns and the matching up columns
  p.n_tiles = (n_cols + p.tile_n - 1) / p.tile_n;
  if (epi == EPI_HEAD) {
    p.n_splits = 1;
    p.k_per_split = (int)align_up(k, (k % 256 == 0) ? 256 : 64);
    return p;
  }
  int s = (kTargetWgs + p.n_tiles / 2) / p.n_tiles;
  const int max_by_k = k / 512 > 0 ? k / 512 : 1;
  if (s > max_by_k) s = max_by_k;
  if (s > kMaxSplitK) s = kMaxSplitK;
  if (s < 1) s = 1;
  const int per = (k + s - 1) / s;
  const int unit = (k % 256 != 0) ? 64 : ((per >= 1024 && k % 512 == 0) ? 512 : 256);
  p.k_per_split = (int)align_up((size_t)per, unit);
  p.n_splits = (k + p.k_per_split - 1) / p.k_per_split;
  return p;
}
inline int tiles_of(int n) { return (n + kGemmTileN - 1) / kGemmTileN; }

// Decomposition of one matmul inside the layer kernel: at most max_items (tile, split) items, every
// split the same whole number of `unit`-deep steps (unit = ring depth x chunk depth of the kernel
// for this row count).  n_splits = 0: not possible for this shape.
SplitPlan plan_layer(int n_cols, int k, int unit, int max_items, int split_cap) {
  SplitPlan p;
  p.tile_n = kGemmTileN;
  p.n_tiles = (n_cols + p.tile_n - 1) / p.tile_n;
  p.n_splits = 0;
  p.k_per_split = 0;
  if (p.n_tiles > max_items || k % unit != 0) return p;
  int smax = max_items / p.n_tiles;
  if (smax > kMaxSplitK) smax = kMaxSplitK;
  if (smax > k / unit) smax = k / unit;
  if (smax > split_cap) smax = split_cap;
  for (int s = smax; s >= 1; --s)
    if (k % s == 0 && (k / s) % unit == 0) {
      p.n_splits = s;
      p.k_per_split = k / s;
      break;
    }
  return p;
}


Layout make_layout(const trispec_model_config &c, int batch, int max_nodes) {
  Layout L;
  memset(&L, 0, sizeof(L));
  const int rows = batch * max_nodes;
  const int rp = rows_pad_for(rows);
  const bool f32 = c.dtype == TRISPEC_F32;
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  const int nqkv = qd + 2 * kvd;
  L.rows_max = rows;
  L.rows_pad_max = rp;
  L.head_tiles = f32 ? 1 : plan_gemm(EPI_HEAD, c.vocab, c.hidden, rp).n_tiles;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.anc = take(sizeof(AncMask) * kMaxRows);
  L.parent = take(sizeof(int32_t) * kMaxRows);
  L.status = take(256);
  L.cos_t = take(sizeof(float) * rows * (c.head_dim / 2));
  L.sin_t = take(sizeof(float) * rows * (c.head_dim / 2));
  L.x = take(sizeof(float) * (size_t)rp * c.hidden);
  L.x2 = take(f32 ? 0 : sizeof(float) * (size_t)rp * c.hidden);   // the layer kernel alternates two copies
  // matmul operands: fp32 models one fp32 panel; bf16 models a bf16 hi panel + a bf16 lo panel
  L.h = take(sizeof(float) * (size_t)rp * c.hidden);
  L.h2 = take(f32 ? 0 : sizeof(float) * (size_t)rp * c.hidden);
  L.q = take(sizeof(float) * (size_t)rp * qd);
  L.qkv_f32 = take(f32 ? 0 : sizeof(float) * (size_t)rp * nqkv);
  L.attn_out = take(sizeof(float) * (size_t)rp * qd);
  L.act = take(sizeof(float) * (size_t)rp * c.ffn);
  if (f32) {
    int m = nqkv;
    if (c.hidden > m) m = c.hidden;
    if (2 * c.ffn > m) m = 2 * c.ffn;
    L.part = take(sizeof(float) * (size_t)rp * m);
  } else {
    // split-K partial tiles: the largest of splits x tiles x tile width over the matmuls of a layer
    const int ep[4] = {EPI_QKV, EPI_RESID, EPI_SWIGLU, EPI_RESID};
    const int nc[4] = {nqkv, c.hidden, 2 * c.ffn, c.hidden};
    const int ks[4] = {c.hidden, qd, c.hidden, c.ffn};
    size_t m = 0;
    for (int i = 0; i < 4; ++i) {
      const SplitPlan p = plan_gemm(ep[i], nc[i], ks[i], rp);
      const size_t e = (size_t)p.n_splits * p.n_tiles * p.tile_n;
      if (e > m) m = e;
      if (p.n_tiles > L.max_tiles) L.max_tiles = p.n_tiles;
    }
    // the layer kernel runs at most kLayerMaxGrid (tile, split) items per matmul and gives each
    // of its matmuls a partial region of its own
    L.part_phase = (size_t)kLayerMaxGrid * kGemmTileN * rp;
    if (kLayerPhases * (size_t)kLayerMaxGrid * kGemmTileN > m) m = kLayerPhases * (size_t)kLayerMaxGrid * kGemmTileN;
    L.part = take(sizeof(float) * m * rp);
  }
  L.bar_index = L.max_tiles + 1;
  L.abort_index = L.bar_index + kLayerPhases * c.n_layers;
  L.n_zero = L.abort_index + 1;
  L.counters = take(sizeof(int32_t) * L.n_zero);
  // sums of squares per (tile, row): two buffers, a matmul reads its producer's while writing its own
  L.ss_part = take(2 * sizeof(float) * (size_t)tiles_of(c.hidden) * rp);   // sized for the narrower tile
  const int group = c.n_q_heads / c.n_kv_heads;
  const size_t prow = f32 ? 0 : (size_t)batch * c.n_kv_heads * kMaxAttnSplits * group * max_nodes;
  L.attn_o = take(sizeof(float) * prow * c.head_dim);
  L.attn_m = take(sizeof(float) * prow);
  L.attn_l = take(sizeof(float) * prow);
  const size_t hs = (size_t)rows * L.head_tiles;
  L.head_l1 = take(sizeof(float) * hs);
  L.head_l2 = take(sizeof(float) * hs);
  L.head_sum = take(sizeof(float) * hs);
  L.head_ent = take(sizeof(float) * hs);
  L.head_idx = take(sizeof(int32_t) * hs);
  L.node_l1 = take(sizeof(float) * kMaxRows);
  L.node_l2 = take(sizeof(float) * kMaxRows);
  L.node_sum = take(sizeof(float) * kMaxRows);
  L.node_ent = take(sizeof(float) * kMaxRows);
  L.node_idx = take(sizeof(int32_t) * kMaxRows);
  L.logits = take(f32 ? sizeof(float) * (size_t)rows * c.vocab : 0);
  L.total = off;
  return L;
}

int check_shape(const trispec_model_config &c) {
  if (c.n_layers < 1 || c.hidden < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.ffn < 1 || c.vocab < 2)
    return TRISPEC_ESHAPE;
  if (c.head_dim != 64 && c.head_dim != 128) return TRISPEC_ESHAPE;
  if (c.n_q_heads % c.n_kv_heads != 0) return TRISPEC_ESHAPE;
  if (c.dtype != TRISPEC_F32 && c.dtype != TRISPEC_BF16) return TRISPEC_ESHAPE;
  if (!(c.rms_eps >= 0.f) || !(c.rope_base > 0.f)) return TRISPEC_ESHAPE;
  if (c.dtype == TRISPEC_BF16) {
    const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
    if (c.hidden % 64 || c.ffn % 64 || qd % 64 || kvd % 32) return TRISPEC_ESHAPE;
    if (c.n_q_heads / c.n_kv_heads > kMaxGroup) return TRISPEC_ESHAPE;
  }
  return TRISPEC_OK;
}

// Validates topological order and the forced chain; the set-up kernel turns the parents into root-path masks.
int build_nodes(const int32_t *parents, int batch, int n_nodes, int n_forced, NodeTable &tab) {
  for (int b = 0; b < batch; ++b) {
    const int32_t *p = parents + (size_t)b * n_nodes;
    if (p[0] != -1) return TRISPEC_ETREE;
    for (int i = 0; i < n_nodes; ++i) {
      if (i > 0 && (p[i] < 0 || p[i] >= i)) return TRISPEC_ETREE;
      if (i > 0 && i < n_forced && p[i] != i - 1) return TRISPEC_EFORCED;
      tab.parent[b * n_nodes + i] = p[i];
    }
  }
  return TRISPEC_OK;
}

int check_opts(const trispec_verify_opts *o, float threshold) {
  if (!o) return TRISPEC_ENULL;
  if (o->criterion != TRISPEC_CRIT_MARGIN && o->criterion != TRISPEC_CRIT_TOP1 && o->criterion != TRISPEC_CRIT_ENTROPY)
    return TRISPEC_EARG;
  if (threshold != threshold) return TRISPEC_EARG;
  if (o->accept_top_k < 0 || (o->accept_top_k > 1 && !o->draft_ranks)) return TRISPEC_EARG;
  if (o->n_feature_layers < 0 || o->n_feature_layers > TRISPEC_MAX_FEATURE_LAYERS) return TRISPEC_EARG;
  if (o->n_feature_layers > 0 && (!o->feature_layers || !o->features_out)) return TRISPEC_ENULL;
  if (o->adapter_w && (!o->adapter_out || o->adapter_dim < 4 || o->adapter_dim % 4)) return TRISPEC_EARG;
  if (!o->workspace) return TRISPEC_EWORKSPACE;
  if (((uintptr_t)o->workspace) & 255) return TRISPEC_EWORKSPACE;
  return TRISPEC_OK;
}

DecideArgs make_decide(const Layout &L, char *ws, const int32_t *tokens, int batch, int n_nodes,
                       float threshold, const trispec_verify_opts *o, const trispec_verify_out *out) {
  DecideArgs d;
  d.tokens = tokens;
  d.parent = (const int32_t *)(ws + L.parent);
  d.batch = batch;
  d.n_nodes = n_nodes;
  d.n_forced = o->n_forced;
  d.criterion = o->criterion;
  d.threshold = threshold;
  d.node_l1 = (float *)(ws + L.node_l1);
  d.node_l2 = (float *)(ws + L.node_l2);
  d.node_sum = (float *)(ws + L.node_sum);
  d.node_ent = (float *)(ws + L.node_ent);
  d.draft_ranks = o->draft_ranks;
  d.accept_top_k = o->accept_top_k;
  d.node_idx = (int32_t *)(ws + L.node_idx);
  d.status_src = (const int32_t *)(ws + L.status);
  d.out = *out;
  return d;
}

}  // namespace

extern "C" {

int trispec_model_create(const trispec_model_config *cfg, const trispec_weights *w, trispec_model **out) {
  if (!cfg || !w || !out) return TRISPEC_ENULL;
  const int rc = check_shape(*cfg);
  if (rc) return rc;
  if (!w->embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate ||
      !w->w_up || !w->w_down || !w->norm_attn || !w->norm_ffn)
    return TRISPEC_ENULL;
  const int L = cfg->n_layers;
  for (int l = 0; l < L; ++l)
    if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->w_gate[l] || !w->w_up[l] || !w->w_down[l] ||
        !w->norm_attn[l] || !w->norm_ffn[l])
      return TRISPEC_ENULL;
  if (cfg->qk_norm != 0 && cfg->qk_norm != 1) return TRISPEC_ESHAPE;
  if (cfg->qk_norm) {
    if (!w->q_norm || !w->k_norm) return TRISPEC_ENULL;
    for (int l = 0; l < L; ++l)
      if (!w->q_norm[l] || !w->k_norm[l]) return TRISPEC_ENULL;
  }
  trispec_model *m = new (std::nothrow) trispec_model;
  if (!m) return TRISPEC_EARG;
  m->cfg = *cfg;
  m->embed = w->embed;
  m->lm_head = w->lm_head;
  m->final_norm = w->final_norm;
  m->wq.assign(w->wq, w->wq + L);
  m->wk.assign(w->wk, w->wk + L);
  m->wv.assign(w->wv, w->wv + L);
  m->wo.assign(w->wo, w->wo + L);
  m->w_gate.assign(w->w_gate, w->w_gate + L);
  m->w_up.assign(w->w_up, w->w_up + L);
  m->w_down.assign(w->w_down, w->w_down + L);
  m->norm_attn.assign(w->norm_attn, w->norm_attn + L);
  m->norm_ffn.assign(w->norm_ffn, w->norm_ffn + L);
  if (cfg->qk_norm) {
    m->q_norm.assign(w->q_norm, w->q_norm + L);
    m->k_norm.assign(w->k_norm, w->k_norm + L);
  }
  m->packed = false;
  for (int i = 0; i < 3; ++i) m->layer_grid[i][0] = m->layer_grid[i][1] = -1;
  m->p_lm_head = nullptr;
  *out = m;
  return TRISPEC_OK;
}

int trispec_model_destroy(trispec_model *m) {
  delete m;
  return TRISPEC_OK;
}

// Packed-buffer layout: per layer wq, wk, wv, wo, w_gate, w_up, w_down, then the LM head.
static size_t pack_plan(const trispec_model_config &c, std::vector<size_t> *offs) {
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  const int rows[7] = {qd, kvd, kvd, c.hidden, c.ffn, c.ffn, c.hidden};
  const int ks[7] = {c.hidden, c.hidden, c.hidden, qd, c.hidden, c.hidden, c.ffn};
  size_t off = 0;
  for (int l = 0; l < c.n_layers; ++l)
    for (int i = 0; i < 7; ++i) {
      if (offs) offs->push_back(off);
      off += packed_weight_bytes(rows[i], ks[i]);
    }
  if (offs) offs->push_back(off);
  off += packed_weight_bytes(c.vocab, c.hidden);
  return off;
}

int trispec_model_pack_bytes(const trispec_model *m, size_t *bytes) {
  if (!m || !bytes) return TRISPEC_ENULL;
  *bytes = m->cfg.dtype == TRISPEC_BF16 ? pack_plan(m->cfg, nullptr) : 0;
  return TRISPEC_OK;
}

int trispec_model_pack(trispec_model *m, void *packed_dev, void *stream) {
  if (!m) return TRISPEC_ENULL;
  if (m->cfg.dtype != TRISPEC_BF16) { m->packed = true; return TRISPEC_OK; }
  if (!packed_dev) return TRISPEC_ENULL;
  if (((uintptr_t)packed_dev) & 255) return TRISPEC_EARG;
  const trispec_model_config &c = m->cfg;
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  std::vector<size_t> offs;
  pack_plan(c, &offs);
  hipStream_t st = (hipStream_t)stream;
  char *base = (char *)packed_dev;
  (void)hipGetLastError();
  const int L = c.n_layers;
  m->p_wq.resize(L); m->p_wk.resize(L); m->p_wv.resize(L); m->p_wo.resize(L);
  m->p_gate.resize(L); m->p_up.resize(L); m->p_down.resize(L);
  for (int l = 0; l < L; ++l) {
    const void *src[7] = {m->wq[l], m->wk[l], m->wv[l], m->wo[l], m->w_gate[l], m->w_up[l], m->w_down[l]};
    const int rows[7] = {qd, kvd, kvd, c.hidden, c.ffn, c.ffn, c.hidden};
    const int ks[7] = {c.hidden, c.hidden, c.hidden, qd, c.hidden, c.hidden, c.ffn};
    const void **dst[7] = {&m->p_wq[l], &m->p_wk[l], &m->p_wv[l], &m->p_wo[l], &m->p_gate[l], &m->p_up[l],
                           &m->p_down[l]};
    for (int i = 0; i < 7; ++i) {
      void *o = base + offs[(size_t)l * 7 + i];
      launch_pack_weights(st, src[i], rows[i], ks[i], o);
      *dst[i] = o;
    }
  }
  void *o = base + offs[(size_t)L * 7];
  launch_pack_weights(st, m->lm_head, c.vocab, c.hidden, o);
  m->p_lm_head = o;
  if (hipGetLastError() != hipSuccess) return TRISPEC_ELAUNCH;
  m->packed = true;
  return TRISPEC_OK;
}

int trispec_pack_matrix_bytes(int32_t n_rows, int32_t k, size_t *bytes) {
  if (!bytes) return TRISPEC_ENULL;
  if (n_rows < 1 || k < 64 || k % 64) return TRISPEC_EARG;
  *bytes = packed_weight_bytes(n_rows, k);
  return TRISPEC_OK;
}

int trispec_pack_matrix(const void *w_dev, int32_t n_rows, int32_t k, void *packed_dev, void *stream) {
  if (!w_dev || !packed_dev) return TRISPEC_ENULL;
  if (n_rows < 1 || k < 64 || k % 64 || (((uintptr_t)packed_dev) & 255) || (((uintptr_t)w_dev) & 15)) return TRISPEC_EARG;
  (void)hipGetLastError();
  launch_pack_weights((hipStream_t)stream, w_dev, n_rows, k, packed_dev);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

int trispec_kv_bytes(const trispec_model *m, int32_t batch, int32_t capacity, size_t *bytes) {
  if (!m || !bytes) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch) return TRISPEC_ENODES;
  if (capacity < 64 || capacity % 64) return TRISPEC_ECAPACITY;
  const trispec_model_config &c = m->cfg;
  *bytes = (size_t)c.n_layers * batch * c.n_kv_heads * capacity * c.head_dim * esize(c.dtype);
  return TRISPEC_OK;
}

int trispec_kv_create(const trispec_model *m, void *k_dev, void *v_dev, int32_t batch, int32_t capacity,
                      trispec_kv **out) {
  if (!m || !k_dev || !v_dev || !out) return TRISPEC_ENULL;
  size_t bytes;
  const int rc = trispec_kv_bytes(m, batch, capacity, &bytes);
  if (rc) return rc;
  if ((((uintptr_t)k_dev) | ((uintptr_t)v_dev)) & 15) return TRISPEC_EARG;
  trispec_kv *kv = new (std::nothrow) trispec_kv;
  if (!kv) return TRISPEC_EARG;
  kv->model = m;
  kv->k = k_dev;
  kv->v = v_dev;
  kv->batch = batch;
  kv->capacity = capacity;
  kv->page_table = nullptr;
  kv->max_pages = kv->n_pages = 0;
  for (int b = 0; b < kMaxBatch; ++b) kv->ctx_len[b] = 0;
  *out = kv;
  return TRISPEC_OK;
}

int trispec_kv_paged_bytes(const trispec_model *m, int32_t n_pages, size_t *bytes) {
  if (!m || !bytes) return TRISPEC_ENULL;
  if (n_pages < 1 || n_pages > (1 << 22)) return TRISPEC_ECAPACITY;
  const trispec_model_config &c = m->cfg;
  *bytes = (size_t)c.n_layers * n_pages * c.n_kv_heads * kKvPage * c.head_dim * esize(c.dtype);
  return TRISPEC_OK;
}

int trispec_kv_create_paged(const trispec_model *m, void *k_pool_dev, void *v_pool_dev, const int32_t *page_table_dev,
                            int32_t batch, int32_t max_pages_per_seq, int32_t n_pages, trispec_kv **out) {
  if (!m || !k_pool_dev || !v_pool_dev || !page_table_dev || !out) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch) return TRISPEC_ENODES;
  size_t bytes;
  const int rc = trispec_kv_paged_bytes(m, n_pages, &bytes);
  if (rc) return rc;
  if (max_pages_per_seq < 1 || max_pages_per_seq > (1 << 22) / kKvPage) return TRISPEC_ECAPACITY;
  if ((((uintptr_t)k_pool_dev) | ((uintptr_t)v_pool_dev)) & 15) return TRISPEC_EARG;
  trispec_kv *kv = new (std::nothrow) trispec_kv;
  if (!kv) return TRISPEC_EARG;
  kv->model = m;
  kv->k = k_pool_dev;
  kv->v = v_pool_dev;
  kv->batch = batch;
  kv->capacity = max_pages_per_seq * kKvPage;
  kv->page_table = page_table_dev;
  kv->max_pages = max_pages_per_seq;
  kv->n_pages = n_pages;
  for (int b = 0; b < kMaxBatch; ++b) kv->ctx_len[b] = 0;
  *out = kv;
  return TRISPEC_OK;
}

int trispec_kv_set_len(trispec_kv *kv, const int32_t *ctx_len_host) {
  if (!kv || !ctx_len_host) return TRISPEC_ENULL;
  for (int b = 0; b < kv->batch; ++b)
    if (ctx_len_host[b] < 0 || ctx_len_host[b] > kv->capacity) return TRISPEC_ECAPACITY;
  for (int b = 0; b < kv->batch; ++b) kv->ctx_len[b] = ctx_len_host[b];
  return TRISPEC_OK;
}

int trispec_kv_get_len(const trispec_kv *kv, int32_t *ctx_len_host) {
  if (!kv || !ctx_len_host) return TRISPEC_ENULL;
  for (int b = 0; b < kv->batch; ++b) ctx_len_host[b] = kv->ctx_len[b];
  return TRISPEC_OK;
}

int trispec_kv_destroy(trispec_kv *kv) {
  delete kv;
  return TRISPEC_OK;
}

int trispec_workspace_bytes(const trispec_model *m, int32_t batch, int32_t max_nodes, size_t *bytes) {
  if (!m || !bytes) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch || max_nodes < 1 || max_nodes > kMaxNodes ||
      batch * max_nodes > kMaxRows)
    return TRISPEC_ENODES;
  *bytes = make_layout(m->cfg, batch, max_nodes).total;
  return TRISPEC_OK;
}

// Test hook: where a named intermediate lives inside the workspace.
int trispec_workspace_region(const trispec_model *m, int32_t batch, int32_t max_nodes, const char *name,
                             size_t *offset, size_t *bytes) {
  if (!m || !name || !offset || !bytes) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch || max_nodes < 1 || max_nodes > kMaxNodes ||
      batch * max_nodes > kMaxRows)
    return TRISPEC_ENODES;
  const Layout L = make_layout(m->cfg, batch, max_nodes);
  const trispec_model_config &c = m->cfg;
  const size_t rp = L.rows_pad_max;
  struct { const char *n; size_t o, b; } tab[] = {
      {"x", L.x, sizeof(float) * rp * c.hidden},
      {"attn_out", L.attn_out, sizeof(float) * rp * c.n_q_heads * c.head_dim},
      {"act", L.act, sizeof(float) * rp * c.ffn},
      {"node_l1", L.node_l1, sizeof(float) * kMaxRows},
      {"node_l2", L.node_l2, sizeof(float) * kMaxRows},
      {"node_sum", L.node_sum, sizeof(float) * kMaxRows},
      {"node_ent", L.node_ent, sizeof(float) * kMaxRows},
      {"node_idx", L.node_idx, sizeof(int32_t) * kMaxRows},
  };
  for (auto &t : tab)
    if (!strcmp(t.n, name)) {
      *offset = t.o;
      *bytes = t.b;
      return TRISPEC_OK;
    }
  return TRISPEC_EARG;
}

int trispec_pass_bytes(const trispec_model *m, int32_t batch, int32_t n_nodes, const int32_t *ctx_len_host,
                       double *bytes) {
  if (!m || !ctx_len_host || !bytes) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch || n_nodes < 1 || n_nodes > kMaxNodes) return TRISPEC_ENODES;
  const trispec_model_config &c = m->cfg;
  const double w = (double)esize(c.dtype);
  const double qd = (double)c.n_q_heads * c.head_dim, kvd = (double)c.n_kv_heads * c.head_dim;
  const double per_layer = 2.0 * c.hidden * qd + 2.0 * c.hidden * kvd + 3.0 * (double)c.hidden * c.ffn +
                           2.0 * c.hidden;
  double kv = 0;
  for (int b = 0; b < batch; ++b) kv += 2.0 * ((double)ctx_len_host[b] + n_nodes) * kvd;
  *bytes = (c.n_layers * per_layer + (double)c.vocab * c.hidden + c.n_layers * kv) * w;
  return TRISPEC_OK;
}

int trispec_verify(trispec_model *m, trispec_kv *kv, const int32_t *draft_tokens,
                   const int32_t *tree_parents, const int32_t *positions, int32_t n_nodes, float threshold,
                   const trispec_verify_opts *opts, const trispec_verify_out *out) {
  if (!m || !kv || !draft_tokens || !tree_parents || !positions || !out) return TRISPEC_ENULL;
  int rc = check_opts(opts, threshold);
  if (rc) return rc;
  if (kv->model != m) return TRISPEC_EMISMATCH;
  const trispec_model_config &c = m->cfg;
  if (c.dtype == TRISPEC_BF16 && !m->packed) return TRISPEC_ESTATE;
  const int B = kv->batch;
  if (n_nodes < 1 || n_nodes > kMaxNodes || B * n_nodes > kMaxRows) return TRISPEC_ENODES;
  if (opts->n_forced < 1 || opts->n_forced > n_nodes) return TRISPEC_EFORCED;
  const int group = c.n_q_heads / c.n_kv_heads;
  if (c.dtype == TRISPEC_BF16 && group * n_nodes > 512) return TRISPEC_ENODES;
  int max_keys = 0;
  for (int b = 0; b < B; ++b) {
    if (kv->ctx_len[b] + n_nodes > kv->capacity) return TRISPEC_ECAPACITY;
    if (kv->ctx_len[b] > max_keys) max_keys = kv->ctx_len[b];
  }
  if (c.dtype == TRISPEC_F32 && max_keys + n_nodes > 12288) return TRISPEC_ECAPACITY;
  NodeTable tab;
  memset(&tab, 0, sizeof(tab));
  rc = build_nodes(tree_parents, B, n_nodes, opts->n_forced, tab);
  if (rc) return rc;
  const Layout L = make_layout(c, B, n_nodes);
  if (opts->workspace_bytes < L.total) return TRISPEC_EWORKSPACE;
  for (int i = 0; i < opts->n_feature_layers; ++i)
    if (opts->feature_layers[i] < 0 || opts->feature_layers[i] >= c.n_layers ||
        (i > 0 && opts->feature_layers[i] <= opts->feature_layers[i - 1]))
      return TRISPEC_EARG;

  hipStream_t st = (hipStream_t)opts->stream;
  char *ws = (char *)opts->workspace;
  const int rows = B * n_nodes, rp = rows_pad_for(rows);
  // residual stream after layer l -> features_out, if l is one of the requested layers
  int next_feature = 0;
  auto export_layer = [&](int l, const float *xs) {
    if (next_feature < opts->n_feature_layers && opts->feature_layers[next_feature] == l) {
      launch_export_hidden(st, c.dtype, xs, nullptr, nullptr, 0, rows, rows_pad_for(rows), c.hidden, c.rms_eps,
                           opts->features_out + (size_t)next_feature * rows * c.hidden);
      ++next_feature;
    }
  };
  const bool f32 = c.dtype == TRISPEC_F32;
  const size_t es = esize(c.dtype);
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, nqkv = qd + 2 * kvd;
  float *x = (float *)(ws + L.x);
  void *attn_out = ws + L.attn_out, *act = ws + L.act;
  const size_t pan_h = (size_t)rp * c.hidden, pan_q = (size_t)rp * qd, pan_f = (size_t)rp * c.ffn;
  float *part = (float *)(ws + L.part);
  float *cos_t = (float *)(ws + L.cos_t), *sin_t = (float *)(ws + L.sin_t);
  int32_t *status = (int32_t *)(ws + L.status);
  CtxLens ctx;
  for (int b = 0; b < kMaxBatch; ++b) ctx.v[b] = b < B ? kv->ctx_len[b] : 0;
  const size_t kv_layer = kv->layer_elems() * es;

  HeadStats hs;
  hs.l1 = (float *)(ws + L.head_l1);
  hs.l2 = (float *)(ws + L.head_l2);
  hs.sumexp = (float *)(ws + L.head_sum);
  hs.ent = (float *)(ws + L.head_ent);
  hs.idx = (int32_t *)(ws + L.head_idx);
  hs.n_tiles = L.head_tiles;

  AttnArgs at;
  memset(&at, 0, sizeof(at));
  at.anc = (const AncMask *)(ws + L.anc);
  at.ctx = ctx;
  at.batch = B; at.n_nodes = n_nodes; at.n_q_heads = c.n_q_heads; at.n_kv_heads = c.n_kv_heads;
  at.head_dim = c.head_dim; at.kv = kv->map();
  {
    // context split: aim at one workgroup per CU over (sequence, kv head, row group, split), at
    // least 256 keys per workgroup, at most kMaxAttnSplits splits.  Long contexts and batches then
    // take few, long splits — the fp32 partial outputs a split writes (rows x head_dim) would
    // otherwise outweigh the K/V it reads.  A tree of more than 128 query rows per kv head over a
    // long context takes 256-row workgroups (eight waves, 64-key tiles), which stage every K/V
    // tile once instead of once per 128-row group; on shorter contexts the two 128-row groups,
    // each with its own CU, finish sooner.
    const int group = c.n_q_heads / c.n_kv_heads;
    const int p_rows = group * n_nodes;
    at.rows_per_wg = (p_rows > 128 && max_keys >= kAttnWideMinKeys) ? 256 : 128;
    at.n_row_groups = (p_rows + at.rows_per_wg - 1) / at.rows_per_wg;
    const int per_split = B * c.n_kv_heads * at.n_row_groups;
    int want = (256 + per_split - 1) / per_split;
    if (want > kMaxAttnSplits) want = kMaxAttnSplits;
    // (a paged cache: every split starts at a multiple of the largest key tile, so that no tile straddles two pages)
    int kps = (int)align_up((size_t)((max_keys + want - 1) / want), kv->page_table ? 128 : 64);
    if (kps < 256) kps = 256;
    at.keys_per_split = kps;
    at.n_splits = (max_keys + kps - 1) / kps;
    if (at.n_splits < 1) at.n_splits = 1;
  }
  at.part_o = (float *)(ws + L.attn_o);
  at.part_m = (float *)(ws + L.attn_m);
  at.part_l = (float *)(ws + L.attn_l);
  at.out = attn_out;
  at.out_panel = (size_t)(rp / 32);   // operand layout: number of 32-row blocks
  auto attention = [&](char *kl, char *vl) {
    at.k_cache = kl;
    at.v_cache = vl;
    double kvb = 0;
    for (int b = 0; b < B; ++b) kvb += 2.0 * (kv->ctx_len[b] + n_nodes) * kvd * es;
    TimedLaunch tl(opts->timer, TRISPEC_K_ATTN, st, kvb);
    if (f32) launch_attn_f32(st, at); else launch_attn_bf16(st, at);
  };

  (void)hipGetLastError();
  launch_setup(st, tab, rows, n_nodes, (AncMask *)(ws + L.anc), (int32_t *)(ws + L.parent), status,
               (int32_t *)(ws + L.counters), L.n_zero);
  launch_rope_table(st, positions, rows, c.head_dim, c.rope_base, cos_t, sin_t);

  if (f32) {
    // ---------------- fp32 models: plain kernels, one per step
    float *h = (float *)(ws + L.h), *q = (float *)(ws + L.q);
    at.q = q;
    launch_embed_norm(st, c.dtype, draft_tokens, m->embed, m->norm_attn[0], rows, c.hidden, c.vocab,
                      c.rms_eps, x, h, 0, nullptr, status);
    auto gemm = [&](const float *xin, int k, int n_seg, const void *w0, int n0, const void *w1, int n1,
                    const void *w2, int n2, float *out) {
      GemmArgs g;
      memset(&g, 0, sizeof(g));
      g.x = xin;
      g.seg[0] = {w0, n0, 0};
      g.seg[1] = {w1, n1, n0};
      g.seg[2] = {w2, n2, n0 + n1};
      g.n_seg = n_seg;
      g.n_total = n0 + n1 + n2;
      g.k = k;
      g.rows = rows;
      g.rows_pad = rp;
      g.n_splits = 1;
      g.out = out;
      TimedLaunch tl(opts->timer, TRISPEC_K_GEMM, st, (double)g.n_total * k * es);
      launch_gemm_f32(st, g);
    };
    for (int l = 0; l < c.n_layers; ++l) {
      gemm(h, c.hidden, 3, m->wq[l], qd, m->wk[l], kvd, m->wv[l], kvd, part);
      char *kl = (char *)kv->k + (size_t)l * kv_layer, *vl = (char *)kv->v + (size_t)l * kv_layer;
      launch_qkv_epilogue(st, c.dtype, part, 1, rows, rp, c.n_q_heads, c.n_kv_heads, c.head_dim, cos_t, sin_t,
                          n_nodes, ctx, kv->map(), q, kl, vl, c.qk_norm ? (const float *)m->q_norm[l] : nullptr,
                          c.qk_norm ? (const float *)m->k_norm[l] : nullptr, c.rms_eps);
      attention(kl, vl);
      gemm((const float *)attn_out, qd, 1, m->wo[l], c.hidden, nullptr, 0, nullptr, 0, part);
      launch_reduce_residual_norm(st, c.dtype, part, 1, rows, rp, c.hidden, m->norm_ffn[l], c.rms_eps, x, h);
      gemm(h, c.hidden, 2, m->w_gate[l], c.ffn, m->w_up[l], c.ffn, nullptr, 0, part);
      launch_reduce_swiglu(st, c.dtype, part, 1, rows, rp, c.ffn, act);
      gemm((const float *)act, c.ffn, 1, m->w_down[l], c.hidden, nullptr, 0, nullptr, 0, part);
      const void *next_norm = (l + 1 < c.n_layers) ? m->norm_attn[l + 1] : m->final_norm;
      launch_reduce_residual_norm(st, c.dtype, part, 1, rows, rp, c.hidden, next_norm, c.rms_eps, x, h);
      export_layer(l, x);
    }
    float *logits = opts->debug_logits ? opts->debug_logits : (float *)(ws + L.logits);
    {
      TimedLaunch tl(opts->timer, TRISPEC_K_HEAD, st, (double)c.vocab * c.hidden * es);
      gemm(h, c.hidden, 1, m->lm_head, c.vocab, nullptr, 0, nullptr, 0, logits);
      launch_stats_from_logits(st, logits, rows, c.vocab, hs);
    }
    if (opts->hidden_out)
      launch_export_hidden(st, c.dtype, h, nullptr, nullptr, 0, rows, rp, c.hidden, c.rms_eps, opts->hidden_out);
    if (opts->adapter_w) {   // y = f W^T + b on the final-norm features (h is already normalised here)
      GemmArgs g;
      memset(&g, 0, sizeof(g));
      g.x = h;
      g.seg[0] = {opts->adapter_w, opts->adapter_dim, 0};
      g.n_seg = 1;
      g.n_total = opts->adapter_dim;
      g.k = c.hidden;
      g.rows = rows;
      g.rows_pad = rp;
      g.n_splits = 1;
      g.out = opts->adapter_out;
      g.bias = opts->adapter_bias;
      launch_gemm_f32(st, g);
    }
  } else {
    // ---------------- bf16 models: per layer QKV, attention (+ merge), O, gate/up, down
    void *h = ws + L.h, *h2 = ws + L.h2;
    float *x2 = (float *)(ws + L.x2);
    int32_t *counters = (int32_t *)(ws + L.counters);
    float *qkv_f32 = (float *)(ws + L.qkv_f32);
    at.qkv = qkv_f32;
    at.q = ws + L.q;
    at.q_panel = pan_q;
    // ss[0]: written by the embedding (1 tile) and by every down projection; ss[1]: by every O projection
    float *ss0 = (float *)(ws + L.ss_part), *ss1 = ss0 + (size_t)tiles_of(c.hidden) * rp;
    launch_embed_norm(st, c.dtype, draft_tokens, m->embed, m->norm_attn[0], rows, c.hidden, c.vocab, c.rms_eps,
                      x, h, (size_t)(rp / 32), ss0, status);
    const int hid_tiles = tiles_of(c.hidden);
    auto base = [&](int epi, const void *xin, size_t xpanel, const float *ss_in, int ss_tiles, int k,
                    int n_total, const SplitPlan &p) {
      GemmArgs g;
      memset(&g, 0, sizeof(g));
      g.epi = epi;
      g.x = xin;
      g.x_panel = xpanel;
      g.ss_in = ss_in;
      g.ss_tiles = ss_tiles;
      g.eps = c.rms_eps;
      g.n_total = n_total;
      g.k = k;
      g.rows = rows;
      g.rows_pad = rp;
      g.tile_n = p.tile_n;
      g.n_tiles = p.n_tiles;
      g.n_splits = p.n_splits;
      g.k_per_split = p.k_per_split;
      g.part = part;
      g.counters = counters;
      return g;
    };
    // The four matmuls of a layer.  `ss_tiles` of a consumer = tiles of its producer (1 after the embedding).
    auto mk_qkv = [&](int l, const SplitPlan &p, int ss_tiles) {
      GemmArgs g = base(EPI_QKV, h, pan_h, ss0, ss_tiles, c.hidden, nqkv, p);
      g.seg[0] = {m->p_wq[l], qd, 0};
      g.seg[1] = {m->p_wk[l], kvd, qd};
      g.seg[2] = {m->p_wv[l], kvd, qd + kvd};
      g.n_seg = 3;
      g.q_out = ws + L.q; g.q_panel = pan_q;
      g.cos_t = cos_t; g.sin_t = sin_t; g.qkv_f32 = qkv_f32; g.ctx = ctx;
      g.k_cache = (char *)kv->k + (size_t)l * kv_layer;
      g.v_cache = (char *)kv->v + (size_t)l * kv_layer;
      g.n_nodes = n_nodes; g.n_q_heads = c.n_q_heads; g.n_kv_heads = c.n_kv_heads; g.head_dim = c.head_dim;
      g.kv = kv->map();
      g.q_norm_w = c.qk_norm ? m->q_norm[l] : nullptr;
      g.k_norm_w = c.qk_norm ? m->k_norm[l] : nullptr;
      return g;
    };
    auto mk_o = [&](int l, const SplitPlan &p, const float *x_in, float *x_out, void *h_out) {
      GemmArgs g = base(EPI_RESID, attn_out, pan_q, nullptr, 0, qd, c.hidden, p);
      g.seg[0] = {m->p_wo[l], c.hidden, 0};
      g.n_seg = 1;
      g.x_resid = x_in; g.x_resid_out = x_out; g.xw_out = h_out; g.out_panel = pan_h;
      g.next_norm_w = m->norm_ffn[l]; g.ss_part = ss1;
      return g;
    };
    auto mk_gu = [&](int l, const SplitPlan &p, const void *h_in) {
      GemmArgs g = base(EPI_SWIGLU, h_in, pan_h, ss1, hid_tiles, c.hidden, 2 * c.ffn, p);
      g.seg[0] = {m->p_gate[l], c.ffn, 0};
      g.seg[1] = {m->p_up[l], c.ffn, c.ffn};
      g.n_seg = 2;
      g.act_out = act; g.ffn = c.ffn; g.out_panel = pan_f;
      return g;
    };
    auto mk_dn = [&](int l, const SplitPlan &p, const float *x_in, float *x_out) {
      GemmArgs g = base(EPI_RESID, act, pan_f, nullptr, 0, c.ffn, c.hidden, p);
      g.seg[0] = {m->p_down[l], c.hidden, 0};
      g.n_seg = 1;
      g.x_resid = x_in; g.x_resid_out = x_out; g.xw_out = h; g.out_panel = pan_h;
      g.next_norm_w = (l + 1 < c.n_layers) ? m->norm_attn[l + 1] : m->final_norm; g.ss_part = ss0;
      return g;
    };
    const SplitPlan pq = plan_gemm(EPI_QKV, nqkv, c.hidden, rp), po = plan_gemm(EPI_RESID, c.hidden, qd, rp);
    const SplitPlan pg = plan_gemm(EPI_SWIGLU, 2 * c.ffn, c.hidden, rp), pd = plan_gemm(EPI_RESID, c.hidden, c.ffn, rp);
    auto timed_gemm = [&](const GemmArgs &g, double bytes) {
      TimedLaunch tl(opts->timer, TRISPEC_K_GEMM, st, bytes);
      launch_gemm_bf16(st, g);
    };
    const double b_qkv = (double)nqkv * c.hidden * es, b_o = (double)c.hidden * qd * es;
    const double b_gu = 2.0 * c.ffn * c.hidden * es, b_dn = (double)c.hidden * c.ffn * es;

    // ---- one launch for O, gate + up, down and the next QKV when the shapes allow it and the
    // whole grid is resident at once on this device (asked once per model and row count)
    bool layered = opts->launch_mode == TRISPEC_LAUNCH_PER_LAYER && rp <= 128;
    SplitPlan lq, lo, lg, ld;
    int lgrid = 0, ring_depth = 0;
    if (layered) {
      const int slot = rp == 32 ? 0 : (rp == 64 ? 1 : 2);
      auto plans = [&](int max_items, int depth) {
        const int unit = layer_step(rp, depth);
        lq = plan_layer(nqkv, c.hidden, unit, max_items, kLayerSplitCap);
        lo = plan_layer(c.hidden, qd, unit, max_items, kLayerSplitCap);
        lg = plan_layer(2 * c.ffn, c.hidden, unit, max_items, 1);
        ld = plan_layer(c.hidden, c.ffn, unit, max_items, kLayerSplitCap);
        return lq.n_splits > 0 && lo.n_splits > 0 && lg.n_splits > 0 && ld.n_splits > 0;
      };
      auto probe_grid = [&](int depth) {
        LayerArgs probe;
        memset(&probe, 0, sizeof(probe));
        probe.n_phases = 3;
        probe.ring_depth = depth;
        probe.ph[0] = mk_o(0, lo, x, x2, h2);
        probe.ph[1] = mk_gu(0, lg, h2);
        probe.ph[2] = mk_dn(0, ld, x2, x);
        return layer_kernel_max_grid(probe);
      };
      layered = false;
      for (int depth = 8; depth >= 4 && !layered; depth -= 4) {
        if (!plans(kLayerMaxGrid, depth)) continue;
        int &cap = m->layer_grid[slot][depth == 8 ? 0 : 1];
        if (cap < 0) cap = probe_grid(depth);
        const int lim = cap < kLayerMaxGrid ? cap : kLayerMaxGrid;
        if (lim <= 0 || !plans(lim, depth)) continue;
        layered = true;
        ring_depth = depth;
      }
      if (layered) {
        auto items = [](const SplitPlan &p) { return p.n_tiles * p.n_splits; };
        lgrid = items(lq);
        if (items(lo) > lgrid) lgrid = items(lo);
        if (items(lg) > lgrid) lgrid = items(lg);
        if (items(ld) > lgrid) lgrid = items(ld);
      }
    }

    if (!layered) {
      int ss0_tiles = 1;
      for (int l = 0; l < c.n_layers; ++l) {
        char *kl = (char *)kv->k + (size_t)l * kv_layer, *vl = (char *)kv->v + (size_t)l * kv_layer;
        timed_gemm(mk_qkv(l, pq, ss0_tiles), b_qkv);
        attention(kl, vl);
        timed_gemm(mk_o(l, po, x, x, h), b_o);
        timed_gemm(mk_gu(l, pg, h), b_gu);
        timed_gemm(mk_dn(l, pd, x, x), b_dn);
        export_layer(l, x);
        ss0_tiles = hid_tiles;
      }
    } else {
      timed_gemm(mk_qkv(0, pq, 1), b_qkv);
      for (int l = 0; l < c.n_layers; ++l) {
        char *kl = (char *)kv->k + (size_t)l * kv_layer, *vl = (char *)kv->v + (size_t)l * kv_layer;
        attention(kl, vl);
        LayerArgs la;
        memset(&la, 0, sizeof(la));
        const bool more = l + 1 < c.n_layers;
        la.n_phases = more ? 4 : 3;
        la.ring_depth = ring_depth;
        la.ph[0] = mk_o(l, lo, x, x2, h2);
        la.ph[1] = mk_gu(l, lg, h2);
        la.ph[2] = mk_dn(l, ld, x2, x);
        if (more) la.ph[3] = mk_qkv(l + 1, lq, hid_tiles);
        for (int p = 0; p < kLayerPhases; ++p) la.ph[p].part = part + (size_t)p * L.part_phase;
        la.bar = counters + L.bar_index + kLayerPhases * l;
        la.abort_word = counters + L.abort_index;
        la.status = status;
        la.spin_limit = g_spin_limit;
        la.stamps = opts->stamps ? (unsigned long long *)opts->stamps + (size_t)16 * l : nullptr;
        la.stamp_wg = 0;
        la.poll_naps = 1;
        TimedLaunch tl(opts->timer, TRISPEC_K_GEMM, st, b_o + b_gu + b_dn + (more ? b_qkv : 0.0));
        if (!launch_layer_bf16(st, la, lgrid)) return TRISPEC_ELAUNCH;
        export_layer(l, x);
      }
    }
    {
      GemmArgs g = base(EPI_HEAD, h, pan_h, ss0, hid_tiles, c.hidden, c.vocab, plan_gemm(EPI_HEAD, c.vocab, c.hidden, rp));
      g.seg[0] = {m->p_lm_head, c.vocab, 0};
      g.n_seg = 1;
      hs.n_tiles = g.n_tiles;
      g.hs = hs;
      g.debug_logits = opts->debug_logits;
      TimedLaunch tl(opts->timer, TRISPEC_K_HEAD, st, (double)c.vocab * c.hidden * es);
      launch_gemm_bf16(st, g);
    }
    if (opts->adapter_w) {
      // the adapter on the final-norm features: the LM head's operand panels and 1/rms again, another
      // matrix, a plain fp32 result (+ bias)
      SplitPlan pa = plan_gemm(EPI_RESID, opts->adapter_dim, c.hidden, rp);
      if (pa.n_splits > 1 && pa.n_tiles > L.max_tiles) {   // no counters for that many tiles: one split
        pa.n_splits = 1;
        pa.k_per_split = (int)align_up(c.hidden, (c.hidden % 256 == 0) ? 256 : 64);
      }
      GemmArgs g = base(EPI_PLAIN, h, pan_h, ss0, hid_tiles, c.hidden, opts->adapter_dim, pa);
      g.seg[0] = {opts->adapter_w, opts->adapter_dim, 0};
      g.n_seg = 1;
      g.out = opts->adapter_out;
      g.bias = opts->adapter_bias;
      launch_gemm_bf16(st, g);
    }
    if (opts->hidden_out)   // x after the last layer, the final norm's weight, the sums of squares the last down projection left
      launch_export_hidden(st, c.dtype, x, m->final_norm, ss0, hid_tiles, rows, rp, c.hidden, c.rms_eps,
                           opts->hidden_out);
  }

  launch_stats_reduce(st, hs, rows, (float *)(ws + L.node_l1), (float *)(ws + L.node_l2),
                      (float *)(ws + L.node_sum), (float *)(ws + L.node_ent), (int32_t *)(ws + L.node_idx));
  DecideArgs d = make_decide(L, ws, draft_tokens, B, n_nodes, threshold, opts, out);
  launch_decide(st, d);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

int trispec_decide(trispec_model *m, int32_t batch, const int32_t *draft_tokens, const int32_t *tree_parents,
                   int32_t n_nodes, float threshold, const trispec_verify_opts *opts,
                   const trispec_verify_out *out) {
  if (!m || !draft_tokens || !tree_parents || !out) return TRISPEC_ENULL;
  int rc = check_opts(opts, threshold);
  if (rc) return rc;
  if (batch < 1 || batch > kMaxBatch || n_nodes < 1 || n_nodes > kMaxNodes || batch * n_nodes > kMaxRows)
    return TRISPEC_ENODES;
  if (opts->n_forced < 1 || opts->n_forced > n_nodes) return TRISPEC_EFORCED;
  NodeTable tab;
  memset(&tab, 0, sizeof(tab));
  rc = build_nodes(tree_parents, batch, n_nodes, opts->n_forced, tab);
  if (rc) return rc;
  const Layout L = make_layout(m->cfg, batch, n_nodes);
  if (opts->workspace_bytes < L.total) return TRISPEC_EWORKSPACE;
  hipStream_t st = (hipStream_t)opts->stream;
  char *ws = (char *)opts->workspace;
  (void)hipGetLastError();
  // the tree of THIS call (it may differ from the last verify's, e.g. after pruning): parents into
  // the workspace, the status word and the counters left alone
  launch_setup(st, tab, batch * n_nodes, n_nodes, (AncMask *)(ws + L.anc), (int32_t *)(ws + L.parent), nullptr, nullptr, 0);
  DecideArgs d = make_decide(L, ws, draft_tokens, batch, n_nodes, threshold, opts, out);
  launch_decide(st, d);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

namespace {
struct SampleLayout {
  size_t z, l1, l2, idx, cs_l1, cs_l2, cs_idx, cs_z, seq_bad, sel_row, sel_mode, chunk_sum, total;
  int n_chunks;
};
SampleLayout sample_layout(int batch, int n_nodes, int vocab) {
  const size_t rows = (size_t)batch * n_nodes;
  SampleLayout L;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.z = take(rows * sizeof(double));
  L.l1 = take(rows * sizeof(float));
  L.l2 = take(rows * sizeof(float));
  L.idx = take(rows * sizeof(int32_t));
  L.n_chunks = (vocab + kSampleChunk - 1) / kSampleChunk;
  L.cs_l1 = take(rows * L.n_chunks * sizeof(float));
  L.cs_l2 = take(rows * L.n_chunks * sizeof(float));
  L.cs_idx = take(rows * L.n_chunks * sizeof(int32_t));
  L.cs_z = take(rows * L.n_chunks * sizeof(double));
  L.seq_bad = take((size_t)batch * sizeof(int32_t));
  L.sel_row = take((size_t)batch * sizeof(int32_t));
  L.sel_mode = take((size_t)batch * sizeof(int32_t));
  L.chunk_sum = take((size_t)batch * 2 * L.n_chunks * sizeof(double));
  L.total = off;
  return L;
}
bool sample_shape_ok(int batch, int n_nodes) {
  return batch >= 1 && batch <= kMaxBatch && n_nodes >= 1 && n_nodes <= kMaxChain && batch * n_nodes <= kMaxRows;
}
}  // namespace

int trispec_sample_scratch_bytes(int32_t batch, int32_t n_nodes, int32_t vocab, size_t *bytes) {
  if (!bytes) return TRISPEC_ENULL;
  if (!sample_shape_ok(batch, n_nodes)) return TRISPEC_ENODES;
  if (vocab < 1 || vocab > kSampleMaxVocab) return TRISPEC_EARG;
  *bytes = sample_layout(batch, n_nodes, vocab).total;
  return TRISPEC_OK;
}

namespace {
// Host-side checks shared by the two sampling entry points (everything but the scratch buffer).
int sample_check(const float *logits, const int32_t *draft_tokens, int32_t batch, int32_t n_nodes, int32_t vocab,
                 float threshold, const trispec_sample_opts *o, const trispec_verify_out *out) {
  if (!logits || !draft_tokens || !o || !out || !o->u_accept || !o->u_sample) return TRISPEC_ENULL;
  if (!sample_shape_ok(batch, n_nodes)) return TRISPEC_ENODES;
  if (n_nodes > 1 && !o->p_draft) return TRISPEC_ENULL;
  if (o->n_forced < 1 || o->n_forced > n_nodes) return TRISPEC_EFORCED;
  if (!(o->temperature > 0.f) || !std::isfinite(o->temperature) || threshold != threshold || vocab < 1 || vocab > kSampleMaxVocab ||
      (o->criterion != TRISPEC_CRIT_MARGIN && o->criterion != TRISPEC_CRIT_TOP1) ||
      (o->resample != TRISPEC_RESAMPLE_RESIDUAL && o->resample != TRISPEC_RESAMPLE_DIRECT))
    return TRISPEC_EARG;
  return TRISPEC_OK;
}

// Carves `ws` (sample_layout bytes, 256-byte aligned) and enqueues the four kernels.
int sample_launch(const float *logits, const int32_t *draft_tokens, int32_t batch, int32_t n_nodes, int32_t vocab,
                  float threshold, const trispec_sample_opts *o, const trispec_verify_out *out,
                  const SampleLayout &L, char *ws);
}  // namespace

int trispec_sample_decide(const float *logits, const int32_t *draft_tokens, int32_t batch, int32_t n_nodes,
                          int32_t vocab, float threshold, const trispec_sample_opts *o,
                          const trispec_verify_out *out) {
  const int rc = sample_check(logits, draft_tokens, batch, n_nodes, vocab, threshold, o, out);
  if (rc) return rc;
  const SampleLayout L = sample_layout(batch, n_nodes, vocab);
  if (!o->scratch || ((uintptr_t)o->scratch & 255) || o->scratch_bytes < L.total) return TRISPEC_EWORKSPACE;
  return sample_launch(logits, draft_tokens, batch, n_nodes, vocab, threshold, o, out, L, (char *)o->scratch);
}

// ---- the entry point that allocates nothing: the scratch of the sampling kernels lives in a
// device array of this library instead of a caller buffer.  Each GPU holds its own copy of the
// array at its own address; in host code the array's NAME is only a handle for
// hipGetSymbolAddress, never a device address, so kernels always get the looked-up pointer.
static __device__ __align__(256) unsigned char scratch[TRISPEC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];   // per device, filled on the first call with that device current

int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TRISPEC_ELAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TRISPEC_ELAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TRISPEC_OK;
}
}  // namespace

int trispec_sample_decide_static(const float *logits, const int32_t *draft_tokens, int32_t batch,
                                 int32_t n_nodes, int32_t vocab, float threshold,
                                 const trispec_sample_opts *o, const trispec_verify_out *out) {
  const int rc = sample_check(logits, draft_tokens, batch, n_nodes, vocab, threshold, o, out);
  if (rc) return rc;
  const SampleLayout L = sample_layout(batch, n_nodes, vocab);
  if (L.total > (size_t)TRISPEC_STATIC_SCRATCH_BYTES) return TRISPEC_EWORKSPACE;
  void *ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs) return rs;
  // Nothing in the scratch has to start at zero: every kernel of the call writes each entry it
  // or a later kernel reads (per chunk statistics, per row merges, the selected row and the
  // chunk masses of the kinds that are drawn from), so the previous call's contents are inert.
  return sample_launch(logits, draft_tokens, batch, n_nodes, vocab, threshold, o, out, L, (char *)ws);
}

namespace {
int sample_launch(const float *logits, const int32_t *draft_tokens, int32_t batch, int32_t n_nodes, int32_t vocab,
                  float threshold, const trispec_sample_opts *o, const trispec_verify_out *out,
                  const SampleLayout &L, char *ws) {
  SampleArgs a;
  memset(&a, 0, sizeof(a));
  a.logits = logits; a.tokens = draft_tokens; a.p_draft = o->p_draft;
  a.u_accept = o->u_accept; a.u_sample = o->u_sample;
  a.batch = batch; a.n_nodes = n_nodes; a.vocab = vocab; a.n_forced = o->n_forced;
  a.criterion = o->criterion; a.resample = o->resample;
  a.inv_temp = 1.0f / o->temperature; a.threshold = threshold;
  a.row_z = (double *)(ws + L.z);
  a.row_l1 = (float *)(ws + L.l1); a.row_l2 = (float *)(ws + L.l2);
  a.row_idx = (int32_t *)(ws + L.idx);
  a.cs_l1 = (float *)(ws + L.cs_l1); a.cs_l2 = (float *)(ws + L.cs_l2);
  a.cs_idx = (int32_t *)(ws + L.cs_idx); a.cs_z = (double *)(ws + L.cs_z);
  a.seq_bad = (int32_t *)(ws + L.seq_bad);
  a.sel_row = (int32_t *)(ws + L.sel_row); a.sel_mode = (int32_t *)(ws + L.sel_mode);
  a.chunk_sum = (double *)(ws + L.chunk_sum); a.n_chunks = L.n_chunks;
  a.out = *out;
  (void)hipGetLastError();
  launch_sample_decide((hipStream_t)o->stream, a);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}
}  // namespace

int trispec_timer_create(int32_t kernel_class, int32_t capacity, trispec_timer **out) {
  if (!out) return TRISPEC_ENULL;
  if (kernel_class < TRISPEC_K_GEMM || kernel_class > TRISPEC_K_ATTN || capacity < 1 || capacity > (1 << 20))
    return TRISPEC_EARG;
  trispec_timer *t = new (std::nothrow) trispec_timer;
  if (!t) return TRISPEC_EARG;
  t->kernel_class = kernel_class;
  t->capacity = capacity;
  t->count = 0;
  t->bytes = 0;
  t->start.resize(capacity);
  t->stop.resize(capacity);
  for (int i = 0; i < capacity; ++i)
    if (hipEventCreate(&t->start[i]) != hipSuccess || hipEventCreate(&t->stop[i]) != hipSuccess) {
      delete t;
      return TRISPEC_ELAUNCH;
    }
  *out = t;
  return TRISPEC_OK;
}

int trispec_timer_reset(trispec_timer *t) {
  if (!t) return TRISPEC_ENULL;
  t->count = 0;
  t->bytes = 0;
  return TRISPEC_OK;
}

int trispec_timer_read(trispec_timer *t, int32_t *n_launches, double *total_ms, double *total_bytes) {
  if (!t || !n_launches || !total_ms || !total_bytes) return TRISPEC_ENULL;
  double ms = 0;
  for (int i = 0; i < t->count; ++i) {
    float e = 0.f;
    if (hipEventElapsedTime(&e, t->start[i], t->stop[i]) != hipSuccess) return TRISPEC_ELAUNCH;
    ms += e;
  }
  *n_launches = t->count;
  *total_ms = ms;
  *total_bytes = t->bytes;
  return TRISPEC_OK;
}

int trispec_timer_destroy(trispec_timer *t) {
  if (!t) return TRISPEC_OK;
  for (size_t i = 0; i < t->start.size(); ++i) {
    (void)hipEventDestroy(t->start[i]);
    (void)hipEventDestroy(t->stop[i]);
  }
  delete t;
  return TRISPEC_OK;
}

int trispec_kv_commit(trispec_kv *kv, const int32_t *nodes_host, const int32_t *n_commit_host, void *stream) {
  if (!kv || !nodes_host || !n_commit_host) return TRISPEC_ENULL;
  const trispec_model_config &c = kv->model->cfg;
  CommitTable t;
  memset(&t, 0, sizeof(t));
  int any = 0;
  for (int b = 0; b < kv->batch; ++b) {
    const int n = n_commit_host[b];
    if (n < 0 || n > kMaxNodes) return TRISPEC_ENODES;
    const int32_t *p = nodes_host + (size_t)b * TRISPEC_PATH_STRIDE;
    for (int i = 0; i < n; ++i) {
      if (p[i] < 0 || p[i] >= kMaxNodes || (i > 0 && p[i] <= p[i - 1])) return TRISPEC_ETREE;
      t.node[b][i] = (uint8_t)p[i];
    }
    if (n > 0 && kv->ctx_len[b] + p[n - 1] >= kv->capacity) return TRISPEC_ECAPACITY;
    t.n[b] = n;
    t.ctx[b] = kv->ctx_len[b];
    any |= n;
  }
  if (any) {
    (void)hipGetLastError();
    launch_kv_commit((hipStream_t)stream, c.dtype, kv->k, kv->v, c.n_layers, kv->layer_elems(), kv->batch, kv->map(),
                     t);
    if (hipGetLastError() != hipSuccess) return TRISPEC_ELAUNCH;
  }
  for (int b = 0; b < kv->batch; ++b) kv->ctx_len[b] += t.n[b];
  return TRISPEC_OK;
}

int trispec_draft_ranks(const float *logits, const int32_t *draft_tokens, const int32_t *tree_parents, int32_t batch,
                        int32_t n_nodes, int32_t vocab, int32_t *ranks, void *stream) {
  if (!logits || !draft_tokens || !tree_parents || !ranks) return TRISPEC_ENULL;
  if (batch < 1 || batch > kMaxBatch || n_nodes < 1 || n_nodes > kMaxNodes || batch * n_nodes > kMaxRows)
    return TRISPEC_ENODES;
  if (vocab < 1) return TRISPEC_EARG;
  NodeTable tab;
  memset(&tab, 0, sizeof(tab));
  const int rc = build_nodes(tree_parents, batch, n_nodes, 1, tab);
  if (rc) return rc;
  (void)hipGetLastError();
  launch_draft_ranks((hipStream_t)stream, logits, draft_tokens, tab, batch, n_nodes, vocab, ranks);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

int trispec_debug_set_spin_limit(uint64_t ticks) {
  g_spin_limit = ticks ? ticks : 200000000ull;
  return TRISPEC_OK;
}

int trispec_wait_probe(int32_t *counter_dev, int32_t expect, uint64_t limit_ticks, int32_t *abort_dev,
                       int32_t *status_dev, void *stream) {
  if (!counter_dev || !abort_dev || !status_dev) return TRISPEC_ENULL;
  (void)hipGetLastError();
  launch_wait_probe((hipStream_t)stream, counter_dev, expect, limit_ticks, abort_dev, status_dev);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

int trispec_prune_reroot(const int32_t *tokens, const int32_t *parents, const int32_t *positions, int32_t n_nodes,
                         const int32_t *path, int32_t path_len, const int32_t *prefix_tokens, int32_t n_prefix,
                         int32_t prefix_pos0, int32_t *out_tokens, int32_t *out_parents, int32_t *out_positions,
                         int32_t *out_old_id, int32_t *out_n_nodes, int32_t *out_n_forced) {
  if (!tokens || !parents || !positions || !path || !out_tokens || !out_parents || !out_positions || !out_old_id ||
      !out_n_nodes || !out_n_forced || (n_prefix > 0 && !prefix_tokens))
    return TRISPEC_ENULL;
  if (n_prefix < 0 || path_len < 1) return TRISPEC_EARG;
  if (n_nodes < 1 || n_nodes > kMaxNodes || path_len > n_nodes) return TRISPEC_ENODES;
  if (parents[0] != -1) return TRISPEC_ETREE;
  for (int i = 1; i < n_nodes; ++i)
    if (parents[i] < 0 || parents[i] >= i) return TRISPEC_ETREE;
  if (path[0] != 0) return TRISPEC_ETREE;
  for (int i = 1; i < path_len; ++i)
    if (path[i] <= 0 || path[i] >= n_nodes || parents[path[i]] != path[i - 1]) return TRISPEC_ETREE;
  // kept nodes: the path, then every descendant of its last node in ascending id order
  // (parents[i] < i, so one ascending sweep marks the whole subtree)
  int keep[kMaxNodes], new_id[kMaxNodes], n_keep = 0;
  bool below[kMaxNodes];
  for (int i = 0; i < n_nodes; ++i) { below[i] = false; new_id[i] = -1; }
  for (int i = 0; i < path_len; ++i) keep[n_keep++] = path[i];
  const int last = path[path_len - 1];
  below[last] = true;
  for (int i = last + 1; i < n_nodes; ++i)
    if (below[parents[i]]) {
      below[i] = true;
      keep[n_keep++] = i;
    }
  if ((long long)n_prefix + n_keep > kMaxNodes) return TRISPEC_ENODES;
  for (int j = 0; j < n_keep; ++j) new_id[keep[j]] = n_prefix + j;
  for (int j = 0; j < n_prefix; ++j) {
    out_tokens[j] = prefix_tokens[j];
    out_parents[j] = j - 1;
    out_positions[j] = prefix_pos0 + j;
    out_old_id[j] = -1;
  }
  for (int j = 0; j < n_keep; ++j) {
    const int old = keep[j], o = n_prefix + j;
    out_tokens[o] = tokens[old];
    out_parents[o] = j == 0 ? n_prefix - 1 : new_id[parents[old]];
    out_positions[o] = positions[old];
    out_old_id[o] = old;
  }
  *out_n_nodes = n_prefix + n_keep;
  *out_n_forced = n_prefix + path_len;
  return TRISPEC_OK;
}

int trispec_copy_probe(void *dst_dev, const void *src_dev, size_t bytes, void *stream) {
  if (!dst_dev || !src_dev) return TRISPEC_ENULL;
  if (bytes == 0 || bytes % 16 || ((((uintptr_t)dst_dev) | ((uintptr_t)src_dev)) & 15)) return TRISPEC_EARG;
  (void)hipGetLastError();
  launch_copy_probe((hipStream_t)stream, dst_dev, src_dev, bytes);
  return hipGetLastError() == hipSuccess ? TRISPEC_OK : TRISPEC_ELAUNCH;
}

const char *trispec_strerror(int code) {
  switch (code) {
    case TRISPEC_OK: return "ok";
    case TRISPEC_ENULL: return "a required pointer is NULL";
    case TRISPEC_ESHAPE: return "model shape not supported";
    case TRISPEC_ENODES: return "n_nodes or batch out of range";
    case TRISPEC_ETREE: return "tree_parents is not a topologically ordered tree";
    case TRISPEC_EFORCED: return "n_forced out of range or forced nodes are not a chain";
    case TRISPEC_ECAPACITY: return "ctx_len + n_nodes exceeds the cache capacity";
    case TRISPEC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case TRISPEC_EARG: return "invalid argument";
    case TRISPEC_EMISMATCH: return "kv cache belongs to another model";
    case TRISPEC_ELAUNCH: return "HIP launch failed";
    case TRISPEC_ESTATE: return "bf16 model has not been packed (trispec_model_pack)";
    default: return "unknown error";
  }
}

}  // extern "C"
