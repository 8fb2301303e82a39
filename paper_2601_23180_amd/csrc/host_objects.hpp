// The objects behind the opaque handles of the C ABI (host memory only).
#pragma once
#include <vector>

#include "internal.hpp"

struct trispec_model {
  trispec_model_config cfg;
  const void *embed, *lm_head, *final_norm;
  std::vector<const void *> wq, wk, wv, wo, w_gate, w_up, w_down, norm_attn, norm_ffn, q_norm, k_norm;
  // bf16 models: packed copies of the matrices (device, inside the caller's pack buffer)
  bool packed;
  int layer_grid[3][2];   // largest resident grid of the layer kernel for rows_pad 32 / 64 / 128 and ring depth 8 / 4 (-1: not asked yet)
  const void *p_lm_head;
  std::vector<const void *> p_wq, p_wk, p_wv, p_wo, p_gate, p_up, p_down;
};

struct trispec_kv {
  const trispec_model *model;
  void *k, *v;
  int32_t batch, capacity;
  int32_t ctx_len[ts::kMaxBatch];
  // paged cache: device page table [batch][max_pages] and the pool size; contiguous cache: nullptr, 0, 0
  const int32_t *page_table;
  int32_t max_pages, n_pages;
  // elements of one layer of K (= of V), and the slot map the kernels address the cache through
  size_t layer_elems() const {
    const trispec_model_config &c = model->cfg;
    return (page_table ? (size_t)n_pages * ts::kKvPage : (size_t)batch * capacity) * c.n_kv_heads * c.head_dim;
  }
  ts::KvMap map() const {
    return ts::KvMap{page_table, max_pages, n_pages, capacity, model->cfg.n_kv_heads, model->cfg.head_dim};
  }
};

struct trispec_timer {
  int32_t kernel_class, capacity, count;
  double bytes;
  std::vector<hipEvent_t> start, stop;
};
