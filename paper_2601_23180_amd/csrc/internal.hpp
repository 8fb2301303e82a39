// Internal declarations shared by the host orchestration (api.cpp) and the kernel
// translation units.  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "trispec.h"

namespace ts {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kMaxRows = TRISPEC_MAX_ROWS;
constexpr int kMaxBatch = TRISPEC_MAX_BATCH;
constexpr int kMaxNodes = TRISPEC_MAX_NODES;
constexpr int kMaxChain = 64;        // nodes of a chain in the sampling form (one lane of a wavefront per node)
constexpr int kMaxGroup = 8;         // query heads per kv head (bf16 attention)
constexpr int kMaxSplitK = 32;       // k-splits of one matmul
constexpr int kMaxAttnSplits = 64;   // context splits of one attention call
constexpr int kAttnWideMinKeys = 6144;   // longest context from which trees of > 128 rows take 256-row workgroups
constexpr int kGemmTileN = 128;      // output columns per workgroup (4 waves x 32)

// Per-call node table, passed to the set-up kernel by value (1 KB of kernel arguments).
struct NodeTable {
  int32_t parent[kMaxRows];
};
// Root path of a node as a bit set over the nodes of its sequence: bit j set <=> node j is an
// ancestor of the node or the node itself.  Built by the set-up kernel from the parents.
// (two named words, selected by comparison: an array indexed by a run-time value would live in
// scratch memory)
struct AncMask {
  uint64_t lo, hi;   // nodes 0..63, nodes 64..127
  static_assert(kMaxNodes == 128, "two mask words");
  __device__ __forceinline__ bool has(int j) const { return (((j < 64) ? lo : hi) >> (j & 63)) & 1ull; }
  __device__ __forceinline__ void set(int j) {
    const uint64_t bit = 1ull << (j & 63);
    if (j < 64) lo |= bit; else hi |= bit;
  }
  __device__ __forceinline__ int count() const { return __popcll(lo) + __popcll(hi); }
  __device__ __forceinline__ int rank(int j) const {   // members below j
    const uint64_t below = (1ull << (j & 63)) - 1ull;
    return j < 64 ? __popcll(lo & below) : __popcll(lo) + __popcll(hi & below);
  }
};

struct CtxLens {
  int32_t v[kMaxBatch];
};

// Per (row, column tile) statistics of the LM-head logits.
struct HeadStats {
  float *l1;      // largest logit
  float *l2;      // second largest logit (-inf if none)
  float *sumexp;  // sum over the tile of exp(logit - l1)
  float *ent;     // sum over the tile of exp(logit - l1) * (logit - l1)   (entropy = ln sum - ent / sum)
  int32_t *idx;   // column of l1 (lowest column among equals)
  int32_t n_tiles;
};

// One weight-streaming matmul  y[r][col] = sum_k X[r][k] * W[col][k]  (see kernels_gemm.hip).
// Where the slots of a sequence live inside ONE layer of the cache.  Contiguous cache:
// K [B][nkv][capacity][d], V^T [B][nkv][d][capacity].  Paged cache: pages of kKvPage slots,
// K [n_pages][nkv][kKvPage][d], V^T [n_pages][nkv][d][kKvPage]; slot s of sequence b is slot
// s % kKvPage of page page_table[b][s / kKvPage].  All results are element offsets from the layer's base.
constexpr int kKvPage = 256;
struct KvMap {
  const int32_t *page_table;   // device [batch][max_pages], or nullptr: contiguous
  int32_t max_pages, n_pages;  // page ids are clamped into [0, n_pages): a bad table reads the wrong page, not foreign memory
  int32_t capacity;            // slots per sequence
  int32_t n_kv, d;
  __device__ __forceinline__ int page_of(int b, int slot) const {
    const int p = page_table[(size_t)b * max_pages + min(slot / kKvPage, max_pages - 1)];
    return min(max(p, 0), n_pages - 1);
  }
  __device__ __forceinline__ size_t k_row(int b, int h, int slot) const {          // K[slot][0]
    if (!page_table) return (((size_t)b * n_kv + h) * capacity + slot) * d;
    const int page = page_of(b, slot);
    return (((size_t)page * n_kv + h) * kKvPage + (slot % kKvPage)) * d;
  }
  __device__ __forceinline__ size_t v_col(int b, int h, int slot) const {          // V^T[0][slot]; feature f is f * v_stride() further
    if (!page_table) return ((size_t)b * n_kv + h) * d * capacity + slot;
    const int page = page_of(b, slot);
    return ((size_t)page * n_kv + h) * d * kKvPage + (slot % kKvPage);
  }
  __device__ __forceinline__ size_t v_stride() const { return page_table ? (size_t)kKvPage : (size_t)capacity; }
};

struct GemmSeg {
  const void *w;   // bf16 models: the PACKED copy of the [n_rows, K] matrix; fp32: the matrix
  int32_t n_rows;
  int32_t col0;    // first output column of this segment
};
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3, EPI_PLAIN = 4 };
struct GemmArgs {
  // fp32 reference-precision path: x is [rows_pad, K] fp32, out is [rows][n_total].
  // bf16 path: x is the bf16 hi panel [rows_pad, K], the lo panel follows x_panel elements later.
  // ss_in (or nullptr): [ss_tiles][rows_pad] sums of squares of the rows of the un-normalised
  // input; the epilogue multiplies the reduced sums by 1/sqrt(sum/K + eps).
  const void *x;
  size_t x_panel;
  const float *ss_in;
  int32_t ss_tiles;
  GemmSeg seg[3];
  int32_t n_seg;
  int32_t n_total;     // total output columns (SWIGLU: 2 * ffn)
  int32_t k;           // reduction length
  int32_t rows;        // valid rows
  int32_t rows_pad;    // 32, 64, 128 or 256
  int32_t k_per_split; // multiple of 64
  int32_t n_splits;
  int32_t n_tiles;
  int32_t tile_n;      // output columns per workgroup (128)
  int32_t epi;
  float *out;          // fp32 path, and the PLAIN epilogue: [rows][n_total] fp32
  const float *bias;   // PLAIN epilogue / fp32 path: [n_total] added to every row, or nullptr
  float *part;         // [n_splits][n_tiles][rows_pad][128] split-K partial tiles
  int32_t *counters;   // [n_tiles + 1], zero between launches
  // QKV epilogue
  const float *cos_t, *sin_t;
  float *qkv_f32;      // [rows][n_total] rotated q, k and v in fp32
  void *q_out;         // bf16 hi/lo panels [rows_pad][nq*d] of the rotated queries
  size_t q_panel;
  void *k_cache, *v_cache;
  const void *q_norm_w, *k_norm_w;   // [head_dim] each, or nullptr: no per-head norm of q / k
  CtxLens ctx;
  int32_t n_nodes, n_q_heads, n_kv_heads, head_dim;
  KvMap kv;
  // RESID epilogue
  const float *x_resid;  // [rows_pad][n_total] residual stream before this matmul
  float *x_resid_out;  // the same after it (may be x_resid itself: every element is read and written by one thread)
  void *xw_out;        // bf16 hi/lo panels [rows_pad][n_total]: x * next norm weight
  const void *next_norm_w;  // bf16 [n_total]
  float *ss_part;      // [n_tiles][rows_pad] sums of squares of the updated rows, per tile
  float eps;
  size_t out_panel;    // panel stride (elements) of xw_out / act_out
  // SWIGLU epilogue
  void *act_out;       // bf16 hi/lo panels [rows_pad][ffn]
  int32_t ffn;
  // HEAD epilogue
  HeadStats hs;
  float *debug_logits;
};

// The matmuls between two attention calls as phases of one launch (kernels_layer.hip): O
// projection, gate + up, down projection and, unless this is the last layer, the next layer's QKV.
constexpr int kLayerPhases = 4;
struct LayerArgs {
  GemmArgs ph[kLayerPhases];
  int32_t n_phases;               // 3 or 4
  int32_t ring_depth;             // 8 or 4 weight chunks in flight per wavefront (see layer_step)
  int32_t *bar;                   // [n_phases] arrival counters of this launch, zero at its start
  int32_t *abort_word;            // sticky: a wait has expired somewhere in this pass
  int32_t *status;                // status word of the pass
  unsigned long long spin_limit;  // longest wait at a barrier, in ticks of the 100 MHz wall clock
  unsigned long long *stamps;     // optional [16]: wall clock of workgroup stamp_wg at the phase boundaries
  int32_t stamp_wg;
  int32_t poll_naps;              // naps of 512 clocks between two polls of a barrier counter
};
// k granularity of a (tile, split) item of the layer kernel: ring depth x chunk depth
inline int layer_step(int rows_pad, int ring_depth) { return ring_depth * (rows_pad <= 64 ? 128 : 64); }
int layer_kernel_max_grid(const LayerArgs &la);
bool launch_layer_bf16(hipStream_t st, const LayerArgs &la, int grid);
// `counter` never reaches `expect`: one workgroup waits `limit` ticks, then reports (test hook)
void launch_wait_probe(hipStream_t st, int32_t *counter, int expect, unsigned long long limit,
                       int32_t *abort_word, int32_t *status);

struct AttnArgs {
  const void *q;        // fp32 path: [rows_pad, nq*d] fp32 queries; bf16 path: bf16 hi panel, lo q_panel later
  size_t q_panel;
  int32_t rows_per_wg;  // query rows (group * n_nodes of them per kv head) one workgroup covers: 128 or 256
  int32_t n_row_groups; // ceil(group * n_nodes / rows_per_wg)
  const void *k_cache;  // this layer's K and V^T, addressed through `kv`
  const void *v_cache;
  KvMap kv;
  const AncMask *anc;   // [B*M]
  const float *qkv;     // [B*M][(nq + 2 nkv) * d] this layer's q, k (rotated) and v in fp32
  CtxLens ctx;
  int32_t batch, n_nodes, n_q_heads, n_kv_heads, head_dim;
  int32_t keys_per_split;   // multiple of 64
  int32_t n_splits;
  float *part_o;        // [B][nkv][n_splits][group*M][d]  unnormalised
  float *part_m;        // [B][nkv][n_splits][group*M]     running max
  float *part_l;        // [B][nkv][n_splits][group*M]     sum of exp
  void *out;            // fp32 path: [rows_pad, nq*d] fp32; bf16 path: bf16 hi/lo panels
  size_t out_panel;     // panel stride (elements) of out
};

constexpr int kSampleChunk = 4096;   // tokens per chunk of the inverse-CDF draw
constexpr int kSampleMaxVocab = kSampleChunk * 1024;   // one thread of the pick kernel per chunk
// Sampling-mode decision on a chain (kernels_sample.hip).  rows = batch * n_nodes.
struct SampleArgs {
  const float *logits;      // [rows, vocab]
  const int32_t *tokens;    // [rows]
  const float *p_draft;     // [batch, n_nodes - 1, vocab]
  const float *u_accept;    // [rows]
  const float *u_sample;    // [batch]
  int32_t batch, n_nodes, vocab, n_forced, criterion, resample;
  float inv_temp, threshold;
  // scratch
  double *row_z;            // [rows] sum exp((l - max) / T)
  float *row_l1, *row_l2;   // [rows] largest and second-largest logit
  int32_t *row_idx;         // [rows] argmax
  float *cs_l1, *cs_l2;     // [rows][n_chunks] per chunk of kSampleChunk tokens: largest / second-largest logit,
  int32_t *cs_idx;          //                  argmax,
  double *cs_z;             //                  sum exp((l - chunk max) / T)
  int32_t *seq_bad;         // [batch] 1: a draft token id of the sequence is outside the vocabulary
  int32_t *sel_row, *sel_mode;   // [batch] node whose distribution yields the token; 0 none, 1 direct, 2 residual
  double *chunk_sum;        // [batch][2][n_chunks] mass per chunk of kSampleChunk tokens: tempered p_v, residual
  int32_t n_chunks;
  trispec_verify_out out;
};
void launch_sample_decide(hipStream_t st, const SampleArgs &a);

struct DecideArgs {
  const int32_t *tokens;   // device [B*M]
  const int32_t *parent;   // device [B*M] (workspace copy)
  int32_t batch, n_nodes, n_forced, criterion;
  float threshold;
  // per-node statistics (workspace)
  float *node_l1, *node_l2, *node_sum, *node_ent;
  int32_t *node_idx;
  const int32_t *draft_ranks;   // [B*M] or nullptr: rank of each node's token in its parent's distribution
  int32_t accept_top_k;         // > 1: a child is followed when its rank is below it (needs draft_ranks)
  const int32_t *status_src;   // device status word of the pass (workspace)
  trispec_verify_out out;
};

// ---- launchers (one per kernel family); all enqueue on `st` and return nothing:
// the caller checks hipGetLastError once at the end of the pass.
void launch_setup(hipStream_t st, const NodeTable &tab, int rows, int n_nodes, AncMask *anc, int32_t *parent,
                  int32_t *status, int32_t *zero, int n_zero);
void launch_rope_table(hipStream_t st, const int32_t *positions, int rows, int head_dim, float base,
                       float *cos_t, float *sin_t);
void launch_embed_norm(hipStream_t st, int dtype, const int32_t *tokens, const void *embed,
                       const void *norm_w, int rows, int hidden, int vocab, float eps, float *x,
                       void *h, size_t h_panel, float *ss_out, int32_t *status);
// nodes / counts of a commit, by value
struct CommitTable {
  uint8_t node[kMaxBatch][kMaxNodes];
  int32_t n[kMaxBatch];
  int32_t ctx[kMaxBatch];
};
void launch_kv_commit(hipStream_t st, int dtype, void *k_cache, void *v_cache, int n_layers, size_t layer_elems,
                      int batch, const KvMap &kv, const CommitTable &t);
void launch_copy_probe(hipStream_t st, void *dst, const void *src, size_t bytes);
// out[r][c] = x[r][c] * rstd(r) * w[c]; rstd from the per-tile sums of squares ss[tile][rows_pad]
// (ss == nullptr: x is already normalised and weighted, plain copy)
void launch_export_hidden(hipStream_t st, int dtype, const float *x, const void *norm_w, const float *ss,
                          int ss_tiles, int rows, int rows_pad, int hidden, float eps, float *out);
void launch_zero_counters(hipStream_t st, int32_t *counters, int n_counters);
void launch_qkv_epilogue(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                         int rows_pad, int n_q_heads, int n_kv_heads, int head_dim,
                         const float *cos_t, const float *sin_t, int n_nodes, CtxLens ctx,
                         const KvMap &kvm, void *q_out, void *k_cache, void *v_cache, const float *q_norm_w,
                         const float *k_norm_w, float eps);
void launch_reduce_residual_norm(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                                 int rows_pad, int hidden, const void *norm_w, float eps, float *x,
                                 void *h);
void launch_reduce_swiglu(hipStream_t st, int dtype, const float *part, int n_splits, int rows,
                          int rows_pad, int ffn, void *act);
void launch_gemm_f32(hipStream_t st, const GemmArgs &a);
size_t packed_weight_bytes(int n_rows, int k);
void launch_pack_weights(hipStream_t st, const void *w, int n_rows, int k, void *out);
void launch_gemm_bf16(hipStream_t st, const GemmArgs &a);   // 4 wavefronts, 128-column tiles
void launch_stats_from_logits(hipStream_t st, const float *logits, int rows, int vocab,
                              const HeadStats &hs);
void launch_attn_f32(hipStream_t st, const AttnArgs &a);
void launch_attn_bf16(hipStream_t st, const AttnArgs &a);
void launch_stats_reduce(hipStream_t st, const HeadStats &hs, int rows, float *node_l1, float *node_l2,
                         float *node_sum, float *node_ent, int32_t *node_idx);
// rank[r] of node r > 0 of every sequence: vocabulary entries that precede tokens[r] in the logits of
// its parent's row (larger, or equal with a lower id); -1 for roots and token ids outside the vocabulary
void launch_draft_ranks(hipStream_t st, const float *logits, const int32_t *tokens, const NodeTable &tab,
                        int batch, int n_nodes, int vocab, int32_t *ranks);
void launch_decide(hipStream_t st, const DecideArgs &a);

}  // namespace ts
