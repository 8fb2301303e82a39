// Round driver of the ternary scheme (Algorithm 1; Sec. 3.2 Cases I / II, Eq. 10): the greedy form on
// draft trees and the sampling form on draft chains.  Host control flow over a few dozen integers per round: every model pass is one
// trispec_verify call, every cache update one trispec_kv_commit call, the Case II hand-over one
// trispec_prune_reroot call.  Each pass is followed by a copy of its decision to the host and a
// stream synchronisation, because which model runs next is decided from it.
#include <string.h>

#include <new>
#include <vector>

#include "host_objects.hpp"

using namespace ts;

struct trispec_ternary {
  trispec_ternary_config cfg;
  std::vector<int32_t> seq;   // the emitted sequence, prompt included; its last token is the next root
  bool started;
};

namespace {

// layout of the device scratch (int32 units)
constexpr int kOffTok = 0, kOffPos = kMaxNodes, kOffDec = 2 * kMaxNodes;   // decision: len, token, escalate, status, path[]
constexpr int kDecInts = 4 + kMaxNodes;
constexpr int kOffU = kOffDec + kDecInts;   // sampling form: u_accept[kMaxNodes], u_sample (floats)
static_assert(kOffU + kMaxNodes + 1 <= TRISPEC_TERNARY_SCRATCH_INTS, "scratch too small");

struct Side {
  trispec_model *model;
  trispec_kv *kv;
  void *ws;
  size_t ws_bytes;
};
Side side(const trispec_ternary *t, bool target) {
  const trispec_ternary_config &c = t->cfg;
  return target ? Side{c.target, c.kv_target, c.workspace_target, c.workspace_target_bytes}
                : Side{c.proxy, c.kv_proxy, c.workspace_proxy, c.workspace_proxy_bytes};
}

int fetch_decision(trispec_ternary *t, trispec_pass_result *r);

// One pass of one model over (tokens, parents, positions) and its decision, on the host.
int run_pass(trispec_ternary *t, bool target, const int32_t *tokens, const int32_t *parents, const int32_t *positions,
             int n, float lambda, int criterion, int n_forced, trispec_pass_result *r) {
  const Side s = side(t, target);
  hipStream_t st = (hipStream_t)t->cfg.stream;
  int32_t *d = t->cfg.scratch_dev;
  if (hipMemcpyAsync(d + kOffTok, tokens, sizeof(int32_t) * n, hipMemcpyHostToDevice, st) != hipSuccess ||
      hipMemcpyAsync(d + kOffPos, positions, sizeof(int32_t) * n, hipMemcpyHostToDevice, st) != hipSuccess)
    return TRISPEC_ELAUNCH;
  trispec_verify_opts o;
  memset(&o, 0, sizeof o);
  o.criterion = criterion;
  o.n_forced = n_forced;
  o.workspace = s.ws;
  o.workspace_bytes = s.ws_bytes;
  o.stream = t->cfg.stream;
  trispec_verify_out out;
  memset(&out, 0, sizeof out);
  out.accepted_len = d + kOffDec;
  out.token = d + kOffDec + 1;
  out.escalate = d + kOffDec + 2;
  out.status = d + kOffDec + 3;
  out.path = d + kOffDec + 4;
  const int rc = trispec_verify(s.model, s.kv, d + kOffTok, parents, d + kOffPos, n, lambda, &o, &out);
  if (rc != TRISPEC_OK) return rc;
  return fetch_decision(t, r);
}

// Host copy of the decision a pass left in the device scratch (after a stream synchronisation).
int fetch_decision(trispec_ternary *t, trispec_pass_result *r) {
  hipStream_t st = (hipStream_t)t->cfg.stream;
  int32_t h[kDecInts];
  if (hipMemcpyAsync(h, t->cfg.scratch_dev + kOffDec, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return TRISPEC_ELAUNCH;
  r->accepted_len = h[0];
  r->token = h[1];
  r->escalate = h[2];
  r->status = h[3];
  r->path_len = 0;
  for (int i = 0; i < kMaxNodes; ++i) {
    r->path[i] = h[4 + i];
    if (h[4 + i] >= 0 && r->path_len == i) r->path_len = i + 1;
  }
  return r->status ? TRISPEC_EARG : TRISPEC_OK;
}

// Sampling form: one pass over a chain with its logits kept, then the temperature > 0 decision on them.
int run_pass_sample(trispec_ternary *t, bool target, const int32_t *tokens, int pos0, int n, const float *p_draft,
                    const float *u_accept, float u_sample, float lambda, int criterion, int n_forced,
                    const trispec_sample_round *sr, trispec_pass_result *r) {
  const Side s = side(t, target);
  hipStream_t st = (hipStream_t)t->cfg.stream;
  int32_t *d = t->cfg.scratch_dev;
  int32_t parents[kMaxNodes], positions[kMaxNodes];
  float u[kMaxNodes + 1];
  for (int i = 0; i < n; ++i) {
    parents[i] = i - 1;
    positions[i] = pos0 + i;
    u[i] = u_accept[i];
  }
  u[kMaxNodes] = u_sample;
  if (hipMemcpyAsync(d + kOffTok, tokens, sizeof(int32_t) * n, hipMemcpyHostToDevice, st) != hipSuccess ||
      hipMemcpyAsync(d + kOffPos, positions, sizeof(int32_t) * n, hipMemcpyHostToDevice, st) != hipSuccess ||
      hipMemcpyAsync(d + kOffU, u, sizeof u, hipMemcpyHostToDevice, st) != hipSuccess)
    return TRISPEC_ELAUNCH;
  trispec_verify_opts o;
  memset(&o, 0, sizeof o);
  o.criterion = TRISPEC_CRIT_MARGIN;
  o.n_forced = n_forced;
  o.workspace = s.ws;
  o.workspace_bytes = s.ws_bytes;
  o.stream = t->cfg.stream;
  o.debug_logits = sr->logits_dev;
  trispec_verify_out none;
  memset(&none, 0, sizeof none);
  int rc = trispec_verify(s.model, s.kv, d + kOffTok, parents, d + kOffPos, n, 0.0f, &o, &none);
  if (rc != TRISPEC_OK) return rc;
  trispec_sample_opts so;
  memset(&so, 0, sizeof so);
  so.temperature = sr->temperature;
  so.resample = sr->resample;
  so.criterion = criterion;
  so.n_forced = n_forced;
  so.p_draft = p_draft;
  so.u_accept = (const float *)(d + kOffU);
  so.u_sample = (const float *)(d + kOffU + kMaxNodes);
  so.stream = t->cfg.stream;
  trispec_verify_out out;
  memset(&out, 0, sizeof out);
  out.accepted_len = d + kOffDec;
  out.token = d + kOffDec + 1;
  out.escalate = d + kOffDec + 2;
  out.status = d + kOffDec + 3;
  out.path = d + kOffDec + 4;
  rc = trispec_sample_decide_static(sr->logits_dev, d + kOffTok, 1, n, s.model->cfg.vocab, lambda, &so, &out);
  if (rc != TRISPEC_OK) return rc;
  return fetch_decision(t, r);
}

int commit(trispec_ternary *t, bool target, const std::vector<int32_t> &nodes) {
  int32_t arr[TRISPEC_PATH_STRIDE];
  memset(arr, 0, sizeof arr);
  const int32_t cnt = (int32_t)nodes.size();
  if (cnt > kMaxNodes) return TRISPEC_ENODES;
  for (int i = 0; i < cnt; ++i) arr[i] = nodes[i];
  return trispec_kv_commit(side(t, target).kv, arr, &cnt, t->cfg.stream);
}

// Plain passes over tokens that are certain: a forced chain, everything committed.
int ingest(trispec_ternary *t, bool target, const int32_t *tokens, int n_tokens, int *n_passes) {
  const Side s = side(t, target);
  int32_t parents[kMaxNodes], positions[kMaxNodes];
  std::vector<int32_t> all;
  for (int done = 0; done < n_tokens;) {
    const int n = n_tokens - done < t->cfg.max_nodes ? n_tokens - done : t->cfg.max_nodes;
    const int c = s.kv->ctx_len[0];
    all.clear();
    for (int i = 0; i < n; ++i) {
      parents[i] = i - 1;
      positions[i] = c + i;
      all.push_back(i);
    }
    trispec_pass_result r;
    int rc = run_pass(t, target, tokens + done, parents, positions, n, 0.0f, TRISPEC_CRIT_MARGIN, n, &r);
    if (rc == TRISPEC_OK) rc = commit(t, target, all);
    if (rc != TRISPEC_OK) return rc;
    done += n;
    if (n_passes) ++*n_passes;
  }
  return TRISPEC_OK;
}

bool tokens_ok(const trispec_ternary *t, const int32_t *tok, int n) {
  const int v = t->cfg.proxy->cfg.vocab;
  for (int i = 0; i < n; ++i)
    if (tok[i] < 0 || tok[i] >= v) return false;
  return true;
}

}  // namespace

extern "C" {

int trispec_ternary_create(const trispec_ternary_config *cfg, trispec_ternary **out) {
  if (!cfg || !out || !cfg->proxy || !cfg->target || !cfg->kv_proxy || !cfg->kv_target || !cfg->scratch_dev)
    return TRISPEC_ENULL;
  if (cfg->max_nodes < 1 || cfg->max_nodes > kMaxNodes || cfg->kv_proxy->batch != 1 || cfg->kv_target->batch != 1)
    return TRISPEC_ENODES;
  if (cfg->kv_proxy->model != cfg->proxy || cfg->kv_target->model != cfg->target ||
      cfg->proxy->cfg.vocab != cfg->target->cfg.vocab)
    return TRISPEC_EMISMATCH;
  if (cfg->criterion != TRISPEC_CRIT_MARGIN && cfg->criterion != TRISPEC_CRIT_TOP1 && cfg->criterion != TRISPEC_CRIT_ENTROPY)
    return TRISPEC_EARG;
  size_t need_p = 0, need_t = 0;
  int rc = trispec_workspace_bytes(cfg->proxy, 1, cfg->max_nodes, &need_p);
  if (rc == TRISPEC_OK) rc = trispec_workspace_bytes(cfg->target, 1, cfg->max_nodes, &need_t);
  if (rc != TRISPEC_OK) return rc;
  if (!cfg->workspace_proxy || !cfg->workspace_target || cfg->workspace_proxy_bytes < need_p ||
      cfg->workspace_target_bytes < need_t)
    return TRISPEC_EWORKSPACE;
  trispec_ternary *t = new (std::nothrow) trispec_ternary;
  if (!t) return TRISPEC_ENULL;
  t->cfg = *cfg;
  t->started = false;
  *out = t;
  return TRISPEC_OK;
}

int trispec_ternary_destroy(trispec_ternary *t) {
  delete t;
  return TRISPEC_OK;
}

int trispec_ternary_start(trispec_ternary *t, const int32_t *prompt_host, int32_t n_prompt) {
  if (!t || !prompt_host) return TRISPEC_ENULL;
  if (n_prompt < 1 || !tokens_ok(t, prompt_host, n_prompt)) return TRISPEC_EARG;
  const int32_t zero = 0;
  int rc = trispec_kv_set_len(t->cfg.kv_proxy, &zero);
  if (rc == TRISPEC_OK) rc = trispec_kv_set_len(t->cfg.kv_target, &zero);
  if (rc != TRISPEC_OK) return rc;
  t->started = false;
  t->seq.assign(prompt_host, prompt_host + n_prompt);
  rc = ingest(t, false, t->seq.data(), n_prompt - 1, nullptr);
  if (rc == TRISPEC_OK) rc = ingest(t, true, t->seq.data(), n_prompt - 1, nullptr);
  if (rc != TRISPEC_OK) return rc;
  t->started = true;
  return TRISPEC_OK;
}

int trispec_ternary_resume(trispec_ternary *t, const int32_t *seq_host, int32_t n_seq) {
  if (!t || !seq_host) return TRISPEC_ENULL;
  if (n_seq < 1 || !tokens_ok(t, seq_host, n_seq) || t->cfg.kv_proxy->ctx_len[0] != n_seq - 1 ||
      t->cfg.kv_target->ctx_len[0] > n_seq - 1)
    return TRISPEC_EARG;
  t->seq.assign(seq_host, seq_host + n_seq);
  t->started = true;
  return TRISPEC_OK;
}

int trispec_ternary_sequence(const trispec_ternary *t, const int32_t **tokens_host, int32_t *n_tokens) {
  if (!t || !tokens_host || !n_tokens) return TRISPEC_ENULL;
  *tokens_host = t->seq.data();
  *n_tokens = (int32_t)t->seq.size();
  return TRISPEC_OK;
}

int trispec_ternary_round(trispec_ternary *t, const int32_t *parents_host, const int32_t *tokens_host, int32_t n_nodes,
                          float lambda, trispec_round_info *info_host) {
  if (!t || !parents_host || !tokens_host) return TRISPEC_ENULL;
  if (!t->started) return TRISPEC_ESTATE;
  if (n_nodes < 1 || n_nodes > t->cfg.max_nodes) return TRISPEC_ENODES;
  if (parents_host[0] != -1) return TRISPEC_ETREE;
  for (int i = 1; i < n_nodes; ++i)
    if (parents_host[i] < 0 || parents_host[i] >= i) return TRISPEC_ETREE;
  if (!tokens_ok(t, tokens_host + 1, n_nodes - 1)) return TRISPEC_EARG;
  trispec_round_info info;
  memset(&info, 0, sizeof info);
  trispec_kv *kvp = t->cfg.kv_proxy, *kvt = t->cfg.kv_target;

  // ---- the proxy verifies the draft tree (Eq. 5 - 9)
  int32_t tokens[kMaxNodes], positions[kMaxNodes], depth[kMaxNodes];
  const int cp = kvp->ctx_len[0];
  for (int i = 0; i < n_nodes; ++i) {
    tokens[i] = i == 0 ? t->seq.back() : tokens_host[i];
    depth[i] = i == 0 ? 0 : depth[parents_host[i]] + 1;
    positions[i] = cp + depth[i];
  }
  int rc = run_pass(t, false, tokens, parents_host, positions, n_nodes, lambda, t->cfg.criterion, 1, &info.proxy);
  if (rc != TRISPEC_OK) return rc;
  const trispec_pass_result &pr = info.proxy;
  info.escalate = pr.escalate;
  std::vector<int32_t> path(pr.path, pr.path + pr.path_len);
  const size_t before = t->seq.size();

  if (!pr.escalate) {
    // ---- Case I: the proxy's decision stands; its own token ends the round
    rc = commit(t, false, path);
    if (rc != TRISPEC_OK) return rc;
    for (size_t i = 1; i < path.size(); ++i) t->seq.push_back(tokens[path[i]]);
    t->seq.push_back(pr.token);
  } else {
    // ---- Case II: the target verifies the approved path as a forced chain, behind the tokens
    // it has not cached yet, and the subtree under v_tau_m (Eq. 10)
    int32_t s_tok[kMaxNodes], s_par[kMaxNodes], s_pos[kMaxNodes], s_old[kMaxNodes], s_n = 0, s_forced = 0;
    int t_len = kvt->ctx_len[0];
    int n_unseen = (int)t->seq.size() - 1 - t_len;            // seq[t_len .. size-2]
    rc = trispec_prune_reroot(tokens, parents_host, positions, n_nodes, path.data(), (int32_t)path.size(),
                              n_unseen > 0 ? t->seq.data() + t_len : nullptr, n_unseen, t_len, s_tok, s_par, s_pos,
                              s_old, &s_n, &s_forced);
    if (rc == TRISPEC_ENODES || (rc == TRISPEC_OK && s_n > t->cfg.max_nodes)) {
      // does not fit one pass: plain target passes take the lagging tokens in first
      rc = ingest(t, true, t->seq.data() + t_len, n_unseen, &info.catch_up);
      if (rc != TRISPEC_OK) return rc;
      rc = trispec_prune_reroot(tokens, parents_host, positions, n_nodes, path.data(), (int32_t)path.size(), nullptr,
                                0, 0, s_tok, s_par, s_pos, s_old, &s_n, &s_forced);
    }
    if (rc != TRISPEC_OK) return rc;
    rc = run_pass(t, true, s_tok, s_par, s_pos, s_n, 0.0f, TRISPEC_CRIT_MARGIN, s_forced, &info.target);
    if (rc != TRISPEC_OK) return rc;
    const trispec_pass_result &tr = info.target;
    info.target_nodes = s_n;
    info.n_forced_target = s_forced;
    // the target's cache takes the forced chain and what it accepted; the proxy's cache takes the
    // approved path and the drafts the target accepted beyond it (in the proxy tree's node ids)
    std::vector<int32_t> t_nodes, p_nodes(path);
    for (int i = 0; i < s_forced - 1; ++i) t_nodes.push_back(i);
    for (int i = 0; i < tr.path_len; ++i) t_nodes.push_back(tr.path[i]);
    for (int i = 1; i < tr.path_len; ++i) p_nodes.push_back(s_old[tr.path[i]]);
    rc = commit(t, true, t_nodes);
    if (rc == TRISPEC_OK) rc = commit(t, false, p_nodes);
    if (rc != TRISPEC_OK) return rc;
    for (size_t i = 1; i < p_nodes.size(); ++i) t->seq.push_back(tokens[p_nodes[i]]);
    t->seq.push_back(tr.token);
  }
  info.n_emitted = (int32_t)(t->seq.size() - before);
  info.ctx_len_proxy = kvp->ctx_len[0];
  info.ctx_len_target = kvt->ctx_len[0];
  if (info_host) *info_host = info;
  return TRISPEC_OK;
}

int trispec_ternary_round_sample(trispec_ternary *t, const int32_t *tokens_host, int32_t n_nodes, float lambda,
                                 const trispec_sample_round *sr, trispec_round_info *info_host) {
  if (!t || !tokens_host || !sr || !sr->logits_dev || !sr->p_draft_work_dev || !sr->u_accept_proxy_host ||
      !sr->u_accept_target_host || (n_nodes > 1 && !sr->p_draft_dev))
    return TRISPEC_ENULL;
  if (!t->started) return TRISPEC_ESTATE;
  // the sampling decision takes chains of up to kMaxChain nodes: that bounds the draft chain and
  // the target's longer chain (lagging tokens + draft chain) alike
  const int chain_cap = t->cfg.max_nodes < kMaxChain ? t->cfg.max_nodes : kMaxChain;
  if (n_nodes < 1 || n_nodes > chain_cap) return TRISPEC_ENODES;
  if (!tokens_ok(t, tokens_host + 1, n_nodes - 1)) return TRISPEC_EARG;
  trispec_round_info info;
  memset(&info, 0, sizeof info);
  trispec_kv *kvp = t->cfg.kv_proxy, *kvt = t->cfg.kv_target;
  hipStream_t st = (hipStream_t)t->cfg.stream;
  const int M = n_nodes, vocab = t->cfg.proxy->cfg.vocab;
  int32_t tokens[2 * kMaxNodes];
  for (int i = 0; i < M; ++i) tokens[i] = i == 0 ? t->seq.back() : tokens_host[i];

  // ---- the proxy's pass over the chain: Bernoulli acceptance (Eq. 6), trusted prefix (Eq. 8 - 9)
  int rc = run_pass_sample(t, false, tokens, kvp->ctx_len[0], M, sr->p_draft_dev, sr->u_accept_proxy_host,
                           sr->u_sample_proxy, lambda, t->cfg.criterion, 1, sr, &info.proxy);
  if (rc != TRISPEC_OK) return rc;
  const trispec_pass_result &pr = info.proxy;
  info.escalate = pr.escalate;
  std::vector<int32_t> path(pr.path, pr.path + pr.path_len);
  const size_t before = t->seq.size();

  if (!pr.escalate) {                                        // Case I
    rc = commit(t, false, path);
    if (rc != TRISPEC_OK) return rc;
    for (size_t i = 1; i < path.size(); ++i) t->seq.push_back(tokens[path[i]]);
    t->seq.push_back(pr.token);
  } else {                                                   // Case II
    const int tau_m = pr.accepted_len;
    int t_len = kvt->ctx_len[0];
    int u = (int)t->seq.size() - 1 - t_len;                  // tokens the target has not cached yet
    if (u + M > chain_cap) {
      rc = ingest(t, true, t->seq.data() + t_len, u, &info.catch_up);
      if (rc != TRISPEC_OK) return rc;
      t_len = kvt->ctx_len[0];
      u = 0;
    }
    // the target's chain: lagging tokens, then the proxy's chain; draft rows and uniforms shifted by u
    int32_t tok_t[2 * kMaxNodes];
    float ua_t[kMaxNodes];
    for (int i = 0; i < u; ++i) { tok_t[i] = t->seq[t_len + i]; ua_t[i] = 0.f; }
    for (int i = 0; i < M; ++i) { tok_t[u + i] = tokens[i]; ua_t[u + i] = sr->u_accept_target_host[i]; }
    const float *pd_t = sr->p_draft_dev;
    if (u > 0 && M > 1) {
      const size_t row = sizeof(float) * (size_t)vocab;
      if (hipMemsetAsync(sr->p_draft_work_dev, 0, row * u, st) != hipSuccess ||
          hipMemcpyAsync(sr->p_draft_work_dev + (size_t)u * vocab, sr->p_draft_dev, row * (M - 1), hipMemcpyDeviceToDevice,
                         st) != hipSuccess)
        return TRISPEC_ELAUNCH;
      pd_t = sr->p_draft_work_dev;
    } else if (u > 0) {
      pd_t = sr->p_draft_work_dev;                           // no draft rows are read: every node is forced
    }
    const int n_forced = u + tau_m + 1;
    rc = run_pass_sample(t, true, tok_t, t_len, u + M, pd_t, ua_t, sr->u_sample_target, 0.0f, TRISPEC_CRIT_MARGIN,
                         n_forced, sr, &info.target);
    if (rc != TRISPEC_OK) return rc;
    const trispec_pass_result &tr = info.target;
    info.target_nodes = u + M;
    info.n_forced_target = n_forced;
    std::vector<int32_t> t_nodes, p_nodes(path);
    for (int i = 0; i < n_forced - 1; ++i) t_nodes.push_back(i);
    for (int i = 0; i < tr.path_len; ++i) t_nodes.push_back(tr.path[i]);
    for (int i = 1; i < tr.path_len; ++i) p_nodes.push_back(tr.path[i] - u);   // chain ids of the proxy's pass
    rc = commit(t, true, t_nodes);
    if (rc == TRISPEC_OK) rc = commit(t, false, p_nodes);
    if (rc != TRISPEC_OK) return rc;
    for (size_t i = 1; i < p_nodes.size(); ++i) t->seq.push_back(tokens[p_nodes[i]]);
    t->seq.push_back(tr.token);
  }
  info.n_emitted = (int32_t)(t->seq.size() - before);
  info.ctx_len_proxy = kvp->ctx_len[0];
  info.ctx_len_target = kvt->ctx_len[0];
  if (info_host) *info_host = info;
  return TRISPEC_OK;
}

}  // extern "C"
