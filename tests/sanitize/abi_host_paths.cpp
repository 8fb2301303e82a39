// Drives the host-only paths of the C ABI (argument validation, size queries, the Case II prune /
// re-root of Sec. 3.2) with seeded valid and invalid inputs.  Meant to be built with the host
// compiler's address and undefined-behaviour sanitizers switched on for the library's host code:
// any out-of-bounds access, overflow or misuse of the arguments ends the run with a report.
// Every call here must return before anything is enqueued on a GPU; none is needed to run it.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "trispec.h"

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() {   // splitmix64, seeded: the run is reproducible
  uint64_t z = (g_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return (uint32_t)((z ^ (z >> 31)) >> 16);
}
static int rint_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

constexpr int kCap = TRISPEC_MAX_NODES + 16;   // room of the driver's own arrays: node counts up to a little past the limit
static long g_calls = 0;
#define EXPECT(cond)                                                              \
  do {                                                                            \
    ++g_calls;                                                                    \
    if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); exit(2); } \
  } while (0)

static trispec_model *make_model(int dtype, std::vector<const void *> &table) {
  trispec_model_config c;
  memset(&c, 0, sizeof c);
  c.n_layers = 3; c.hidden = 256; c.n_q_heads = 4; c.n_kv_heads = 2; c.head_dim = 64;
  c.ffn = 512; c.vocab = 4099; c.dtype = dtype; c.rms_eps = 1e-6f; c.rope_base = 1e4f;
  table.assign(3, (const void *)0x1000);   // never dereferenced on the host
  trispec_weights w;
  memset(&w, 0, sizeof w);
  w.embed = w.lm_head = w.final_norm = (const void *)0x1000;
  w.wq = w.wk = w.wv = w.wo = w.w_gate = w.w_up = w.w_down = w.norm_attn = w.norm_ffn = table.data();
  trispec_model *m = nullptr;
  EXPECT(trispec_model_create(&c, &w, &m) == TRISPEC_OK && m);
  return m;
}

static void shapes() {
  std::vector<const void *> t;
  for (int i = 0; i < 400; ++i) {
    trispec_model_config c;
    memset(&c, 0, sizeof c);
    c.n_layers = rint_in(-1, 4); c.hidden = rint_in(-64, 640); c.n_q_heads = rint_in(-1, 20);
    c.n_kv_heads = rint_in(-1, 9); c.head_dim = (rnd() & 1) ? 64 * rint_in(0, 3) : rint_in(-8, 200);
    c.ffn = rint_in(-64, 1024); c.vocab = rint_in(-5, 70000); c.dtype = rint_in(-1, 2);
    c.rms_eps = 1e-6f; c.rope_base = 1e4f; c.qk_norm = rint_in(-1, 2);
    t.assign(c.n_layers > 0 ? c.n_layers : 1, (const void *)0x1000);
    trispec_weights w;
    memset(&w, 0, sizeof w);
    w.embed = w.lm_head = w.final_norm = (const void *)0x1000;
    w.wq = w.wk = w.wv = w.wo = w.w_gate = w.w_up = w.w_down = w.norm_attn = w.norm_ffn = t.data();
    if (rnd() & 1) w.q_norm = w.k_norm = t.data();
    trispec_model *m = nullptr;
    const int rc = trispec_model_create(&c, &w, &m);
    EXPECT(rc == TRISPEC_OK || rc == TRISPEC_ESHAPE || rc == TRISPEC_ENULL);
    if (rc == TRISPEC_OK) {
      size_t b = 0;
      for (int j = 0; j < 8; ++j) {
        int r = trispec_workspace_bytes(m, rint_in(-1, 10), rint_in(-1, kCap - 10), &b);
        EXPECT(r == TRISPEC_OK || r == TRISPEC_ENODES || r == TRISPEC_ESHAPE);
        r = trispec_kv_bytes(m, rint_in(-1, 10), 64 * rint_in(-1, 40) + (rnd() % 5 == 0), &b);
        EXPECT(r == TRISPEC_OK || r == TRISPEC_ENODES || r == TRISPEC_ECAPACITY);
        double bytes = 0;
        int32_t ctx[TRISPEC_MAX_BATCH];
        for (int &x : ctx) x = rint_in(0, 5000);
        r = trispec_pass_bytes(m, rint_in(-1, 9), rint_in(-1, 66), ctx, &bytes);
        EXPECT(r == TRISPEC_OK || r == TRISPEC_ENODES || r == TRISPEC_EARG);
      }
      EXPECT(trispec_model_pack_bytes(m, &b) == TRISPEC_OK);
      EXPECT(trispec_model_destroy(m) == TRISPEC_OK);
    }
  }
  size_t b = 0;
  EXPECT(trispec_pack_matrix_bytes(20, 256, &b) == TRISPEC_OK && b >= 20u * 256u * 2u);
  EXPECT(trispec_pack_matrix_bytes(0, 256, &b) != TRISPEC_OK);
  EXPECT(trispec_pack_matrix_bytes(20, 100, &b) != TRISPEC_OK);
  EXPECT(trispec_pack_matrix_bytes(20, 256, nullptr) == TRISPEC_ENULL);
  for (int code = 1; code >= -14; --code) EXPECT(trispec_strerror(code) != nullptr);
}

// Random tree, random root path (or a broken one), random prefix: the outputs must stay inside
// their TRISPEC_MAX_NODES entries and, when the call succeeds, describe a valid tree.
static void prune() {
  int32_t tok[kCap], par[kCap], pos[kCap], path[kCap], pre[kCap];
  int32_t o_tok[TRISPEC_MAX_NODES + 1], o_par[TRISPEC_MAX_NODES + 1], o_pos[TRISPEC_MAX_NODES + 1],
      o_old[TRISPEC_MAX_NODES + 1];
  const int32_t guard = 0x5a5a5a5a;
  for (int it = 0; it < 20000; ++it) {
    const int n = (rnd() % 50 == 0) ? rint_in(-2, kCap - 10) : rint_in(1, TRISPEC_MAX_NODES);
    const int nn = n < 1 ? 1 : (n > kCap ? kCap : n);
    par[0] = -1; pos[0] = 100; tok[0] = rint_in(0, 999);
    for (int i = 1; i < nn; ++i) {
      par[i] = rint_in(0, i - 1);
      pos[i] = pos[par[i]] + 1;
      tok[i] = rint_in(0, 999);
    }
    const bool break_tree = rnd() % 40 == 0;
    if (break_tree && nn > 2) par[rint_in(1, nn - 1)] = rint_in(-3, nn + 3);
    // a root path by walking down, sometimes damaged
    int plen = 0, cur = 0;
    path[plen++] = 0;
    while (true) {
      int kids[kCap], nk = 0;
      for (int i = cur + 1; i < nn; ++i) if (par[i] == cur) kids[nk++] = i;
      if (!nk || rnd() % 3 == 0) break;
      cur = kids[rnd() % nk];
      path[plen++] = cur;
    }
    const bool break_path = rnd() % 40 == 0;
    if (break_path) path[rint_in(0, plen - 1)] = rint_in(-2, nn + 2);
    const int n_pre = (rnd() % 4 == 0) ? rint_in(-1, kCap - 10) : 0;
    for (int i = 0; i < kCap; ++i) pre[i] = rint_in(0, 999);
    o_tok[TRISPEC_MAX_NODES] = o_par[TRISPEC_MAX_NODES] = o_pos[TRISPEC_MAX_NODES] = o_old[TRISPEC_MAX_NODES] = guard;
    int32_t on = -7, of = -7;
    const int rc = trispec_prune_reroot(tok, par, pos, n, path, (rnd() % 60 == 0) ? rint_in(-1, kCap - 10) : plen,
                                        n_pre > 0 ? pre : nullptr, n_pre, 100 - (n_pre > 0 ? n_pre : 0),
                                        o_tok, o_par, o_pos, o_old, &on, &of);
    EXPECT(o_tok[TRISPEC_MAX_NODES] == guard && o_par[TRISPEC_MAX_NODES] == guard &&
           o_pos[TRISPEC_MAX_NODES] == guard && o_old[TRISPEC_MAX_NODES] == guard);
    EXPECT(rc == TRISPEC_OK || rc == TRISPEC_ENODES || rc == TRISPEC_ETREE || rc == TRISPEC_EARG || rc == TRISPEC_ENULL);
    if (rc == TRISPEC_OK) {
      EXPECT(on >= 1 && on <= TRISPEC_MAX_NODES && of >= 1 && of <= on);
      EXPECT(o_par[0] == -1);
      for (int i = 1; i < on; ++i) EXPECT(o_par[i] >= 0 && o_par[i] < i);
      if (!break_tree)   // positions were depths: they still are
        for (int i = 1; i < on; ++i) EXPECT(o_pos[i] == o_pos[o_par[i]] + 1);
      for (int i = 1; i < of; ++i) EXPECT(o_par[i] == i - 1);   // the forced part is a chain
    }
  }
  EXPECT(trispec_prune_reroot(nullptr, par, pos, 3, path, 1, nullptr, 0, 0, o_tok, o_par, o_pos, o_old, nullptr, nullptr) == TRISPEC_ENULL);
}

// trispec_verify / trispec_decide / trispec_kv_* with arguments that must be refused on the host.
static void verify_args() {
  std::vector<const void *> t;
  trispec_model *m = make_model(TRISPEC_F32, t);
  size_t kvb = 0, wsb = 0;
  EXPECT(trispec_kv_bytes(m, 2, 256, &kvb) == TRISPEC_OK && kvb > 0);
  EXPECT(trispec_workspace_bytes(m, 2, 16, &wsb) == TRISPEC_OK && wsb > 0);
  trispec_kv *kv = nullptr;
  EXPECT(trispec_kv_create(m, (void *)0x10000, (void *)0x20000, 2, 256, &kv) == TRISPEC_OK && kv);
  EXPECT(trispec_kv_create(m, nullptr, (void *)0x20000, 2, 256, &kv) == TRISPEC_ENULL);
  EXPECT(trispec_kv_create(m, (void *)0x10000, (void *)0x20000, 2, 100, &kv) == TRISPEC_ECAPACITY);
  int32_t len[2] = {10, 300};
  EXPECT(trispec_kv_set_len(kv, len) == TRISPEC_ECAPACITY);
  len[1] = 250;
  EXPECT(trispec_kv_set_len(kv, len) == TRISPEC_OK);
  trispec_verify_opts o;
  trispec_verify_out out;
  memset(&out, 0, sizeof out);
  int32_t parents[2 * kCap];
  for (int it = 0; it < 3000; ++it) {
    memset(&o, 0, sizeof o);
    o.criterion = (rnd() % 8 == 0) ? rint_in(-1, 4) : TRISPEC_CRIT_MARGIN;
    o.n_forced = (rnd() % 4 == 0) ? rint_in(-1, 20) : 1;
    o.workspace = (rnd() % 8 == 0) ? nullptr : (void *)(uintptr_t)(0x100000 + ((rnd() % 8 == 0) ? 4 : 0));
    o.workspace_bytes = (rnd() % 8 == 0) ? wsb / 2 : wsb;
    o.launch_mode = rint_in(-1, 2);
    o.n_feature_layers = (rnd() % 6 == 0) ? rint_in(-1, 10) : 0;
    int32_t fl[10];
    for (int &x : fl) x = rint_in(-1, 4);
    o.feature_layers = (rnd() & 1) ? fl : nullptr;
    o.features_out = (rnd() & 1) ? (float *)0x300000 : nullptr;
    o.accept_top_k = (rnd() % 6 == 0) ? rint_in(-1, 5) : 0;
    o.adapter_dim = (rnd() % 6 == 0) ? rint_in(-4, 9) : 0;
    o.adapter_w = (rnd() % 6 == 0) ? (const void *)0x400000 : nullptr;
    const int n = (rnd() % 6 == 0) ? rint_in(-1, kCap - 10) : 16;
    // Two sequences of 16 nodes would be a valid call: something is wrong every time, so that
    // nothing is ever enqueued (a parent that is not an earlier node; NaN threshold for one node).
    const int stride = n > 0 ? n : 1;
    for (int b = 0; b < 2; ++b) {
      parents[b * stride] = -1;
      for (int i = 1; i < stride; ++i) parents[b * stride + i] = rint_in(0, i - 1);
    }
    if (stride > 1) { const int i = rint_in(1, stride - 1); parents[stride + i] = i + rint_in(0, 3); }
    const float thr = (stride == 1 || rnd() % 10 == 0) ? __builtin_nanf("") : 0.5f;
    int rc = trispec_verify(m, kv, (const int32_t *)0x500000, parents, (const int32_t *)0x600000, n, thr, &o, &out);
    EXPECT(rc < 0 && rc != TRISPEC_ELAUNCH);
    rc = trispec_decide(m, 2, (const int32_t *)0x500000, parents, n, thr, &o, &out);
    EXPECT(rc < 0 && rc != TRISPEC_ELAUNCH);
  }
  // commit: node lists that are not increasing, counts out of range, capacity
  int32_t nodes[2 * TRISPEC_PATH_STRIDE], cnt[2];
  for (int it = 0; it < 2000; ++it) {
    for (int &x : nodes) x = rint_in(-1, TRISPEC_MAX_NODES + 1);
    cnt[0] = rint_in(2, TRISPEC_MAX_NODES + 2);
    cnt[1] = rint_in(2, 8);
    nodes[TRISPEC_PATH_STRIDE + 1] = nodes[TRISPEC_PATH_STRIDE];   // never strictly increasing
    const int rc = trispec_kv_commit(kv, nodes, cnt, nullptr);
    EXPECT(rc == TRISPEC_ENODES || rc == TRISPEC_ETREE || rc == TRISPEC_ECAPACITY);
  }
  EXPECT(trispec_kv_destroy(kv) == TRISPEC_OK);
  EXPECT(trispec_model_destroy(m) == TRISPEC_OK);
  // the sampling decision's argument checks
  size_t sb = 0;
  EXPECT(trispec_sample_scratch_bytes(2, 9, 50000, &sb) == TRISPEC_OK && sb > 0);
  EXPECT(trispec_sample_scratch_bytes(0, 9, 50000, &sb) != TRISPEC_OK);
  EXPECT(trispec_sample_scratch_bytes(2, 9, 0, &sb) != TRISPEC_OK);
  EXPECT(trispec_sample_scratch_bytes(2, 9, 50000, nullptr) == TRISPEC_ENULL);
}

// The round driver's host-side checks (Algorithm 1's routing lives behind the boundary).
static void ternary_args() {
  std::vector<const void *> tp, tt;
  trispec_model *mp = make_model(TRISPEC_F32, tp), *mt = make_model(TRISPEC_F32, tt);
  trispec_kv *kp = nullptr, *kt = nullptr;
  EXPECT(trispec_kv_create(mp, (void *)0x10000, (void *)0x20000, 1, 256, &kp) == TRISPEC_OK);
  EXPECT(trispec_kv_create(mt, (void *)0x30000, (void *)0x40000, 1, 256, &kt) == TRISPEC_OK);
  trispec_ternary_config c;
  memset(&c, 0, sizeof c);
  c.proxy = mp; c.target = mt; c.kv_proxy = kp; c.kv_target = kt;
  c.workspace_proxy = (void *)0x100000; c.workspace_target = (void *)0x200000;
  c.workspace_proxy_bytes = c.workspace_target_bytes = (size_t)1 << 40;
  c.scratch_dev = (int32_t *)0x300000; c.criterion = TRISPEC_CRIT_MARGIN; c.max_nodes = 24;
  trispec_ternary *t = nullptr;
  for (int it = 0; it < 200; ++it) {
    trispec_ternary_config d = c;
    switch (rnd() % 6) {
      case 0: d.max_nodes = rint_in(-3, kCap); break;
      case 1: d.criterion = rint_in(-2, 6); break;
      case 2: d.kv_target = kp; break;
      case 3: d.workspace_proxy_bytes = rnd() % 4096; break;
      case 4: d.scratch_dev = nullptr; break;
      default: break;
    }
    trispec_ternary *x = nullptr;
    const int rc = trispec_ternary_create(&d, &x);
    EXPECT(rc == TRISPEC_OK || rc == TRISPEC_ENULL || rc == TRISPEC_ENODES || rc == TRISPEC_EMISMATCH ||
           rc == TRISPEC_EARG || rc == TRISPEC_EWORKSPACE);
    if (rc == TRISPEC_OK) EXPECT(trispec_ternary_destroy(x) == TRISPEC_OK);
  }
  EXPECT(trispec_ternary_create(&c, &t) == TRISPEC_OK && t);
  int32_t par[kCap], tok[kCap];
  trispec_round_info info;
  EXPECT(trispec_ternary_round(t, par, tok, 4, 0.5f, &info) == TRISPEC_ESTATE);
  const int32_t one = 17;
  EXPECT(trispec_ternary_resume(t, &one, 1) == TRISPEC_OK);
  for (int it = 0; it < 3000; ++it) {
    const int n = rint_in(-1, 30);
    const int nn = n < 1 ? 1 : n;
    par[0] = (rnd() % 20 == 0) ? 0 : -1;
    for (int i = 1; i < nn; ++i) par[i] = rint_in(0, i - 1);
    for (int i = 0; i < nn; ++i) tok[i] = rint_in(0, 4098);
    // always wrong somewhere, so that no pass is ever launched: too many nodes, a bad parent or a bad token
    if (n >= 2 && n <= 24) {
      if (rnd() & 1) par[rint_in(1, n - 1)] = n + rint_in(0, 5);
      else tok[rint_in(1, n - 1)] = (rnd() & 1) ? -1 - (int)(rnd() % 9) : 4099 + (int)(rnd() % 9);
    } else if (n == 1) {
      par[0] = 0;
    }
    const int rc = trispec_ternary_round(t, par, tok, n, 0.5f, (rnd() & 1) ? &info : nullptr);
    EXPECT(rc == TRISPEC_ENODES || rc == TRISPEC_ETREE || rc == TRISPEC_EARG);
  }
  const int32_t *seq = nullptr;
  int32_t nseq = 0;
  EXPECT(trispec_ternary_sequence(t, &seq, &nseq) == TRISPEC_OK && nseq == 1 && seq[0] == 17);
  EXPECT(trispec_ternary_destroy(t) == TRISPEC_OK);
  EXPECT(trispec_kv_destroy(kp) == TRISPEC_OK && trispec_kv_destroy(kt) == TRISPEC_OK);
  EXPECT(trispec_model_destroy(mp) == TRISPEC_OK && trispec_model_destroy(mt) == TRISPEC_OK);
}

int main() {
  ternary_args();
  shapes();
  prune();
  verify_args();
  printf("ok %ld checks\n", g_calls);
  return 0;
}
