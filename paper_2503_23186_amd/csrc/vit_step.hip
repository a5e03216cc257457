// cnnk_vit_train_step: one training step of a pre-norm Vision Transformer classifier on one device
// (Section IV-A's second model; Algorithm 1's inner loop: forward pass, loss, backward pass, update).
// Host code: the order of the calls, the layout of the arena, the parameter table.  Everything runs
// through the entry points of cnnk_vit.h (and the classifier head and the residual sums through
// cnnk_fc_softmax_xent / cnnk_add of cnnk.h).
#include <stdio.h>
#include <string.h>
#include "common.h"
#include "sgd.h"
#include "../../include/cnnk_vit.h"

int cnnk_fill_zero(void* p, size_t bytes, hipStream_t st);   // vit_ops.hip

namespace {
enum { P_WE = 0, P_BE, P_CLS, P_POS, P_BLOCK0 };                          // model parameters
enum { B_G1 = 0, B_B1, B_WQKV, B_BQKV, B_WO, B_BO, B_G2, B_B2, B_W1, B_C1, B_W2, B_C2, B_COUNT };
// internal tensors of the arena behind the public ones
enum { X_Z0 = CNNK_VIT_TENSORS, X_DZ0, X_STATS1, X_STATS2, X_LSE, X_STATSF, X_TENSORS };

struct Geo {
  int B, n, T, d, m, K0, L, classes, dtype, heads;
  size_t rows, es;
};

bool make_geo(const cnnk_vit_desc* v, Geo* g) {
  if (!v) return false;
  if (v->B <= 0 || v->image <= 0 || v->patch <= 0 || v->dim <= 0 || v->heads <= 0 || v->layers <= 0 || v->mlp <= 0 ||
      v->classes <= 0 || v->image % v->patch != 0 || v->dim % v->heads != 0)
    return false;
  g->B = v->B;
  g->n = (v->image / v->patch) * (v->image / v->patch);
  g->T = g->n + 1;
  g->d = v->dim;
  g->m = v->mlp;
  g->K0 = v->patch * v->patch * 3;
  g->L = v->layers;
  g->classes = v->classes;
  g->dtype = v->dtype;
  g->heads = v->heads;
  g->rows = (size_t)g->B * g->T;
  g->es = elem_size(v->dtype);
  return true;
}

int validate(const cnnk_vit_desc* v, Geo* g) {
  if (!v) return CNNK_ERR_NULL;
  if (!make_geo(v, g)) return CNNK_ERR_SHAPE;
  if (v->dtype != CNNK_F32 && v->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  const int dh = v->dim / v->heads;
  if ((dh != 16 && dh != 32 && dh != 64) || (long long)g->T * dh > 16384) return CNNK_ERR_UNSUPPORTED;
  if (v->dim % 8 != 0 || v->mlp % 8 != 0 || g->K0 % 8 != 0 || v->dim > 2048 || v->mlp > 65536) return CNNK_ERR_UNSUPPORTED;
  if ((double)g->rows * (v->mlp > 3 * v->dim ? v->mlp : 3 * v->dim) > 2147483647.0) return CNNK_ERR_UNSUPPORTED;
  if (!(v->ln_eps >= 0.f)) return CNNK_ERR_SHAPE;
  return CNNK_OK;
}

// bytes of one instance of a tensor (0: not a per-layer tensor id / unused)
size_t tensor_bytes(const Geo& g, int id) {
  const size_t r = g.rows, es = g.es;
  switch (id) {
    case CNNK_VIT_PATCHES: return (size_t)g.B * g.n * g.K0 * es;
    case CNNK_VIT_TOK: case CNNK_VIT_DTOK: return r * g.d * es;
    case CNNK_VIT_H: case CNNK_VIT_O: case CNNK_VIT_XMID: case CNNK_VIT_H2: case CNNK_VIT_XOUT:
    case CNNK_VIT_DH: case CNNK_VIT_DO: case CNNK_VIT_DXMID: case CNNK_VIT_DH2: case CNNK_VIT_DXOUT:
      return r * g.d * es;
    case CNNK_VIT_QKV: case CNNK_VIT_DQKV: return r * 3 * g.d * es;
    case CNNK_VIT_U: case CNNK_VIT_G: case CNNK_VIT_DU: case CNNK_VIT_DG: return r * g.m * es;
    case CNNK_VIT_F: case CNNK_VIT_DF: return (size_t)g.B * g.d * es;
    case X_Z0: case X_DZ0: return (size_t)g.B * g.n * g.d * es;
    case X_STATS1: case X_STATS2: return r * 2 * sizeof(float);
    case X_LSE: return (size_t)g.B * g.heads * g.T * sizeof(float);
    case X_STATSF: return (size_t)g.B * 2 * sizeof(float);
    default: return 0;
  }
}
bool per_layer(int id) {
  switch (id) {
    case CNNK_VIT_H: case CNNK_VIT_QKV: case CNNK_VIT_O: case CNNK_VIT_XMID: case CNNK_VIT_H2: case CNNK_VIT_U:
    case CNNK_VIT_G: case CNNK_VIT_XOUT: case CNNK_VIT_DH: case CNNK_VIT_DQKV: case CNNK_VIT_DO: case CNNK_VIT_DXMID:
    case CNNK_VIT_DH2: case CNNK_VIT_DU: case CNNK_VIT_DG: case CNNK_VIT_DXOUT: case X_STATS1: case X_STATS2: case X_LSE:
      return true;
    default: return false;
  }
}

struct Arena {
  size_t off[X_TENSORS];      // offset of instance 0
  size_t size[X_TENSORS];     // bytes of one instance, rounded up to 256
  size_t total;
};

void layout(const Geo& g, Arena* a) {
  size_t at = 0;
  for (int id = 0; id < X_TENSORS; ++id) {
    const size_t b = tensor_bytes(g, id);
    a->size[id] = align_up(b, 256);
    a->off[id] = at;
    at += a->size[id] * (per_layer(id) ? (size_t)g.L : 1);
  }
  a->total = at;
}

size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

size_t workspace(const cnnk_vit_desc* v, const Geo& g) {
  size_t w = 0;
  const long long shapes[5][3] = {{(long long)g.B * g.n, g.K0, g.d}, {(long long)g.rows, g.d, 3 * g.d}, {(long long)g.rows, g.d, g.d},
                                  {(long long)g.rows, g.d, g.m}, {(long long)g.rows, g.m, g.d}};
  for (int i = 0; i < 5; ++i) w = max_sz(w, cnnk_linear_workspace_bytes(shapes[i][0], (int)shapes[i][1], (int)shapes[i][2], g.dtype));
  cnnk_ln_desc ln = {(int)g.rows, g.d, g.dtype, v->ln_eps, 0};
  w = max_sz(w, cnnk_layernorm_workspace_bytes(&ln));
  w = max_sz(w, cnnk_bias_act_workspace_bytes((long long)g.rows, 3 * g.d));
  w = max_sz(w, cnnk_bias_act_workspace_bytes((long long)g.rows, g.m));
  cnnk_fc_desc fc = {g.B, g.d, g.classes, g.dtype};
  w = max_sz(w, cnnk_fc_workspace_bytes(&fc));
  return align_up(w, 256);
}

// Walks the step's calls in order.  In enumeration mode nothing runs: the walk counts the calls and
// copies the name of call `want`.
struct Walk {
  bool run;
  int idx, want;
  char* name_out;
  int name_n;
  int rc;
  void** events;
  hipStream_t st;
  template <typename F>
  void call(int layer, const char* name, F&& f) {
    if (!run) {
      if (idx == want && name_out && name_n > 0) {
        if (layer >= 0) snprintf(name_out, (size_t)name_n, "block%d.%s", layer, name);
        else snprintf(name_out, (size_t)name_n, "%s", name);
      }
      ++idx;
      return;
    }
    if (rc != CNNK_OK) { ++idx; return; }
    if (events) (void)hipEventRecord((hipEvent_t)events[2 * idx], st);
    rc = f();
    if (events) (void)hipEventRecord((hipEvent_t)events[2 * idx + 1], st);
    ++idx;
  }
};

int walk(const cnnk_vit_desc* v, const Geo& g, const cnnk_vit_buffers* buf, float lr, float mu, float wd, Walk& w,
         bool forward_only = false) {
  Arena A;
  layout(g, &A);
  char* base = buf ? (char*)buf->arena : nullptr;
  auto at = [&](int id, int l) -> void* { return base ? base + A.off[id] + A.size[id] * (size_t)(per_layer(id) ? l : 0) : nullptr; };
  // Calls that only the update waits for go to the second stream when there is one: `st`, `ws` and
  // `wsb` are what the call lambdas below read, and forked() points them at the second stream and the
  // upper half of the workspace for the duration of one call.
  const bool two = w.run && buf && buf->aux_stream && buf->ev_fork && buf->ev_join && !w.events;
  void* const ws_main = buf ? buf->ws : nullptr;
  const size_t wsb_main = buf ? (two ? buf->ws_bytes / 2 / 256 * 256 : buf->ws_bytes) : 0;
  void* ws = ws_main;
  size_t wsb = wsb_main;
  hipStream_t st = w.st;
  auto forked = [&](int layer, const char* name, auto&& f) {
    if (!two) { w.call(layer, name, f); return; }
    if (w.rc != CNNK_OK) { ++w.idx; return; }
    hipStream_t aux = (hipStream_t)buf->aux_stream;
    if (hipEventRecord((hipEvent_t)buf->ev_fork, w.st) != hipSuccess || hipStreamWaitEvent(aux, (hipEvent_t)buf->ev_fork, 0) != hipSuccess) {
      w.rc = CNNK_ERR_HIP;
      ++w.idx;
      return;
    }
    st = aux; ws = (char*)ws_main + wsb_main; wsb = wsb_main;
    w.rc = f();
    st = w.st; ws = ws_main; wsb = wsb_main;
    ++w.idx;
  };
  const bool bf = g.dtype == CNNK_BF16;
  auto P = [&](int k) -> float* { return buf ? (float*)buf->param[k] : nullptr; };
  auto Wm = [&](int k) -> const void* { return buf ? (bf ? buf->param_lp[k] : buf->param[k]) : nullptr; };
  auto Gr = [&](int k) -> float* { return buf ? (float*)buf->grad[k] : nullptr; };
  const int d = g.d, m = g.m, T = g.T;
  const long long rows = (long long)g.rows;
  const cnnk_embed_desc ed = {g.B, v->image, v->patch, d, g.dtype};
  const long long prow = (long long)g.B * g.n;     // patch rows
  const int dt = g.dtype;
  const cnnk_ln_desc ln = {(int)g.rows, d, g.dtype, v->ln_eps, 0};
  const cnnk_ln_desc ln_cls = {g.B, d, g.dtype, v->ln_eps, (long long)T * d};
  const cnnk_attn_desc ad = {g.B, T, v->heads, d / v->heads, g.dtype};
  const cnnk_fc_desc fc = {g.B, d, g.classes, g.dtype};
  const int p_tail = P_BLOCK0 + B_COUNT * g.L;     // gf, bf, Wh, bh

  // ---- forward ----
  w.call(-1, "embed.patchify", [&] { return cnnk_vit_patchify(&ed, buf->x, at(CNNK_VIT_PATCHES, 0), st); });
  w.call(-1, "embed.gemm", [&] { return cnnk_linear_fwd(prow, g.K0, d, dt, at(CNNK_VIT_PATCHES, 0), Wm(P_WE), nullptr, nullptr, CNNK_ACT_NONE, nullptr, at(X_Z0, 0), ws, wsb, st); });
  w.call(-1, "embed.tokens", [&] { return cnnk_vit_embed_fwd(&ed, at(X_Z0, 0), P(P_BE), P(P_CLS), P(P_POS), at(CNNK_VIT_TOK, 0), st); });
  for (int l = 0; l < g.L; ++l) {
    const int p0 = P_BLOCK0 + B_COUNT * l;
    void* xin = l ? at(CNNK_VIT_XOUT, l - 1) : at(CNNK_VIT_TOK, 0);
    w.call(l, "ln1", [&] { return cnnk_layernorm_fwd(&ln, xin, P(p0 + B_G1), P(p0 + B_B1), at(CNNK_VIT_H, l), (float*)at(X_STATS1, l), st); });
    w.call(l, "qkv.gemm", [&] { return cnnk_linear_fwd(rows, d, 3 * d, dt, at(CNNK_VIT_H, l), Wm(p0 + B_WQKV), P(p0 + B_BQKV), nullptr, CNNK_ACT_NONE, nullptr, at(CNNK_VIT_QKV, l), ws, wsb, st); });
    w.call(l, "attn", [&] { return cnnk_attention_fwd(&ad, at(CNNK_VIT_QKV, l), at(CNNK_VIT_O, l), (float*)at(X_LSE, l), st); });
    w.call(l, "proj.gemm_res", [&] { return cnnk_linear_fwd(rows, d, d, dt, at(CNNK_VIT_O, l), Wm(p0 + B_WO), P(p0 + B_BO), xin, CNNK_ACT_NONE, nullptr, at(CNNK_VIT_XMID, l), ws, wsb, st); });
    w.call(l, "ln2", [&] { return cnnk_layernorm_fwd(&ln, at(CNNK_VIT_XMID, l), P(p0 + B_G2), P(p0 + B_B2), at(CNNK_VIT_H2, l), (float*)at(X_STATS2, l), st); });
    w.call(l, "fc1.gemm_gelu", [&] { return cnnk_linear_fwd(rows, d, m, dt, at(CNNK_VIT_H2, l), Wm(p0 + B_W1), P(p0 + B_C1), nullptr, CNNK_ACT_GELU, at(CNNK_VIT_U, l), at(CNNK_VIT_G, l), ws, wsb, st); });
    w.call(l, "fc2.gemm_res", [&] { return cnnk_linear_fwd(rows, m, d, dt, at(CNNK_VIT_G, l), Wm(p0 + B_W2), P(p0 + B_C2), at(CNNK_VIT_XMID, l), CNNK_ACT_NONE, nullptr, at(CNNK_VIT_XOUT, l), ws, wsb, st); });
  }
  void* xlast = at(CNNK_VIT_XOUT, g.L - 1);
  w.call(-1, "head.ln", [&] { return cnnk_layernorm_fwd(&ln_cls, xlast, P(p_tail), P(p_tail + 1), at(CNNK_VIT_F, 0), (float*)at(X_STATSF, 0), st); });
  if (forward_only) {
    w.call(-1, "head.loss", [&] {
      return cnnk_fc_softmax_xent(&fc, at(CNNK_VIT_F, 0), P(p_tail + 2), P(p_tail + 3), buf->labels, buf->loss, buf->pred,
                                  buf->probs, nullptr, nullptr, nullptr, ws, wsb, st);
    });
    return w.rc;
  }
  w.call(-1, "head.loss", [&] {
    return cnnk_fc_softmax_xent(&fc, at(CNNK_VIT_F, 0), P(p_tail + 2), P(p_tail + 3), buf->labels, buf->loss, buf->pred, buf->probs,
                                at(CNNK_VIT_DF, 0), Gr(p_tail + 2), Gr(p_tail + 3), ws, wsb, st);
  });
  // ---- backward ----
  void* dxlast = at(CNNK_VIT_DXOUT, g.L - 1);
  w.call(-1, "head.zero", [&] { return cnnk_fill_zero(dxlast, A.size[CNNK_VIT_DXOUT], st); });
  w.call(-1, "head.ln.bwd", [&] {
    return cnnk_layernorm_bwd(&ln_cls, at(CNNK_VIT_DF, 0), xlast, P(p_tail), (const float*)at(X_STATSF, 0), nullptr, dxlast, Gr(p_tail),
                              Gr(p_tail + 1), ws, wsb, st);
  });
  for (int l = g.L - 1; l >= 0; --l) {
    const int p0 = P_BLOCK0 + B_COUNT * l;
    void* xin = l ? at(CNNK_VIT_XOUT, l - 1) : at(CNNK_VIT_TOK, 0);
    void* dxin = l ? at(CNNK_VIT_DXOUT, l - 1) : at(CNNK_VIT_DTOK, 0);
    void* dxo = at(CNNK_VIT_DXOUT, l);
    forked(l, "fc2.dbias", [&] { return cnnk_bias_act_bwd(rows, d, g.dtype, CNNK_ACT_NONE, dxo, nullptr, nullptr, Gr(p0 + B_C2), ws, wsb, st); });
    forked(l, "fc2.wgrad", [&] { return cnnk_linear_wgrad(rows, m, d, dt, at(CNNK_VIT_G, l), dxo, Gr(p0 + B_W2), ws, wsb, st); });
    w.call(l, "fc2.dgrad", [&] { return cnnk_linear_dgrad(rows, m, d, dt, dxo, Wm(p0 + B_W2), at(CNNK_VIT_DG, l), ws, wsb, st); });
    w.call(l, "fc1.gelu.bwd", [&] { return cnnk_bias_act_bwd(rows, m, g.dtype, CNNK_ACT_GELU, at(CNNK_VIT_DG, l), at(CNNK_VIT_U, l), at(CNNK_VIT_DU, l), Gr(p0 + B_C1), ws, wsb, st); });
    forked(l, "fc1.wgrad", [&] { return cnnk_linear_wgrad(rows, d, m, dt, at(CNNK_VIT_H2, l), at(CNNK_VIT_DU, l), Gr(p0 + B_W1), ws, wsb, st); });
    w.call(l, "fc1.dgrad", [&] { return cnnk_linear_dgrad(rows, d, m, dt, at(CNNK_VIT_DU, l), Wm(p0 + B_W1), at(CNNK_VIT_DH2, l), ws, wsb, st); });
    w.call(l, "ln2.bwd", [&] {
      return cnnk_layernorm_bwd(&ln, at(CNNK_VIT_DH2, l), at(CNNK_VIT_XMID, l), P(p0 + B_G2), (const float*)at(X_STATS2, l), dxo,
                                at(CNNK_VIT_DXMID, l), Gr(p0 + B_G2), Gr(p0 + B_B2), ws, wsb, st);
    });
    void* dxm = at(CNNK_VIT_DXMID, l);
    forked(l, "proj.dbias", [&] { return cnnk_bias_act_bwd(rows, d, g.dtype, CNNK_ACT_NONE, dxm, nullptr, nullptr, Gr(p0 + B_BO), ws, wsb, st); });
    forked(l, "proj.wgrad", [&] { return cnnk_linear_wgrad(rows, d, d, dt, at(CNNK_VIT_O, l), dxm, Gr(p0 + B_WO), ws, wsb, st); });
    w.call(l, "proj.dgrad", [&] { return cnnk_linear_dgrad(rows, d, d, dt, dxm, Wm(p0 + B_WO), at(CNNK_VIT_DO, l), ws, wsb, st); });
    w.call(l, "attn.bwd", [&] { return cnnk_attention_bwd(&ad, at(CNNK_VIT_QKV, l), at(CNNK_VIT_O, l), at(CNNK_VIT_DO, l), (const float*)at(X_LSE, l), at(CNNK_VIT_DQKV, l), st); });
    forked(l, "qkv.dbias", [&] { return cnnk_bias_act_bwd(rows, 3 * d, g.dtype, CNNK_ACT_NONE, at(CNNK_VIT_DQKV, l), nullptr, nullptr, Gr(p0 + B_BQKV), ws, wsb, st); });
    forked(l, "qkv.wgrad", [&] { return cnnk_linear_wgrad(rows, d, 3 * d, dt, at(CNNK_VIT_H, l), at(CNNK_VIT_DQKV, l), Gr(p0 + B_WQKV), ws, wsb, st); });
    w.call(l, "qkv.dgrad", [&] { return cnnk_linear_dgrad(rows, d, 3 * d, dt, at(CNNK_VIT_DQKV, l), Wm(p0 + B_WQKV), at(CNNK_VIT_DH, l), ws, wsb, st); });
    w.call(l, "ln1.bwd", [&] {
      return cnnk_layernorm_bwd(&ln, at(CNNK_VIT_DH, l), xin, P(p0 + B_G1), (const float*)at(X_STATS1, l), dxm, dxin, Gr(p0 + B_G1),
                                Gr(p0 + B_B1), ws, wsb, st);
    });
  }
  w.call(-1, "embed.tokens.bwd", [&] { return cnnk_vit_embed_bwd(&ed, at(CNNK_VIT_DTOK, 0), at(X_DZ0, 0), Gr(P_BE), Gr(P_CLS), Gr(P_POS), st); });
  forked(-1, "embed.wgrad", [&] { return cnnk_linear_wgrad(prow, g.K0, d, dt, at(CNNK_VIT_PATCHES, 0), at(X_DZ0, 0), Gr(P_WE), ws, wsb, st); });
  // ---- update ----
  if (two && w.rc == CNNK_OK) {
    if (hipEventRecord((hipEvent_t)buf->ev_join, (hipStream_t)buf->aux_stream) != hipSuccess ||
        hipStreamWaitEvent(w.st, (hipEvent_t)buf->ev_join, 0) != hipSuccess)
      w.rc = CNNK_ERR_HIP;
  }
  w.call(-1, "update", [&] {
    const int np = p_tail + 4;
    const size_t sizes_blk[B_COUNT] = {(size_t)d, (size_t)d, (size_t)3 * d * d, (size_t)3 * d, (size_t)d * d, (size_t)d, (size_t)d, (size_t)d,
                                       (size_t)m * d, (size_t)m, (size_t)d * m, (size_t)d};
    SgdTable t;
    t.count = 0;
    int rc = CNNK_OK;
    for (int k = 0; k < np && rc == CNNK_OK; ++k) {
      size_t n;
      if (k == P_WE) n = (size_t)d * g.K0;
      else if (k == P_BE || k == P_CLS) n = (size_t)d;
      else if (k == P_POS) n = (size_t)T * d;
      else if (k < p_tail) n = sizes_blk[(k - P_BLOCK0) % B_COUNT];
      else if (k == p_tail || k == p_tail + 1) n = (size_t)d;
      else if (k == p_tail + 2) n = (size_t)g.classes * d;
      else n = (size_t)g.classes;
      const int i = t.count++;
      t.w[i] = (float*)buf->param[k]; t.v[i] = (float*)buf->mom[k]; t.g[i] = (const float*)buf->grad[k];
      t.wlp[i] = bf ? buf->param_lp[k] : nullptr; t.n[i] = n;
      if (t.count == kSgdMaxTensors || k == np - 1) { rc = sgd_multi(t, lr, mu, wd, st); t.count = 0; }
    }
    return rc;
  });
  return w.rc;
}
}  // namespace

extern "C" size_t cnnk_vit_arena_bytes(const cnnk_vit_desc* v) {
  Geo g;
  if (validate(v, &g) != CNNK_OK) return 0;
  Arena a;
  layout(g, &a);
  return a.total;
}

extern "C" size_t cnnk_vit_workspace_bytes(const cnnk_vit_desc* v) {
  Geo g;
  if (validate(v, &g) != CNNK_OK) return 0;
  return workspace(v, g);
}

extern "C" int cnnk_vit_tensor(const cnnk_vit_desc* v, int id, int layer, size_t* offset, size_t* bytes) {
  Geo g;
  const int rc = validate(v, &g);
  if (rc != CNNK_OK) return rc;
  if (!offset || !bytes) return CNNK_ERR_NULL;
  if (id < 0 || id >= CNNK_VIT_TENSORS) return CNNK_ERR_SHAPE;
  if (per_layer(id) && (layer < 0 || layer >= g.L)) return CNNK_ERR_SHAPE;
  Arena a;
  layout(g, &a);
  *offset = a.off[id] + a.size[id] * (size_t)(per_layer(id) ? layer : 0);
  *bytes = tensor_bytes(g, id);
  return CNNK_OK;
}

extern "C" int cnnk_vit_step_calls(const cnnk_vit_desc* v) {
  Geo g;
  if (validate(v, &g) != CNNK_OK) return 0;
  Walk w = {false, 0, -1, nullptr, 0, CNNK_OK, nullptr, nullptr};
  walk(v, g, nullptr, 0.f, 0.f, 0.f, w);
  return w.idx;
}

extern "C" int cnnk_vit_step_call_name(const cnnk_vit_desc* v, int i, char* out, int n) {
  Geo g;
  const int rc = validate(v, &g);
  if (rc != CNNK_OK) return rc;
  if (!out || n <= 0) return CNNK_ERR_NULL;
  out[0] = 0;
  Walk w = {false, 0, i, out, n, CNNK_OK, nullptr, nullptr};
  walk(v, g, nullptr, 0.f, 0.f, 0.f, w);
  return (i >= 0 && i < w.idx) ? CNNK_OK : CNNK_ERR_SHAPE;
}

static int check_buffers(const cnnk_vit_desc* v, const Geo& g, const cnnk_vit_buffers* buf, bool training) {
  if (!buf || !buf->param || !buf->x || !buf->labels || !buf->loss || !buf->pred || !buf->arena) return CNNK_ERR_NULL;
  if (training && (!buf->grad || !buf->mom)) return CNNK_ERR_NULL;
  const int np = P_BLOCK0 + B_COUNT * g.L + 4;
  if (buf->n_params != np) return CNNK_ERR_SHAPE;
  const bool bf = g.dtype == CNNK_BF16;
  if (bf && !buf->param_lp) return CNNK_ERR_NULL;
  for (int k = 0; k < np; ++k) {
    if (!buf->param[k] || (training && (!buf->grad[k] || !buf->mom[k]))) return CNNK_ERR_NULL;
    const int r = k >= P_BLOCK0 && k < np - 4 ? (k - P_BLOCK0) % B_COUNT : -1;
    const bool matrix = k == P_WE || r == B_WQKV || r == B_WO || r == B_W1 || r == B_W2;
    if (bf && matrix && !buf->param_lp[k]) return CNNK_ERR_NULL;
  }
  if (buf->arena_bytes < cnnk_vit_arena_bytes(v)) return CNNK_ERR_WORKSPACE;
  if ((((size_t)buf->arena) & 255) != 0 || (((size_t)buf->ws) & 255) != 0) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

extern "C" int cnnk_vit_eval_step(const cnnk_vit_desc* v, const cnnk_vit_buffers* buf, int* n_correct, void* stream) {
  Geo g;
  int rc = validate(v, &g);
  if (rc != CNNK_OK) return rc;
  rc = check_buffers(v, g, buf, false);
  if (rc != CNNK_OK) return rc;
  if (!buf->ws || buf->ws_bytes < workspace(v, g)) return CNNK_ERR_WORKSPACE;
  cnnk_vit_buffers b = *buf;          // one stream, no per-call events
  b.events = nullptr; b.n_events = 0; b.aux_stream = nullptr;
  Walk w = {true, 0, -1, nullptr, 0, CNNK_OK, nullptr, (hipStream_t)stream};
  rc = walk(v, g, &b, 0.f, 0.f, 0.f, w, true);
  if (rc != CNNK_OK || !n_correct) return rc;
  return cnnk_count_correct(g.B, buf->pred, buf->labels, n_correct, stream);
}

extern "C" int cnnk_vit_train_step(const cnnk_vit_desc* v, const cnnk_vit_buffers* buf, float lr, float momentum,
                                   float weight_decay, void* stream) {
  Geo g;
  const int rc = validate(v, &g);
  if (rc != CNNK_OK) return rc;
  const int rcb = check_buffers(v, g, buf, true);
  if (rcb != CNNK_OK) return rcb;
  const bool two_streams = buf->aux_stream && buf->ev_fork && buf->ev_join && !buf->events;
  if (!buf->ws || buf->ws_bytes < workspace(v, g) * (two_streams ? 2 : 1)) return CNNK_ERR_WORKSPACE;
  if ((((size_t)buf->arena) & 255) != 0 || (((size_t)buf->ws) & 255) != 0) return CNNK_ERR_UNSUPPORTED;
  Walk w = {true, 0, -1, nullptr, 0, CNNK_OK, nullptr, (hipStream_t)stream};
  if (buf->events) {
    Walk c = {false, 0, -1, nullptr, 0, CNNK_OK, nullptr, nullptr};
    walk(v, g, nullptr, 0.f, 0.f, 0.f, c);
    if (buf->n_events < 2 * c.idx) return CNNK_ERR_WORKSPACE;
    w.events = buf->events;
  }
  return walk(v, g, buf, lr, momentum, weight_decay, w);
}
