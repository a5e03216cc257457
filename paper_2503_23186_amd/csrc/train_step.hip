// cnnk_train_step: forward over a layer list, loss, backward over the reversed list, SGD-momentum
// update of every parameter (the inner mini-batch loop of the paper's Algorithm 1 for one
// data-parallel replica).  Host code only: it validates the whole list first, then enqueues the
// kernels of the other entry points on one stream, with no host synchronisation in between.
#include <vector>
#include "common.h"
#include "sgd.h"
#include "conv.h"

namespace {

// grid budget (in compute units) of a weight gradient that runs beside the backward pass: measured
// optimum on ResNet-18 b256 (96..128 are within 1 %, 64 and 192 are 3 % slower)
constexpr int kAuxWgradCus = 112;
constexpr int kStatSlots = 4;   // convolutions whose per-channel sums may be pending at once
constexpr size_t kStatBytes = kStatSlots * 2 * 2048 * sizeof(float);

struct Walk {
  std::vector<size_t> slot_elems;   // 0 = not seen yet
  std::vector<size_t> param_elems;
  size_t ws = 0;
  size_t wt_bytes = 0;               // transposed bf16 weights of every conv whose data gradient runs on MFMA
  std::vector<size_t> wt_off;        // per layer: offset into that region, or (size_t)-1
  int x8_layer = -1;                 // first-layer convolution with fewer than 8 input channels, if any:
  size_t x8_off = 0;                 // its 8-channel copy of the network input lives in the same region
  int dtype = -1;
};

bool dgrad_pretransposed(const cnnk_layer& l) {
  if (l.op != CNNK_OP_CONV || l.in0 == 0 || l.d.conv.dtype != CNNK_BF16) return false;
  return conv_mfma_supported(make_geom(&l.d.conv), CNNK_PASS_DGRAD);
}

bool set_elems(std::vector<size_t>& v, int id, size_t n) {
  if (id < 0 || id >= (int)v.size()) return false;
  if (v[id] == 0) { v[id] = n; return true; }
  return v[id] == n;
}

size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

// Checks every layer and gathers tensor sizes and the workspace need.  n_slots/n_params < 0:
// sizes are unknown (workspace query), ids are only checked for being non-negative.
int walk_layers(const cnnk_layer* L, int n, int n_slots, int n_params, Walk* w) {
  if (!L) return CNNK_ERR_NULL;
  if (n <= 0) return CNNK_ERR_SHAPE;
  int max_slot = 0, max_param = 0;
  for (int i = 0; i < n; ++i) {
    const int ids[3] = {L[i].in0, L[i].in1, L[i].out};
    for (int k = 0; k < 3; ++k) if (ids[k] > max_slot) max_slot = ids[k];
    if (L[i].p0 > max_param) max_param = L[i].p0;
    if (L[i].p1 > max_param) max_param = L[i].p1;
  }
  if (n_slots >= 0 && max_slot >= n_slots) return CNNK_ERR_SHAPE;
  if (n_params >= 0 && max_param >= n_params) return CNNK_ERR_SHAPE;
  w->slot_elems.assign(max_slot + 1, 0);
  w->param_elems.assign(max_param + 1, 0);
  w->wt_off.assign(n, (size_t)-1);
  for (int i = 0; i < n; ++i) {
    const cnnk_layer& l = L[i];
    int dt = -1;
    bool ok = true;
    switch (l.op) {
      case CNNK_OP_CONV: {
        const cnnk_conv_desc& d = l.d.conv;
        int rc = cnnk_validate_conv(&d);
        if (rc != CNNK_OK) return rc;
        dt = d.dtype;
        const int Ho = conv_out(d.H, d.pad, d.R, d.stride), Wo = conv_out(d.W, d.pad, d.S, d.stride);
        ok = l.in0 >= 0 && l.out > 0 && l.p0 >= 0 &&
             set_elems(w->slot_elems, l.in0, (size_t)d.N * d.H * d.W * d.Cin) &&
             set_elems(w->slot_elems, l.out, (size_t)d.N * Ho * Wo * d.Cout) &&
             set_elems(w->param_elems, l.p0, (size_t)d.Cout * d.R * d.S * d.Cin);
        for (int p = 0; p < 3; ++p) w->ws = max_sz(w->ws, cnnk_conv2d_workspace_bytes(&d, p));
        if (dgrad_pretransposed(l)) {
          w->wt_off[i] = w->wt_bytes;
          w->wt_bytes += align_up((size_t)d.Cout * d.R * d.S * d.Cin * sizeof(bf16_t), 256);
        }
        if (w->x8_layer < 0 && l.in0 == 0 && d.dtype == CNNK_BF16 && conv_pad_supported(make_geom(&d))) {
          w->x8_layer = i;
          w->x8_off = w->wt_bytes;
          w->wt_bytes += conv_pad_x8_bytes(make_geom(&d));
        }
        break;
      }
      case CNNK_OP_BN: {
        const cnnk_bn_desc& d = l.d.bn;
        const size_t e = (size_t)d.N * d.H * d.W * d.C;
        dt = d.dtype;
        if (d.N <= 0 || d.H <= 0 || d.W <= 0 || d.C <= 0) return CNNK_ERR_SHAPE;
        if (d.C % 8 != 0 || d.C > 2048) return CNNK_ERR_UNSUPPORTED;
        if (l.in0 == 0) return CNNK_ERR_UNSUPPORTED;  // batch norm directly on the network input
        ok = l.in0 > 0 && l.out > 0 && l.p0 >= 0 && l.p1 >= 0 && set_elems(w->slot_elems, l.in0, e) &&
             set_elems(w->slot_elems, l.out, e) && (l.in1 < 0 || set_elems(w->slot_elems, l.in1, e)) &&
             set_elems(w->param_elems, l.p0, d.C) && set_elems(w->param_elems, l.p1, d.C);
        w->ws = max_sz(w->ws, cnnk_bn_workspace_bytes(&d));
        break;
      }
      case CNNK_OP_POOL: {
        const cnnk_pool_desc& d = l.d.pool;
        dt = d.dtype;
        if (d.N <= 0 || d.H <= 0 || d.W <= 0 || d.C <= 0) return CNNK_ERR_SHAPE;
        if (d.C % 8 != 0) return CNNK_ERR_UNSUPPORTED;
        size_t eo;
        if (d.mode == CNNK_POOL_MAX2) {
          if ((d.H & 1) || (d.W & 1)) return CNNK_ERR_SHAPE;
          eo = (size_t)d.N * (d.H / 2) * (d.W / 2) * d.C;
        } else if (d.mode == CNNK_POOL_GAP) {
          eo = (size_t)d.N * d.C;
        } else {
          return CNNK_ERR_UNSUPPORTED;
        }
        ok = l.in0 >= 0 && l.out > 0 && set_elems(w->slot_elems, l.in0, (size_t)d.N * d.H * d.W * d.C) &&
             set_elems(w->slot_elems, l.out, eo);
        break;
      }
      case CNNK_OP_ADD: {
        const cnnk_pool_desc& d = l.d.pool;
        dt = d.dtype;
        if (d.N <= 0 || d.H <= 0 || d.W <= 0 || d.C <= 0) return CNNK_ERR_SHAPE;
        const size_t e = (size_t)d.N * d.H * d.W * d.C;
        ok = l.in0 >= 0 && l.in1 >= 0 && l.out > 0 && set_elems(w->slot_elems, l.in0, e) &&
             set_elems(w->slot_elems, l.in1, e) && set_elems(w->slot_elems, l.out, e);
        break;
      }
      case CNNK_OP_FC_LOSS: {
        const cnnk_fc_desc& d = l.d.fc;
        dt = d.dtype;
        if (i != n - 1) return CNNK_ERR_UNSUPPORTED;
        if (d.N <= 0 || d.F <= 0 || d.classes <= 0) return CNNK_ERR_SHAPE;
        if (d.classes > 4096 || d.N > 65535) return CNNK_ERR_UNSUPPORTED;
        ok = l.in0 > 0 && l.p0 >= 0 && l.p1 >= 0 && set_elems(w->slot_elems, l.in0, (size_t)d.N * d.F) &&
             set_elems(w->param_elems, l.p0, (size_t)d.classes * d.F) && set_elems(w->param_elems, l.p1, d.classes);
        w->ws = max_sz(w->ws, cnnk_fc_workspace_bytes(&d));
        break;
      }
      default:
        return CNNK_ERR_UNSUPPORTED;
    }
    if (!ok) return CNNK_ERR_SHAPE;
    if (dt != CNNK_F32 && dt != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
    if (w->dtype < 0) w->dtype = dt;
    if (dt != w->dtype) return CNNK_ERR_UNSUPPORTED;
  }
  if (L[n - 1].op != CNNK_OP_FC_LOSS) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

}  // namespace

extern "C" int cnnk_train_step_event_groups(int n_layers) { return n_layers > 0 ? 3 * n_layers - 1 : 0; }

namespace {
// Records the caller's events around one group of launches when timing was requested.
struct GroupTimer {
  void** ev;
  hipStream_t st;
  GroupTimer(const cnnk_buffers* B, int n_layers, void* stream) : ev(nullptr), st((hipStream_t)stream) {
    if (B->events && B->n_events >= 2 * cnnk_train_step_event_groups(n_layers)) ev = B->events;
  }
  void begin(int g) { if (ev) (void)hipEventRecord((hipEvent_t)ev[2 * g], st); }
  void end(int g) { if (ev) (void)hipEventRecord((hipEvent_t)ev[2 * g + 1], st); }
};
}  // namespace

extern "C" size_t cnnk_train_step_workspace_bytes(const cnnk_layer* layers, int n_layers) {
  Walk w;
  if (walk_layers(layers, n_layers, -1, -1, &w) != CNNK_OK) return 0;
  return align_up(align_up(w.ws, 256) + kStatBytes + w.wt_bytes, 256);
}

extern "C" int cnnk_train_step(const cnnk_layer* L, int n, const cnnk_buffers* B, const int* labels, float lr,
                               float momentum, float weight_decay, float* loss, int* pred, void* stream) {
  if (!B || !labels || !loss || !pred) return CNNK_ERR_NULL;
  if (!B->act || !B->dact || !B->param || !B->grad || !B->mom || !B->bn_save || !B->pool_idx) return CNNK_ERR_NULL;
  Walk w;
  int rc = walk_layers(L, n, B->n_slots, B->n_params, &w);
  if (rc != CNNK_OK) return rc;
  if (!B->ws || B->ws_bytes < align_up(w.ws, 256) + kStatBytes + w.wt_bytes) return CNNK_ERR_WORKSPACE;
  const bool bf16 = w.dtype == CNNK_BF16;
  for (size_t s = 0; s < w.slot_elems.size(); ++s) {
    if (w.slot_elems[s] == 0) continue;
    if (!B->act[s] || (s != 0 && !B->dact[s])) return CNNK_ERR_NULL;
  }
  for (size_t p = 0; p < w.param_elems.size(); ++p) {
    if (w.param_elems[p] == 0) continue;
    if (!B->param[p] || !B->grad[p] || !B->mom[p]) return CNNK_ERR_NULL;
  }
  for (int i = 0; i < n; ++i) {
    if (L[i].op == CNNK_OP_CONV && bf16 && (!B->param_lp || !B->param_lp[L[i].p0])) return CNNK_ERR_NULL;
    if (L[i].op == CNNK_OP_BN && !B->bn_save[i]) return CNNK_ERR_NULL;
    if (L[i].op == CNNK_OP_POOL && L[i].d.pool.mode == CNNK_POOL_MAX2 && !B->pool_idx[i]) return CNNK_ERR_NULL;
  }
  // every tensor that the backward pass reads a gradient from must receive one
  {
    std::vector<char> has(w.slot_elems.size(), 0);
    for (int i = n - 1; i >= 0; --i) {
      const cnnk_layer& l = L[i];
      if (l.op != CNNK_OP_FC_LOSS && !has[l.out]) return CNNK_ERR_SHAPE;
      has[l.in0] = 1;
      if ((l.op == CNNK_OP_BN || l.op == CNNK_OP_ADD) && l.in1 >= 0) has[l.in1] = 1;
    }
  }

  // The first kStatBytes of the workspace carry the per-channel sums from a convolution to the
  // batch norm that follows it; the calls themselves get the rest.
  float* const stat_base = reinterpret_cast<float*>(B->ws);
  int stat_slot[kStatSlots];   // tensor slot whose sums each buffer holds, -1 = free
  for (int k = 0; k < kStatSlots; ++k) stat_slot[k] = -1;
  // second stream for the weight gradients (off while per-call timing is requested)
  const bool timing = B->events && B->n_events >= 2 * cnnk_train_step_event_groups(n);
  const size_t ws_one = align_up(align_up(w.ws, 256) + kStatBytes + w.wt_bytes, 256);
  hipStream_t aux = nullptr;
  if (B->aux_stream && B->ev_fork && B->ev_join && !timing) {
    if (B->ws_bytes < 2 * ws_one) return CNNK_ERR_WORKSPACE;
    aux = (hipStream_t)B->aux_stream;
  }
  void* const aux_ws = static_cast<char*>(B->ws) + ws_one;
  const size_t aux_wsb = aux ? B->ws_bytes - ws_one : 0;
  char* const wt_region = static_cast<char*>(B->ws) + kStatBytes;
  void* ws = wt_region + w.wt_bytes;
  const size_t wsb = (aux ? ws_one : B->ws_bytes) - kStatBytes - w.wt_bytes;
  GroupTimer timer(B, n, stream);
  // Side branches of the forward pass: a convolution i whose output goes through a plain batch norm
  // (i+1: no ReLU, no residual) into nothing but the residual input of a later batch norm j - the
  // projection shortcut of a residual block.  With a second stream the pair runs there, launched
  // when the main stream reaches the first other reader a < i of the same input, and joined in
  // front of j.
  std::vector<int> side_of(n, -1);     // side_of[a] = i: launch the branch that starts at i before layer a
  std::vector<char> on_side(n, 0), join_before(n, 0);
  if (aux && bf16) {
    for (int i = 0; i + 1 < n; ++i) {
      const cnnk_layer& c = L[i];
      const cnnk_layer& b = L[i + 1];
      if (c.op != CNNK_OP_CONV || b.op != CNNK_OP_BN || b.in0 != c.out || b.in1 >= 0 || b.d.bn.relu) continue;
      int readers_c = 0, readers_b = 0, j = -1, a = -1;
      for (int k = 0; k < n; ++k) {
        if (L[k].op == CNNK_OP_FC_LOSS) { if (L[k].in0 == c.out || L[k].in0 == b.out) readers_b = 99; continue; }
        const bool two = L[k].op == CNNK_OP_BN || L[k].op == CNNK_OP_ADD;
        if (L[k].in0 == c.out || (two && L[k].in1 == c.out)) ++readers_c;
        if (L[k].in0 == b.out) readers_b = 99;
        if (two && L[k].in1 == b.out) { ++readers_b; j = (L[k].op == CNNK_OP_BN) ? k : -1; }
        if (a < 0 && k < i && (L[k].in0 == c.in0 || (two && L[k].in1 == c.in0))) a = k;
      }
      if (readers_c != 1 || readers_b != 1 || j <= i + 1 || a < 0 || side_of[a] >= 0) continue;
      side_of[a] = i;
      on_side[i] = on_side[i + 1] = 1;
      join_before[j] = 1;
    }
  }
  float* const aux_stat = reinterpret_cast<float*>(aux_ws);              // sums hand-off of a side branch
  void* const aux_scratch = static_cast<char*>(aux_ws) + 2 * 2048 * sizeof(float);
  const size_t aux_scratch_b = aux ? aux_wsb - 2 * 2048 * sizeof(float) : 0;
  // All weight transpositions of the data-gradient kernels in one launch (per 32 layers).  With a
  // second stream they run there beside the classifier head, whose few small launches leave the
  // device almost idle (tune key 12 = -1 keeps them on the main stream).
  auto transpose_all = [&](hipStream_t s_) -> int {
    TransposeTable t;
    t.count = 0;
    int r = CNNK_OK;
    for (int i = 0; i < n; ++i) {
      if (w.wt_off[i] == (size_t)-1) continue;
      const cnnk_conv_desc& d = L[i].d.conv;
      const int k = t.count++;
      t.src[k] = static_cast<const bf16_t*>(B->param_lp[L[i].p0]);
      t.dst[k] = reinterpret_cast<bf16_t*>(wt_region + w.wt_off[i]);
      t.Cout[k] = d.Cout; t.T[k] = d.R * d.S; t.Cin[k] = d.Cin;
      if (t.count == kMaxTranspose) {
        r = conv_transpose_weights_multi(t, s_);
        if (r != CNNK_OK) return r;
        t.count = 0;
      }
    }
    if (t.count > 0) r = conv_transpose_weights_multi(t, s_);
    return r;
  };
  bool wt_forked = false;
  bool x8_valid = false;   // the forward pass left the first layer's 8-channel input copy in place
  // ---- forward pass and loss ---------------------------------------------------------------
  for (int i = 0; i < n; ++i) {
    const cnnk_layer& l = L[i];
    if (side_of[i] >= 0) {
      const int s0 = side_of[i];
      const cnnk_layer& c = L[s0];
      const cnnk_layer& b = L[s0 + 1];
      if (hipEventRecord((hipEvent_t)B->ev_fork, (hipStream_t)stream) != hipSuccess ||
          hipStreamWaitEvent(aux, (hipEvent_t)B->ev_fork, 0) != hipSuccess)
        return CNNK_ERR_HIP;
      const bool sums = c.d.conv.Cout % 8 == 0 && c.d.conv.Cout <= 2048;
      rc = cnnk_conv2d_fwd(&c.d.conv, B->act[c.in0], B->param_lp[c.p0], B->act[c.out], sums ? aux_stat : nullptr,
                           sums ? aux_stat + 2048 : nullptr, aux_scratch, aux_scratch_b, aux);
      if (rc != CNNK_OK) return rc;
      float* run = B->bn_running ? B->bn_running[s0 + 1] : nullptr;
      rc = cnnk_bn_relu_fwd(&b.d.bn, B->act[b.in0], nullptr, B->param[b.p0], B->param[b.p1], B->act[b.out],
                            B->bn_save[s0 + 1], B->bn_save[s0 + 1] + b.d.bn.C, run, run ? run + b.d.bn.C : nullptr,
                            sums ? aux_stat : nullptr, sums ? aux_stat + 2048 : nullptr, aux_scratch, aux_scratch_b,
                            aux);
      if (rc != CNNK_OK) return rc;
      if (hipEventRecord((hipEvent_t)B->ev_join, aux) != hipSuccess) return CNNK_ERR_HIP;
    }
    if (on_side[i]) continue;
    if (join_before[i] && hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)B->ev_join, 0) != hipSuccess)
      return CNNK_ERR_HIP;
    timer.begin(i);
    switch (l.op) {
      case CNNK_OP_CONV: {
        const void* wt = bf16 ? B->param_lp[l.p0] : (const void*)B->param[l.p0];
        // hand the per-channel sums to the batch norm that consumes this output, if one does and
        // a buffer is free
        int sb = -1;
        if (bf16 && l.d.conv.Cout % 8 == 0 && l.d.conv.Cout <= 2048) {
          bool wanted = false;
          for (int j = i + 1; j < n && !wanted; ++j) wanted = L[j].op == CNNK_OP_BN && L[j].in0 == l.out;
          for (int k = 0; wanted && k < kStatSlots && sb < 0; ++k)
            if (stat_slot[k] < 0) sb = k;
        }
        float* ssum = sb >= 0 ? stat_base + (size_t)sb * 4096 : nullptr;
        // the 8-channel copy of the network input is kept for this layer's weight gradient
        X8Cache x8c{reinterpret_cast<bf16_t*>(wt_region + w.x8_off), false};
        if (i == w.x8_layer) t_cnnk_x8_cache = &x8c;
        rc = cnnk_conv2d_fwd(&l.d.conv, B->act[l.in0], wt, B->act[l.out], ssum, ssum ? ssum + 2048 : nullptr, ws, wsb,
                             stream);
        t_cnnk_x8_cache = nullptr;
        if (i == w.x8_layer) x8_valid = x8c.valid;
        if (sb >= 0) stat_slot[sb] = l.out;
        break;
      }
      case CNNK_OP_BN: {
        const int C = l.d.bn.C;
        float* run = B->bn_running ? B->bn_running[i] : nullptr;
        int sb = -1;
        for (int k = 0; k < kStatSlots; ++k)
          if (stat_slot[k] == l.in0) sb = k;
        const float* ssum = sb >= 0 ? stat_base + (size_t)sb * 4096 : nullptr;
        rc = cnnk_bn_relu_fwd(&l.d.bn, B->act[l.in0], l.in1 >= 0 ? B->act[l.in1] : nullptr, B->param[l.p0],
                              B->param[l.p1], B->act[l.out], B->bn_save[i], B->bn_save[i] + C, run,
                              run ? run + C : nullptr, ssum, ssum ? ssum + 2048 : nullptr, ws, wsb, stream);
        if (sb >= 0) stat_slot[sb] = -1;
        break;
      }
      case CNNK_OP_POOL:
        rc = cnnk_pool_fwd(&l.d.pool, B->act[l.in0], B->act[l.out], B->pool_idx[i], stream);
        break;
      case CNNK_OP_ADD:
        rc = cnnk_add(w.slot_elems[l.out], w.dtype, B->act[l.in0], B->act[l.in1], B->act[l.out], stream);
        break;
      case CNNK_OP_FC_LOSS:
        if (aux && g_cnnk_tune[12] >= 0) {
          if (hipEventRecord((hipEvent_t)B->ev_fork, (hipStream_t)stream) != hipSuccess ||
              hipStreamWaitEvent(aux, (hipEvent_t)B->ev_fork, 0) != hipSuccess)
            return CNNK_ERR_HIP;
          rc = transpose_all(aux);
          if (rc != CNNK_OK) return rc;
          if (hipEventRecord((hipEvent_t)B->ev_join, aux) != hipSuccess) return CNNK_ERR_HIP;
          wt_forked = true;
        }
        rc = cnnk_fc_softmax_xent(&l.d.fc, B->act[l.in0], B->param[l.p0], B->param[l.p1], labels, loss, pred,
                                  B->probs, B->dact[l.in0], B->grad[l.p0], B->grad[l.p1], ws, wsb, stream);
        break;
    }
    timer.end(i);
    if (rc != CNNK_OK) return rc;
  }
  // ---- backward pass ---------------------------------------------------------------------------
  if (!wt_forked) {
    rc = transpose_all((hipStream_t)stream);
    if (rc != CNNK_OK) return rc;
  } else if (hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)B->ev_join, 0) != hipSuccess) {
    return CNNK_ERR_HIP;
  }
  std::vector<char> written(w.slot_elems.size(), 0);
  std::vector<char> updated(w.param_elems.size(), 0);   // parameters already updated on the second stream
  written[L[n - 1].in0] = 1;
  // Tried and dropped (ResNet-18 b256, same-box A/B): (1) the backward pass of a projection shortcut
  // on the second stream - queued behind the weight gradients there it made the main stream wait,
  // 2.45 vs 2.37 ms; (2) per-channel sums through exact 64-bit integer atomics (three fixed-point
  // limbs, 8 replicas) instead of partials + a finalising launch - same-address atomics serialise
  // in L2 at 10-20 ns each: 3.29 ms with one copy, 2.42 vs 2.40 ms with eight; (3) the finalising
  // reduction inside the consuming batch-norm launch (its first workgroups reduce and publish, all
  // wait on flags with device-scope release / acquire) - the cache write-back and invalidate of
  // those fences cost far more than the launch they save: 2.68 vs 2.33 ms; (4) the weight
  // transpositions on the second stream beside the forward pass: no change (2.334 vs 2.334 ms).
  for (int i = n - 2; i >= 0; --i) {
    const cnnk_layer& l = L[i];
    const int g0 = n + 2 * (n - 2 - i);
    timer.begin(g0);
    switch (l.op) {
      case CNNK_OP_CONV: {
        // data gradient of this layer (main stream); with a second stream it is enqueued first so
        // that the event behind it exists when the weight gradient's reduction needs it
        auto dgrad = [&]() -> int {
          if (l.in0 == 0) return CNNK_OK;
          int r;
          if (w.wt_off[i] != (size_t)-1) {
            r = conv_mfma_dgrad_pt(make_geom(&l.d.conv), static_cast<const bf16_t*>(B->dact[l.out]),
                                   reinterpret_cast<const bf16_t*>(wt_region + w.wt_off[i]),
                                   static_cast<bf16_t*>(B->dact[l.in0]), written[l.in0], (hipStream_t)stream);
          } else {
            const void* wt = bf16 ? B->param_lp[l.p0] : (const void*)B->param[l.p0];
            r = cnnk_conv2d_dgrad(&l.d.conv, B->dact[l.out], wt, B->dact[l.in0], written[l.in0], ws, wsb, stream);
          }
          written[l.in0] = 1;
          return r;
        };
        if (!aux) {
          X8Cache x8c{reinterpret_cast<bf16_t*>(wt_region + w.x8_off), x8_valid};
          if (i == w.x8_layer && x8_valid) t_cnnk_x8_cache = &x8c;
          rc = cnnk_conv2d_wgrad(&l.d.conv, B->act[l.in0], B->dact[l.out], B->grad[l.p0], ws, wsb, stream);
          t_cnnk_x8_cache = nullptr;
          timer.end(g0);
          timer.begin(g0 + 1);
          if (rc == CNNK_OK) rc = dgrad();
          break;
        }
        // dy and x are final here: fork the weight gradient onto the second stream
        if (hipEventRecord((hipEvent_t)B->ev_fork, (hipStream_t)stream) != hipSuccess ||
            hipStreamWaitEvent(aux, (hipEvent_t)B->ev_fork, 0) != hipSuccess)
          return CNNK_ERR_HIP;
        rc = dgrad();
        if (rc != CNNK_OK) return rc;
        // The update of this layer's weights follows its weight gradient on the second stream, once
        // the data gradient (the last reader of the weights in this step) is done: the event is
        // re-recorded behind it, and the split-K reduction of the weight gradient waits for it and
        // applies the update in the same launch (a separate launch where nothing is reduced).
        const bool after_dgrad = l.in0 != 0;
        if (after_dgrad && hipEventRecord((hipEvent_t)B->ev_fork, (hipStream_t)stream) != hipSuccess)
          return CNNK_ERR_HIP;
        SgdFuse fuse{B->param[l.p0], B->mom[l.p0], (bf16 && B->param_lp) ? B->param_lp[l.p0] : nullptr,
                     lr, momentum, weight_decay, after_dgrad ? (hipEvent_t)B->ev_fork : nullptr, false};
        t_cnnk_sgd_fuse = &fuse;
        t_cnnk_wgrad_cus = kAuxWgradCus;
        X8Cache x8c{reinterpret_cast<bf16_t*>(wt_region + w.x8_off), x8_valid};
        if (i == w.x8_layer && x8_valid) t_cnnk_x8_cache = &x8c;
        rc = cnnk_conv2d_wgrad(&l.d.conv, B->act[l.in0], B->dact[l.out], B->grad[l.p0], aux_ws, aux_wsb, aux);
        t_cnnk_x8_cache = nullptr;
        t_cnnk_wgrad_cus = 256;
        t_cnnk_sgd_fuse = nullptr;
        if (rc != CNNK_OK) return rc;
        if (!fuse.done) {
          if (after_dgrad && hipStreamWaitEvent(aux, (hipEvent_t)B->ev_fork, 0) != hipSuccess) return CNNK_ERR_HIP;
          SgdTable t1;
          t1.count = 1;
          t1.w[0] = B->param[l.p0];
          t1.v[0] = B->mom[l.p0];
          t1.g[0] = B->grad[l.p0];
          t1.wlp[0] = (bf16 && B->param_lp) ? B->param_lp[l.p0] : nullptr;
          t1.n[0] = w.param_elems[l.p0];
          rc = sgd_multi(t1, lr, momentum, weight_decay, aux);
        }
        updated[l.p0] = 1;
        break;
      }
      case CNNK_OP_BN: {
        const int C = l.d.bn.C;
        const bool res = l.in1 > 0;
        const int flags = (written[l.in0] ? 1 : 0) | ((res && written[l.in1]) ? 2 : 0);
        // without a residual branch the ReLU mask is recomputed from x (y is not read)
        const void* ymask = (l.d.bn.relu && !res && g_cnnk_tune[9] >= 0) ? nullptr : B->act[l.out];
        rc = cnnk_bn_relu_bwd(&l.d.bn, B->dact[l.out], B->act[l.in0], ymask, B->param[l.p0], B->param[l.p1],
                              B->bn_save[i], B->bn_save[i] + C, B->dact[l.in0], res ? B->dact[l.in1] : nullptr, flags,
                              B->grad[l.p0], B->grad[l.p1], ws, wsb, stream);
        written[l.in0] = 1;
        if (res) written[l.in1] = 1;
        break;
      }
      case CNNK_OP_POOL:
        if (l.in0 != 0) {
          rc = cnnk_pool_bwd(&l.d.pool, B->dact[l.out], B->pool_idx[i], B->dact[l.in0], written[l.in0], stream);
          written[l.in0] = 1;
        }
        break;
      case CNNK_OP_ADD: {
        const int ins[2] = {l.in0, l.in1};
        for (int k = 0; k < 2 && rc == CNNK_OK; ++k) {
          if (ins[k] == 0) continue;
          rc = cnnk_grad_route(w.slot_elems[l.out], w.dtype, B->dact[l.out], B->dact[ins[k]], written[ins[k]], stream);
          written[ins[k]] = 1;
        }
        break;
      }
      default:
        break;
    }
    if (l.op != CNNK_OP_CONV) {
      timer.end(g0);
      timer.begin(g0 + 1);
    }
    timer.end(g0 + 1);
    if (rc != CNNK_OK) return rc;
  }
  // ---- parameter update -----------------------------------------------------------------------
  // With a second stream the parameters that are left (batch-norm and classifier parameters: their
  // gradients were computed on this stream) are updated first; the wait for the tail of the other
  // stream (the first layer's weight gradient and update) comes last, so the two overlap.
  const int g_upd = cnnk_train_step_event_groups(n) - 1;
  timer.begin(g_upd);
  SgdTable t;
  t.count = 0;
  for (size_t p = 0; p < w.param_elems.size(); ++p) {
    if (w.param_elems[p] == 0 || updated[p]) continue;
    const int k = t.count++;
    t.w[k] = B->param[p];
    t.v[k] = B->mom[p];
    t.g[k] = B->grad[p];
    t.wlp[k] = (bf16 && B->param_lp) ? B->param_lp[p] : nullptr;
    t.n[k] = w.param_elems[p];
    if (t.count == kSgdMaxTensors) {
      rc = sgd_multi(t, lr, momentum, weight_decay, (hipStream_t)stream);
      if (rc != CNNK_OK) return rc;
      t.count = 0;
    }
  }
  if (t.count > 0) rc = sgd_multi(t, lr, momentum, weight_decay, (hipStream_t)stream);
  timer.end(g_upd);
  if (aux && rc == CNNK_OK) {
    if (hipEventRecord((hipEvent_t)B->ev_join, aux) != hipSuccess ||
        hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)B->ev_join, 0) != hipSuccess)
      return CNNK_ERR_HIP;
  }
  return rc;
}

// Validation pass: the forward half of the step in inference mode.
extern "C" int cnnk_eval_step(const cnnk_layer* L, int n, const cnnk_buffers* B, const int* labels, float* loss,
                              int* pred, int* n_correct, void* stream) {
  if (!B || !labels || !loss || !pred) return CNNK_ERR_NULL;
  if (!B->act || !B->param || !B->bn_running || !B->pool_idx) return CNNK_ERR_NULL;
  Walk w;
  int rc = walk_layers(L, n, B->n_slots, B->n_params, &w);
  if (rc != CNNK_OK) return rc;
  if (!B->ws || B->ws_bytes < align_up(w.ws, 256) + kStatBytes + w.wt_bytes) return CNNK_ERR_WORKSPACE;
  const bool bf16 = w.dtype == CNNK_BF16;
  for (size_t s = 0; s < w.slot_elems.size(); ++s)
    if (w.slot_elems[s] != 0 && !B->act[s]) return CNNK_ERR_NULL;
  for (size_t p = 0; p < w.param_elems.size(); ++p)
    if (w.param_elems[p] != 0 && !B->param[p]) return CNNK_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    if (L[i].op == CNNK_OP_CONV && bf16 && (!B->param_lp || !B->param_lp[L[i].p0])) return CNNK_ERR_NULL;
    if (L[i].op == CNNK_OP_BN && !B->bn_running[i]) return CNNK_ERR_NULL;
    if (L[i].op == CNNK_OP_POOL && L[i].d.pool.mode == CNNK_POOL_MAX2 && !B->pool_idx[i]) return CNNK_ERR_NULL;
  }
  void* ws = static_cast<char*>(B->ws) + kStatBytes + w.wt_bytes;
  const size_t wsb = B->ws_bytes - kStatBytes - w.wt_bytes;
  for (int i = 0; i < n && rc == CNNK_OK; ++i) {
    const cnnk_layer& l = L[i];
    switch (l.op) {
      case CNNK_OP_CONV: {
        const void* wt = bf16 ? B->param_lp[l.p0] : (const void*)B->param[l.p0];
        rc = cnnk_conv2d_fwd(&l.d.conv, B->act[l.in0], wt, B->act[l.out], nullptr, nullptr, ws, wsb, stream);
        break;
      }
      case CNNK_OP_BN: {
        const float* run = B->bn_running[i];
        rc = cnnk_bn_relu_infer(&l.d.bn, B->act[l.in0], l.in1 >= 0 ? B->act[l.in1] : nullptr, B->param[l.p0],
                                B->param[l.p1], run, run + l.d.bn.C, B->act[l.out], stream);
        break;
      }
      case CNNK_OP_POOL:
        rc = cnnk_pool_fwd(&l.d.pool, B->act[l.in0], B->act[l.out], B->pool_idx[i], stream);
        break;
      case CNNK_OP_ADD:
        rc = cnnk_add(w.slot_elems[l.out], w.dtype, B->act[l.in0], B->act[l.in1], B->act[l.out], stream);
        break;
      case CNNK_OP_FC_LOSS:
        rc = cnnk_fc_softmax_xent(&l.d.fc, B->act[l.in0], B->param[l.p0], B->param[l.p1], labels, loss, pred,
                                  B->probs, nullptr, nullptr, nullptr, ws, wsb, stream);
        if (rc == CNNK_OK && n_correct) rc = cnnk_count_correct(l.d.fc.N, pred, labels, n_correct, stream);
        break;
    }
  }
  return rc;
}
