"""Pins of the Vision Transformer oracle (oracle/vit.py) to things other than itself: torch's CPU
operators and autograd in float64 (an independently written model out of library routines), finite
differences of the whole step, closed forms and invariants of the single operators."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as WL
from oracle import vit as V


def small(batch=3, dtype="f32", **kw):
    net = WL.vit_mini(batch=batch, dtype=dtype, image=16, patch=4, dim=32, heads=2, layers=2, mlp=48, classes=10, **kw)
    return net, WL.make_vit_inputs(net, config_id=61)


def torch_loss(net, x, labels, P):
    """The same model out of torch's own operators (unfold, layer_norm, softmax, gelu, cross_entropy)."""
    p, d, h = net.patch, net.dim, net.heads
    B = x.shape[0]
    # unfold wants NCHW and orders a patch (channel, row, column): reorder to (row, column, channel)
    cols = F.unfold(x.permute(0, 3, 1, 2), kernel_size=p, stride=p)           # [B, 3 p p, n]
    n = cols.shape[-1]
    patches = cols.reshape(B, 3, p, p, n).permute(0, 4, 2, 3, 1).reshape(B, n, p * p * 3)
    X = torch.cat([(P["cls"] + P["pos"][0]).expand(B, 1, d), patches @ P["We"].T + P["be"] + P["pos"][1:]], dim=1)
    for l in range(net.layers):
        g = lambda k: P["%s.%d" % (k, l)]
        H = F.layer_norm(X, (d,), g("g1"), g("b1"), eps=1e-6)
        qkv = F.linear(H, g("Wqkv"), g("bqkv")).reshape(B, n + 1, 3, h, d // h).permute(2, 0, 3, 1, 4)
        A = torch.softmax(qkv[0] @ qkv[1].transpose(-1, -2) / math.sqrt(d // h), dim=-1)
        O = (A @ qkv[2]).permute(0, 2, 1, 3).reshape(B, n + 1, d)
        X = X + F.linear(O, g("Wo"), g("bo"))
        H2 = F.layer_norm(X, (d,), g("g2"), g("b2"), eps=1e-6)
        X = X + F.linear(F.gelu(F.linear(H2, g("W1"), g("c1"))), g("W2"), g("c2"))
    f = F.layer_norm(X[:, 0], (d,), P["gf"], P["bf"], eps=1e-6)
    return F.cross_entropy(F.linear(f, P["Wh"], P["bh"]), labels)


def test_step_matches_torch_autograd():
    net, inp = small()
    loss, c = V.forward(net.cfg(), inp["x"], inp["labels"], inp["params"])
    grads, _ = V.backward(net.cfg(), inp["params"], c)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in inp["params"].items()}
    tl = torch_loss(net, torch.tensor(inp["x"]), torch.tensor(inp["labels"], dtype=torch.long), P)
    tl.backward()
    assert loss == pytest.approx(tl.item(), rel=1e-12)
    assert set(grads) == set(P)
    for k in P:
        want = P[k].grad.numpy()
        assert np.abs(grads[k] - want).max() <= 1e-11 * max(1.0, np.abs(want).max()), k


def test_step_finite_differences():
    net, inp = small(batch=2)
    cfg = net.cfg()
    loss, c = V.forward(cfg, inp["x"], inp["labels"], inp["params"])
    grads, _ = V.backward(cfg, inp["params"], c)
    rng = np.random.default_rng(5)
    for name in ("We", "cls", "pos", "g1.0", "b1.1", "Wqkv.0", "bqkv.1", "Wo.1", "bo.0", "g2.1", "W1.0", "c1.1",
                 "W2.1", "c2.0", "gf", "bf", "Wh", "bh", "be"):
        a = inp["params"][name]
        for _ in range(2):
            idx = tuple(rng.integers(0, s) for s in a.shape)
            h = 1e-5
            keep = a[idx]
            a[idx] = keep + h
            lp, _ = V.forward(cfg, inp["x"], inp["labels"], inp["params"])
            a[idx] = keep - h
            lm, _ = V.forward(cfg, inp["x"], inp["labels"], inp["params"])
            a[idx] = keep
            assert grads[name][idx] == pytest.approx((lp - lm) / (2 * h), rel=2e-5, abs=1e-8), (name, idx)


def test_patchify_by_index():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 12, 8, 3))
    out = V.patchify(x, 4)
    assert out.shape == (2, 6, 48)
    for b, py, px, r, s, ch in [(0, 0, 0, 0, 0, 0), (1, 2, 1, 3, 2, 1), (0, 1, 1, 0, 3, 2), (1, 0, 1, 2, 0, 0)]:
        assert out[b, py * 2 + px, (r * 4 + s) * 3 + ch] == x[b, py * 4 + r, px * 4 + s, ch]


def test_layernorm_closed_forms():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 7, 64)) * 3 + 1.5
    g, b = rng.standard_normal(64), rng.standard_normal(64)
    y, mean, rstd = V.layernorm_fwd(x, np.ones(64), np.zeros(64), eps=0.0)
    assert np.abs(y.mean(-1)).max() < 1e-12 and np.abs((y * y).mean(-1) - 1).max() < 1e-12
    # a constant row normalises to the offset; eps decides the scale of a row of variance v
    yc, _, _ = V.layernorm_fwd(np.full((1, 64), 4.0), g, b)
    assert np.abs(yc - b).max() < 1e-9
    row = np.tile([1.0, -1.0], 32)[None]            # mean 0, variance 1
    ye, _, _ = V.layernorm_fwd(row, np.ones(64), np.zeros(64), eps=3.0)
    assert np.abs(ye - row / 2.0).max() < 1e-15
    # the gradient is orthogonal to the two directions the normalisation removes
    dy = rng.standard_normal(x.shape)
    y2, mean, rstd = V.layernorm_fwd(x, g, b)
    dx, dg, db = V.layernorm_bwd(dy, x, g, mean, rstd)
    xh = (x - mean[..., None]) * rstd[..., None]
    assert np.abs(dx.sum(-1)).max() < 1e-12
    # ... exactly so without eps; with it, mean(xh^2) = var / (var + eps) leaves the factor eps * rstd^2
    want = rstd * ((dy * g) * xh).sum(-1) * (1e-6 * rstd * rstd)
    assert np.abs((dx * xh).sum(-1) - want).max() < 1e-13
    assert np.abs(db - dy.sum((0, 1))).max() < 1e-12
    t = torch.tensor(x, requires_grad=True)
    tg, tb = torch.tensor(g, requires_grad=True), torch.tensor(b, requires_grad=True)
    F.layer_norm(t, (64,), tg, tb, eps=1e-6).backward(torch.tensor(dy))
    assert np.abs(dx - t.grad.numpy()).max() < 1e-12 and np.abs(dg - tg.grad.numpy()).max() < 1e-12


def test_gelu_values():
    # Phi(1) = 0.8413447460685429 (standard normal distribution function), phi(1) = exp(-1/2)/sqrt(2 pi)
    assert V.gelu(np.array(1.0)) == pytest.approx(0.8413447460685429, rel=1e-15)
    assert V.gelu(np.array(0.0)) == 0.0 and V.gelu_grad(np.array(0.0)) == 0.5
    assert V.gelu_grad(np.array(1.0)) == pytest.approx(0.8413447460685429 + 0.24197072451914337, rel=1e-15)
    u = np.linspace(-6, 6, 241)
    assert np.abs(V.gelu(u) - V.gelu(-u) - u).max() < 1e-15            # u Phi(u) - (-u) Phi(-u) = u
    assert np.abs(V.gelu(np.array([30.0, -30.0])) - [30.0, 0.0]).max() < 1e-300
    h = 1e-6
    assert np.abs((V.gelu(u + h) - V.gelu(u - h)) / (2 * h) - V.gelu_grad(u)).max() < 1e-9
    assert np.abs(V.gelu(u) - F.gelu(torch.tensor(u)).numpy()).max() < 1e-15


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    B, T, h, dh = 2, 9, 3, 8
    d = h * dh
    qkv = rng.standard_normal((B, T, 3 * d))
    O, A = V.attention_fwd(qkv, h)
    assert np.abs(A.sum(-1) - 1).max() < 1e-14 and (A > 0).all()
    # zero queries: every key weighs the same, the output is the mean value vector of the head
    z = qkv.copy()
    z[:, :, :d] = 0
    Oz, Az = V.attention_fwd(z, h)
    assert np.abs(Az - 1.0 / T).max() < 1e-15
    assert np.abs(Oz - np.broadcast_to(z[:, :, 2 * d:].mean(axis=1, keepdims=True), Oz.shape)).max() < 1e-14
    # one key far closer than the rest: the output is that key's value
    s = qkv.copy()
    s[:, :, :d] = 0
    s[:, :, d:2 * d] = 0
    s[:, :, 0:dh] = 100.0                     # head 0 queries
    s[:, 4, d:d + dh] = 100.0                 # head 0, key 4
    Os, _ = V.attention_fwd(s, h)
    assert np.abs(Os[:, :, :dh] - s[:, 4:5, 2 * d:2 * d + dh]).max() < 1e-12
    # permuting keys and values together changes nothing; heads do not mix
    perm = rng.permutation(T)
    p2 = qkv.copy()
    p2[:, :, d:] = qkv[:, perm, d:]
    assert np.abs(V.attention_fwd(p2, h)[0] - O).max() < 1e-13
    m = qkv.copy()
    m[:, :, 2 * d + dh:] += 1.0               # values of heads 1, 2
    assert np.abs(V.attention_fwd(m, h)[0][:, :, :dh] - O[:, :, :dh]).max() == 0.0
    # brute force, one output element at a time
    for b, t, hh, j in [(0, 0, 0, 0), (1, 8, 2, 7), (0, 3, 1, 4)]:
        qv = qkv[b, t, hh * dh:(hh + 1) * dh]
        sc = np.array([qv @ qkv[b, u, d + hh * dh:d + (hh + 1) * dh] for u in range(T)]) / math.sqrt(dh)
        w = np.exp(sc - sc.max())
        w /= w.sum()
        want = sum(w[u] * qkv[b, u, 2 * d + hh * dh + j] for u in range(T))
        assert O[b, t, hh * dh + j] == pytest.approx(want, rel=1e-13)
    # backward against autograd through torch's fused attention
    dO = rng.standard_normal(O.shape)
    t = torch.tensor(qkv, requires_grad=True)
    q, k, v = (t[:, :, i * d:(i + 1) * d].reshape(B, T, h, dh).transpose(1, 2) for i in range(3))
    to = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, T, d)
    assert np.abs(to.detach().numpy() - O).max() < 1e-13
    to.backward(torch.tensor(dO))
    assert np.abs(V.attention_bwd(dO, qkv, A, h) - t.grad.numpy()).max() < 1e-13


def test_loss_and_update_rules():
    net, inp = small()
    cfg = net.cfg()
    # zero classifier: uniform probabilities, loss ln(classes)
    P = dict(inp["params"])
    P["Wh"] = np.zeros_like(P["Wh"])
    P["bh"] = np.zeros_like(P["bh"])
    loss, c = V.forward(cfg, inp["x"], inp["labels"], P)
    assert loss == pytest.approx(math.log(10), rel=1e-14)
    assert (c["pred"] == 0).all()                          # equal maxima: the lowest class index
    # lr = 0 leaves the parameters alone and still advances the momentum buffers
    out = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], inp["mom"], lr=0.0, momentum=0.9)
    assert all((out["params"][k] == inp["params"][k]).all() for k in inp["params"])
    assert any((out["mom"][k] != inp["mom"][k]).any() for k in inp["params"])
    # mu = 0, no decay: Algorithm 1's plain rule w <- w - eta * grad
    zero = {k: np.zeros_like(v) for k, v in inp["mom"].items()}
    out = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], zero, lr=0.05, momentum=0.0)
    for k in ("Wqkv.0", "pos", "bh"):
        assert np.abs(out["params"][k] - (inp["params"][k] - 0.05 * out["grads"][k])).max() < 1e-16
    # a small step along the negative gradient lowers the loss by about lr * |grad|^2
    out = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], zero, lr=1e-3, momentum=0.0)
    l2, _ = V.forward(cfg, inp["x"], inp["labels"], out["params"])
    g2 = sum(float((g * g).sum()) for g in out["grads"].values())
    assert out["loss"] - l2 == pytest.approx(1e-3 * g2, rel=5e-2)
    # the buffer enters linearly: a buffer V moves the new buffer by mu V and the new weights by -lr mu V
    withv = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], inp["mom"], lr=0.25, momentum=0.5)
    nov = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], zero, lr=0.25, momentum=0.5)
    for k in ("W1.0", "cls", "gf"):
        assert np.abs(withv["mom"][k] - nov["mom"][k] - 0.5 * inp["mom"][k]).max() < 1e-16
        assert np.abs(withv["params"][k] - nov["params"][k] + 0.125 * inp["mom"][k]).max() < 1e-16
    # weight decay: grad + wd * w enters the buffer
    out = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], zero, lr=0.1, momentum=0.0, weight_decay=0.5)
    assert np.abs(out["mom"]["Wo.1"] - (out["grads"]["Wo.1"] + 0.5 * inp["params"]["Wo.1"])).max() < 1e-16


def test_bf16_storage_points():
    net, inp = small(dtype="bf16")
    out = V.train_step(net.cfg(), inp["x"], inp["labels"], inp["params"], inp["mom"], storage="bf16")
    c, da = out["cache"], out["dacts"]
    for k in ("X0", "H.0", "QKV.1", "O.0", "Xmid.1", "H2.0", "U.1", "G.0", "Xout", "F"):
        assert (V.round_bf16(c[k]) == c[k]).all(), k
    for k, v in da.items():
        assert (V.round_bf16(v) == v).all(), k
    assert any((V.round_bf16(g) != g).any() for g in out["grads"].values())     # parameter gradients stay exact
    ref = V.train_step(net.cfg(), inp["x"], inp["labels"], inp["params"], inp["mom"])
    assert abs(out["loss"] - ref["loss"]) < 2e-2
    # round_bf16 itself: ties to even on hand-computed cases (1 + 2^-8 is the midpoint above 1)
    assert V.round_bf16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20])).tolist() == \
        [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]
    assert (V.round_bf16(np.array([0.1, -3.3])) == torch.tensor([0.1, -3.3]).to(torch.bfloat16).double().numpy()).all()


def test_epoch_loop_chains_steps_and_keeps_the_best_checkpoint():
    net = WL.vit_mini(batch=4, dtype="f32", image=16, patch=4, dim=32, heads=2, layers=1, mlp=48, classes=5)
    cfg = net.cfg()
    inp = WL.make_vit_inputs(net, config_id=65)
    ds = WL.make_vit_dataset(net, 65, n_train=16, n_val=8, signal=1.0)
    orders = WL.epoch_orders(65, 16, 4, 3)
    lrs = [0.05] * 12
    out = V.fit(cfg, 4, ds["train_x"], ds["train_y"], ds["val_x"], ds["val_y"], inp["params"], inp["mom"], orders, lrs)
    # the loop is nothing but the step chained over the mini-batches in the given order
    P, M = inp["params"], inp["mom"]
    losses = []
    for e in range(3):
        for b in range(4):
            idx = orders[e][4 * b:4 * b + 4]
            r = V.train_step(cfg, ds["train_x"][idx], ds["train_y"][idx], P, M, 0.05, 0.9, 0.0)
            P, M = r["params"], r["mom"]
            losses.append(r["loss"])
    assert all((out["params"][k] == P[k]).all() for k in P)
    assert [h[0] for h in out["history"]] == [float(np.mean(losses[4 * e:4 * e + 4])) for e in range(3)]
    # validation: accuracy is the fraction of the oracle's own predictions that match; best = first maximum
    acc, vloss, pred = V.evaluate(cfg, 4, ds["val_x"], ds["val_y"], P)
    assert acc == float(np.mean(pred == ds["val_y"])) and (acc, vloss) == out["history"][-1][1:]
    accs = [h[1] for h in out["history"]]
    assert out["best"]["epoch"] == int(np.argmax(accs)) and out["best"]["acc"] == max(accs)
    # zero learning rate: parameters stay, every epoch validates the same
    z = V.fit(cfg, 4, ds["train_x"], ds["train_y"], ds["val_x"], ds["val_y"], inp["params"], inp["mom"], orders[:2], [0.0] * 8)
    assert all((z["params"][k] == inp["params"][k]).all() for k in inp["params"]) and z["history"][0][1:] == z["history"][1][1:]
    # a set that can be learnt is learnt: the training loss falls over a few epochs
    more = V.fit(cfg, 4, ds["train_x"], ds["train_y"], ds["val_x"], ds["val_y"], inp["params"], inp["mom"],
                 WL.epoch_orders(65, 16, 4, 12), [0.05] * 48)
    assert more["history"][-1][0] < 0.75 * more["history"][0][0]
