"""Pins of the fp64 oracle against things other than itself: brute force on tiny tensors,
closed forms, adjoint identities, finite differences, special cases that reduce to a matrix
product, and torch's CPU float64 library operators.  CPU only."""
import os
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as WL
from oracle import ops, train_step, forward_loss

RNG = np.random.default_rng(1234)
GOLDEN = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")) as fh:
    for line in fh:
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            GOLDEN[k] = float(v)

CONV_CASES = [  # N,H,W,Cin,Cout,R,stride,pad
    (2, 5, 5, 3, 4, 3, 1, 1), (2, 6, 6, 3, 5, 3, 2, 1), (1, 7, 5, 2, 3, 3, 2, 1),
    (2, 4, 4, 3, 2, 1, 1, 0), (2, 6, 6, 4, 3, 1, 2, 0), (1, 5, 5, 2, 2, 3, 1, 0), (1, 8, 8, 2, 3, 3, 3, 1),
]


def nchw(a):
    return torch.from_numpy(np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2))))


def nhwc(t):
    return np.transpose(t.detach().numpy(), (0, 2, 3, 1))


def w_oihw(w):
    return torch.from_numpy(np.ascontiguousarray(np.transpose(w, (0, 3, 1, 2))))


def relerr(a, b):
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def brute_conv(x, w, stride, pad):
    """Independent definition: explicit zero-padded image, patch matrix, naive dot products."""
    N, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, Cin))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, Ho, Wo, Cout))
    for n in range(N):
        for i in range(Ho):
            for j in range(Wo):
                patch = xp[n, i * stride:i * stride + R, j * stride:j * stride + S, :].reshape(-1)
                for k in range(Cout):
                    y[n, i, j, k] = sum(float(a) * float(b) for a, b in zip(patch, w[k].reshape(-1)))
    return y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_brute_force_and_torch(case):
    N, H, W, Cin, Cout, R, st, p = case
    x = RNG.standard_normal((N, H, W, Cin))
    w = RNG.standard_normal((Cout, R, R, Cin))
    y = ops.conv2d_fwd(x, w, st, p)
    assert y.shape == (N, (H + 2 * p - R) // st + 1, (W + 2 * p - R) // st + 1, Cout)
    assert relerr(y, brute_conv(x, w, st, p)) < 1e-12
    assert relerr(y, nhwc(TF.conv2d(nchw(x), w_oihw(w), stride=st, padding=p))) < 1e-12


def test_conv_1x1_is_matrix_product():
    x = RNG.standard_normal((3, 4, 5, 6))
    w = RNG.standard_normal((7, 1, 1, 6))
    y = ops.conv2d_fwd(x, w, 1, 0)
    assert relerr(y.reshape(-1, 7), x.reshape(-1, 6) @ w.reshape(7, 6).T) < 1e-13


def test_conv_delta_kernels_shift_with_zero_fill():
    x = RNG.standard_normal((2, 6, 7, 3))
    for r in range(3):
        for s in range(3):
            w = np.zeros((3, 3, 3, 3))
            for c in range(3):
                w[c, r, s, c] = 1.0
            y = ops.conv2d_fwd(x, w, 1, 1)
            expect = np.zeros_like(x)
            for h in range(6):
                for ww in range(7):
                    hi, wi = h + r - 1, ww + s - 1
                    if 0 <= hi < 6 and 0 <= wi < 7:
                        expect[:, h, ww, :] = x[:, hi, wi, :]
            assert np.array_equal(y, expect)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identities(case):
    N, H, W, Cin, Cout, R, st, p = case
    x = RNG.standard_normal((N, H, W, Cin))
    w = RNG.standard_normal((Cout, R, R, Cin))
    y = ops.conv2d_fwd(x, w, st, p)
    dy = RNG.standard_normal(y.shape)
    dx = ops.conv2d_dgrad(dy, w, x.shape, st, p)
    dw = ops.conv2d_wgrad(x, dy, w.shape, st, p)
    lhs = np.sum(y * dy)
    assert abs(lhs - np.sum(x * dx)) <= 1e-12 * max(1.0, abs(lhs))
    assert abs(lhs - np.sum(w * dw)) <= 1e-12 * max(1.0, abs(lhs))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_grads_match_torch_autograd(case):
    N, H, W, Cin, Cout, R, st, p = case
    x = RNG.standard_normal((N, H, W, Cin))
    w = RNG.standard_normal((Cout, R, R, Cin))
    tx = nchw(x).requires_grad_(True)
    tw = w_oihw(w).requires_grad_(True)
    ty = TF.conv2d(tx, tw, stride=st, padding=p)
    dy = RNG.standard_normal(nhwc(ty).shape)
    ty.backward(nchw(dy))
    assert relerr(ops.conv2d_dgrad(dy, w, x.shape, st, p), nhwc(tx.grad)) < 1e-12
    assert relerr(ops.conv2d_wgrad(x, dy, w.shape, st, p), np.transpose(tw.grad.numpy(), (0, 2, 3, 1))) < 1e-12


def test_conv_grads_finite_differences():
    N, H, W, Cin, Cout, R, st, p = 2, 6, 6, 3, 4, 3, 2, 1
    x = RNG.standard_normal((N, H, W, Cin))
    w = RNG.standard_normal((Cout, R, R, Cin))
    dy = RNG.standard_normal(ops.conv2d_fwd(x, w, st, p).shape)
    phi = lambda xx, ww: float(np.sum(ops.conv2d_fwd(xx, ww, st, p) * dy))
    dx = ops.conv2d_dgrad(dy, w, x.shape, st, p)
    dw = ops.conv2d_wgrad(x, dy, w.shape, st, p)
    h = 1e-6
    for _ in range(20):
        i = tuple(RNG.integers(0, s) for s in x.shape)
        e = np.zeros_like(x); e[i] = h
        fd = (phi(x + e, w) - phi(x - e, w)) / (2 * h)
        assert abs(fd - dx[i]) <= 1e-7 * max(1.0, abs(dx[i]))
        j = tuple(RNG.integers(0, s) for s in w.shape)
        e = np.zeros_like(w); e[j] = h
        fd = (phi(x, w + e) - phi(x, w - e)) / (2 * h)
        assert abs(fd - dw[j]) <= 1e-7 * max(1.0, abs(dw[j]))


def test_bn_fwd_invariants_and_torch():
    x = 3.0 + 2.0 * RNG.standard_normal((4, 5, 6, 7))
    C = 7
    y, mean, invstd = ops.bn_relu_fwd(x, np.ones(C), np.zeros(C), relu=False)
    var = x.reshape(-1, C).var(axis=0)
    assert np.max(np.abs(y.reshape(-1, C).mean(axis=0))) < 1e-12
    assert np.allclose(y.reshape(-1, C).var(axis=0), var / (var + 1e-5), rtol=1e-12)
    assert np.allclose(mean, x.reshape(-1, C).mean(axis=0), rtol=1e-13)
    assert np.allclose(invstd, 1 / np.sqrt(var + 1e-5), rtol=1e-13)
    beta = RNG.standard_normal(C)
    yc, _, _ = ops.bn_relu_fwd(np.full((2, 3, 3, C), 5.0), RNG.standard_normal(C), beta, relu=False)
    assert np.allclose(yc, beta.reshape(1, 1, 1, C), atol=1e-12)
    # library cross-check incl. running statistics (momentum 0.1, unbiased running variance)
    g = 1 + 0.1 * RNG.standard_normal(C)
    rm = RNG.standard_normal(C); rv = 1 + RNG.random(C)
    trm, trv = torch.from_numpy(rm.copy()), torch.from_numpy(rv.copy())
    ty = TF.batch_norm(nchw(x), trm, trv, torch.from_numpy(g), torch.from_numpy(beta), True, 0.1, 1e-5)
    res = RNG.standard_normal(x.shape)
    y2, _, _ = ops.bn_relu_fwd(x, g, beta, relu=True, residual=res, running_mean=rm, running_var=rv)
    assert relerr(y2, np.maximum(nhwc(ty) + res, 0)) < 1e-12
    assert np.allclose(rm, trm.numpy(), rtol=1e-12) and np.allclose(rv, trv.numpy(), rtol=1e-12)


@pytest.mark.parametrize("relu,with_res", [(False, False), (True, False), (True, True), (False, True)])
def test_bn_bwd_invariants_fd_and_torch(relu, with_res):
    C = 5
    x = 1.0 + RNG.standard_normal((3, 4, 4, C))
    g = 1 + 0.1 * RNG.standard_normal(C)
    b = 0.1 * RNG.standard_normal(C)
    res = RNG.standard_normal(x.shape) if with_res else None
    y, mean, invstd = ops.bn_relu_fwd(x, g, b, relu=relu, residual=res)
    dy = RNG.standard_normal(x.shape)
    dx, dres, dg, db = ops.bn_relu_bwd(dy, x, y, g, mean, invstd, relu=relu, want_dres=with_res)
    xhat = (x - mean) * invstd
    assert np.max(np.abs(dx.reshape(-1, C).sum(axis=0))) < 1e-12
    # sum(dx*xhat) = gamma*invstd*dgamma*(1 - var/(var+eps)): zero up to the eps regulariser
    assert np.allclose((dx * xhat).reshape(-1, C).sum(axis=0), g * invstd * dg * 1e-5 * invstd ** 2,
                       rtol=1e-6, atol=1e-13)
    mask = (y > 0) if relu else np.ones_like(y, dtype=bool)
    if with_res:
        assert np.array_equal(dres, dy * mask)
    # torch autograd through the batch statistics
    tx = nchw(x).requires_grad_(True)
    tg = torch.from_numpy(g).requires_grad_(True)
    tb = torch.from_numpy(b).requires_grad_(True)
    tu = TF.batch_norm(tx, None, None, tg, tb, True, 0.1, 1e-5)
    if with_res:
        tr = nchw(res).requires_grad_(True)
        tu = tu + tr
    ty = torch.relu(tu) if relu else tu
    ty.backward(nchw(dy))
    assert relerr(dx, nhwc(tx.grad)) < 1e-11
    assert relerr(dg, tg.grad.numpy()) < 1e-12 and relerr(db, tb.grad.numpy()) < 1e-12
    if with_res:
        assert relerr(dres, nhwc(tr.grad)) < 1e-13
    # finite differences of sum(y*dy) w.r.t. x, through mean and variance
    f = lambda xx: float(np.sum(ops.bn_relu_fwd(xx, g, b, relu=relu, residual=res)[0] * dy))
    h = 1e-6
    for _ in range(10):
        i = tuple(RNG.integers(0, s) for s in x.shape)
        e = np.zeros_like(x); e[i] = h
        fd = (f(x + e) - f(x - e)) / (2 * h)
        assert abs(fd - dx[i]) <= 2e-7 * max(1.0, abs(dx[i]))


def test_pool_brute_force_ties_and_torch():
    x = RNG.standard_normal((2, 4, 6, 3))
    y, am = ops.pool_fwd(x, "max2")
    for n in range(2):
        for i in range(2):
            for j in range(3):
                for c in range(3):
                    win = [x[n, 2 * i + dr, 2 * j + dc, c] for dr in range(2) for dc in range(2)]
                    assert y[n, i, j, c] == max(win)
                    assert am[n, i, j, c] == win.index(max(win))
    assert relerr(y, nhwc(TF.max_pool2d(nchw(x), 2))) == 0.0
    # ties: first maximal element in (row, col) scan order
    xt = np.zeros((1, 2, 2, 4))
    xt[0, :, :, 1] = [[1, 5], [5, 5]]
    xt[0, :, :, 2] = [[0, 0], [7, 7]]
    xt[0, :, :, 3] = [[-1, -1], [-1, -0.5]]
    _, amt = ops.pool_fwd(xt, "max2")
    assert amt.reshape(-1).tolist() == [0, 1, 2, 3]
    dy = RNG.standard_normal(y.shape)
    dx = ops.pool_bwd(dy, am, x.shape, "max2")
    assert abs(dx.sum() - dy.sum()) < 1e-12 and np.count_nonzero(dx) == dy.size
    tx = nchw(x).requires_grad_(True)
    TF.max_pool2d(tx, 2).backward(nchw(dy))
    assert np.array_equal(dx, nhwc(tx.grad))
    # global average pool
    g, _ = ops.pool_fwd(x, "gap")
    assert np.allclose(g.reshape(2, 3), x.mean(axis=(1, 2)), rtol=1e-13)
    dg = RNG.standard_normal((2, 1, 1, 3))
    dxg = ops.pool_bwd(dg, None, x.shape, "gap")
    assert np.allclose(dxg, np.broadcast_to(dg / 24.0, x.shape), rtol=1e-15)


def test_fc_softmax_xent_closed_forms_fd_and_torch():
    N, F, K = 6, 9, 100
    x = RNG.standard_normal((N, F)); Wm = RNG.standard_normal((K, F)) * 0.3; b = RNG.standard_normal(K) * 0.1
    lab = RNG.integers(0, K, N).astype(np.int32)
    r = ops.fc_softmax_xent(x, Wm, b, lab)
    assert np.max(np.abs(r["probs"].sum(axis=1) - 1)) < 1e-14
    z = np.array([[sum(x[n, f] * Wm[j, f] for f in range(F)) + b[j] for j in range(K)] for n in range(N)])
    assert np.array_equal(r["pred"], z.argmax(axis=1))
    dz = (r["probs"] - np.eye(K)[lab]) / N
    assert np.max(np.abs(dz.sum(axis=1))) < 1e-15
    assert relerr(r["dW"], dz.T @ x) < 1e-13 and relerr(r["db"], dz.sum(0)) < 1e-13 and relerr(r["dx"], dz @ Wm) < 1e-13
    # zero logits: L = ln(100), uniform probabilities
    r0 = ops.fc_softmax_xent(x, np.zeros((K, F)), np.zeros(K), lab)
    assert abs(r0["loss"] - GOLDEN["ln_100"]) < 1e-14
    assert np.allclose(r0["probs"], GOLDEN["uniform_prob_100"], rtol=1e-14)
    assert all(p == 0 for p in r0["pred"])          # lowest index on ties
    # shift invariance
    r1 = ops.fc_softmax_xent(x, Wm, b + 123.0, lab)
    assert abs(r1["loss"] - r["loss"]) < 1e-12 and relerr(r1["dW"], r["dW"]) < 1e-11
    # library cross-check
    tx = torch.from_numpy(x).requires_grad_(True); tW = torch.from_numpy(Wm).requires_grad_(True)
    tb = torch.from_numpy(b).requires_grad_(True)
    tl = TF.cross_entropy(tx @ tW.T + tb, torch.from_numpy(lab.astype(np.int64)))
    tl.backward()
    assert abs(tl.item() - r["loss"]) < 1e-13
    assert relerr(r["dW"], tW.grad.numpy()) < 1e-12 and relerr(r["dx"], tx.grad.numpy()) < 1e-12
    assert relerr(r["db"], tb.grad.numpy()) < 1e-12
    # finite differences
    h = 1e-6
    L = lambda xx, WW, bb: ops.fc_softmax_xent(xx, WW, bb, lab)["loss"]
    for _ in range(10):
        i = tuple(RNG.integers(0, s) for s in Wm.shape); e = np.zeros_like(Wm); e[i] = h
        assert abs((L(x, Wm + e, b) - L(x, Wm - e, b)) / (2 * h) - r["dW"][i]) < 1e-8
        i = tuple(RNG.integers(0, s) for s in x.shape); e = np.zeros_like(x); e[i] = h
        assert abs((L(x + e, Wm, b) - L(x - e, Wm, b)) / (2 * h) - r["dx"][i]) < 1e-8


def test_sgd_momentum_closed_form():
    mu, lr, k = 0.9, 0.1, 3
    w = np.zeros(4); v = np.zeros(4); g = np.ones(4)
    for _ in range(k):
        ops.sgd_momentum(w, v, g, lr, mu)
    assert np.allclose(v, GOLDEN["sgd_v_3"], rtol=1e-14) and np.allclose(w, GOLDEN["sgd_w_3"], rtol=1e-14)
    assert np.allclose(v, (1 - mu ** k) / (1 - mu)) and np.allclose(w, -lr * (k - mu * (1 - mu ** k) / (1 - mu)) / (1 - mu))
    # mu = 0, no decay: the plain rule theta <- theta - eta*grad
    w = RNG.standard_normal(5); w0 = w.copy(); v = RNG.standard_normal(5); g = RNG.standard_normal(5)
    ops.sgd_momentum(w, v, g, 0.05, 0.0)
    assert np.allclose(w, w0 - 0.05 * g, rtol=1e-15)
    # weight decay enters the gradient
    w = np.ones(3); v = np.zeros(3)
    ops.sgd_momentum(w, v, np.zeros(3), 0.1, 0.9, 0.5)
    assert np.allclose(v, 0.5) and np.allclose(w, 0.95)


NETS = {"tiny": lambda: WL.tiny_cnn(batch=4, size=8, cout=8), "mini_resnet": WL.mini_resnet,
        "mini_preact": WL.mini_preact}


@pytest.mark.parametrize("name", list(NETS))
def test_whole_step_finite_differences(name):
    net = NETS[name]()
    inp = WL.make_inputs(net, 77, perturb_bn=True)
    out = train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"], lr=0.1, momentum=0.9)
    rng = np.random.default_rng(5)
    h = 1e-6
    for k, p in enumerate(inp["params"]):
        g = out["grads"][k]
        scale = max(np.max(np.abs(g)), 1e-3)
        for _ in range(min(p.size, 6)):
            i = tuple(rng.integers(0, s) for s in p.shape)
            ps = [q.copy() for q in inp["params"]]
            ps[k][i] += h
            lp = forward_loss(net, inp["x"], inp["labels"], ps)[0]
            ps[k][i] -= 2 * h
            lm = forward_loss(net, inp["x"], inp["labels"], ps)[0]
            assert abs((lp - lm) / (2 * h) - g[i]) <= 2e-6 * scale, (name, k, i)
    # update rule applied to every parameter
    for p, v, g, p2, v2 in zip(inp["params"], inp["mom"], out["grads"], out["params"], out["mom"]):
        assert np.allclose(v2, 0.9 * v + g, rtol=1e-13, atol=1e-300)
        assert np.allclose(p2, p - 0.1 * (0.9 * v + g), rtol=1e-13, atol=1e-300)


def test_whole_step_first_order_descent():
    net = WL.mini_resnet()
    inp = WL.make_inputs(net, 78, zero_momentum=True)
    eta = 1e-5
    out = train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"], lr=eta, momentum=0.0)
    l1 = forward_loss(net, inp["x"], inp["labels"], out["params"])[0]
    gnorm2 = sum(float(np.sum(g * g)) for g in out["grads"])
    assert abs((out["loss"] - l1) - eta * gnorm2) <= 1e-3 * eta * gnorm2


def test_step_matches_torch_autograd_on_mini_resnet():
    """Independent chain: the same layer list evaluated with torch float64 library ops + autograd."""
    for net in (WL.mini_resnet(), WL.mini_preact()):
        inp = WL.make_inputs(net, 79, perturb_bn=True)
        out = train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"])
        tp = [torch.from_numpy(p.copy()).requires_grad_(True) for p in inp["params"]]
        acts = {0: nchw(inp["x"])}
        for L in net.layers:
            if L["op"] == "conv":
                acts[L["y"]] = TF.conv2d(acts[L["x"]], tp[L["w"]].permute(0, 3, 1, 2), stride=L["stride"], padding=L["pad"])
            elif L["op"] == "bn":
                u = TF.batch_norm(acts[L["x"]], None, None, tp[L["gamma"]], tp[L["beta"]], True, 0.1, 1e-5)
                if L["res"] >= 0:
                    u = u + acts[L["res"]]
                acts[L["y"]] = torch.relu(u) if L["relu"] else u
            elif L["op"] == "pool":
                acts[L["y"]] = TF.max_pool2d(acts[L["x"]], 2) if L["mode"] == "max2" else acts[L["x"]].mean(dim=(2, 3), keepdim=True)
            elif L["op"] == "add":
                acts[L["y"]] = acts[L["a"]] + acts[L["b"]]
            else:
                z = acts[L["x"]].reshape(L["N"], L["F"]) @ tp[L["W"]].T + tp[L["b"]]
                loss = TF.cross_entropy(z, torch.from_numpy(inp["labels"].astype(np.int64)))
        loss.backward()
        assert abs(loss.item() - out["loss"]) < 1e-12
        for k, t in enumerate(tp):
            assert relerr(out["grads"][k], t.grad.numpy()) < 1e-9, (net.name, k)


def test_round_bf16_matches_library_conversion_and_ties():
    a = np.concatenate([RNG.standard_normal(5000) * 10.0 ** RNG.integers(-6, 6, 5000), [0.0, -0.0, 1.0, -3.5]])
    a = a.astype(np.float32).astype(np.float64)
    got = ops.round_bf16(a)
    lib = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, lib)
    # ties go to the even significand: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert ops.round_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert ops.round_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert ops.round_bf16(np.array([1 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1 + 2.0 ** -7
    # already representable values are fixed points (the seeded bf16 inputs stay untouched)
    assert np.array_equal(ops.round_bf16(WL.to_bf16_representable(a)), WL.to_bf16_representable(a))


def test_storage_emulation_only_rounds_stores():
    net = WL.mini_resnet()
    inp = WL.make_inputs(net, 81)
    pure = train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"])
    emu = train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"], storage="bf16")
    for s, a in emu["acts"].items():
        if s != 0:
            assert np.array_equal(a, ops.round_bf16(a))
    for s, g in emu["dacts"].items():
        assert np.array_equal(g, ops.round_bf16(g))
    assert abs(emu["loss"] - pure["loss"]) < 2e-2 * pure["loss"]
    for ge, gp in zip(emu["grads"], pure["grads"]):
        assert np.max(np.abs(ge - gp)) <= 0.25 * np.max(np.abs(gp))   # tiny net: a sanity bound only


def test_storage_jitter_is_a_bounded_seeded_perturbation_of_the_rounding_only():
    """The jittered bf16-storage walk: amplitude 0 is the plain bf16-storage walk bit for bit; a
    seed fixes the walk; everything stored is still a bf16 value; and the first stored tensor (the
    first convolution's output, whose inputs no jitter has touched yet) lies within the stated
    amplitude plus half a bf16 unit in the last place of the exact value."""
    net = WL.mini_resnet()
    inp = WL.make_inputs(net, 82)
    args = (net, inp["x"], inp["labels"], inp["params"], inp["mom"])
    plain = train_step(*args, storage="bf16")
    zero = train_step(*args, storage="bf16", jitter=(5, 0.0))
    for k in range(len(plain["grads"])):
        assert np.array_equal(plain["grads"][k], zero["grads"][k])
    rel = 2.0 ** -12     # exaggerated so that many roundings move
    a = train_step(*args, storage="bf16", jitter=(5, rel))
    b = train_step(*args, storage="bf16", jitter=(5, rel))
    c = train_step(*args, storage="bf16", jitter=(6, rel))
    assert all(np.array_equal(x, y) for x, y in zip(a["grads"], b["grads"]))
    assert any(not np.array_equal(x, y) for x, y in zip(a["grads"], c["grads"]))
    for s, t in a["acts"].items():
        if s != 0:
            assert np.array_equal(t, ops.round_bf16(t))
    first = net.layers[0]
    assert first["op"] == "conv" and first["x"] == 0
    exact = ops.conv2d_fwd(inp["x"], inp["params"][first["w"]], first["stride"], first["pad"])
    rms = np.sqrt(np.mean(exact ** 2))
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 1e-300))) - 7)
    assert np.all(np.abs(a["acts"][first["y"]] - exact) <= rel * rms + 0.5 * ulp * (1 + 1e-9) + rel * rms * 2.0 ** -7)
    assert not np.array_equal(a["acts"][first["y"]], plain["acts"][first["y"]])
    with pytest.raises(ValueError):
        train_step(*args, jitter=(5, rel))


def test_storage_jitter_keeps_zeros_and_signs():
    """Clamped activations and masked gradients are exact zeros in any implementation: the jitter
    leaves them (and every sign) alone, so the ensemble's ReLU masks differ only through values
    computed downstream of a moved rounding, and a member stays as close to the float64 walk as
    the plain bf16-storage walk is (same order of magnitude, not the O(1) of a randomised mask)."""
    net = WL.mini_resnet(batch=8, size=8, widths=(16, 32))
    inp = WL.make_inputs(net, 83)
    args = (net, inp["x"], inp["labels"], inp["params"], inp["mom"])
    pure = train_step(*args)
    plain = train_step(*args, storage="bf16")
    from oracle.ensemble import JITTER_REL, JITTER_SEEDS
    for seed in JITTER_SEEDS:
        m = train_step(*args, storage="bf16", jitter=(seed, JITTER_REL))
        relu_out = [L["y"] for L in net.layers if L["op"] == "bn" and L["relu"]]
        for s in relu_out:
            assert np.all(m["acts"][s] >= 0.0)
            assert 0.2 < np.mean(m["acts"][s] == 0.0) < 0.8          # about half the units are clamped
        for k, g in enumerate(pure["grads"]):
            dm = np.linalg.norm(m["grads"][k] - g)
            dp = np.linalg.norm(plain["grads"][k] - g)
            assert dm <= 3.0 * dp + 2e-2 * np.linalg.norm(g), (seed, k, dm, dp)
