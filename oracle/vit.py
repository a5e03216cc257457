"""fp64 oracle of one training step of a Vision Transformer classifier (the paper's second model
family, Section IV-A: ViT-B/16; the step is the inner loop of Algorithm 1: forward pass, loss,
backward pass, parameter update).  TEST INFRASTRUCTURE ONLY; numpy, no blocking, no fusion.

The paper names the model and nothing else.  The reading taken is the standard pre-norm ViT:

  patches   P[b, i] = the p x p x 3 pixels of patch i (row-major over the patch grid), flattened in
            (row, column, channel) order
  tokens    X0[b, 0] = cls + pos[0];   X0[b, 1 + i] = P[b, i] @ We^T + be + pos[1 + i]
  block l   H  = LN(X; g1, b1)                          QKV = H @ Wqkv^T + bqkv   (q | k | v, head-major)
            S  = q k^T / sqrt(dh) per head,  A = softmax(S) over keys,  O = A v   (heads concatenated)
            X  = X + O @ Wo^T + bo
            H2 = LN(X; g2, b2)                          U = H2 @ W1^T + c1,   G = gelu(U)   (exact, erf)
            X  = X + G @ W2^T + c2
  head      F = LN(X[:, 0]; gf, bf)                     logits = F @ Wh^T + bh,  mean cross-entropy
  LN(x)     = (x - mean) / sqrt(var + eps) * g + b over the feature axis, biased variance, eps 1e-6
  update    v <- mu v + (grad + wd w);  w <- w - lr v   on every parameter (Algorithm 1's update)

storage='bf16' rounds every activation and activation gradient to bfloat16 where a bf16-storage
implementation keeps it (tokens, LN outputs, QKV, attention output, the residual stream after each
sum, U, G, F, and the gradient of each of them); parameter gradients are not rounded.  `q` replaces
that rounding (used for the seeded ensemble of equally legal bf16 walks).
"""
from __future__ import annotations
import numpy as np
from scipy.special import erf

LN_EPS = 1e-6

# parameter order of one encoder block and of the whole model
BLOCK_PARAMS = ("g1", "b1", "Wqkv", "bqkv", "Wo", "bo", "g2", "b2", "W1", "c1", "W2", "c2")


def param_names(layers):
    names = ["We", "be", "cls", "pos"]
    for l in range(layers):
        names += ["%s.%d" % (n, l) for n in BLOCK_PARAMS]
    return names + ["gf", "bf", "Wh", "bh"]


def round_bf16(a):
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def patchify(x, p):
    """x [B, H, W, C] -> [B, (H/p)(W/p), p*p*C]."""
    B, H, W, C = x.shape
    gh, gw = H // p, W // p
    out = np.empty((B, gh * gw, p * p * C))
    for py in range(gh):
        for px in range(gw):
            out[:, py * gw + px] = x[:, py * p:(py + 1) * p, px * p:(px + 1) * p, :].reshape(B, -1)
    return out


def layernorm_fwd(x, g, b, eps=LN_EPS):
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    return (x - mean) * rstd * g + b, mean[..., 0], rstd[..., 0]


def layernorm_bwd(dy, x, g, mean, rstd):
    """Gradient of layernorm_fwd.  Returns (dx, dg, db)."""
    xh = (x - mean[..., None]) * rstd[..., None]
    dxh = dy * g
    C = x.shape[-1]
    dx = rstd[..., None] * (dxh - dxh.mean(axis=-1, keepdims=True) - xh * (dxh * xh).sum(axis=-1, keepdims=True) / C)
    red = tuple(range(x.ndim - 1))
    return dx, (dy * xh).sum(axis=red), dy.sum(axis=red)


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def gelu_grad(u):
    return 0.5 * (1.0 + erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def attention_fwd(qkv, heads):
    """qkv [B, T, 3 d] (q | k | v, each head-major) -> (O [B, T, d], A [B, heads, T, T])."""
    B, T, d3 = qkv.shape
    d = d3 // 3
    dh = d // heads
    q, k, v = (qkv[:, :, i * d:(i + 1) * d].reshape(B, T, heads, dh).transpose(0, 2, 1, 3) for i in range(3))
    S = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    S = S - S.max(axis=-1, keepdims=True)
    A = np.exp(S)
    A /= A.sum(axis=-1, keepdims=True)
    O = (A @ v).transpose(0, 2, 1, 3).reshape(B, T, d)
    return O, A


def attention_bwd(dO, qkv, A, heads):
    B, T, d3 = qkv.shape
    d = d3 // 3
    dh = d // heads
    q, k, v = (qkv[:, :, i * d:(i + 1) * d].reshape(B, T, heads, dh).transpose(0, 2, 1, 3) for i in range(3))
    dOh = dO.reshape(B, T, heads, dh).transpose(0, 2, 1, 3)
    dv = A.transpose(0, 1, 3, 2) @ dOh
    dA = dOh @ v.transpose(0, 1, 3, 2)
    dS = A * (dA - (dA * A).sum(axis=-1, keepdims=True)) / np.sqrt(dh)
    dq = dS @ k
    dk = dS.transpose(0, 1, 3, 2) @ q
    back = lambda t: t.transpose(0, 2, 1, 3).reshape(B, T, d)
    return np.concatenate([back(dq), back(dk), back(dv)], axis=-1)


def softmax_xent(logits, labels):
    """Mean cross-entropy, predictions (lowest index among equal maxima), d loss / d logits."""
    N = logits.shape[0]
    z = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    loss = float(-np.mean(np.log(p[np.arange(N), labels])))
    pred = np.argmax(logits, axis=1).astype(np.int32)
    dl = p.copy()
    dl[np.arange(N), labels] -= 1.0
    return loss, pred, p, dl / N


def _quantiser(storage, q):
    if q is not None:
        return q
    if storage is None:
        return lambda a: a
    if storage == "bf16":
        return round_bf16
    raise ValueError(storage)


def forward(cfg, x, labels, P, storage=None, q=None):
    """cfg: dict(patch, dim, heads, layers, mlp, classes); P: {name: array}.  Returns (loss, cache)."""
    q = _quantiser(storage, q)
    B = x.shape[0]
    d = cfg["dim"]
    c = {}
    c["patches"] = patchify(np.asarray(x, dtype=np.float64), cfg["patch"])
    n = c["patches"].shape[1]
    X = np.empty((B, n + 1, d))
    X[:, 0] = P["cls"] + P["pos"][0]
    X[:, 1:] = c["patches"] @ P["We"].T + P["be"] + P["pos"][1:]
    X = q(X)
    c["X0"] = X
    for l in range(cfg["layers"]):
        g = lambda name: P["%s.%d" % (name, l)]
        c["Xin.%d" % l] = X
        H, c["m1.%d" % l], c["r1.%d" % l] = layernorm_fwd(X, g("g1"), g("b1"))
        H = q(H)
        QKV = q(H @ g("Wqkv").T + g("bqkv"))
        O, A = attention_fwd(QKV, cfg["heads"])
        O = q(O)
        X = q(X + O @ g("Wo").T + g("bo"))
        c["H.%d" % l], c["QKV.%d" % l], c["A.%d" % l], c["O.%d" % l], c["Xmid.%d" % l] = H, QKV, A, O, X
        H2, c["m2.%d" % l], c["r2.%d" % l] = layernorm_fwd(X, g("g2"), g("b2"))
        H2 = q(H2)
        U = q(H2 @ g("W1").T + g("c1"))
        G = q(gelu(U))
        X = q(X + G @ g("W2").T + g("c2"))
        c["H2.%d" % l], c["U.%d" % l], c["G.%d" % l] = H2, U, G
    c["Xout"] = X
    F, c["mf"], c["rf"] = layernorm_fwd(X[:, 0], P["gf"], P["bf"])
    F = q(F)
    c["F"] = F
    logits = F @ P["Wh"].T + P["bh"]
    loss, pred, probs, dlogits = softmax_xent(logits, np.asarray(labels))
    c.update(logits=logits, pred=pred, probs=probs, dlogits=dlogits)
    return loss, c


def backward(cfg, P, c, storage=None, q=None):
    """Chain rule through `forward` in reverse.  Returns ({name: gradient}, {name: activation gradient})."""
    q = _quantiser(storage, q)
    G, dA = {}, {}
    dl = c["dlogits"]
    G["Wh"] = dl.T @ c["F"]
    G["bh"] = dl.sum(axis=0)
    dF = q(dl @ P["Wh"])
    dA["F"] = dF
    dx0, G["gf"], G["bf"] = layernorm_bwd(dF, c["Xout"][:, 0], P["gf"], c["mf"], c["rf"])
    dX = np.zeros_like(c["Xout"])
    dX[:, 0] = dx0
    dX = q(dX)
    dA["Xout"] = dX
    for l in range(cfg["layers"] - 1, -1, -1):
        g = lambda name: P["%s.%d" % (name, l)]
        n = lambda name: "%s.%d" % (name, l)
        B, T, d = dX.shape
        # X = Xmid + G @ W2^T + c2
        G[n("W2")] = dX.reshape(B * T, d).T @ c[n("G")].reshape(B * T, -1)
        G[n("c2")] = dX.sum(axis=(0, 1))
        dG = q(dX @ g("W2"))
        dU = q(dG * gelu_grad(c[n("U")]))
        G[n("W1")] = dU.reshape(B * T, -1).T @ c[n("H2")].reshape(B * T, d)
        G[n("c1")] = dU.sum(axis=(0, 1))
        dH2 = q(dU @ g("W1"))
        dln, G[n("g2")], G[n("b2")] = layernorm_bwd(dH2, c[n("Xmid")], g("g2"), c[n("m2")], c[n("r2")])
        dX = q(dX + dln)
        dA[n("G")], dA[n("U")], dA[n("H2")], dA[n("Xmid")] = dG, dU, dH2, dX
        # Xmid = Xin + O @ Wo^T + bo
        G[n("Wo")] = dX.reshape(B * T, d).T @ c[n("O")].reshape(B * T, d)
        G[n("bo")] = dX.sum(axis=(0, 1))
        dO = q(dX @ g("Wo"))
        dQKV = q(attention_bwd(dO, c[n("QKV")], c[n("A")], cfg["heads"]))
        G[n("Wqkv")] = dQKV.reshape(B * T, -1).T @ c[n("H")].reshape(B * T, d)
        G[n("bqkv")] = dQKV.sum(axis=(0, 1))
        dH = q(dQKV @ g("Wqkv"))
        dln, G[n("g1")], G[n("b1")] = layernorm_bwd(dH, c[n("Xin")], g("g1"), c[n("m1")], c[n("r1")])
        dX = q(dX + dln)
        dA[n("O")], dA[n("QKV")], dA[n("H")], dA[n("Xin")] = dO, dQKV, dH, dX
    # X0[:, 0] = cls + pos[0];  X0[:, 1:] = patches @ We^T + be + pos[1:]
    B, T, d = dX.shape
    G["pos"] = dX.sum(axis=0)
    G["cls"] = dX[:, 0].sum(axis=0)
    dE = dX[:, 1:].reshape(B * (T - 1), d)
    G["We"] = dE.T @ c["patches"].reshape(B * (T - 1), -1)
    G["be"] = dE.sum(axis=0)
    return G, dA


def train_step(cfg, x, labels, P, V, lr=0.1, momentum=0.9, weight_decay=0.0, storage=None, q=None):
    """One step.  P, V: {name: parameter / momentum buffer}.  Returns dict(loss, pred, probs, cache,
    dacts, grads, params, mom); the inputs are not modified."""
    loss, c = forward(cfg, x, labels, P, storage, q)
    grads, dacts = backward(cfg, P, c, storage, q)
    newP, newV = {}, {}
    for k in P:
        v = momentum * np.asarray(V[k], dtype=np.float64) + (grads[k] + weight_decay * P[k])
        newV[k] = v
        newP[k] = P[k] - lr * v
    return dict(loss=loss, pred=c["pred"], probs=c["probs"], cache=c, dacts=dacts, grads=grads, params=newP, mom=newV)


def evaluate(cfg, batch, xs, ys, P, storage=None):
    """The validation pass (Algorithm 1: "evaluate model on validation data"): forward and loss over xs in
    batches of `batch` (xs.shape[0] a multiple of it).  Returns (accuracy, mean loss over batches, predictions)."""
    assert xs.shape[0] % batch == 0
    correct, losses, preds = 0, [], []
    for b in range(xs.shape[0] // batch):
        yb = np.asarray(ys[b * batch:(b + 1) * batch])
        loss, c = forward(cfg, xs[b * batch:(b + 1) * batch], yb, P, storage)
        correct += int(np.sum(c["pred"] == yb))
        losses.append(loss)
        preds.append(c["pred"])
    return correct / xs.shape[0], float(np.mean(losses)), np.concatenate(preds)


def fit(cfg, batch, train_x, train_y, val_x, val_y, P, V, orders, lrs, momentum=0.9, weight_decay=0.0, storage=None):
    """The epoch loop of Algorithm 1 on one device: per epoch one train_step per mini-batch (orders[e]:
    the epoch's sample order, consecutive slices of `batch` are the mini-batches; lrs: the learning
    rate of every step), then the validation metric and "save checkpoint if it improved".
    Returns dict(params, mom, history, best): history[e] = (mean train loss, val accuracy, val loss)."""
    P = {k: np.array(v, dtype=np.float64) for k, v in P.items()}
    V = {k: np.array(v, dtype=np.float64) for k, v in V.items()}
    history, best, k = [], None, 0
    for e, order in enumerate(orders):
        order = np.asarray(order)
        assert order.size % batch == 0
        losses = []
        for b in range(order.size // batch):
            idx = order[b * batch:(b + 1) * batch]
            r = train_step(cfg, train_x[idx], train_y[idx], P, V, lrs[k], momentum, weight_decay, storage)
            P, V = r["params"], r["mom"]
            losses.append(r["loss"])
            k += 1
        acc, vloss, _ = evaluate(cfg, batch, val_x, val_y, P, storage)
        history.append((float(np.mean(losses)), acc, vloss))
        if best is None or acc > best["acc"]:
            best = dict(epoch=e, acc=acc, params={n: a.copy() for n, a in P.items()}, mom={n: a.copy() for n, a in V.items()})
    return dict(params=P, mom=V, history=history, best=best)
