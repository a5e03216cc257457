"""Oracle walker: one training step over a layer list, in float64.  Test infrastructure.

Follows the inner loop of the paper's Algorithm 1 in its printed order: forward pass, loss,
backward pass (chain rule through the layer list in reverse), parameter update.  A tensor
that feeds two consumers receives the sum of both gradients; the network input (slot 0)
receives none.

storage=None   : pure float64, no intermediate rounding.
storage='bf16' : every activation and activation gradient is rounded to bfloat16 at the point
                 where the bf16 mode stores it (conv / BN / pool / add outputs, every gradient
                 contribution and every sum of contributions); arithmetic between the stores
                 stays float64 and parameter gradients are not rounded.  The ReLU masks,
                 max-pool winners and predicted classes are then decided on values of the same
                 precision as the stored ones.
jitter=(seed, rel), bf16 storage only: before each of those roundings a seeded perturbation drawn
                 uniformly from +-rel * rms(tensor) is added to every element that is not exactly
                 zero (unless it would change the element's sign).  The paper fixes no
                 precision; in a bf16-storage / fp32-accumulate implementation the value that gets
                 rounded differs from the exact one by the fp32 accumulation error of that
                 implementation, which decides the rounding of the values that lie that close to a
                 rounding boundary.  Walks with different seeds are therefore equally legal results
                 of the same method, and their spread measures how far two correct bf16
                 implementations may lie apart (tests grade the HIP step against that spread).
"""
from __future__ import annotations
import numpy as np
from . import ops

BN_EPS = 1e-5
BN_MOMENTUM = 0.1


def _q(storage, jitter=None):
    if storage is None:
        if jitter is not None:
            raise ValueError("jitter belongs to a storage mode")
        return lambda a: a
    if storage == "bf16":
        if jitter is None:
            return ops.round_bf16
        seed, rel = jitter
        rng = np.random.default_rng(seed)

        def q(a):
            a = np.asarray(a, dtype=np.float64)
            rms = float(np.sqrt(np.mean(a * a))) if a.size else 0.0
            b = a + (rel * rms) * rng.uniform(-1.0, 1.0, size=a.shape)
            # exact zeros (a clamped activation, a masked or unrouted gradient, padding) are exact in
            # any implementation, and rounding noise never changes a sign: those elements stay as
            # they are, so that no ReLU mask is decided by the perturbation itself
            keep = (a == 0.0) | (np.sign(b) != np.sign(a))
            return ops.round_bf16(np.where(keep, a, b))
        return q
    raise ValueError(storage)


def forward_loss(net, x, labels, params, storage=None, running=None, infer=False, q=None):
    """Forward pass and loss only.  Returns (loss, fc_result, acts, saved).

    running: {layer index: [running_mean, running_var]} (float64 arrays).  Training mode
    (infer=False) updates them in place; inference mode (infer=True) normalises with them
    instead of the batch statistics and changes nothing."""
    q = _q(storage) if q is None else q
    if infer and running is None:
        raise ValueError("inference mode needs running statistics")
    acts = {0: np.asarray(x, dtype=np.float64)}
    saved = {}
    out = None
    for i, L in enumerate(net.layers):
        op = L["op"]
        if op == "conv":
            acts[L["y"]] = q(ops.conv2d_fwd(acts[L["x"]], params[L["w"]], L["stride"], L["pad"]))
        elif op == "bn":
            res = acts[L["res"]] if L["res"] >= 0 else None
            if infer:
                rm, rv = running[i]
                acts[L["y"]] = q(ops.bn_relu_infer(acts[L["x"]], params[L["gamma"]], params[L["beta"]], rm, rv,
                                                   relu=bool(L["relu"]), residual=res, eps=BN_EPS))
                continue
            rm, rv = running[i] if running is not None else (None, None)
            y, mean, invstd = ops.bn_relu_fwd(acts[L["x"]], params[L["gamma"]], params[L["beta"]],
                                              relu=bool(L["relu"]), residual=res, eps=BN_EPS,
                                              momentum=BN_MOMENTUM, running_mean=rm, running_var=rv)
            acts[L["y"]] = q(y)
            saved[i] = (mean, invstd)
        elif op == "pool":
            y, am = ops.pool_fwd(acts[L["x"]], L["mode"])
            acts[L["y"]] = q(y)
            saved[i] = am
        elif op == "add":
            acts[L["y"]] = q(acts[L["a"]] + acts[L["b"]])
        elif op == "fc_loss":
            xin = acts[L["x"]].reshape(L["N"], L["F"])
            out = ops.fc_softmax_xent(xin, params[L["W"]], params[L["b"]], labels)
        else:
            raise ValueError(op)
    return out["loss"], out, acts, saved


def initial_running(net):
    """Running statistics before the first step: mean 0, variance 1."""
    return {i: [np.zeros(L["C"]), np.ones(L["C"])] for i, L in enumerate(net.layers) if L["op"] == "bn"}


def eval_forward(net, x, labels, params, running, storage=None):
    """Validation pass: forward in inference mode.  Returns dict(loss, pred, probs, n_correct)."""
    loss, fc, _, _ = forward_loss(net, x, labels, params, storage, running=running, infer=True)
    labels = np.asarray(labels)
    return dict(loss=loss, pred=fc["pred"], probs=fc["probs"], n_correct=int(np.sum(fc["pred"] == labels)))


def train_step(net, x, labels, params, mom, lr=0.1, momentum=0.9, weight_decay=0.0, storage=None,
               running=None, jitter=None):
    """One step.  Returns dict(loss, pred, acts, dacts, grads, params, mom[, running]); inputs are
    not modified (the running statistics, if given, are copied and the copy is advanced)."""
    q = _q(storage, jitter)
    if running is not None:
        running = {i: [np.array(rm, dtype=np.float64), np.array(rv, dtype=np.float64)]
                   for i, (rm, rv) in running.items()}
    loss, fc, acts, saved = forward_loss(net, x, labels, params, storage, running=running, q=q)
    grads = [None] * len(params)
    dacts = {}

    def contribute(slot, g):
        if slot == 0:
            return
        g = q(g)
        dacts[slot] = g if slot not in dacts else q(dacts[slot] + g)

    for i in range(len(net.layers) - 1, -1, -1):
        L = net.layers[i]
        op = L["op"]
        if op == "fc_loss":
            grads[L["W"]] = fc["dW"]
            grads[L["b"]] = fc["db"]
            contribute(L["x"], fc["dx"].reshape(L["N"], 1, 1, L["F"]))
        elif op == "pool":
            contribute(L["x"], ops.pool_bwd(dacts[L["y"]], saved[i], acts[L["x"]].shape, L["mode"]))
        elif op == "add":
            contribute(L["a"], dacts[L["y"]])
            contribute(L["b"], dacts[L["y"]])
        elif op == "bn":
            mean, invstd = saved[i]
            dx, dres, dg, db = ops.bn_relu_bwd(dacts[L["y"]], acts[L["x"]], acts[L["y"]],
                                               params[L["gamma"]], mean, invstd,
                                               relu=bool(L["relu"]), want_dres=L["res"] >= 0)
            grads[L["gamma"]] = dg
            grads[L["beta"]] = db
            contribute(L["x"], dx)
            if L["res"] >= 0:
                contribute(L["res"], dres)
        elif op == "conv":
            dy = dacts[L["y"]]
            grads[L["w"]] = ops.conv2d_wgrad(acts[L["x"]], dy, params[L["w"]].shape, L["stride"], L["pad"])
            if L["x"] != 0:
                contribute(L["x"], ops.conv2d_dgrad(dy, params[L["w"]], acts[L["x"]].shape,
                                                    L["stride"], L["pad"]))
    new_params, new_mom = [], []
    for p, v, g in zip(params, mom, grads):
        w2 = np.array(p, dtype=np.float64, copy=True, order="C")
        v2 = np.array(v, dtype=np.float64, copy=True, order="C")
        ops.sgd_momentum(w2.reshape(-1), v2.reshape(-1), np.asarray(g).reshape(-1), lr, momentum, weight_decay)
        new_params.append(w2)
        new_mom.append(v2)
    return dict(loss=loss, pred=fc["pred"], probs=fc["probs"], acts=acts, dacts=dacts, grads=grads,
                params=new_params, mom=new_mom, saved=saved, running=running)
