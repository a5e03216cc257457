"""Oracle training loop for one device, in float64.  Test infrastructure.

The epoch loop of the paper's Algorithm 1 with every multi-device line dropped (one device has
nothing to distribute or synchronise): for each epoch, for each mini-batch the step of
oracle.step (forward, loss, backward, update), then the validation metric on held-out data in
inference mode and "save checkpoint if the metric improved".  The caller supplies the
learning rate of every step and the sample order of every epoch, so the loop itself draws no
random numbers and holds no schedule formula.
"""
from __future__ import annotations
import numpy as np
from . import step as ostep


def evaluate(net, xs, ys, params, running, storage=None):
    """Inference-mode pass over xs in batches of the net's batch size (xs.shape[0] must be a
    multiple of it).  Returns (accuracy, mean loss over batches, predictions)."""
    B = net.slots[0][0]
    assert xs.shape[0] % B == 0
    correct, losses, preds = 0, [], []
    for b in range(xs.shape[0] // B):
        r = ostep.eval_forward(net, xs[b * B:(b + 1) * B], ys[b * B:(b + 1) * B], params, running, storage)
        correct += r["n_correct"]
        losses.append(r["loss"])
        preds.append(r["pred"])
    return correct / xs.shape[0], float(np.mean(losses)), np.concatenate(preds)


def fit(net, train_x, train_y, val_x, val_y, params, mom, orders, lrs, momentum=0.9, weight_decay=0.0,
        storage=None, jitter=None):
    """jitter=(seed, rel): every training step k is the jittered bf16-storage walk of oracle.step with
    seed `seed + k` (validation passes are not perturbed).
    orders: one index array per epoch (a multiple of the batch size long; consecutive slices are
    the mini-batches); lrs: the learning rate of every step, in order.
    Returns dict(params, mom, running, history, best): history[e] = (mean train loss, val accuracy,
    val loss); best = dict(epoch, acc, params, mom, running) of the last improvement ("checkpoint")."""
    B = net.slots[0][0]
    params = [np.array(p, dtype=np.float64) for p in params]
    mom = [np.array(v, dtype=np.float64) for v in mom]
    running = ostep.initial_running(net)
    history, best, k = [], None, 0
    for e, order in enumerate(orders):
        order = np.asarray(order)
        assert order.size % B == 0
        losses = []
        for b in range(order.size // B):
            idx = order[b * B:(b + 1) * B]
            r = ostep.train_step(net, train_x[idx], train_y[idx], params, mom, lr=lrs[k], momentum=momentum,
                                 weight_decay=weight_decay, storage=storage, running=running,
                                 jitter=None if jitter is None else (jitter[0] + k, jitter[1]))
            params, mom, running = r["params"], r["mom"], r["running"]
            losses.append(r["loss"])
            k += 1
        acc, vloss, _ = evaluate(net, val_x, val_y, params, running, storage)
        history.append((float(np.mean(losses)), acc, vloss))
        if best is None or acc > best["acc"]:
            best = dict(epoch=e, acc=acc, params=[p.copy() for p in params], mom=[v.copy() for v in mom],
                        running={i: [a.copy(), b_.copy()] for i, (a, b_) in running.items()})
    return dict(params=params, mom=mom, running=running, history=history, best=best)
