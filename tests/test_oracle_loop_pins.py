"""Pins of the oracle's inference-mode batch norm, validation pass and epoch loop against things
other than themselves: reduction to the (separately pinned) training-mode operator, torch's CPU
float64 library operator, closed forms of the running-statistics recurrence, batch independence,
and descent on a learnable synthetic set.  CPU only."""
import numpy as np
import torch
import torch.nn.functional as TF

import workloads as WL
from oracle import ops, train_step, forward_loss, eval_forward, initial_running, loop

RNG = np.random.default_rng(4321)


def nchw(a):
    return torch.from_numpy(np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2))))


def test_bn_infer_reduces_to_training_mode_and_matches_torch():
    x = RNG.standard_normal((3, 4, 5, 6)) * 2.0 + 0.7
    res = RNG.standard_normal(x.shape)
    g = 1.0 + 0.3 * RNG.standard_normal(6)
    b = 0.2 * RNG.standard_normal(6)
    # running statistics equal to the batch's own (biased variance): the training-mode output
    mu = x.reshape(-1, 6).mean(0)
    var = x.reshape(-1, 6).var(0)
    for relu in (False, True):
        for r in (None, res):
            y_train, _, _ = ops.bn_relu_fwd(x, g, b, relu=relu, residual=r)
            y_inf = ops.bn_relu_infer(x, g, b, mu, var, relu=relu, residual=r)
            assert np.max(np.abs(y_train - y_inf)) < 1e-13
    # arbitrary running statistics: torch's library operator in evaluation mode
    rm = RNG.standard_normal(6)
    rv = RNG.uniform(0.3, 2.0, 6)
    ref = TF.batch_norm(nchw(x), torch.from_numpy(rm), torch.from_numpy(rv), torch.from_numpy(g),
                        torch.from_numpy(b), False, 0.1, 1e-5)
    ref = np.transpose(ref.numpy(), (0, 2, 3, 1))
    assert np.max(np.abs(ops.bn_relu_infer(x, g, b, rm, rv, relu=False) - ref)) < 1e-13
    assert np.max(np.abs(ops.bn_relu_infer(x, g, b, rm, rv, relu=True, residual=res) - np.maximum(ref + res, 0))) < 1e-13
    # closed forms: x == running_mean gives beta; one standard deviation above it gives gamma + beta
    eps = 1e-5
    x0 = np.broadcast_to(rm, x.shape)
    assert np.max(np.abs(ops.bn_relu_infer(x0, g, b, rm, rv, relu=False) - b)) < 1e-15
    x1 = np.broadcast_to(rm + np.sqrt(rv + eps), x.shape)
    assert np.max(np.abs(ops.bn_relu_infer(x1, g, b, rm, rv, relu=False) - (g + b))) < 1e-14
    # the inputs are not touched
    rm2, rv2 = rm.copy(), rv.copy()
    ops.bn_relu_infer(x, g, b, rm2, rv2)
    assert np.array_equal(rm, rm2) and np.array_equal(rv, rv2)


def test_running_statistics_recurrence_closed_form():
    x = RNG.standard_normal((4, 3, 3, 5)) * 1.5 - 0.4
    g, b = np.ones(5), np.zeros(5)
    rm, rv = np.zeros(5), np.ones(5)
    mu = x.reshape(-1, 5).mean(0)
    unb = x.reshape(-1, 5).var(0, ddof=1)
    alpha = 0.1
    for k in range(1, 6):
        ops.bn_relu_fwd(x, g, b, relu=False, momentum=alpha, running_mean=rm, running_var=rv)
        d = (1 - alpha) ** k
        assert np.max(np.abs(rm - (1 - d) * mu)) < 1e-14
        assert np.max(np.abs(rv - (d + (1 - d) * unb))) < 1e-14


def test_eval_forward_is_batch_independent_and_reduces_to_training_forward():
    net = WL.mini_resnet(batch=4)
    inp = WL.make_inputs(net, 91, perturb_bn=True)
    # (a) with the running statistics set to each layer's own (biased) batch statistics the
    #     inference pass is the training pass
    _, fc, acts, saved = forward_loss(net, inp["x"], inp["labels"], inp["params"])
    running = {}
    for i, L in enumerate(net.layers):
        if L["op"] == "bn":
            mean, invstd = saved[i]
            running[i] = [mean.copy(), 1.0 / invstd ** 2 - 1e-5]
    ev = eval_forward(net, inp["x"], inp["labels"], inp["params"], running)
    assert abs(ev["loss"] - fc["loss"]) < 1e-12
    assert np.array_equal(ev["pred"], fc["pred"])
    assert ev["n_correct"] == int(np.sum(fc["pred"] == inp["labels"]))
    # (b) inference mode: a sample's output does not depend on the rest of the batch (training mode does)
    running = initial_running(net)
    for v in running.values():
        v[0] += 0.1 * RNG.standard_normal(v[0].shape)
        v[1] *= RNG.uniform(0.5, 1.5, v[1].shape)
    x2 = inp["x"].copy()
    x2[1:] = RNG.standard_normal(x2[1:].shape)
    p1 = eval_forward(net, inp["x"], inp["labels"], inp["params"], running)["probs"][0]
    p2 = eval_forward(net, x2, inp["labels"], inp["params"], running)["probs"][0]
    assert np.max(np.abs(p1 - p2)) < 1e-14
    t1 = forward_loss(net, inp["x"], inp["labels"], inp["params"])[1]["probs"][0]
    t2 = forward_loss(net, x2, inp["labels"], inp["params"])[1]["probs"][0]
    assert np.max(np.abs(t1 - t2)) > 1e-6
    # (c) the pass changes nothing it was given
    before = {i: [a.copy(), b.copy()] for i, (a, b) in running.items()}
    eval_forward(net, inp["x"], inp["labels"], inp["params"], running)
    assert all(np.array_equal(before[i][0], running[i][0]) and np.array_equal(before[i][1], running[i][1]) for i in running)


def test_eval_forward_matches_torch_eval_mode():
    net = WL.mini_preact(batch=4)
    inp = WL.make_inputs(net, 92, perturb_bn=True)
    running = initial_running(net)
    for v in running.values():
        v[0] += 0.2 * RNG.standard_normal(v[0].shape)
        v[1] *= RNG.uniform(0.5, 1.5, v[1].shape)
    ev = eval_forward(net, inp["x"], inp["labels"], inp["params"], running)
    tp = [torch.from_numpy(p.copy()) for p in inp["params"]]
    acts = {0: nchw(inp["x"])}
    for i, L in enumerate(net.layers):
        if L["op"] == "conv":
            acts[L["y"]] = TF.conv2d(acts[L["x"]], tp[L["w"]].permute(0, 3, 1, 2), stride=L["stride"], padding=L["pad"])
        elif L["op"] == "bn":
            u = TF.batch_norm(acts[L["x"]], torch.from_numpy(running[i][0]), torch.from_numpy(running[i][1]),
                              tp[L["gamma"]], tp[L["beta"]], False, 0.1, 1e-5)
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
    assert abs(loss.item() - ev["loss"]) < 1e-12
    assert np.array_equal(z.argmax(1).numpy(), ev["pred"])


def test_loop_with_zero_learning_rate_moves_only_the_running_statistics():
    net = WL.mini_resnet(batch=4, classes=5)
    inp = WL.make_inputs(net, 93, zero_momentum=True)
    data = WL.make_dataset(net, 93, n_train=4, n_val=4)
    orders = [np.arange(4)] * 3                       # the same batch three times
    out = loop.fit(net, data["train_x"], data["train_y"], data["val_x"], data["val_y"], inp["params"],
                   inp["mom"], orders, lrs=[0.0] * 3, momentum=0.0)
    for p, q in zip(inp["params"], out["params"]):
        assert np.array_equal(p, q)
    # first BN layer reads the stem convolution of the fixed batch: closed-form recurrence, k = 3
    i_bn = next(i for i, L in enumerate(net.layers) if L["op"] == "bn")
    conv = net.layers[i_bn - 1]
    y = ops.conv2d_fwd(data["train_x"], inp["params"][conv["w"]], conv["stride"], conv["pad"])
    mu = y.reshape(-1, y.shape[-1]).mean(0)
    unb = y.reshape(-1, y.shape[-1]).var(0, ddof=1)
    d = 0.9 ** 3
    assert np.max(np.abs(out["running"][i_bn][0] - (1 - d) * mu)) < 1e-13
    assert np.max(np.abs(out["running"][i_bn][1] - (d + (1 - d) * unb))) < 1e-13
    # nothing improved after epoch 0, so the checkpoint is epoch 0's
    assert out["best"]["epoch"] == 0


def test_loop_chains_steps_and_keeps_the_best_checkpoint():
    net = WL.mini_resnet(batch=4, classes=3)
    inp = WL.make_inputs(net, 94)
    data = WL.make_dataset(net, 94, n_train=12, n_val=8, signal=1.0)
    epochs = 4
    orders = WL.epoch_orders(94, 12, 4, epochs)
    lrs = [0.05 * 0.9 ** k for k in range(3 * epochs)]          # a different rate at every step
    out = loop.fit(net, data["train_x"], data["train_y"], data["val_x"], data["val_y"], inp["params"],
                   inp["mom"], orders, lrs, momentum=0.9, weight_decay=1e-3)
    # the same chain by hand: step k consumes lrs[k] and slice (k mod 3) of its epoch's order
    params, mom, running = inp["params"], inp["mom"], initial_running(net)
    for k in range(3 * epochs):
        e, b = divmod(k, 3)
        idx = orders[e][4 * b:4 * b + 4]
        r = train_step(net, data["train_x"][idx], data["train_y"][idx], params, mom, lr=lrs[k], momentum=0.9,
                       weight_decay=1e-3, running=running)
        params, mom, running = r["params"], r["mom"], r["running"]
        if k == 2:
            acc0, vloss0, _ = loop.evaluate(net, data["val_x"], data["val_y"], params, running)
            assert abs(out["history"][0][1] - acc0) < 1e-15 and abs(out["history"][0][2] - vloss0) < 1e-12
    for p, q in zip(params, out["params"]):
        assert np.array_equal(p, q)
    for i in running:
        assert np.array_equal(running[i][0], out["running"][i][0]) and np.array_equal(running[i][1], out["running"][i][1])
    # the checkpoint is the first epoch that reached the best accuracy, and re-evaluating its
    # contents reproduces that accuracy
    accs = [h[1] for h in out["history"]]
    assert out["best"]["acc"] == max(accs) and out["best"]["epoch"] == accs.index(max(accs))
    acc_b, _, _ = loop.evaluate(net, data["val_x"], data["val_y"], out["best"]["params"], out["best"]["running"])
    assert acc_b == out["best"]["acc"]


def test_loop_learns_a_learnable_set():
    """Descent across the loop: on a set whose labels follow from the inputs the training loss
    falls and the validation accuracy rises well above chance (1/4)."""
    net = WL.mini_resnet(batch=16, classes=4)
    inp = WL.make_inputs(net, 95, zero_momentum=True)
    data = WL.make_dataset(net, 95, n_train=64, n_val=32, signal=1.0)
    epochs = 6
    orders = WL.epoch_orders(95, 64, 16, epochs)
    out = loop.fit(net, data["train_x"], data["train_y"], data["val_x"], data["val_y"], inp["params"],
                   inp["mom"], orders, lrs=[0.1] * (4 * epochs), momentum=0.9)
    h = out["history"]
    assert h[-1][0] < 0.5 * h[0][0]
    assert h[-1][1] >= 0.75
    assert h[-1][2] < h[0][2]
