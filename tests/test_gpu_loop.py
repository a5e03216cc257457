"""GPU parity of the epoch-loop entry points against the oracle: inference-mode batch norm,
the forward-only classifier head, the correct-prediction count, cnnk_eval_step on every
architecture, and the whole loop (mini-batches, schedule, validation, checkpoint, resume)."""
import ctypes as C
import numpy as np
import pytest
import torch

import workloads as WL
from util import TOL, DEV, dev, dev_f32, host, max_rel_err, rep

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from oracle import ops, loop as oloop  # noqa: E402

RNG = np.random.default_rng(777)


def cnnk():
    from paper_2503_23186_amd import cnnk as m
    return m


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 5, 8), (4, 8, 8, 64), (3, 7, 5, 24), (2, 4, 4, 512), (5, 16, 16, 128),
                                   (1, 1, 1, 2048), (64, 32, 32, 64)])
@pytest.mark.parametrize("relu,with_res", [(0, 0), (1, 0), (1, 1), (0, 1)])
def test_bn_infer_matches_oracle(dtype, shape, relu, with_res):
    k = cnnk()
    N, H, W, Cc = shape
    x = rep(RNG.standard_normal(shape) * 1.7 + 0.3, dtype)
    res = rep(RNG.standard_normal(shape), dtype) if with_res else None
    g = rep(1.0 + 0.2 * RNG.standard_normal(Cc), "f32")
    b = rep(0.3 * RNG.standard_normal(Cc), "f32")
    rm = rep(0.5 * RNG.standard_normal(Cc), "f32")
    rv = rep(RNG.uniform(0.2, 3.0, Cc), "f32")
    ref = ops.bn_relu_infer(x, g, b, rm, rv, relu=bool(relu), residual=res)
    d = k.bn_desc(N, H, W, Cc, k.BF16 if dtype == "bf16" else k.F32, relu, 1e-5, 0.1)
    xd, yd = dev(x, dtype), torch.empty(shape, dtype=dev(x, dtype).dtype, device=DEV)
    rd = dev(res, dtype) if with_res else None
    gd, bd, rmd, rvd = dev_f32(g), dev_f32(b), dev_f32(rm), dev_f32(rv)
    keep = (rmd.clone(), rvd.clone())
    k.cnnk_bn_relu_infer(d, xd, rd, gd, bd, rmd, rvd, yd)
    torch.cuda.synchronize()
    assert max_rel_err(host(yd), ref) <= (5e-3 if dtype == "bf16" else 1e-5)
    assert torch.equal(rmd, keep[0]) and torch.equal(rvd, keep[1])
    if relu:    # the zero pattern is a decision: same inputs, so the same zeros up to values at the rounding edge
        got0, ref0 = host(yd) == 0, ref == 0
        edge = np.abs(ref) < (2e-2 if dtype == "bf16" else 1e-5) * np.max(np.abs(ref))
        assert np.all((got0 == ref0) | edge)


def test_bn_infer_rejects_bad_arguments():
    k = cnnk()
    d = k.bn_desc(2, 4, 4, 12, k.F32, 1, 1e-5, 0.1)      # C not a multiple of 8
    t = torch.zeros(2 * 4 * 4 * 12, device=DEV)
    with pytest.raises(k.CnnkError) as e:
        k.cnnk_bn_relu_infer(d, t, None, t, t, t, t, t)
    assert e.value.status == 3
    d = k.bn_desc(2, 4, 4, 16, k.F32, 1, 1e-5, 0.1)
    with pytest.raises(k.CnnkError) as e:
        k.cnnk_bn_relu_infer(d, t, None, t, t, None, t, t)
    assert e.value.status == 1


@pytest.mark.parametrize("n", [1, 7, 256, 1000])
def test_count_correct_is_exact_and_accumulates(n):
    k = cnnk()
    pred = RNG.integers(0, 5, n).astype(np.int32)
    lab = RNG.integers(0, 5, n).astype(np.int32)
    cnt = torch.tensor([11], dtype=torch.int32, device=DEV)
    pd, ld = torch.from_numpy(pred).to(DEV), torch.from_numpy(lab).to(DEV)
    k.cnnk_count_correct(n, pd, ld, cnt)
    k.cnnk_count_correct(n, pd, ld, cnt)
    torch.cuda.synchronize()
    assert cnt.item() == 11 + 2 * int(np.sum(pred == lab))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fc_forward_only_matches_the_full_call_and_writes_no_gradient(dtype):
    k = cnnk()
    N, F, K = 32, 64, 10
    x = rep(RNG.standard_normal((N, F)), dtype)
    W = rep(RNG.standard_normal((K, F)) / 8, "f32")
    b = rep(0.1 * RNG.standard_normal(K), "f32")
    lab = RNG.integers(0, K, N).astype(np.int32)
    ref = ops.fc_softmax_xent(x, W, b, lab)
    d = k.fc_desc(N, F, K, k.BF16 if dtype == "bf16" else k.F32)
    wsb = k.cnnk_fc_workspace_bytes(d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    xd, Wd, bd, ld = dev(x, dtype), dev_f32(W), dev_f32(b), torch.from_numpy(lab).to(DEV)
    loss = torch.zeros(1, device=DEV)
    pred = torch.zeros(N, dtype=torch.int32, device=DEV)
    probs = torch.zeros(N, K, device=DEV)
    k.cnnk_fc_softmax_xent(d, xd, Wd, bd, ld, loss, pred, probs, None, None, None, ws, wsb)
    torch.cuda.synchronize()
    assert abs(loss.item() - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert np.array_equal(pred.cpu().numpy(), ref["pred"])
    assert max_rel_err(host(probs), ref["probs"]) <= 1e-5
    # two of the three gradient pointers: an argument error, nothing is launched
    dx = torch.zeros(N, F, dtype=xd.dtype, device=DEV)
    with pytest.raises(k.CnnkError) as e:
        k.cnnk_fc_softmax_xent(d, xd, Wd, bd, ld, loss, pred, probs, dx, None, None, ws, wsb)
    assert e.value.status == 1


NETS = {
    "tiny_f32": lambda: WL.build_config(1),
    "vgg_bf16": lambda: WL.build_config(2, batch=8),
    "vgg_f32": lambda: WL.build_config(2, batch=4, dtype="f32"),
    "resnet18_bf16": lambda: WL.build_config(3, batch=8),
    "resnet18_f32": lambda: WL.build_config(3, batch=4, dtype="f32"),
    "resnet50_bf16": lambda: WL.build_config(4, batch=4),
    "wrn_bf16": lambda: WL.build_config(5, batch=4, widths=(32, 64, 128), per_group=2),
    "mini_preact_f32": lambda: WL.mini_preact(batch=8),
}


def perturbed_running(net, seed):
    r = np.random.default_rng(seed)
    run = oracle.initial_running(net)
    for v in run.values():
        v[0] = rep(v[0] + 0.1 * r.standard_normal(v[0].shape), "f32")
        v[1] = rep(v[1] * r.uniform(0.6, 1.6, v[1].shape), "f32")
    return run


@pytest.mark.parametrize("name", sorted(NETS))
def test_eval_step_matches_oracle_and_touches_no_training_state(name):
    from paper_2503_23186_amd import StepRunner
    k = cnnk()
    net = NETS[name]()
    inp = WL.make_inputs(net, 31, perturb_bn=True)
    running = perturbed_running(net, 5)
    ref = oracle.eval_forward(net, inp["x"], inp["labels"], inp["params"], running)
    run = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype)
    run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    for i, (rm, rv) in running.items():
        run.bn_running[i].copy_(torch.from_numpy(np.stack([rm, rv]).astype(np.float32)))
    for g in run.grad:
        g.fill_(3.0)
    state = [t.clone() for t in run.param + run.mom + run.grad + [t for t in run.bn_running + run.bn_save if t is not None]]
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    s = torch.cuda.current_stream().cuda_stream
    k.cnnk_eval_step(run.c_layers, len(net.layers), run.buffers, run.labels, run.loss, run.pred, cnt, s)
    torch.cuda.synchronize()
    tol = TOL[net.dtype]
    assert abs(run.loss.item() - ref["loss"]) <= tol * abs(ref["loss"])
    assert max_rel_err(host(run.probs), ref["probs"]) <= tol
    # argmax: exact wherever the oracle's top-2 margin exceeds the error of the probabilities
    pr = np.sort(ref["probs"], axis=1)
    clear = (pr[:, -1] - pr[:, -2]) > 2 * tol * np.max(ref["probs"])
    got = run.pred.cpu().numpy()
    assert np.array_equal(got[clear], ref["pred"][clear])
    assert cnt.item() == int(np.sum(got == inp["labels"]))
    if clear.all():
        assert cnt.item() == ref["n_correct"]
    after = run.param + run.mom + run.grad + [t for t in run.bn_running + run.bn_save if t is not None]
    assert all(torch.equal(a, b) for a, b in zip(after, state))
    # without running statistics the call is an argument error and launches nothing
    keep = run.buffers.bn_running
    run.buffers.bn_running = None
    with pytest.raises(k.CnnkError) as e:
        k.cnnk_eval_step(run.c_layers, len(net.layers), run.buffers, run.labels, run.loss, run.pred, None, s)
    assert e.value.status == 1
    run.buffers.bn_running = keep


def _fit_case(net, cfg, n_train, n_val, epochs, signal=1.0):
    inp = WL.make_inputs(net, cfg)
    data = WL.make_dataset(net, cfg, n_train, n_val, signal=signal)
    orders = WL.epoch_orders(cfg, n_train, net.batch, epochs)
    return inp, data, orders


def test_fit_matches_the_oracle_loop_fp32(tmp_path):
    from paper_2503_23186_amd.trainer import Trainer, cosine_lr
    net = WL.mini_resnet(batch=8, classes=4)
    epochs, n_train, n_val = 4, 32, 16
    inp, data, orders = _fit_case(net, 41, n_train, n_val, epochs)
    lrs = cosine_lr(0.05, epochs * (n_train // 8), warmup_steps=2)
    ref = oloop.fit(net, data["train_x"], data["train_y"], data["val_x"], data["val_y"], inp["params"],
                    inp["mom"], orders, lrs, momentum=0.9, weight_decay=5e-4)
    tr = Trainer(net)
    tr.load_state(inp["params"], inp["mom"])
    tx, ty = tr.to_device(data["train_x"], data["train_y"])
    vx, vy = tr.to_device(data["val_x"], data["val_y"])
    ck = str(tmp_path / "best.safetensors")
    hist = tr.fit(tx, ty, vx, vy, orders, lrs, momentum=0.9, weight_decay=5e-4, ckpt_path=ck)
    print("\nfit fp32: hip", [tuple(round(v, 5) for v in h) for h in hist])
    print("fit fp32: ref", [tuple(round(v, 5) for v in h) for h in ref["history"]])
    for h, r in zip(hist, ref["history"]):
        assert abs(h[0] - r[0]) <= 1e-4 * abs(r[0]) and abs(h[2] - r[2]) <= 1e-4 * abs(r[2])
        assert h[1] == r[1]
    for k_, p in enumerate(ref["params"]):
        assert max_rel_err(host(tr.run.param[k_]), p) <= 1e-4
        assert max_rel_err(host(tr.run.mom[k_]), ref["mom"][k_]) <= 1e-4
    for i, (rm, rv) in ref["running"].items():
        assert max_rel_err(host(tr.run.bn_running[i][0]), rm) <= 1e-4
        assert max_rel_err(host(tr.run.bn_running[i][1]), rv) <= 1e-4
    assert tr.best_epoch == ref["best"]["epoch"] and tr.best_acc == ref["best"]["acc"]
    # the checkpoint holds the state of the best epoch
    tr2 = Trainer(net)
    tr2.load_checkpoint(ck)
    assert tr2.epoch == ref["best"]["epoch"] + 1 and tr2.best_acc == ref["best"]["acc"]
    for k_, p in enumerate(ref["best"]["params"]):
        assert max_rel_err(host(tr2.run.param[k_]), p) <= 1e-4
    acc, _ = tr2.evaluate(vx, vy)
    assert acc == ref["best"]["acc"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_resume_from_checkpoint_is_bit_identical(tmp_path, dtype):
    from paper_2503_23186_amd.trainer import Trainer, step_lr
    net = WL.mini_resnet(batch=8, dtype=dtype, size=16, widths=(16, 32), classes=4)
    epochs, n_train, n_val = 4, 32, 16
    inp, data, orders = _fit_case(net, 42, n_train, n_val, epochs)
    lrs = step_lr(0.05, n_train // 8, epochs, milestones=(2,), gamma=0.5)
    straight = Trainer(net)
    straight.load_state(inp["params"], inp["mom"])
    tx, ty = straight.to_device(data["train_x"], data["train_y"])
    vx, vy = straight.to_device(data["val_x"], data["val_y"])
    h_all = straight.fit(tx, ty, vx, vy, orders, lrs)
    first = Trainer(net)
    first.load_state(inp["params"], inp["mom"])
    h1 = first.fit(tx, ty, vx, vy, orders[:2], lrs)
    ck = str(tmp_path / "mid.safetensors")
    first.save_checkpoint(ck)
    second = Trainer(net)
    second.load_checkpoint(ck)
    assert second.epoch == 2 and second.step == 2 * (n_train // 8)
    h2 = second.fit(tx, ty, vx, vy, orders[2:], lrs)
    assert h1 + h2 == h_all
    for a, b in zip(straight.run.param + straight.run.mom, second.run.param + second.run.mom):
        assert torch.equal(a, b)
    for a, b in zip(straight.run.bn_running, second.run.bn_running):
        assert a is None or torch.equal(a, b)
    for a, b in zip(straight.run.param_lp, second.run.param_lp):
        assert a is None or torch.equal(a, b)
    assert (second.best_acc, second.best_epoch) == (straight.best_acc, straight.best_epoch)


def test_fit_bf16_tracks_the_oracle_within_its_own_bf16_floor():
    """bf16 storage over several steps: on every epoch's train loss and validation loss the HIP loop
    has to be indistinguishable from a member of the oracle's ensemble of legal bf16 loops (distance
    to the float64 loop no larger than the members' mean + 3 standard deviations, plus the 2e-2
    bar); the validation accuracy may differ from the float64 loop's by no more samples than the
    members' do, plus two."""
    from paper_2503_23186_amd.trainer import Trainer, constant_lr
    from util import JITTER_REL, JITTER_SEEDS, SCALE_TO_EXACT, ensemble_bound
    net = WL.mini_resnet(batch=8, dtype="bf16", size=16, widths=(16, 32), classes=4)
    epochs, n_train, n_val = 3, 32, 16
    inp, data, orders = _fit_case(net, 43, n_train, n_val, epochs)
    lrs = constant_lr(0.02, epochs * 4)
    fit = lambda **kw: oloop.fit(net, data["train_x"], data["train_y"], data["val_x"], data["val_y"],
                                 inp["params"], inp["mom"], orders, lrs, **kw)
    pure = fit()
    members = [fit(storage="bf16")] + [fit(storage="bf16", jitter=(1000 * s, JITTER_REL)) for s in JITTER_SEEDS]
    tr = Trainer(net)
    tr.load_state(inp["params"], inp["mom"])
    tx, ty = tr.to_device(data["train_x"], data["train_y"])
    vx, vy = tr.to_device(data["val_x"], data["val_y"])
    hist = tr.fit(tx, ty, vx, vy, orders, lrs)
    print("\nfit bf16: hip", [tuple(round(v, 4) for v in h) for h in hist])
    print("fit bf16: f64", [tuple(round(v, 4) for v in h) for h in pure["history"]])
    for m in members:
        print("fit bf16: member", [tuple(round(v, 4) for v in h) for h in m["history"]])
    for e, (h, p) in enumerate(zip(hist, pure["history"])):
        for j in (0, 2):
            bound = ensemble_bound([abs(m["history"][e][j] - p[j]) for m in members], 2e-2 * abs(p[j]), SCALE_TO_EXACT)
            assert abs(h[j] - p[j]) <= bound, (e, j, h[j], p[j], bound)
        worst = max(abs(m["history"][e][1] - p[1]) for m in members)
        assert abs(h[1] - p[1]) <= worst + 2.0 / n_val


def test_profile_returns_layer_times_and_leaves_the_state_alone():
    from paper_2503_23186_amd.trainer import Trainer
    net = WL.mini_resnet(batch=8, dtype="bf16", size=16, widths=(16, 32))
    inp = WL.make_inputs(net, 44)
    tr = Trainer(net)
    tr.load_state(inp["params"], inp["mom"])
    tr.run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    before = [t.clone() for t in tr.run.param + tr.run.mom + [t for t in tr.run.bn_running if t is not None]]
    rows = tr.profile(steps=2)
    n = len(net.layers)
    assert len(rows) == 3 * n - 1
    assert all(ms >= 0.0 for _, _, ms in rows)
    assert sum(ms for _, ph, ms in rows if ph == "fwd") > 0.0
    after = tr.run.param + tr.run.mom + [t for t in tr.run.bn_running if t is not None]
    assert all(torch.equal(a, b) for a, b in zip(after, before))


def test_batch_gather_and_bf16_rounding_match_the_definitions():
    """cnnk_gather_rows against numpy indexing (bit exact; 16-byte, 4-byte and unaligned rows;
    repeated and out-of-range indices), cnnk_round_bf16 against the oracle's rounding (bit exact)."""
    from paper_2503_23186_amd import cnnk as K
    from oracle import ops as ref
    rng = np.random.default_rng(91)
    for n_src, row_elems, dt in [(50, 32 * 32 * 3, torch.bfloat16), (33, 7, torch.float32), (9, 1, torch.int32),
                                 (20, 10, torch.bfloat16)]:
        if dt == torch.int32:
            src = torch.from_numpy(rng.integers(0, 100, (n_src, row_elems)).astype(np.int32)).to("cuda:0")
        else:
            src = torch.from_numpy(rng.standard_normal((n_src, row_elems)).astype(np.float32)).to("cuda:0").to(dt)
        idx = rng.integers(0, n_src, 24).astype(np.int64)
        idx[3] = idx[4]                                            # a repeated sample
        gidx = torch.from_numpy(idx).to("cuda:0")
        dst = torch.full((24, row_elems), 7, dtype=dt, device="cuda:0")
        bad = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        K.cnnk_gather_rows(24, n_src, row_elems * src.element_size(), src, gidx, dst, bad)
        torch.cuda.synchronize()
        assert torch.equal(dst, src[gidx]) and bad.item() == 0
        for wrong in (n_src, -1):
            idx2 = idx.copy(); idx2[5] = wrong
            K.cnnk_gather_rows(24, n_src, row_elems * src.element_size(), src, torch.from_numpy(idx2).to("cuda:0"), dst, bad)
            torch.cuda.synchronize()
            want = src[gidx].clone(); want[5] = 0
            assert torch.equal(dst, want) and bad.item() == 1
            bad.zero_()
    for n in (1, 5, 1000, 4099, 1 << 20):
        w = (rng.standard_normal(n) * 10.0 ** rng.integers(-3, 3, n)).astype(np.float32)
        gw = torch.from_numpy(w).to("cuda:0")
        glp = torch.zeros(n, dtype=torch.bfloat16, device="cuda:0")
        K.cnnk_round_bf16(n, gw, glp)
        torch.cuda.synchronize()
        assert np.array_equal(glp.to(torch.float64).cpu().numpy(), ref.round_bf16(w.astype(np.float64)))


def test_strategy_selection_from_a_measured_profile():
    """Algorithm 1's "profile, estimate, solve" on a real profile: the per-call times of the HIP step
    become components, and the solver's plan for four devices equals the oracle's brute-force
    minimum of the same objective."""
    from paper_2503_23186_amd.trainer import Trainer
    from paper_2503_23186_amd import asa
    from oracle import asa_ref
    net = WL.mini_resnet(batch=32, dtype="bf16", size=16, widths=(32, 64))
    inp = WL.make_inputs(net, 45)
    tr = Trainer(net)
    tr.load_state(inp["params"], inp["mom"])
    tr.run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    rows = tr.profile(steps=3)
    comps = asa.components_from_tape(net.layers, rows, net.dtype)
    assert len(comps) == 7 and all(c.t > 0 for c in comps)
    comps = comps[:6]                                   # 6^6 assignments for the brute force
    as_dicts = [dict(t=c.t, G=c.G, O=c.O, S=c.S, A=c.A) for c in comps]
    need = sum(c.S + c.A for c in comps)
    for caps, bw in (([need] * 4, 100e9), ([need / 3] * 4, 100e9), ([need / 3] * 4, 1e9)):
        plan = asa.solve(comps, asa.Cluster(K=4, mem=list(caps), bw=bw, lat=5e-6, d=2))
        want_t, want_a = asa_ref.solve_brute_force(as_dicts, 4, 2, bw, 5e-6, caps)
        assert want_a is not None and plan.time == pytest.approx(want_t, rel=1e-12)
        assert asa_ref.feasible(as_dicts, plan.assignment, 4, 2, caps)
