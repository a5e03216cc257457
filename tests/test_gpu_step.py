"""GPU parity of cnnk_train_step against the oracle walker: loss, every activation, every
activation gradient, every parameter gradient, updated weights and momentum, labels/argmax."""
import numpy as np
import pytest
import torch

import workloads as WL
from util import JITTER_REL, JITTER_SEEDS, SCALE_TO_EXACT, SCALE_TO_MEMBER, TOL, ensemble_bound, host, max_rel_err

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402


def run_both(net, config_id, lr=0.1, momentum=0.9, wd=0.0, steps=1, **gen):
    """Runs the HIP step and the oracle walker(s) on the same seeded inputs.  For the bf16 mode the
    oracle is walked in pure float64 (key None) and as an ensemble of equally legal bf16-storage
    walks: the plain one (key "bf16") and one per seed of JITTER_SEEDS (key ("bf16", seed)) whose
    roundings are decided on values perturbed by an fp32-accumulation-sized amount (see
    oracle/step.py)."""
    from paper_2503_23186_amd import StepRunner
    inp = WL.make_inputs(net, config_id, **gen)
    runner = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype)
    runner.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    modes = [None]
    if net.dtype == "bf16":
        modes += ["bf16"] + [("bf16", s) for s in JITTER_SEEDS]
    outs = {}
    state = {m: (inp["params"], inp["mom"]) for m in modes}
    for k in range(steps):
        runner.step(lr, momentum, wd)
        for m in modes:
            storage = None if m is None else "bf16"
            jitter = (1000 * m[1] + k, JITTER_REL) if isinstance(m, tuple) else None
            outs[m] = oracle.train_step(net, inp["x"], inp["labels"], state[m][0], state[m][1], lr, momentum, wd,
                                        storage=storage, jitter=jitter)
            state[m] = (outs[m]["params"], outs[m]["mom"])
    torch.cuda.synchronize()
    return inp, runner, outs


def l2_rel_err(got, ref):
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


def runner_tensors(runner, like):
    """The HIP step's tensors as host float64 arrays, in the layout of an oracle result."""
    return dict(loss=runner.loss.item(),
                acts={s: host(runner.act[s]).reshape(a.shape) for s, a in like["acts"].items()},
                dacts={s: host(runner.dact[s]).reshape(g.shape) for s, g in like["dacts"].items()},
                grads=[host(runner.grad[k]).reshape(g.shape) for k, g in enumerate(like["grads"])],
                params=[host(runner.param[k]).reshape(g.shape) for k, g in enumerate(like["params"])],
                mom=[host(runner.mom[k]).reshape(g.shape) for k, g in enumerate(like["mom"])],
                probs=host(runner.probs))


def errors(got, out):
    """Per tensor class: worst max-norm error (max|got-ref| / max|ref|) and worst L2 relative error
    of `got` against `out` (both in the layout of an oracle result)."""
    e = {}

    def upd(kind, a, b):
        m, l = max_rel_err(a, b), l2_rel_err(a, b)
        pm, pl = e.get(kind, (0.0, 0.0))
        e[kind] = (max(pm, m), max(pl, l))

    upd("loss", np.array([got["loss"]]), np.array([out["loss"]]))
    for s, a in out["acts"].items():
        if s != 0:
            upd("act", got["acts"][s], a)
    for s, g in out["dacts"].items():
        upd("dact", got["dacts"][s], g)
    for k, g in enumerate(out["grads"]):
        upd("grad", got["grads"][k], g)
        upd("param", got["params"][k], out["params"][k])
        upd("mom", got["mom"][k], out["mom"][k])
    upd("probs", got["probs"], out["probs"])
    return e


def check_step(net, inp, runner, outs, tol):
    """fp32 mode: every tensor within `tol` (max-norm) of the float64 oracle.

    bf16 mode: a free-running bf16 step and the float64 walk decide ReLU masks and pool winners on
    values that differ by storage rounding, and at random initialisation the gradients are
    incoherent sums, so a fraction f of flipped decisions moves a gradient by about sqrt(f) of its
    norm whatever the implementation.  How far a correct bf16 implementation may lie from the
    float64 walk, and from another correct one, is measured on the oracle alone: an ensemble of
    bf16-storage walks that differ only in roundings an fp32 accumulation could decide either way.
    The HIP step has to be statistically indistinguishable from a member (oracle.ensemble: the
    members' mean figure, scaled for the factor of two to which the ensemble's noise amplitude
    models the implementation's, + 3 standard deviations of the members' own figures + `tol`) in
      (a) its L2 distance to the float64 walk, per tensor class,
      (b) its mean L2 distance to the members, against the members' pairwise distances,
      (c) for the forward quantities (activations, probabilities), which are not chaotic, also
          the max-norm distance to the float64 walk;
    the loss is within `tol` of the float64 loss outright.  The max-norm of a gradient is one
    worst element of a chaotic quantity and is graded where it is well posed: element-wise bf16
    parity of every layer on identical inputs (test_gpu_layers.py, test_gpu_fullsize.py)."""
    assert torch.equal(runner.labels.cpu(), torch.from_numpy(inp["labels"]))        # labels pass through
    for k in range(len(net.params)):
        if runner.param_lp[k] is not None:
            assert torch.equal(runner.param_lp[k], runner.param[k].to(torch.bfloat16))
    pure = outs[None]
    hip = runner_tensors(runner, pure)
    e = errors(hip, pure)
    print("\n%s [%s] b%d vs float64 oracle (max-norm/L2): %s"
          % (net.name, net.dtype, net.batch, {k: "%.1e/%.1e" % v for k, v in e.items()}))
    p = pure["probs"]
    top2 = np.sort(p, axis=1)[:, -2:]
    pred = runner.pred.cpu().numpy()
    if net.dtype == "f32":
        for kind, (m, _) in e.items():
            assert m <= tol, (kind, m)
        safe = (top2[:, 1] - top2[:, 0]) > 4 * tol * top2[:, 1]
    else:
        members = [outs["bf16"]] + [outs[("bf16", s)] for s in JITTER_SEEDS]
        to_pure = [errors(m, pure) for m in members]
        pairs = [errors(members[i], members[j]) for i in range(len(members)) for j in range(i)]
        to_members = [errors(hip, m) for m in members]
        assert e["loss"][0] <= tol, e["loss"]
        report = {}
        for kind in ("act", "dact", "grad", "param", "mom", "probs"):
            b_pure = ensemble_bound([t[kind][1] for t in to_pure], tol, SCALE_TO_EXACT)
            b_pair = ensemble_bound([t[kind][1] for t in pairs], tol, SCALE_TO_MEMBER)
            d_mem = float(np.mean([t[kind][1] for t in to_members]))
            report[kind] = "%.1e<=%.1e %.1e<=%.1e" % (e[kind][1], b_pure, d_mem, b_pair)
            assert e[kind][1] <= b_pure, (kind, "L2 distance to the float64 walk", e[kind][1], b_pure)
            assert d_mem <= b_pair, (kind, "mean L2 distance to the ensemble", d_mem, b_pair)
            if kind in ("act", "probs"):
                b_max = ensemble_bound([t[kind][0] for t in to_pure], tol, SCALE_TO_EXACT)
                assert e[kind][0] <= b_max, (kind, "max-norm distance to the float64 walk", e[kind][0], b_max)
        print("%s L2: to float64 <= ensemble bound, to members <= pairwise bound: %s" % (net.name, report))
        safe = (top2[:, 1] - top2[:, 0]) > 4 * max(tol, e["probs"][0]) * top2[:, 1]
    assert np.array_equal(pred[safe], pure["pred"][safe])                            # argmax: bit exact
    print("argmax compared on %d of %d samples" % (int(safe.sum()), len(safe)))


def test_config1_tiny_cnn_fp32():
    net = WL.build_config(1)
    inp, runner, out = run_both(net, 1)
    check_step(net, inp, runner, out, TOL["f32"])


def test_config1_three_steps_zero_initial_momentum():
    net = WL.build_config(1)
    inp, runner, out = run_both(net, 1, steps=3, zero_momentum=True)
    check_step(net, inp, runner, out, TOL["f32"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", ["mini_resnet", "mini_preact"])
def test_mini_nets(name, dtype):
    net = getattr(WL, name)(batch=6, dtype=dtype, size=8, widths=(16, 32))
    inp, runner, out = run_both(net, 60, perturb_bn=True, wd=5e-4)
    check_step(net, inp, runner, out, TOL[dtype])


def test_config2_vgg_bf16_batch16():
    net = WL.build_config(2, batch=16)
    inp, runner, out = run_both(net, 2)
    check_step(net, inp, runner, out, TOL["bf16"])


def test_config3_resnet18_bf16_batch8():
    net = WL.build_config(3, batch=8)
    inp, runner, out = run_both(net, 3)
    check_step(net, inp, runner, out, TOL["bf16"])


def test_config4_resnet50_bf16_batch4():
    net = WL.build_config(4, batch=4)
    inp, runner, out = run_both(net, 4)
    check_step(net, inp, runner, out, TOL["bf16"])


def test_config5_wrn_bf16_small():
    net = WL.wrn28_10(batch=4, widths=(32, 64, 128), per_group=2)
    inp, runner, out = run_both(net, 5)
    check_step(net, inp, runner, out, TOL["bf16"])


def test_fp32_resnet18_narrow():
    net = WL.resnet18(batch=4, dtype="f32", size=16, widths=(16, 32, 64, 128))
    inp, runner, out = run_both(net, 30)
    check_step(net, inp, runner, out, TOL["f32"])


def test_two_streams_match_one_stream():
    """The weight gradients forked onto a second stream give the results of the single-stream
    order over several consecutive steps (workspace halves and events reused).  The forked
    weight gradients split their pixel range over fewer workgroups, so the fp32 partial sums are
    grouped differently: equal up to fp32 rounding, and each mode is bit-reproducible."""
    from paper_2503_23186_amd import StepRunner
    net = WL.mini_resnet(batch=16, dtype="bf16", widths=(64, 128))
    inp = WL.make_inputs(net, 0)
    runs = []
    for two in (False, True, True):
        r = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype, two_streams=two)
        r.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
        for _ in range(3):
            r.step(0.1, 0.9, 1e-4)
        torch.cuda.synchronize()
        runs.append(r)
    a, b, c = runs
    assert abs(a.loss.item() - b.loss.item()) <= 1e-5 * abs(a.loss.item())
    for k in range(len(net.params)):
        for name in ("grad", "param", "mom"):
            ta, tb, tc = (getattr(r, name)[k] for r in (a, b, c))
            assert torch.equal(tb, tc), "%s %d differs between two identical runs" % (name, k)
            scale = ta.abs().max().item() + 1e-30
            assert (ta - tb).abs().max().item() <= 1e-4 * scale, "%s %d" % (name, k)


def _run_steps(net, inp, tune, two_streams, steps=2):
    from paper_2503_23186_amd import StepRunner, cnnk
    for k, v in tune.items():
        cnnk.cnnk_tune(k, v)
    try:
        r = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype, two_streams=two_streams)
        r.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
        for _ in range(steps):
            r.step(0.1, 0.9, 1e-4)
        torch.cuda.synchronize()
    finally:
        for k in tune:
            cnnk.cnnk_tune(k, 0)
    return r


def _assert_same_bits(net, a, b):
    assert torch.equal(a.loss, b.loss)
    for s in range(1, len(net.slots)):
        assert torch.equal(a.act[s], b.act[s]), "activation %d" % s
        assert torch.equal(a.dact[s], b.dact[s]), "activation gradient %d" % s
    for k in range(len(net.params)):
        for name in ("grad", "param", "mom"):
            assert torch.equal(getattr(a, name)[k], getattr(b, name)[k]), "%s %d" % (name, k)


@pytest.mark.parametrize("name", ["mini_resnet", "mini_preact"])
def test_bn_backward_mask_from_y_equals_mask_recomputed_from_x(name):
    """Without a residual branch the step recomputes the ReLU mask from x instead of reading y
    (the forward kernel's own arithmetic on the same operands); handing y to every batch-norm
    backward call instead (tune key 9) must give the same bits everywhere, and the oracle's result."""
    net = getattr(WL, name)(batch=16, dtype="bf16", widths=(64, 128))
    inp = WL.make_inputs(net, 0, perturb_bn=True)
    a = _run_steps(net, inp, {}, two_streams=False)
    b = _run_steps(net, inp, {9: -1}, two_streams=False)
    _assert_same_bits(net, a, b)
    from paper_2503_23186_amd import cnnk
    cnnk.cnnk_tune(9, -1)
    try:
        inp2, runner, outs = run_both(net, 0, perturb_bn=True)
        check_step(net, inp2, runner, outs, TOL["bf16"])
    finally:
        cnnk.cnnk_tune(9, 0)


def test_weight_transposes_on_either_stream_give_the_same_bits():
    """With a second stream the weight transpositions of the data-gradient kernels run there beside
    the classifier head; tune key 12 keeps them on the main stream.  Same bits either way."""
    net = WL.mini_resnet(batch=16, dtype="bf16", widths=(64, 128))
    inp = WL.make_inputs(net, 0)
    a = _run_steps(net, inp, {}, two_streams=True, steps=3)
    b = _run_steps(net, inp, {12: -1}, two_streams=True, steps=3)
    _assert_same_bits(net, a, b)
