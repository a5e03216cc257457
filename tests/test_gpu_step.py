"""GPU parity of cnnk_train_step against the oracle walker: loss, every activation, every
activation gradient, every parameter gradient, updated weights and momentum, labels/argmax."""
import numpy as np
import pytest
import torch

import workloads as WL
from util import TOL, host, max_rel_err

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402


def run_both(net, config_id, lr=0.1, momentum=0.9, wd=0.0, steps=1, **gen):
    from paper_2503_23186_amd import StepRunner
    inp = WL.make_inputs(net, config_id, **gen)
    runner = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype)
    runner.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    params, mom = inp["params"], inp["mom"]
    out = None
    for _ in range(steps):
        runner.step(lr, momentum, wd)
        out = oracle.train_step(net, inp["x"], inp["labels"], params, mom, lr, momentum, wd)
        params, mom = out["params"], out["mom"]
    torch.cuda.synchronize()
    return inp, runner, out


def check_step(net, inp, runner, out, tol):
    worst = {}
    loss = runner.loss.item()
    assert abs(loss - out["loss"]) <= tol * abs(out["loss"]), (loss, out["loss"])
    assert torch.equal(runner.labels.cpu(), torch.from_numpy(inp["labels"]))        # labels pass through
    for s, a in out["acts"].items():
        e = max_rel_err(host(runner.act[s]).reshape(a.shape), a)
        worst["act"] = max(worst.get("act", 0), e)
        assert e <= tol, ("act", s, e)
    for s, g in out["dacts"].items():
        e = max_rel_err(host(runner.dact[s]).reshape(g.shape), g)
        worst["dact"] = max(worst.get("dact", 0), e)
        assert e <= tol, ("dact", s, e)
    for k, g in enumerate(out["grads"]):
        e = max_rel_err(host(runner.grad[k]), g)
        worst["grad"] = max(worst.get("grad", 0), e)
        assert e <= tol, ("grad", k, net.params[k]["kind"], e)
        e = max_rel_err(host(runner.param[k]), out["params"][k])
        assert e <= tol, ("param", k, e)
        e = max_rel_err(host(runner.mom[k]), out["mom"][k])
        assert e <= tol, ("mom", k, e)
        if runner.param_lp[k] is not None:
            assert torch.equal(runner.param_lp[k], runner.param[k].to(torch.bfloat16))
    # predicted classes: exact wherever the oracle's top-2 probability margin exceeds the tolerance
    p = out["probs"]
    top2 = np.sort(p, axis=1)[:, -2:]
    safe = (top2[:, 1] - top2[:, 0]) > 4 * tol * top2[:, 1]
    pred = runner.pred.cpu().numpy()
    assert np.array_equal(pred[safe], out["pred"][safe])
    assert max_rel_err(host(runner.probs), p) <= tol
    print("%s: loss %.6f vs %.6f, worst errors %s, argmax compared on %d/%d samples"
          % (net.name, loss, out["loss"], {k: "%.2e" % v for k, v in worst.items()}, int(safe.sum()), len(safe)))


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
