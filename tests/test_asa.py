"""The strategy-selection solver (paper_2503_23186_amd/asa.py) against the oracle's brute-force
minimisation of the same objective (oracle/asa_ref.py), closed forms of the cost model, and the
component extraction from a layer list.  CPU only: the row is control plane, it has no kernels."""
import math

import numpy as np
import pytest

import workloads as WL
from oracle import asa_ref as ref
from paper_2503_23186_amd import asa


def random_instance(rng, L, K):
    comps = []
    for i in range(L):
        t = float(rng.uniform(0.2e-3, 3e-3))
        n_p = float(rng.integers(1_000, 3_000_000))
        out = float(rng.integers(50_000, 30_000_000))
        comps.append(dict(t=t, G=4 * n_p, O=out, S=14 * n_p, A=out * rng.uniform(1.0, 3.0)))
    return comps


def to_components(comps):
    return [asa.Component(name="c%d" % i, t=c["t"], G=c["G"], O=c["O"], S=c["S"], A=c["A"]) for i, c in enumerate(comps)]


@pytest.mark.parametrize("seed", range(40))
def test_solver_matches_brute_force(seed):
    rng = np.random.default_rng(1000 + seed)
    K = int(rng.choice([2, 3, 4]))
    d = 2
    L = int(rng.integers(1, 6))
    comps = random_instance(rng, L, K)
    bw = float(rng.choice([5e9, 50e9, 400e9]))
    lat = float(rng.choice([0.0, 5e-6, 50e-6]))
    need_dp = sum(c["S"] + c["A"] / K for c in comps)
    need_one = sum(c["S"] + c["A"] for c in comps)
    kind = seed % 4
    if kind == 0:
        caps = [need_one * 2] * K                                   # everything fits everywhere
    elif kind == 1:
        caps = [need_dp * float(rng.uniform(0.5, 1.0))] * K          # full replication does not fit
    elif kind == 2:
        caps = [need_dp * float(rng.uniform(0.3, 1.5)) for _ in range(K)]   # unequal devices
    else:
        caps = [need_one / K * float(rng.uniform(0.2, 0.9))] * K     # often nothing fits
    want_t, want_a = ref.solve_brute_force(comps, K, d, bw, lat, caps)
    plan = asa.solve(to_components(comps), asa.Cluster(K=K, mem=list(caps), bw=bw, lat=lat, d=d))
    if want_a is None:
        assert math.isinf(plan.time) and plan.assignment == []
        return
    assert plan.time == pytest.approx(want_t, rel=1e-12, abs=1e-18)
    # the plan itself, priced and checked by the oracle
    assert ref.feasible(comps, plan.assignment, K, d, caps)
    assert ref.objective(comps, plan.assignment, K, d, bw, lat) == pytest.approx(want_t, rel=1e-12)
    assert asa.predict(to_components(comps), plan.assignment, asa.Cluster(K=K, mem=list(caps), bw=bw, lat=lat, d=d)) \
        == pytest.approx(want_t, rel=1e-12)


def test_cost_model_closed_forms():
    c = asa.Component("c", t=8e-3, G=4e6, O=2e6, S=14e6, A=6e6)
    one = asa.Cluster(K=1, mem=1e12, bw=1e9)
    assert asa.t_comm(c, ("DP",), one) == 0.0 and asa.t_device(c, ("DP",), one) == 8e-3
    cl = asa.Cluster(K=8, mem=1e12, bw=100e9, lat=2e-6, d=2)
    # ring all-reduce over 8: 2 * 7/8 * bytes / bw + 14 latencies
    assert asa.t_comm(c, ("DP",), cl) == pytest.approx(2 * 7 / 8 * 4e6 / 100e9 + 14 * 2e-6)
    # hybrid: half the gradient over 4 replicas, and two all-gathers of the output inside a pair
    assert asa.t_comm(c, ("HP",), cl) == pytest.approx(2 * 3 / 4 * 2e6 / 100e9 + 6 * 2e-6 + 2 * (0.5 * 2e6 / 100e9 + 2e-6))
    assert asa.t_comm(c, ("MP", 3), cl) == 0.0
    assert asa.t_device(c, ("MP", 3), cl) == 8e-3 and asa.t_device(c, ("DP",), cl) == pytest.approx(1e-3 + asa.t_comm(c, ("DP",), cl))
    assert asa.mem_per_device(c, ("DP",), cl) == [14e6 + 6e6 / 8] * 8
    assert asa.mem_per_device(c, ("HP",), cl) == [7e6 + 6e6 / 8] * 8
    assert asa.mem_per_device(c, ("MP", 2), cl) == [0, 0, 20e6, 0, 0, 0, 0, 0]
    assert asa.t_relayout(c, ("MP", 1), ("MP", 1), cl) == 0.0
    assert asa.t_relayout(c, ("MP", 1), ("MP", 2), cl) == pytest.approx(2 * (2e6 / 100e9 + 2e-6))
    assert asa.t_relayout(c, ("DP",), ("MP", 2), cl) == pytest.approx(2 * (7 / 8 * 2e6 / 100e9 + 2e-6))
    assert asa.t_relayout(c, ("DP",), ("HP",), cl) == pytest.approx(2 * (0.5 * 2e6 / 100e9 + 2e-6))


def test_limits_of_the_plan():
    rng = np.random.default_rng(7)
    comps = to_components(random_instance(rng, 12, 8))
    total = sum(c.t for c in comps)
    # free communication, plenty of memory: every component is split over all devices
    fast = asa.solve(comps, asa.Cluster(K=8, mem=1e15, bw=1e18, lat=0.0, d=2))
    assert fast.time == pytest.approx(total / 8, rel=1e-6)
    assert all(s[0] in ("DP", "HP") for s in fast.assignment)
    # one device: the measured step itself
    assert asa.solve(comps, asa.Cluster(K=1, mem=1e15, bw=1e9)).time == pytest.approx(total, rel=1e-12)
    # a network that is useless: everything stays on one device (no transfers), the step is the sum
    slow = asa.solve(comps, asa.Cluster(K=8, mem=1e15, bw=1.0, lat=1.0, d=2))
    assert slow.time == pytest.approx(total, rel=1e-12)
    assert len({s for s in slow.assignment}) == 1 and slow.assignment[0][0] == "MP"
    # replication does not fit: the model is spread over devices, and every device stays within its memory
    S = sum(c.S + c.A for c in comps)
    tight = asa.solve(comps, asa.Cluster(K=8, mem=S / 5, bw=300e9, lat=2e-6, d=2))
    assert math.isfinite(tight.time) and tight.time > fast.time
    assert all(u <= S / 5 * (1 + 1e-12) for u in tight.mem_used)
    assert any(s[0] == "MP" for s in tight.assignment) or any(s[0] == "HP" for s in tight.assignment)
    # more memory never makes the optimum slower
    roomy = asa.solve(comps, asa.Cluster(K=8, mem=S / 3, bw=300e9, lat=2e-6, d=2))
    assert roomy.time <= tight.time * (1 + 1e-12)


def test_components_from_a_layer_list():
    net = WL.mini_resnet(batch=8, dtype="bf16", size=16, widths=(32, 64))
    n = len(net.layers)
    rows = [(i, "fwd", 1.0) for i in range(n)] + [(i, "bwd", 2.0) for i in range(n - 1)] + [(-1, "update", 10.0)]
    comps = asa.components_from_tape(net.layers, rows, "bf16")
    convs = [i for i, L in enumerate(net.layers) if L["op"] == "conv"]
    assert len(comps) == len(convs) + 1                          # one per convolution, and the head
    assert [c.layers[0] for c in comps[:-1]] == convs
    assert sorted(i for c in comps for i in c.layers) == list(range(n))
    # times: every layer's rows land in its component, the update is spread by parameter count
    assert sum(c.t for c in comps) == pytest.approx((n * 1.0 + (n - 1) * 2.0 + 10.0) * 1e-3)
    first = net.layers[convs[0]]
    c0 = comps[0]
    w = first["Cout"] * 9 * first["Cin"]
    bn_c = first["Cout"]
    assert c0.G == 4 * (w + 2 * bn_c)                            # fp32 gradients of the weights and of gamma, beta
    assert c0.S == 14 * w + 12 * 2 * bn_c                        # + momentum, master copy, bf16 copy of the conv weights
    assert c0.O == 8 * 16 * 16 * first["Cout"] * 2               # the batch norm's bf16 output
    head = comps[-1]
    assert head.G == 4 * (100 * 64 + 100)


def test_replanning_criterion():
    assert not asa.changed_significantly([1.0, 2.0, 3.0], [1.05, 2.0, 3.1])
    assert asa.changed_significantly([1.0, 2.0, 3.0], [1.0, 2.0, 4.0])
    assert asa.changed_significantly([1.0, 2.0], [1.0, 2.0, 3.0])
