"""Writes tests/golden/resnet18_b256_step.json: what the float64 oracle computes for one training
step of the benchmark workload (ResNet-18, 32x32x3, 100 classes, batch 256; seeded synthetic
inputs of workloads.make_inputs(config 3)), as a small sample that a GPU test can check the
full-size HIP step against.

Calls only the oracle and the shared input generators.  Takes several minutes and ~20 GB of host
memory:

    python tests/golden/make_resnet18_b256_fixture.py

Per tensor (every activation slot, every activation gradient, every parameter gradient) it
stores: the L2 norm and the max magnitude of the pure float64 result, the values at 24 seeded
positions, and the oracle's own bf16-storage walk at the same positions together with its
relative L2 distance from the pure walk (the floor that any bf16 implementation sits on: ReLU
masks and pool winners decided on bf16-rounded values flip against the float64 walk).
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import workloads as WL  # noqa: E402
import oracle  # noqa: E402

CONFIG = 3
SAMPLES = 24
LR, MOMENTUM, WD = 0.1, 0.9, 0.0


def sig(v):
    """9 significant digits: far below every tolerance the fixture is used with."""
    return float("%.9g" % float(v))


def sample_positions(name, size):
    seed = int.from_bytes(name.encode().ljust(8, b"\0")[:8], "little") % (2 ** 32)   # stable across runs
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(size, size=min(SAMPLES, size), replace=False))


def main():
    net = WL.build_config(CONFIG)
    inp = WL.make_inputs(net, CONFIG)
    walks = {}
    for mode in (None, "bf16"):
        print("oracle walk, storage =", mode, flush=True)
        walks[mode] = oracle.train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"], LR, MOMENTUM, WD,
                                        storage=mode)
    pure, emu = walks[None], walks["bf16"]
    out = {"config": CONFIG, "batch": net.batch, "lr": LR, "momentum": MOMENTUM, "weight_decay": WD,
           "loss": sig(pure["loss"]), "loss_bf16_storage": sig(emu["loss"]), "tensors": {}}

    def add(name, a, b):
        a = np.asarray(a, dtype=np.float64).ravel()
        b = np.asarray(b, dtype=np.float64).ravel()
        pos = sample_positions(name, a.size)
        na = float(np.linalg.norm(a))
        out["tensors"][name] = {
            "size": int(a.size),
            "l2": sig(na),
            "max": sig(np.abs(a).max()),
            "floor_l2": sig(np.linalg.norm(a - b) / max(na, 1e-300)),
            "pos": [int(p) for p in pos],
            "pure": [sig(v) for v in a[pos]],
            "bf16_storage": [sig(v) for v in b[pos]],
        }

    for s in sorted(pure["acts"]):
        if s != 0:
            add("act%d" % s, pure["acts"][s], emu["acts"][s])
    for s in sorted(pure["dacts"]):
        add("dact%d" % s, pure["dacts"][s], emu["dacts"][s])
    for k in range(len(pure["grads"])):
        add("grad%d" % k, pure["grads"][k], emu["grads"][k])
    path = os.path.join(HERE, "resnet18_b256_step.json")
    with open(path, "w") as f:
        json.dump(out, f, separators=(",", ":"))
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
