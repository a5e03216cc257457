"""Host logic of the epoch loop: learning-rate schedules against their closed forms, and the
checkpoint file round trip.  CPU only (no kernel is launched)."""
import math
import numpy as np
import pytest
import torch

from paper_2503_23186_amd.trainer import constant_lr, step_lr, cosine_lr, write_checkpoint, read_checkpoint


def test_schedules_closed_forms():
    assert constant_lr(0.1, 5) == [0.1] * 5
    s = step_lr(0.1, steps_per_epoch=3, epochs=6, milestones=(2, 4), gamma=0.5)
    assert len(s) == 18
    assert s[:6] == [0.1] * 6 and s[6:12] == [0.05] * 6 and s[12:] == [0.025] * 6
    c = cosine_lr(0.2, total_steps=12, warmup_steps=4, floor=0.02)
    assert len(c) == 12
    assert np.allclose(c[:4], [0.05, 0.1, 0.15, 0.2])
    assert c[4] == pytest.approx(0.2)                       # the cosine starts at the base rate
    assert c[8] == pytest.approx(0.02 + 0.18 * 0.5)         # half way: mean of base and floor
    assert all(a >= b for a, b in zip(c[4:], c[5:]))        # monotone down
    assert c[-1] == pytest.approx(0.02 + 0.09 * (1 + math.cos(math.pi * 7 / 8)))
    assert min(c) >= 0.02
    assert cosine_lr(0.1, 1) == [0.1]


def test_checkpoint_file_round_trip(tmp_path):
    g = torch.Generator().manual_seed(3)
    t = {"param.0": torch.randn(4, 3, 3, 2, generator=g), "mom.0": torch.randn(4, 3, 3, 2, generator=g),
         "bn_running.1": torch.rand(2, 8, generator=g)}
    t["param.0"][0, 0, 0, 0] = float.fromhex("0x1.fffffep-127")     # a subnormal survives bit for bit
    meta = dict(net="mini", dtype="bf16", epoch=3, step=17, best_acc=0.8125, best_epoch=2)
    p = str(tmp_path / "ck.safetensors")
    write_checkpoint(p, t, meta)
    t2, m2 = read_checkpoint(p)
    assert set(t2) == set(t)
    for k in t:
        assert t2[k].dtype == t[k].dtype and torch.equal(t2[k].view(torch.int32), t[k].view(torch.int32))
    assert m2["net"] == "mini" and m2["dtype"] == "bf16"
    assert int(m2["epoch"]) == 3 and int(m2["step"]) == 17 and int(m2["best_epoch"]) == 2
    assert float(m2["best_acc"]) == 0.8125
    # floats are stored with repr: an accuracy like 1/3 comes back exactly
    write_checkpoint(p, t, dict(meta, best_acc=1.0 / 3.0))
    assert float(read_checkpoint(p)[1]["best_acc"]) == 1.0 / 3.0
