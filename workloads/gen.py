"""Seeded synthetic inputs standing in for CIFAR-100-shaped data (32x32 RGB, 100 classes).

Values: images i.i.d. N(0,1); labels uniform integers in [0, classes); convolution weights
He-normal on fan-in; FC weights N(0, 1/F), bias 0; BN gamma=1, beta=0 (or perturbed on request);
momentum buffers N(0,1)*1e-2 so that the momentum term is visible after a single step.
Everything is drawn in float64 on the host; for the bf16 storage mode the tensors that the
HIP path stores in bf16 are first rounded to bf16-representable values so that neither side
is charged for input quantisation.
"""
from __future__ import annotations
import numpy as np


def rng_for(config_id: int, stream_id: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([2503, 23186, int(config_id), int(stream_id)]))


def to_bf16_representable(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even) and return them as float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(a.shape)


def make_inputs(net, config_id=0, perturb_bn=False, zero_momentum=False):
    """Return dict(x, labels, params[list], mom[list]) of float64 / int32 host arrays."""
    bf16 = net.dtype == "bf16"
    N, H, W, C = net.slots[0]
    x = rng_for(config_id, 0).standard_normal((N, H, W, C))
    labels = rng_for(config_id, 1).integers(0, net.classes, size=N).astype(np.int32)
    if bf16:
        x = to_bf16_representable(x)
    params, mom = [], []
    vr = rng_for(config_id, 2)
    for k, p in enumerate(net.params):
        r = rng_for(config_id, 100 + k)
        shp, kind = p["shape"], p["kind"]
        if kind == "conv_w":
            a = r.standard_normal(shp) * np.sqrt(2.0 / p["fan_in"])
        elif kind == "fc_w":
            a = r.standard_normal(shp) * np.sqrt(1.0 / p["fan_in"])
        elif kind == "bn_gamma":
            a = 1.0 + (0.1 * r.standard_normal(shp) if perturb_bn else np.zeros(shp))
        else:  # bn_beta, fc_b
            a = 0.1 * r.standard_normal(shp) if (perturb_bn and kind == "bn_beta") else np.zeros(shp)
        if bf16 and kind == "conv_w":
            a = to_bf16_representable(a)
        else:
            a = a.astype(np.float32).astype(np.float64)   # fp32 master copies are exact on both sides
        params.append(np.ascontiguousarray(a))
        v = np.zeros(shp) if zero_momentum else 1e-2 * vr.standard_normal(shp)
        mom.append(np.ascontiguousarray(v.astype(np.float32).astype(np.float64)))
    return dict(x=np.ascontiguousarray(x), labels=labels, params=params, mom=mom)


def make_dataset(net, config_id, n_train, n_val, signal=0.5):
    """A seeded synthetic train/validation set of the net's input shape, standing in for a labelled
    image set: every class has a fixed N(0,1) template image, a sample is N(0,1) noise plus
    `signal` times its class's template, labels are uniform in [0, classes).  With signal > 0
    the labels can be learnt, so a validation metric has something to improve on.
    Returns dict(train_x, train_y, val_x, val_y) (float64 NHWC / int32)."""
    _, H, W, C = net.slots[0]
    templates = rng_for(config_id, 10).standard_normal((net.classes, H, W, C))
    out = {}
    for name, n, sid in (("train", n_train, 11), ("val", n_val, 13)):
        y = rng_for(config_id, sid).integers(0, net.classes, size=n).astype(np.int32)
        x = rng_for(config_id, sid + 1).standard_normal((n, H, W, C)) + signal * templates[y]
        x = to_bf16_representable(x) if net.dtype == "bf16" else x.astype(np.float32).astype(np.float64)
        out[name + "_x"] = np.ascontiguousarray(x)
        out[name + "_y"] = y
    return out


def epoch_orders(config_id, n_train, batch, epochs):
    """The sample order of every epoch: a seeded permutation of range(n_train) cut to a whole
    number of mini-batches (consecutive slices of `batch` indices are the mini-batches)."""
    keep = (n_train // batch) * batch
    return [rng_for(config_id, 1000 + e).permutation(n_train)[:keep].astype(np.int64) for e in range(epochs)]
