"""Vision Transformer workload descriptions and seeded synthetic inputs (no arithmetic of the
method: shapes, parameter tables and random numbers only).

The paper (Section IV-A) names ViT-B/16 with about 86 million parameters on CIFAR-100 and states
neither the input resolution nor the batch size.  Reading: the standard ViT-B/16 (width 768, 12
blocks, 12 heads, MLP 3072, 16 x 16 patches) on images scaled to 224 x 224 (196 patches + a class
token), 100 classes: 85.9 M parameters.  Inputs are synthetic N(0, 1) images of that shape,
standing in for the scaled data set; labels uniform in [0, classes).

Initial values: linear weights N(0, 0.02^2) (the usual truncated-normal scale, untruncated), biases
N(0, 0.02^2) so that every bias gradient path is exercised, LayerNorm gains 1 + N(0, 0.1^2) and
offsets N(0, 0.1^2), class token and position table N(0, 0.02^2); momentum buffers N(0, 1) * 1e-3.
"""
from __future__ import annotations
from dataclasses import dataclass
import numpy as np
from .gen import rng_for, to_bf16_representable

BLOCK_PARAMS = ("g1", "b1", "Wqkv", "bqkv", "Wo", "bo", "g2", "b2", "W1", "c1", "W2", "c2")


@dataclass
class ViT:
    name: str
    batch: int
    dtype: str          # 'f32' or 'bf16' storage mode of the HIP path
    image: int
    patch: int
    dim: int
    heads: int
    layers: int
    mlp: int
    classes: int = 100

    @property
    def tokens(self):
        return (self.image // self.patch) ** 2 + 1

    def cfg(self):
        return dict(patch=self.patch, dim=self.dim, heads=self.heads, layers=self.layers, mlp=self.mlp,
                    classes=self.classes)

    def param_table(self):
        """[(name, shape, kind)] in the library's parameter order.  kind: 'w' (matrix used by a GEMM:
        kept in bf16 as well in the bf16 mode), 'v' (vector or table, fp32 only)."""
        d, m, p = self.dim, self.mlp, self.patch
        t = [("We", (d, p * p * 3), "w"), ("be", (d,), "v"), ("cls", (d,), "v"), ("pos", (self.tokens, d), "v")]
        for l in range(self.layers):
            shapes = dict(g1=(d,), b1=(d,), Wqkv=(3 * d, d), bqkv=(3 * d,), Wo=(d, d), bo=(d,), g2=(d,), b2=(d,),
                          W1=(m, d), c1=(m,), W2=(d, m), c2=(d,))
            for n in BLOCK_PARAMS:
                t.append(("%s.%d" % (n, l), shapes[n], "w" if n[0] == "W" else "v"))
        t += [("gf", (d,), "v"), ("bf", (d,), "v"), ("Wh", (self.classes, d), "v"), ("bh", (self.classes,), "v")]
        return t

    def n_params(self):
        return int(sum(np.prod(s) for _, s, _ in self.param_table()))

    def flops(self):
        """Multiply-add flops (x2) of one training step's matrix products: forward, data gradient
        and weight gradient of every linear layer, and the attention products."""
        B, T, d, m = self.batch, self.tokens, self.dim, self.mlp
        rows = B * T
        lin = 2 * rows * (3 * d * d + d * d + 2 * d * m) * self.layers
        emb = 2 * B * (T - 1) * d * (self.patch * self.patch * 3)
        att_f = 2 * 2 * B * self.heads * T * T * (d // self.heads) * self.layers
        return 3 * lin + 2 * emb + att_f * 3.5      # attention backward: five products against two


def vit_b16(batch=64, dtype="bf16"):
    return ViT("vit_b16", batch, dtype, image=224, patch=16, dim=768, heads=12, layers=12, mlp=3072)


def vit_mini(batch=4, dtype="f32", image=32, patch=8, dim=128, heads=2, layers=2, mlp=256, classes=100):
    return ViT("vit_mini", batch, dtype, image, patch, dim, heads, layers, mlp, classes)


def make_vit_inputs(net: ViT, config_id=6, zero_momentum=False):
    """dict(x [B, H, W, 3], labels, params {name: array}, mom {name: array}) of float64 / int32 arrays.
    In the bf16 mode the images and the GEMM weights are bf16-representable, so that neither side is
    charged for input quantisation; everything else is fp32-representable."""
    bf16 = net.dtype == "bf16"
    x = rng_for(config_id, 0).standard_normal((net.batch, net.image, net.image, 3))
    x = to_bf16_representable(x) if bf16 else x.astype(np.float32).astype(np.float64)
    labels = rng_for(config_id, 1).integers(0, net.classes, size=net.batch).astype(np.int32)
    params, mom = {}, {}
    vr = rng_for(config_id, 2)
    for k, (name, shape, kind) in enumerate(net.param_table()):
        r = rng_for(config_id, 100 + k)
        base = name.split(".")[0]
        if base in ("g1", "g2", "gf"):
            a = 1.0 + 0.1 * r.standard_normal(shape)
        elif base in ("b1", "b2", "bf"):
            a = 0.1 * r.standard_normal(shape)
        else:
            a = 0.02 * r.standard_normal(shape)
        a = to_bf16_representable(a) if (bf16 and kind == "w") else a.astype(np.float32).astype(np.float64)
        params[name] = np.ascontiguousarray(a)
        v = np.zeros(shape) if zero_momentum else 1e-3 * vr.standard_normal(shape)
        mom[name] = np.ascontiguousarray(v.astype(np.float32).astype(np.float64))
    return dict(x=np.ascontiguousarray(x), labels=labels, params=params, mom=mom)


def make_vit_dataset(net: ViT, config_id, n_train, n_val, signal=0.5):
    """A seeded synthetic train / validation set of the net's input shape: every class has a fixed N(0, 1)
    template image, a sample is N(0, 1) noise plus `signal` times its class's template, labels uniform.
    Returns dict(train_x, train_y, val_x, val_y) (float64 NHWC / int32)."""
    shape = (net.image, net.image, 3)
    templates = rng_for(config_id, 10).standard_normal((net.classes,) + shape)
    out = {}
    for name, n, sid in (("train", n_train, 11), ("val", n_val, 13)):
        y = rng_for(config_id, sid).integers(0, net.classes, size=n).astype(np.int32)
        x = rng_for(config_id, sid + 1).standard_normal((n,) + shape) + signal * templates[y]
        x = to_bf16_representable(x) if net.dtype == "bf16" else x.astype(np.float32).astype(np.float64)
        out[name + "_x"] = np.ascontiguousarray(x)
        out[name + "_y"] = y
    return out
