"""Layer lists ("tapes") of the image-classification CNNs whose train step is measured.

A Net is plain data: tensor slots with NHWC shapes, parameter slots with shapes and kinds,
and an ordered list of layer records.  Both executors (the fp64 oracle walker and the HIP
library's cnnk_train_step) consume the same records; nothing here computes anything.

Layer records (dicts):
  conv    : x, y, w, N,H,W,Cin,Cout,R,S,stride,pad        (no bias; y is Ho x Wo)
  bn      : x, res(-1 if none), y, gamma, beta, N,H,W,C, relu   (y = relu?(bn(x) [+ res]))
  pool    : x, y, mode('max2'|'gap'), N,H,W,C
  add     : a, b, y, N,H,W,C
  fc_loss : x, W, b, N,F,classes                           (x is the N x F pooled features)

The networks are the 32x32-input, 100-class adaptations of the paper's CNN workload
(Section IV-A names ResNet-50 on CIFAR-100; the inner loop of Algorithm 1 is the step).
"""
from __future__ import annotations
from dataclasses import dataclass, field


@dataclass
class Net:
    name: str
    batch: int
    dtype: str                      # 'f32' or 'bf16' storage mode of the HIP path
    layers: list = field(default_factory=list)
    slots: list = field(default_factory=list)      # [(N,H,W,C)]
    params: list = field(default_factory=list)     # [dict(shape, kind, fan_in)]
    classes: int = 100

    # -- construction helpers -------------------------------------------------
    def slot(self, N, H, W, C):
        self.slots.append((N, H, W, C))
        return len(self.slots) - 1

    def param(self, shape, kind, fan_in=0):
        self.params.append(dict(shape=tuple(shape), kind=kind, fan_in=fan_in))
        return len(self.params) - 1

    def conv(self, x, Cout, k, stride):
        N, H, W, Cin = self.slots[x]
        pad = 1 if k == 3 else 0
        Ho = (H + 2 * pad - k) // stride + 1
        Wo = (W + 2 * pad - k) // stride + 1
        w = self.param((Cout, k, k, Cin), "conv_w", fan_in=Cin * k * k)
        y = self.slot(N, Ho, Wo, Cout)
        self.layers.append(dict(op="conv", x=x, y=y, w=w, N=N, H=H, W=W, Cin=Cin, Cout=Cout,
                                R=k, S=k, stride=stride, pad=pad))
        return y

    def bn(self, x, relu=True, res=-1):
        N, H, W, C = self.slots[x]
        g = self.param((C,), "bn_gamma")
        b = self.param((C,), "bn_beta")
        y = self.slot(N, H, W, C)
        self.layers.append(dict(op="bn", x=x, res=res, y=y, gamma=g, beta=b, N=N, H=H, W=W, C=C,
                                relu=1 if relu else 0))
        return y

    def pool(self, x, mode):
        N, H, W, C = self.slots[x]
        y = self.slot(N, H // 2, W // 2, C) if mode == "max2" else self.slot(N, 1, 1, C)
        self.layers.append(dict(op="pool", x=x, y=y, mode=mode, N=N, H=H, W=W, C=C))
        return y

    def add(self, a, b):
        N, H, W, C = self.slots[a]
        assert self.slots[b] == (N, H, W, C)
        y = self.slot(N, H, W, C)
        self.layers.append(dict(op="add", a=a, b=b, y=y, N=N, H=H, W=W, C=C))
        return y

    def fc_loss(self, x):
        N, H, W, C = self.slots[x]
        assert H == 1 and W == 1
        Wp = self.param((self.classes, C), "fc_w", fan_in=C)
        bp = self.param((self.classes,), "fc_b")
        self.layers.append(dict(op="fc_loss", x=x, W=Wp, b=bp, N=N, F=C, classes=self.classes))

    # -- bookkeeping ----------------------------------------------------------
    def n_params(self):
        t = 0
        for p in self.params:
            n = 1
            for d in p["shape"]:
                n *= d
            t += n
        return t

    def conv_flops(self):
        """(forward, forward+backward) convolution flops at true K; a conv reading slot 0
        (the network input) has no data gradient."""
        fwd = 0
        tot = 0
        for L in self.layers:
            if L["op"] != "conv":
                continue
            Ho = (L["H"] + 2 * L["pad"] - L["R"]) // L["stride"] + 1
            Wo = (L["W"] + 2 * L["pad"] - L["S"]) // L["stride"] + 1
            f = 2 * L["N"] * Ho * Wo * L["Cout"] * L["R"] * L["S"] * L["Cin"]
            fwd += f
            tot += f * (2 if L["x"] == 0 else 3)
        return fwd, tot


def tiny_cnn(batch=8, dtype="f32", size=32, cout=16, classes=100):
    n = Net("tiny_cnn", batch, dtype, classes=classes)
    x = n.slot(batch, size, size, 3)
    t = n.bn(n.conv(x, cout, 3, 1))
    n.fc_loss(n.pool(t, "gap"))
    return n


def vgg_style(batch=128, dtype="bf16", size=32, widths=(64, 64, "M", 128, 128, "M", 256, 256, "M")):
    n = Net("vgg_style", batch, dtype)
    t = n.slot(batch, size, size, 3)
    for wdt in widths:
        t = n.pool(t, "max2") if wdt == "M" else n.bn(n.conv(t, wdt, 3, 1))
    n.fc_loss(n.pool(t, "gap"))
    return n


def _basic_block(n, x, width, stride):
    t = n.bn(n.conv(x, width, 3, stride))
    t = n.conv(t, width, 3, 1)
    if stride != 1 or n.slots[x][3] != width:
        r = n.bn(n.conv(x, width, 1, stride), relu=False)
    else:
        r = x
    return n.bn(t, relu=True, res=r)


def resnet18(batch=256, dtype="bf16", size=32, widths=(64, 128, 256, 512), blocks=(2, 2, 2, 2)):
    n = Net("resnet18", batch, dtype)
    t = n.slot(batch, size, size, 3)
    t = n.bn(n.conv(t, widths[0], 3, 1))
    for i, (wdt, nb) in enumerate(zip(widths, blocks)):
        for b in range(nb):
            t = _basic_block(n, t, wdt, (1 if i == 0 else 2) if b == 0 else 1)
    n.fc_loss(n.pool(t, "gap"))
    return n


def _bottleneck(n, x, width, stride, first):
    t = n.bn(n.conv(x, width, 1, 1))
    t = n.bn(n.conv(t, width, 3, stride))
    t = n.conv(t, 4 * width, 1, 1)
    r = n.bn(n.conv(x, 4 * width, 1, stride), relu=False) if first else x
    return n.bn(t, relu=True, res=r)


def resnet50(batch=256, dtype="bf16", size=32, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3)):
    n = Net("resnet50", batch, dtype)
    t = n.slot(batch, size, size, 3)
    t = n.bn(n.conv(t, 64, 3, 1))
    for i, (wdt, nb) in enumerate(zip(widths, blocks)):
        for b in range(nb):
            t = _bottleneck(n, t, wdt, (1 if i == 0 else 2) if b == 0 else 1, b == 0)
    n.fc_loss(n.pool(t, "gap"))
    return n


def _preact_block(n, x, width, stride):
    a = n.bn(x)
    t = n.bn(n.conv(a, width, 3, stride))
    t = n.conv(t, width, 3, 1)
    if stride != 1 or n.slots[x][3] != width:
        r = n.conv(a, width, 1, stride)
    else:
        r = x
    return n.add(t, r)


def wrn28_10(batch=128, dtype="bf16", size=32, widths=(160, 320, 640), per_group=4, stem=16):
    n = Net("wrn28_10", batch, dtype)
    t = n.slot(batch, size, size, 3)
    t = n.conv(t, stem, 3, 1)
    for i, wdt in enumerate(widths):
        for b in range(per_group):
            t = _preact_block(n, t, wdt, (1 if i == 0 else 2) if b == 0 else 1)
    t = n.bn(t)
    n.fc_loss(n.pool(t, "gap"))
    return n


def mini_resnet(batch=4, dtype="f32", size=8, widths=(8, 16), classes=100):
    """Shrunken post-activation ResNet with one identity block and one strided projection block."""
    n = Net("mini_resnet", batch, dtype, classes=classes)
    t = n.slot(batch, size, size, 3)
    t = n.bn(n.conv(t, widths[0], 3, 1))
    t = _basic_block(n, t, widths[0], 1)
    t = _basic_block(n, t, widths[1], 2)
    n.fc_loss(n.pool(t, "gap"))
    return n


def mini_preact(batch=4, dtype="f32", size=8, widths=(8, 16), stem=8, classes=100):
    """Shrunken pre-activation network: add op, projection from the pre-activated tensor, max-pool."""
    n = Net("mini_preact", batch, dtype, classes=classes)
    t = n.slot(batch, size, size, 3)
    t = n.conv(t, stem, 3, 1)
    t = _preact_block(n, t, widths[0], 1)
    t = _preact_block(n, t, widths[1], 2)
    t = n.bn(t)
    t = n.pool(t, "max2")
    n.fc_loss(n.pool(t, "gap"))
    return n


CONFIGS = {
    1: lambda **kw: tiny_cnn(**{**dict(batch=8, dtype="f32"), **kw}),
    2: lambda **kw: vgg_style(**{**dict(batch=128, dtype="bf16"), **kw}),
    3: lambda **kw: resnet18(**{**dict(batch=256, dtype="bf16"), **kw}),
    4: lambda **kw: resnet50(**{**dict(batch=256, dtype="bf16"), **kw}),
    5: lambda **kw: wrn28_10(**{**dict(batch=128, dtype="bf16"), **kw}),
}


def build_config(config_id, **overrides):
    return CONFIGS[config_id](**overrides)
