"""Full-size parity: the benchmark workload's shapes, in the launch configuration bench.py times.

The oracle cannot walk batch 256 inside a test, so:
  * the hot kernels run at their full ResNet-18 batch-256 shapes and are checked on sampled
    outputs that the oracle computes one by one (its own routines on cropped operands), BN on
    the whole tensor;
  * the whole step (two streams, as bench.py runs it) is checked against a small fixture that
    tests/golden/make_resnet18_b256_fixture.py wrote from the oracle alone: the loss, and per
    tensor the norm and 24 sampled values of the float64 walk plus the oracle's own bf16-storage
    walk, which measures the floor any bf16 implementation sits on (see test_gpu_step.py).
"""
import json
import os

import numpy as np
import pytest
import torch

import workloads as WL
from util import dev, dev_f32, host, max_rel_err, rep

pytestmark = pytest.mark.gpu

from oracle import ops as ref  # noqa: E402

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "resnet18_b256_step.json")


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    from paper_2503_23186_amd import cnnk
    return cnnk


def ws_for(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0"), max(int(nbytes), 256)


# the four 3x3 stride-1 shapes of ResNet-18 at batch 256, one strided 3x3, one 1x1 projection, the stem
FULL_CONVS = [(256, 32, 32, 64, 64, 3, 1), (256, 16, 16, 128, 128, 3, 1), (256, 8, 8, 256, 256, 3, 1),
              (256, 4, 4, 512, 512, 3, 1), (256, 32, 32, 64, 128, 3, 2), (256, 16, 16, 128, 256, 1, 2),
              (256, 32, 32, 3, 64, 3, 1)]


# distinct shapes of the other configurations at their full batch: ResNet-50 b256 (1x1 bottleneck
# GEMMs incl. K = 64 single-stage tiles and the widest layers, a strided 3x3, a strided projection),
# WRN-28-10 b128 (160/320/640 channels: ragged 64-channel tiles; 16-channel and 3-channel inputs),
# VGG b128 (a 3x3 stride-1 layer that changes the channel count)
OTHER_FULL_CONVS = [(256, 32, 32, 64, 256, 1, 1), (256, 32, 32, 256, 64, 1, 1), (256, 32, 32, 128, 128, 3, 2),
                    (256, 8, 8, 256, 1024, 1, 1), (256, 4, 4, 2048, 512, 1, 1), (256, 8, 8, 1024, 2048, 1, 2),
                    (128, 32, 32, 160, 160, 3, 1), (128, 16, 16, 320, 320, 3, 1), (128, 8, 8, 640, 640, 3, 1),
                    (128, 32, 32, 160, 320, 3, 2), (128, 32, 32, 16, 160, 3, 1), (128, 32, 32, 3, 16, 3, 1),
                    (128, 16, 16, 64, 128, 3, 1)]


@pytest.mark.parametrize("shape", FULL_CONVS + OTHER_FULL_CONVS)
def test_conv_full_size_sampled(K, shape):
    N, H, W, Cin, Cout, R, st = shape
    pad = R // 2
    rng = np.random.default_rng(77)
    x = rep(rng.standard_normal((N, H, W, Cin)), "bf16")
    w = rep(rng.standard_normal((Cout, R, R, Cin)) * np.sqrt(2.0 / (Cin * R * R)), "bf16")
    Ho, Wo = ref.out_hw(H, W, R, R, st, pad)
    dy = rep(rng.standard_normal((N, Ho, Wo, Cout)), "bf16")
    d = K.conv_desc(N, H, W, Cin, Cout, R, R, st, pad, K.BF16)
    gx, gw, gdy = dev(x, "bf16"), dev(w, "bf16"), dev(dy, "bf16")
    nb = max(K.cnnk_conv2d_workspace_bytes(d, p) for p in range(3))
    ws, nb = ws_for(nb)
    gy = torch.empty((N, Ho, Wo, Cout), dtype=torch.bfloat16, device="cuda:0")
    gdx = torch.empty((N, H, W, Cin), dtype=torch.bfloat16, device="cuda:0")
    gdw = torch.empty((Cout, R, R, Cin), dtype=torch.float32, device="cuda:0")
    K.cnnk_conv2d_fwd(d, gx, gw, gy, None, None, ws, nb)
    K.cnnk_conv2d_wgrad(d, gx, gdy, gdw, ws, nb)
    K.cnnk_conv2d_dgrad(d, gdy, gw, gdx, 0, ws, nb)
    torch.cuda.synchronize()
    y, dx, dw = host(gy), host(gdx), host(gdw)
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))

    # forward: one output pixel (all channels) = the oracle's convolution of the R x R window
    got, want = [], []
    for _ in range(96):
        n, ho, wo = int(rng.integers(N)), int(rng.integers(Ho)), int(rng.integers(Wo))
        if _ < 8:   # corners and edges first
            n, ho, wo = [0, N - 1][_ & 1], [0, Ho - 1][(_ >> 1) & 1], [0, Wo - 1][(_ >> 2) & 1]
        win = xp[n:n + 1, ho * st:ho * st + R, wo * st:wo * st + R, :]
        want.append(ref.conv2d_fwd(win, w, 1, 0)[0, 0, 0, :])
        got.append(y[n, ho, wo, :])
    assert max_rel_err(np.array(got), np.array(want)) <= 1e-2

    # data gradient: one input pixel (all channels) needs the dy positions that its R x R
    # neighbourhood of outputs covers: the oracle's dgrad on that crop, embedded with its offset
    got, want = [], []
    for _ in range(64):
        n, h, wi = int(rng.integers(N)), int(rng.integers(H)), int(rng.integers(W))
        if _ < 8:
            n, h, wi = [0, N - 1][_ & 1], [0, H - 1][(_ >> 1) & 1], [0, W - 1][(_ >> 2) & 1]
        # outputs (ho, wo) with ho*st - pad <= h <= ho*st - pad + R - 1
        ho0, ho1 = max(0, -(-(h + pad - R + 1) // st)), min(Ho - 1, (h + pad) // st)
        wo0, wo1 = max(0, -(-(wi + pad - R + 1) // st)), min(Wo - 1, (wi + pad) // st)
        if ho0 > ho1 or wo0 > wo1:
            want.append(np.zeros(Cin)); got.append(dx[n, h, wi, :]); continue
        dyc = dy[n:n + 1, ho0:ho1 + 1, wo0:wo1 + 1, :]
        # crop of the input that these outputs read, without padding: rows ho0*st-pad .. ho1*st-pad+R-1
        r0, c0 = ho0 * st - pad, wo0 * st - pad
        hh, ww = (ho1 - ho0) * st + R, (wo1 - wo0) * st + R
        dxc = ref.conv2d_dgrad(dyc, w, (1, hh, ww, Cin), st, 0)
        want.append(dxc[0, h - r0, wi - c0, :])
        got.append(dx[n, h, wi, :])
    assert max_rel_err(np.array(got), np.array(want)) <= 1e-2

    # weight gradient: one (k, c) pair (all taps) = the oracle's wgrad on single-channel slices,
    # a reduction over all N*Ho*Wo positions
    got, want = [], []
    for _ in range(12):
        k, c = int(rng.integers(Cout)), int(rng.integers(Cin))
        dwk = ref.conv2d_wgrad(x[..., c:c + 1], dy[..., k:k + 1], (1, R, R, 1), st, pad)
        want.append(dwk[0, :, :, 0])
        got.append(dw[k, :, :, c])
    assert max_rel_err(np.array(got), np.array(want)) <= 1e-4 * 20   # fp32 sums over 2.6e5 bf16 products


@pytest.mark.parametrize("shape", [(256, 32, 32, 64), (256, 8, 8, 1024), (256, 4, 4, 2048), (128, 32, 32, 160)])
def test_bn_full_size(K, shape):
    """BN + ReLU forward (statistics from sums, as after a convolution) and backward (mask
    recomputed from x), whole tensor against the oracle: the 64-channel 32x32 batch-256 tensor of
    the benchmark, the widest ResNet-50 tensors (few, long-lived reducing workgroups) and a
    WRN tensor whose channel count does not divide the workgroup."""
    N, H, W, C = shape
    rng = np.random.default_rng(5)
    x = rep(0.3 + 1.1 * rng.standard_normal((N, H, W, C)), "bf16")
    gamma = (1 + 0.1 * rng.standard_normal(C)).astype(np.float32).astype(np.float64)
    beta = (0.1 * rng.standard_normal(C)).astype(np.float32).astype(np.float64)
    dy = rep(rng.standard_normal((N, H, W, C)), "bf16")
    y_ref, mean_ref, invstd_ref = ref.bn_relu_fwd(x, gamma, beta, relu=True)
    d = K.bn_desc(N, H, W, C, K.BF16, 1)
    ws, nb = ws_for(K.cnnk_bn_workspace_bytes(d))
    gx, gg, gb = dev(x, "bf16"), dev_f32(gamma), dev_f32(beta)
    s1 = dev_f32(x.reshape(-1, C).sum(0)); s2 = dev_f32((x ** 2).reshape(-1, C).sum(0))
    gy = torch.empty_like(gx)
    gm = torch.empty(C, device="cuda:0"); gi = torch.empty(C, device="cuda:0")
    K.cnnk_bn_relu_fwd(d, gx, None, gg, gb, gy, gm, gi, None, None, s1, s2, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gm), mean_ref) <= 1e-5 and max_rel_err(host(gi), invstd_ref) <= 1e-4
    assert max_rel_err(host(gy), y_ref) <= 4e-3
    # backward with the mask of the kernel's own forward output (what the recomputation reproduces)
    dx_ref, _, dg_ref, db_ref = ref.bn_relu_bwd(dy, x, host(gy), gamma, host(gm), host(gi), relu=True, want_dres=False)
    gdx = torch.empty_like(gx)
    gdg = torch.empty(C, device="cuda:0"); gdb = torch.empty(C, device="cuda:0")
    K.cnnk_bn_relu_bwd(d, dev(dy, "bf16"), gx, None, gg, gb, gm, gi, gdx, None, 0, gdg, gdb, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdg), dg_ref) <= 1e-4 and max_rel_err(host(gdb), db_ref) <= 1e-4
    assert max_rel_err(host(gdx), dx_ref) <= 4e-3


def test_step_full_size_against_fixture():
    """One step of the benchmark workload exactly as bench.py runs it (config 3, two streams)."""
    from paper_2503_23186_amd import StepRunner
    with open(GOLDEN) as f:
        G = json.load(f)
    net = WL.build_config(G["config"])
    assert net.batch == G["batch"]
    inp = WL.make_inputs(net, G["config"])
    run = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype, two_streams=True)
    run.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    run.step(G["lr"], G["momentum"], G["weight_decay"])
    torch.cuda.synchronize()
    loss = run.loss.item()
    print("\nfull-size loss: hip %.6f, oracle float64 %.6f, oracle bf16 storage %.6f"
          % (loss, G["loss"], G["loss_bf16_storage"]))
    assert abs(loss - G["loss"]) <= 2e-2 * abs(G["loss"])
    worst = {}
    for name, t in G["tensors"].items():
        kind = name.rstrip("0123456789")
        idx = int(name[len(kind):])
        buf = {"act": run.act, "dact": run.dact, "grad": run.grad}[kind][idx]
        flat = buf.reshape(-1)
        assert flat.numel() == t["size"], name
        pos = torch.tensor(t["pos"], device=flat.device)
        got = flat[pos].to(torch.float64).cpu().numpy()
        pure, emu = np.array(t["pure"]), np.array(t["bf16_storage"])
        norm = float(torch.linalg.vector_norm(flat.to(torch.float32)).item())
        # the norm over the whole tensor, and the sampled values, no farther from the float64 walk
        # than 1.5x the oracle's own bf16-storage walk (plus the bf16 bar)
        floor = t["floor_l2"]
        nerr = abs(norm / max(t["l2"], 1e-300) - 1.0)
        scale = max(t["max"], 1e-300)
        serr = float(np.max(np.abs(got - pure))) / scale
        sfloor = float(np.max(np.abs(emu - pure))) / scale
        worst[kind] = max(worst.get(kind, 0.0), nerr)
        assert nerr <= 1.5 * floor + 2e-2, (name, nerr, floor)
        assert serr <= 1.5 * sfloor + 4.0 * floor * (t["l2"] / np.sqrt(t["size"])) / scale + 2e-2, (name, serr, sfloor)
    print("worst norm deviation per class:", {k: "%.1e" % v for k, v in worst.items()})


def test_conv_beyond_2gib_falls_back(K):
    """A tensor of 2^30 elements or more is outside what the buffer-load kernels address (byte
    offset 2^31 marks padding); the library must route it to the pointer-based kernels.  Forward
    and data gradient of a thin 3x3 convolution on a 1 x 11600 x 11600 x 8 image (2.15 GB per
    tensor), generated on the device and checked on windows sampled at both ends of the tensor."""
    N, H, W, C = 1, 11600, 11600, 8
    assert N * H * W * C >= 1 << 30
    gen = torch.Generator(device="cuda:0").manual_seed(3)
    gx = torch.randn((N, H, W, C), generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    gw = (torch.randn((C, 3, 3, C), generator=gen, device="cuda:0", dtype=torch.float32) * 0.1).to(torch.bfloat16)
    d = K.conv_desc(N, H, W, C, C, 3, 3, 1, 1, K.BF16)
    ws, nb = ws_for(max(K.cnnk_conv2d_workspace_bytes(d, p) for p in (0, 1)))
    gy = torch.empty((N, H, W, C), dtype=torch.bfloat16, device="cuda:0")
    K.cnnk_conv2d_fwd(d, gx, gw, gy, None, None, ws, nb)
    torch.cuda.synchronize()
    w = host(gw)
    rng = np.random.default_rng(4)
    spots = [(0, 0), (0, W - 1), (H - 1, 0), (H - 1, W - 1), (H - 2, W - 3)]
    spots += [(int(rng.integers(1, H - 1)), int(rng.integers(1, W - 1))) for _ in range(11)]
    got, want = [], []
    for h, wi in spots:
        h0, h1, w0, w1 = max(h - 1, 0), min(h + 2, H), max(wi - 1, 0), min(wi + 2, W)
        win = np.zeros((1, 3, 3, C))
        win[0, h0 - (h - 1):h1 - (h - 1), w0 - (wi - 1):w1 - (wi - 1), :] = host(gx[0, h0:h1, w0:w1, :])
        want.append(ref.conv2d_fwd(win, w, 1, 0)[0, 0, 0, :])
        got.append(host(gy[0, h, wi, :]))
    assert max_rel_err(np.array(got), np.array(want)) <= 1e-2
    # data gradient, written into the buffer that held x (dy := y)
    K.cnnk_conv2d_dgrad(d, gy, gw, gx, 0, ws, nb)
    torch.cuda.synchronize()
    got, want = [], []
    for h, wi in spots:
        h0, h1, w0, w1 = max(h - 1, 0), min(h + 2, H), max(wi - 1, 0), min(wi + 2, W)
        dyc = np.zeros((1, 3, 3, C))
        dyc[0, h0 - (h - 1):h1 - (h - 1), w0 - (wi - 1):w1 - (wi - 1), :] = host(gy[0, h0:h1, w0:w1, :])
        # the 3x3 block of outputs around (h, wi) read a 5x5 block of inputs whose centre is (h, wi)
        want.append(ref.conv2d_dgrad(dyc, w, (1, 5, 5, C), 1, 0)[0, 2, 2, :])
        got.append(host(gx[0, h, wi, :]))
    assert max_rel_err(np.array(got), np.array(want)) <= 1e-2
