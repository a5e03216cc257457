"""Layer-by-layer bf16/fp32 parity on identical inputs: the oracle walks the network (with bf16
stores in the bf16 mode), and every layer's HIP kernel is then run on the ORACLE's input tensors of
that layer and compared element by element with the oracle's outputs: activations, activation
gradients, parameter gradients; pool winners bit exact.  Inputs flow oracle -> HIP only."""
import numpy as np
import pytest
import torch

import workloads as WL
from util import dev, dev_f32, host, max_rel_err

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from oracle import ops as ref  # noqa: E402


def ws_for(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0"), max(int(nbytes), 256)


NETS = [
    ("vgg_b8", lambda: WL.build_config(2, batch=8), 2),
    ("resnet18_b4", lambda: WL.build_config(3, batch=4), 3),
    ("resnet50_b2", lambda: WL.build_config(4, batch=2), 4),
    ("wrn_small", lambda: WL.wrn28_10(batch=2, widths=(160, 320, 640), per_group=1), 5),
    ("resnet18_f32", lambda: WL.resnet18(batch=2, dtype="f32", size=16, widths=(16, 32, 64, 128)), 31),
]


@pytest.mark.parametrize("name,make,cid", NETS, ids=[n[0] for n in NETS])
def test_every_layer_on_oracle_inputs(name, make, cid):
    layerwise_case(name, make(), cid)


def layerwise_case(name, net, cid):
    """Walks `net` with the oracle, then runs every layer's HIP kernels on the oracle's tensors and
    compares whole outputs (also used at the benchmark's full batch by test_gpu_fullsize.py)."""
    from paper_2503_23186_amd import cnnk as K
    dtype = net.dtype
    dt = K.BF16 if dtype == "bf16" else K.F32
    st = "bf16" if dtype == "bf16" else None
    q = ref.round_bf16 if dtype == "bf16" else (lambda a: a)
    # bf16 outputs: both sides round (nearly) the same value once, so they differ by at most one
    # unit in the last place of an element, 2^-8 of the largest one
    out_tol = 4e-3 if dtype == "bf16" else 1e-5
    acc_tol = 2e-4 if dtype == "bf16" else 2e-5
    inp = WL.make_inputs(net, cid, perturb_bn=True)
    o = oracle.train_step(net, inp["x"], inp["labels"], inp["params"], inp["mom"], storage=st)
    acts, dacts, P = o["acts"], o["dacts"], inp["params"]
    worst = {}

    def chk(kind, got, want, tol):
        e = max_rel_err(host(got).reshape(want.shape), want)
        worst[kind] = max(worst.get(kind, 0.0), e)
        assert e <= tol, (name, kind, e)

    for i, L in enumerate(net.layers):
        op = L["op"]
        if op == "conv":
            d = K.conv_desc(L["N"], L["H"], L["W"], L["Cin"], L["Cout"], L["R"], L["S"], L["stride"], L["pad"], dt)
            x, w, dy = acts[L["x"]], P[L["w"]], dacts[L["y"]]
            gx, gw, gdy = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
            gy = torch.empty(acts[L["y"]].shape, dtype=gx.dtype, device="cuda:0")
            ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_FWD))
            K.cnnk_conv2d_fwd(d, gx, gw, gy, None, None, ws, nb)
            chk("conv_y", gy, acts[L["y"]], out_tol)
            gdw = torch.empty(w.shape, dtype=torch.float32, device="cuda:0")
            ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_WGRAD))
            K.cnnk_conv2d_wgrad(d, gx, gdy, gdw, ws, nb)
            chk("conv_dw", gdw, o["grads"][L["w"]], acc_tol)
            if L["x"] != 0:
                gdx = torch.empty(x.shape, dtype=gx.dtype, device="cuda:0")
                ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_DGRAD))
                K.cnnk_conv2d_dgrad(d, gdy, gw, gdx, 0, ws, nb)
                chk("conv_dx", gdx, q(ref.conv2d_dgrad(dy, w, x.shape, L["stride"], L["pad"])), out_tol)
        elif op == "bn":
            d = K.bn_desc(L["N"], L["H"], L["W"], L["C"], dt, L["relu"])
            ws, nb = ws_for(K.cnnk_bn_workspace_bytes(d))
            x, y, dy = acts[L["x"]], acts[L["y"]], dacts[L["y"]]
            res = acts[L["res"]] if L["res"] >= 0 else None
            gx = dev(x, dtype)
            gg, gb = dev_f32(P[L["gamma"]]), dev_f32(P[L["beta"]])
            gy = torch.empty(x.shape, dtype=gx.dtype, device="cuda:0")
            gm = torch.empty(L["C"], device="cuda:0"); gi = torch.empty(L["C"], device="cuda:0")
            K.cnnk_bn_relu_fwd(d, gx, None if res is None else dev(res, dtype), gg, gb, gy, gm, gi,
                               None, None, None, None, ws, nb)
            mean, invstd = o["saved"][i]
            chk("bn_mean", gm, mean, 1e-5); chk("bn_invstd", gi, invstd, 1e-5)
            chk("bn_y", gy, y, out_tol)
            dx_ref, dres_ref, dg_ref, db_ref = ref.bn_relu_bwd(dy, x, y, P[L["gamma"]], mean, invstd,
                                                               relu=bool(L["relu"]), want_dres=res is not None)
            gdx = torch.empty(x.shape, dtype=gx.dtype, device="cuda:0")
            gdr = torch.empty(x.shape, dtype=gx.dtype, device="cuda:0") if res is not None else None
            gdg = torch.empty(L["C"], device="cuda:0"); gdb = torch.empty(L["C"], device="cuda:0")
            K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, dev(y, dtype), gg, gb, dev_f32(mean), dev_f32(invstd), gdx, gdr, 0,
                               gdg, gdb, ws, nb)
            chk("bn_dgamma", gdg, dg_ref, acc_tol); chk("bn_dbeta", gdb, db_ref, acc_tol)
            chk("bn_dx", gdx, q(dx_ref), out_tol)
            if res is not None:
                if dtype == "bf16":
                    assert np.array_equal(host(gdr), dres_ref)      # masked copy of dy: exact
                else:
                    chk("bn_dres", gdr, dres_ref, out_tol)          # inputs were rounded to float on upload
        elif op == "pool":
            mode = K.POOL_MAX2 if L["mode"] == "max2" else K.POOL_GAP
            d = K.pool_desc(L["N"], L["H"], L["W"], L["C"], dt, mode)
            x, y, dy = acts[L["x"]], acts[L["y"]], dacts[L["y"]]
            gy = torch.empty(y.shape, dtype=dev(x, dtype).dtype, device="cuda:0")
            gam = torch.empty(y.shape, dtype=torch.uint8, device="cuda:0") if mode == K.POOL_MAX2 else None
            K.cnnk_pool_fwd(d, dev(x, dtype), gy, gam)
            chk("pool_y", gy, y, out_tol)
            if mode == K.POOL_MAX2:
                assert np.array_equal(gam.cpu().numpy(), o["saved"][i])     # winners: bit exact
            gdx = torch.empty(x.shape, dtype=gy.dtype, device="cuda:0")
            K.cnnk_pool_bwd(d, dev(dy, dtype), gam, gdx, 0)
            chk("pool_dx", gdx, q(ref.pool_bwd(dy, o["saved"][i], x.shape, L["mode"])), out_tol)
        elif op == "add":
            a, b = acts[L["a"]], acts[L["b"]]
            gy = torch.empty(a.shape, dtype=dev(a, dtype).dtype, device="cuda:0")
            K.cnnk_add(a.size, dt, dev(a, dtype), dev(b, dtype), gy)
            chk("add_y", gy, acts[L["y"]], out_tol)
        elif op == "fc_loss":
            d = K.fc_desc(L["N"], L["F"], L["classes"], dt)
            ws, nb = ws_for(K.cnnk_fc_workspace_bytes(d))
            x = acts[L["x"]].reshape(L["N"], L["F"])
            gl = torch.empty(1, device="cuda:0"); gp = torch.empty(L["N"], dtype=torch.int32, device="cuda:0")
            gdx = torch.empty(x.shape, dtype=dev(x, dtype).dtype, device="cuda:0")
            gdW = torch.empty(P[L["W"]].shape, device="cuda:0"); gdb = torch.empty(L["classes"], device="cuda:0")
            K.cnnk_fc_softmax_xent(d, dev(x, dtype), dev_f32(P[L["W"]]), dev_f32(P[L["b"]]),
                                   torch.from_numpy(inp["labels"]).to("cuda:0"), gl, gp, None, gdx, gdW, gdb, ws, nb)
            assert abs(gl.item() - o["loss"]) <= 1e-5 * o["loss"]
            chk("fc_dW", gdW, o["grads"][L["W"]], acc_tol); chk("fc_db", gdb, o["grads"][L["b"]], acc_tol)
            chk("fc_dx", gdx, q(dacts[L["x"]].reshape(x.shape)), out_tol)
            top2 = np.sort(o["probs"], axis=1)[:, -2:]
            safe = (top2[:, 1] - top2[:, 0]) > 1e-5
            assert np.array_equal(gp.cpu().numpy()[safe], o["pred"][safe])
    torch.cuda.synchronize()
    print("\n%s: worst max-norm error per kernel output: %s" % (name, {k: "%.1e" % v for k, v in worst.items()}))
