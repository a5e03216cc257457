"""GPU parity of the Vision Transformer path (include/cnnk_vit.h) against oracle/vit.py: every
operator on seeded tensors, whole tensors element by element, and the whole training step (every
activation, activation gradient, parameter gradient, updated parameter and momentum buffer)."""
import numpy as np
import pytest
import torch

import workloads as WL
from util import (JITTER_REL, JITTER_SEEDS, SCALE_TO_EXACT, SCALE_TO_MEMBER, dev, dev_f32, ensemble_bound, host,
                  max_rel_err, rep)

pytestmark = pytest.mark.gpu

from oracle import vit as V  # noqa: E402
from oracle.step import _q as oracle_quantiser  # noqa: E402


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    from paper_2503_23186_amd import vit
    return vit


def dt_of(K, dtype):
    return K.BF16 if dtype == "bf16" else K.F32


def ws_for(nbytes):
    n = max(int(nbytes), 256)
    return torch.empty(n, dtype=torch.uint8, device="cuda:0"), n


# one unit in the last place of the largest element for bf16 outputs; fp32 sums of bf16-sized terms
OUT_TOL = {"f32": 2e-6, "bf16": 4e-3}
SUM_TOL = {"f32": 2e-5, "bf16": 2e-5}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,C,stride", [(37, 32, 0), (394, 768, 0), (101, 128, 0), (50, 1024, 0), (9, 4096, 0),
                                           (13, 768, 197 * 768), (1, 4, 0), (5, 260, 0)])
def test_layernorm(K, rows, C, stride, dtype):
    rng = np.random.default_rng(rows * 1000 + C)
    xs = stride or C
    xfull = rep(rng.standard_normal((rows, xs)) * 2.0 + 0.7, dtype)
    x = xfull[:, :C]
    g = rep(1.0 + 0.2 * rng.standard_normal(C), "f32")
    b = rep(0.3 * rng.standard_normal(C), "f32")
    dy = rep(rng.standard_normal((rows, C)), dtype)
    dresfull = rep(rng.standard_normal((rows, xs)), dtype)
    y, mean, rstd = V.layernorm_fwd(x, g, b)
    dx, dg, db = V.layernorm_bwd(dy, x, g, mean, rstd)
    d = K.ln_desc(rows, C, dt_of(K, dtype), 1e-6, stride)
    gx, gy = dev(xfull, dtype), dev(np.zeros((rows, C)), dtype)
    stats = torch.zeros((rows, 2), device="cuda:0")
    K.cnnk_layernorm_fwd(d, gx, dev_f32(g), dev_f32(b), gy, stats)
    torch.cuda.synchronize()
    assert max_rel_err(host(gy), y) <= OUT_TOL[dtype]
    assert max_rel_err(host(stats)[:, 0], mean) <= 1e-5 and max_rel_err(host(stats)[:, 1], rstd) <= 1e-5
    ws, nb = ws_for(K.cnnk_layernorm_workspace_bytes(d))
    for with_res in (False, True):
        gdx = dev(np.full((rows, xs), 7.0), dtype)
        gdg, gdb = torch.zeros(C, device="cuda:0"), torch.zeros(C, device="cuda:0")
        K.cnnk_layernorm_bwd(d, dev(dy, dtype), gx, dev_f32(g), stats, dev(dresfull, dtype) if with_res else None, gdx, gdg,
                             gdb, ws, nb)
        torch.cuda.synchronize()
        want = dx + (dresfull[:, :C] if with_res else 0.0)
        got = host(gdx)
        assert max_rel_err(got[:, :C], want) <= OUT_TOL[dtype] * (2 if with_res else 1)
        assert (got[:, C:] == 7.0).all()                     # nothing outside the rows' C elements is touched
        assert max_rel_err(host(gdg), dg) <= SUM_TOL[dtype] and max_rel_err(host(gdb), db) <= SUM_TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,C", [(37, 32), (394, 3072), (100, 2304), (1000, 768), (3, 8), (129, 264)])
def test_bias_activation_residual(K, rows, C, dtype):
    rng = np.random.default_rng(rows + C)
    z = rep(rng.standard_normal((rows, C)) * 1.5, dtype)
    bias = rep(0.5 * rng.standard_normal(C), "f32")
    res = rep(rng.standard_normal((rows, C)), dtype)
    dy = rep(rng.standard_normal((rows, C)), dtype)
    dt = dt_of(K, dtype)
    ws, nb = ws_for(K.cnnk_bias_act_workspace_bytes(rows, C))
    # bias only, bias + residual
    for r in (None, res):
        gy = dev(np.zeros((rows, C)), dtype)
        K.cnnk_bias_act_fwd(rows, C, dt, K.ACT_NONE, dev(z, dtype), dev_f32(bias), None if r is None else dev(r, dtype), None, gy)
        torch.cuda.synchronize()
        assert max_rel_err(host(gy), z + bias + (0.0 if r is None else r)) <= OUT_TOL[dtype]
    gdb = torch.zeros(C, device="cuda:0")
    K.cnnk_bias_act_bwd(rows, C, dt, K.ACT_NONE, dev(dy, dtype), None, None, gdb, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdb), dy.sum(0)) <= SUM_TOL[dtype]
    # bias + GELU: the stored pre-activation, the activation of the STORED value, and the gradient
    gu, gy = dev(np.zeros((rows, C)), dtype), dev(np.zeros((rows, C)), dtype)
    K.cnnk_bias_act_fwd(rows, C, dt, K.ACT_GELU, dev(z, dtype), dev_f32(bias), None, gu, gy)
    torch.cuda.synchronize()
    u = host(gu)
    assert max_rel_err(u, z + bias) <= OUT_TOL[dtype]
    assert max_rel_err(host(gy), V.gelu(u)) <= OUT_TOL[dtype]
    gdz = dev(np.zeros((rows, C)), dtype)
    K.cnnk_bias_act_bwd(rows, C, dt, K.ACT_GELU, dev(dy, dtype), gu, gdz, gdb, ws, nb)
    torch.cuda.synchronize()
    want = dy * V.gelu_grad(u)
    assert max_rel_err(host(gdz), want) <= OUT_TOL[dtype]
    assert max_rel_err(host(gdb), want.sum(0)) <= SUM_TOL[dtype]
    # in place: u over z
    gz = dev(z, dtype)
    K.cnnk_bias_act_fwd(rows, C, dt, K.ACT_GELU, gz, dev_f32(bias), None, gz, gy)
    torch.cuda.synchronize()
    assert (host(gz) == u).all()


# bf16 runs on the dense matrix-core kernels (256 x 128 tiles, 32 reduction elements per stage: ragged
# row and column tiles, ragged last stages, one to many stages, split and unsplit weight gradients);
# fp32 and "bf16-conv" on the 1 x 1 convolution kernels.  The last shapes are ViT-B/16's at batch 64.
LINEAR_SHAPES = [(64, 32, 32), (288, 64, 160), (1056, 768, 96), (68, 128, 256), (100, 40, 24), (512, 3072, 128),
                 (12608, 768, 2304), (12608, 3072, 768), (12544, 768, 768)]


@pytest.mark.parametrize("dtype", ["f32", "bf16", "bf16-rows64", "bf16-rows128", "bf16-conv"])
@pytest.mark.parametrize("rows,Kd,N", LINEAR_SHAPES)
def test_linear_layers(K, rows, Kd, N, dtype):
    from paper_2503_23186_amd import cnnk
    if dtype == "f32" and rows > 2000:
        pytest.skip("the fp32 mode is a small-shape validation mode")
    if dtype == "bf16-conv":
        if rows > 2000:
            pytest.skip("covered by the convolution tests")
        cnnk.cnnk_tune(15, -1)
    if dtype in ("bf16-rows64", "bf16-rows128"):
        # the matrix-core kernels with 64-byte / 128-byte operand rows in LDS whatever the shape
        cnnk.cnnk_tune(15, 1 if dtype == "bf16-rows64" else 2)
    try:
        _linear_case(K, rows, Kd, N, "bf16" if dtype.startswith("bf16-") else dtype)
    finally:
        cnnk.cnnk_tune(15, 0)


def _linear_case(K, rows, Kd, N, dtype):
    rng = np.random.default_rng(rows + Kd + N)
    x = rep(rng.standard_normal((rows, Kd)), dtype)
    w = rep(rng.standard_normal((N, Kd)) / np.sqrt(Kd), dtype)
    bias = rep(0.5 * rng.standard_normal(N), "f32")
    dy = rep(rng.standard_normal((rows, N)), dtype)
    dt = dt_of(K, dtype)
    ws, nb = ws_for(K.cnnk_linear_workspace_bytes(rows, Kd, N, dt))
    gx, gw, gdy = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    tol = OUT_TOL[dtype] if dtype == "bf16" else 2e-5
    z = x @ w.T
    for b in (None, bias):
        gy = dev(np.zeros((rows, N)), dtype)
        K.cnnk_linear_fwd(rows, Kd, N, dt, gx, gw, None if b is None else dev_f32(b), K.ACT_NONE, None, gy, ws, nb)
        torch.cuda.synchronize()
        # convolution path in bf16: the product is rounded before the bias is added, and again after
        assert max_rel_err(host(gy), z + (0.0 if b is None else b)) <= tol * (2 if (dtype == "bf16" and b is not None) else 1)
    # residual connection: the sum of the stored product and the residual
    res = rep(rng.standard_normal((rows, N)), dtype)
    gy = dev(np.zeros((rows, N)), dtype)
    K.cnnk_linear_fwd(rows, Kd, N, dt, gx, gw, dev_f32(bias), K.ACT_NONE, None, gy, ws, nb, res=dev(res, dtype))
    torch.cuda.synchronize()
    assert max_rel_err(host(gy), z + bias + res) <= tol * (2 if dtype == "bf16" else 1)
    gu, gy = dev(np.zeros((rows, N)), dtype), dev(np.zeros((rows, N)), dtype)
    K.cnnk_linear_fwd(rows, Kd, N, dt, gx, gw, dev_f32(bias), K.ACT_GELU, gu, gy, ws, nb)
    torch.cuda.synchronize()
    u = host(gu)
    assert max_rel_err(u, z + bias) <= tol * (2 if dtype == "bf16" else 1)
    assert max_rel_err(host(gy), V.gelu(u)) <= tol
    gdx = dev(np.zeros((rows, Kd)), dtype)
    K.cnnk_linear_dgrad(rows, Kd, N, dt, gdy, gw, gdx, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdx), dy @ w) <= tol
    gdw = torch.full((N, Kd), 3.0, device="cuda:0")
    K.cnnk_linear_wgrad(rows, Kd, N, dt, gx, gdy, gdw, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdw), dy.T @ x) <= 2e-5
    # bit-reproducible
    gdw2 = torch.zeros((N, Kd), device="cuda:0")
    K.cnnk_linear_wgrad(rows, Kd, N, dt, gx, gdy, gdw2, ws, nb)
    torch.cuda.synchronize()
    assert torch.equal(gdw, gdw2)


# bf16 with head size 64 runs on the matrix cores (one 32-token block per wavefront: 17, 197, 256, 33
# tokens = 1, 7, 8, 2 blocks with ragged and full last blocks); "bf16-valu" forces the general kernels
@pytest.mark.parametrize("dtype", ["f32", "bf16", "bf16-valu"])
@pytest.mark.parametrize("B,T,heads,dh", [(2, 17, 2, 64), (1, 197, 3, 64), (2, 5, 2, 16), (1, 50, 4, 32), (1, 300, 1, 32),
                                          (3, 1, 2, 16), (1, 256, 1, 64), (2, 33, 12, 64), (1, 1, 1, 64)])
def test_attention(K, B, T, heads, dh, dtype):
    from paper_2503_23186_amd import cnnk
    if dtype == "bf16-valu":
        if dh != 64:
            pytest.skip("already on the general kernels")
        cnnk.cnnk_tune(10, -1)
        try:
            _attention_case(K, B, T, heads, dh, "bf16")
        finally:
            cnnk.cnnk_tune(10, 0)
    else:
        _attention_case(K, B, T, heads, dh, dtype)


def _attention_case(K, B, T, heads, dh, dtype):
    rng = np.random.default_rng(B * 7 + T * 13 + heads + dh)
    d = heads * dh
    qkv = rep(rng.standard_normal((B, T, 3 * d)) * 1.3, dtype)
    dO = rep(rng.standard_normal((B, T, d)), dtype)
    O, A = V.attention_fwd(qkv, heads)
    ad = K.attn_desc(B, T, heads, dh, dt_of(K, dtype))
    gq, go = dev(qkv, dtype), dev(np.zeros((B, T, d)), dtype)
    lse = torch.zeros((B, heads, T), device="cuda:0")
    K.cnnk_attention_fwd(ad, gq, go, lse)
    torch.cuda.synchronize()
    assert max_rel_err(host(go), O) <= (OUT_TOL[dtype] if dtype == "bf16" else 5e-5)
    q, k = (qkv[:, :, i * d:(i + 1) * d].reshape(B, T, heads, dh).transpose(0, 2, 1, 3) for i in range(2))
    S = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    want_lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(host(lse) - want_lse).max() <= 1e-4
    # backward from the oracle's own output (both sides differentiate at the same point)
    Oq = rep(O, dtype)
    want = V.attention_bwd(dO, qkv, A, heads)
    gd = dev(np.zeros((B, T, 3 * d)), dtype)
    K.cnnk_attention_bwd(ad, gq, dev(Oq, dtype), dev(dO, dtype), lse, gd)
    torch.cuda.synchronize()
    got = host(gd)
    assert np.all(np.isfinite(got))
    for i, name in enumerate("qkv"):
        # D = do . o is taken of the stored (rounded) output: one more rounding than the oracle's exact D.
        # With a single key the query and key gradients are exactly zero: the error is then measured
        # against the size of the value gradient.
        part, ref = got[:, :, i * d:(i + 1) * d], want[:, :, i * d:(i + 1) * d]
        scale = max(np.abs(ref).max(), 1e-2 * np.abs(want).max())
        assert np.abs(part - ref).max() / scale <= (OUT_TOL[dtype] * 2 if dtype == "bf16" else 5e-5), name


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,image,patch,dim", [(2, 16, 4, 32), (3, 32, 8, 128), (1, 224, 16, 768), (2, 24, 8, 64)])
def test_patches_and_tokens(K, B, image, patch, dim, dtype):
    rng = np.random.default_rng(image + dim)
    n = (image // patch) ** 2
    x = rep(rng.standard_normal((B, image, image, 3)), dtype)
    ed = K.embed_desc(B, image, patch, dim, dt_of(K, dtype))
    gp = dev(np.zeros((B, n, patch * patch * 3)), dtype)
    K.cnnk_vit_patchify(ed, dev(x, dtype), gp)
    torch.cuda.synchronize()
    assert (host(gp) == V.patchify(x, patch)).all()
    z = rep(rng.standard_normal((B, n, dim)), dtype)
    be, cls, pos = (rep(rng.standard_normal(s), "f32") for s in ((dim,), (dim,), (n + 1, dim)))
    gt = dev(np.zeros((B, n + 1, dim)), dtype)
    K.cnnk_vit_embed_fwd(ed, dev(z, dtype), dev_f32(be), dev_f32(cls), dev_f32(pos), gt)
    torch.cuda.synchronize()
    want = np.empty((B, n + 1, dim))
    want[:, 0] = cls + pos[0]
    want[:, 1:] = z + be + pos[1:]
    assert max_rel_err(host(gt), want) <= OUT_TOL[dtype]
    dtok = rep(rng.standard_normal((B, n + 1, dim)), dtype)
    gdz = dev(np.zeros((B, n, dim)), dtype)
    gdbe, gdcls, gdpos = (torch.zeros(s, device="cuda:0") for s in ((dim,), (dim,), (n + 1, dim)))
    K.cnnk_vit_embed_bwd(ed, dev(dtok, dtype), gdz, gdbe, gdcls, gdpos)
    torch.cuda.synchronize()
    assert (host(gdz) == dtok[:, 1:]).all()
    assert max_rel_err(host(gdpos), dtok.sum(0)) <= SUM_TOL[dtype]
    assert max_rel_err(host(gdcls), dtok[:, 0].sum(0)) <= SUM_TOL[dtype]
    assert max_rel_err(host(gdbe), dtok[:, 1:].sum((0, 1))) <= SUM_TOL[dtype]


# ---- the whole step -------------------------------------------------------------------------------------
ACTS = {"TOK": "X0", "H": "H", "QKV": "QKV", "O": "O", "XMID": "Xmid", "H2": "H2", "U": "U", "G": "G", "F": "F"}
DACTS = {"DH": "H", "DQKV": "QKV", "DO": "O", "DXMID": "Xmid", "DH2": "H2", "DU": "U", "DG": "G", "DF": "F"}


def run_hip(net, inp, lr, momentum, wd, two_streams=True):
    from paper_2503_23186_amd.vit import VitRunner
    r = VitRunner(net, two_streams=two_streams)
    r.load(inp["x"], inp["labels"], inp["params"], inp["mom"])
    r.step(lr, momentum, wd)
    torch.cuda.synchronize()
    return r


def hip_tensors(r, net):
    """The HIP step's tensors by the oracle's names: (acts, dacts, grads, params, mom)."""
    B, T, L = net.batch, net.tokens, net.layers
    acts, dacts = {}, {}
    for name, on in ACTS.items():
        if name in ("TOK", "F"):
            acts[on] = host(r.tensor(name))
        else:
            for l in range(L):
                acts["%s.%d" % (on, l)] = host(r.tensor(name, l))
    for l in range(L):
        acts["Xout.%d" % l] = host(r.tensor("XOUT", l))
    for name, on in DACTS.items():
        if name == "DF":
            dacts[on] = host(r.tensor(name))
        else:
            for l in range(L):
                dacts["%s.%d" % (on, l)] = host(r.tensor(name, l))
    for l in range(L):
        dacts["Xin.%d" % l] = host(r.tensor("DXOUT", l - 1)) if l else host(r.tensor("DTOK"))
    dacts["Xout"] = host(r.tensor("DXOUT", L - 1))
    grads = {n: host(r.grad[k]) for k, n in enumerate(r.names)}
    params = {n: host(r.param[k]) for k, n in enumerate(r.names)}
    mom = {n: host(r.mom[k]) for k, n in enumerate(r.names)}
    return acts, dacts, grads, params, mom


def oracle_tensors(out, net):
    c, L = out["cache"], net.layers
    acts = {k: v for k, v in c.items() if k.split(".")[0] in ("X0", "H", "QKV", "O", "Xmid", "H2", "U", "G", "F")}
    for l in range(L):
        acts["Xout.%d" % l] = c["Xin.%d" % (l + 1)] if l + 1 < L else c["Xout"]
    return acts, out["dacts"], out["grads"], out["params"], out["mom"]


def compare(got, want, metric):
    """Worst figure per tensor class over all tensors of the class."""
    worst = {}
    for cls, g, w in zip(("acts", "dacts", "grads", "params", "mom"), got, want):
        assert set(g) == set(w), (cls, set(g) ^ set(w))
        worst[cls] = max(metric(g[k].reshape(w[k].shape), w[k]) for k in w)
    return worst


def l2_rel(got, ref):
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


STEP_NETS = {
    "b16": dict(batch=2, image=224, patch=16, dim=768, heads=12, layers=2, mlp=3072),  # ViT-B/16's geometry, two blocks
    "b16-full-depth": dict(batch=8, image=224, patch=16, dim=768, heads=12, layers=12, mlp=3072),  # ViT-B/16 itself, batch 8
    "mini": dict(batch=4, image=32, patch=8, dim=128, heads=2, layers=2, mlp=256),
    "tall": dict(batch=2, image=64, patch=8, dim=64, heads=4, layers=3, mlp=192),     # 65 tokens, dh 16
    "wide": dict(batch=3, image=32, patch=16, dim=256, heads=4, layers=1, mlp=1024),  # 5 tokens, dh 64
}


@pytest.mark.parametrize("name", [n for n in STEP_NETS if not n.startswith("b16")])
def test_step_fp32(K, name):
    net = WL.vit_mini(dtype="f32", **STEP_NETS[name])
    inp = WL.make_vit_inputs(net, config_id=62)
    lr, mu, wd = 0.05, 0.9, 1e-3
    r = run_hip(net, inp, lr, mu, wd)
    out = V.train_step(net.cfg(), inp["x"], inp["labels"], inp["params"], inp["mom"], lr, mu, wd)
    assert abs(r.loss.item() - out["loss"]) <= 1e-4 * abs(out["loss"])
    assert (host(r.pred) == out["pred"]).all()
    assert np.abs(host(r.probs) - out["probs"]).max() <= 1e-5
    worst = compare(hip_tensors(r, net), oracle_tensors(out, net), max_rel_err)
    assert all(v <= 1e-4 for v in worst.values()), worst


@pytest.mark.parametrize("name", list(STEP_NETS))
def test_step_bf16_against_the_ensemble_of_legal_walks(K, name):
    """The free-running bf16 step against the float64 walk and against the oracle's own bf16 walks
    (plain and seeded, as for the convolutional networks): per tensor class the L2 distance to the
    float64 walk and the mean distance to the members must lie inside the band that the members
    themselves span; loss within 2e-2; predictions equal wherever the oracle's margin is clear."""
    net = WL.vit_mini(dtype="bf16", **STEP_NETS[name])
    inp = WL.make_vit_inputs(net, config_id=63)
    lr, mu, wd = 0.05, 0.9, 1e-3
    r = run_hip(net, inp, lr, mu, wd)
    cfg = net.cfg()
    exact = V.train_step(cfg, inp["x"], inp["labels"], inp["params"], inp["mom"], lr, mu, wd)
    members = [V.train_step(cfg, inp["x"], inp["labels"], inp["params"], inp["mom"], lr, mu, wd, storage="bf16")]
    members += [V.train_step(cfg, inp["x"], inp["labels"], inp["params"], inp["mom"], lr, mu, wd,
                             q=oracle_quantiser("bf16", (s, JITTER_REL))) for s in JITTER_SEEDS]
    assert abs(r.loss.item() - exact["loss"]) <= 2e-2
    got = hip_tensors(r, net)
    ex = oracle_tensors(exact, net)
    mem = [oracle_tensors(m, net) for m in members]
    d_exact = compare(got, ex, l2_rel)
    m_exact = [compare(m, ex, l2_rel) for m in mem]
    d_mem = [compare(got, m, l2_rel) for m in mem]
    m_mem = [compare(mem[i], mem[j], l2_rel) for i in range(len(mem)) for j in range(i + 1, len(mem))]
    for cls in d_exact:
        tol = 1e-6 if cls in ("params", "mom") else 2e-2
        assert d_exact[cls] <= ensemble_bound([m[cls] for m in m_exact], tol, SCALE_TO_EXACT), (cls, d_exact, m_exact)
        assert np.mean([d[cls] for d in d_mem]) <= ensemble_bound([m[cls] for m in m_mem], tol, SCALE_TO_MEMBER), (cls, d_mem, m_mem)
    logits = exact["cache"]["logits"]
    top2 = np.sort(logits, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 5e-2
    assert (host(r.pred)[clear] == exact["pred"][clear]).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_second_stream_changes_no_bit(K, dtype):
    """The weight and bias gradients forked onto a second stream: same kernels, same order of every
    sum, so two consecutive steps give bit-identical parameters, momentum buffers and gradients."""
    net = WL.vit_mini(dtype=dtype, **STEP_NETS["mini"])
    inp = WL.make_vit_inputs(net, config_id=64)
    runs = []
    for two in (False, True):
        r = run_hip(net, inp, 0.05, 0.9, 1e-3, two_streams=two)
        r.step(0.05, 0.9, 1e-3)
        torch.cuda.synchronize()
        runs.append(r)
    a, b = runs
    assert a.loss.item() == b.loss.item()
    for k in range(len(a.names)):
        assert torch.equal(a.param[k], b.param[k]) and torch.equal(a.mom[k], b.mom[k]) and torch.equal(a.grad[k], b.grad[k]), a.names[k]


# ---- the epoch loop around the step ---------------------------------------------------------------------
def _loop_case(dtype):
    net = WL.vit_mini(batch=4, dtype=dtype, image=32, patch=8, dim=128, heads=2, layers=2, mlp=256, classes=10)
    inp = WL.make_vit_inputs(net, config_id=66)
    ds = WL.make_vit_dataset(net, 66, n_train=24, n_val=8, signal=1.0)
    return net, inp, ds


def test_eval_step_matches_the_oracle_and_touches_no_training_state(K):
    from paper_2503_23186_amd.vit import VitRunner
    for dtype in ("f32", "bf16"):
        net, inp, ds = _loop_case(dtype)
        r = VitRunner(net)
        r.load(ds["val_x"][:4], ds["val_y"][:4], inp["params"], inp["mom"])
        before = [t.clone() for t in r.param + r.mom + r.grad]
        nc = torch.full((1,), 5, dtype=torch.int32, device="cuda:0")
        K.cnnk_vit_eval_step(r.desc, r.buffers, nc)
        torch.cuda.synchronize()
        loss, c = V.forward(net.cfg(), ds["val_x"][:4], ds["val_y"][:4], inp["params"], storage=None)
        tol = 1e-5 if dtype == "f32" else 2e-2
        assert abs(r.loss.item() - loss) <= tol * max(1.0, abs(loss))
        assert np.abs(host(r.probs) - c["probs"]).max() <= tol
        top2 = np.sort(c["logits"], axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > (1e-4 if dtype == "f32" else 5e-2)
        assert (host(r.pred)[clear] == c["pred"][clear]).all()
        assert nc.item() == 5 + int(np.sum(host(r.pred) == ds["val_y"][:4]))
        assert all(torch.equal(a, b) for a, b in zip(before, r.param + r.mom + r.grad))


def test_fit_matches_the_oracle_loop_fp32(K, tmp_path):
    from paper_2503_23186_amd.trainer import VitTrainer, cosine_lr
    net, inp, ds = _loop_case("f32")
    epochs, nb = 3, 24 // 4
    orders = WL.epoch_orders(66, 24, 4, epochs)
    lrs = cosine_lr(0.05, epochs * nb, warmup_steps=3)
    want = V.fit(net.cfg(), 4, ds["train_x"], ds["train_y"], ds["val_x"], ds["val_y"], inp["params"], inp["mom"], orders, lrs,
                 momentum=0.9, weight_decay=1e-3)
    t = VitTrainer(net)
    t.load_state(inp["params"], inp["mom"])
    tx, ty = t.to_device(ds["train_x"], ds["train_y"])
    vx, vy = t.to_device(ds["val_x"], ds["val_y"])
    ck = str(tmp_path / "best.safetensors")
    hist = t.fit(tx, ty, vx, vy, orders, lrs, 0.9, 1e-3, ckpt_path=ck)
    for (gl, ga, gv), (wl, wa, wv) in zip(hist, want["history"]):
        assert abs(gl - wl) <= 1e-4 * abs(wl) and ga == wa and abs(gv - wv) <= 1e-4 * abs(wv)
    for k, name in enumerate(t.run.names):
        assert max_rel_err(host(t.run.param[k]), want["params"][name].reshape(t.run.param[k].shape)) <= 1e-4, name
        assert max_rel_err(host(t.run.mom[k]), want["mom"][name].reshape(t.run.mom[k].shape)) <= 1e-4, name
    assert t.best_epoch == want["best"]["epoch"] and t.best_acc == want["best"]["acc"]
    # the checkpoint holds the best epoch's parameters and reproduces its accuracy
    t2 = VitTrainer(net)
    t2.load_checkpoint(ck)
    assert t2.epoch == want["best"]["epoch"] + 1
    for k, name in enumerate(t2.run.names):
        assert max_rel_err(host(t2.run.param[k]), want["best"]["params"][name].reshape(t2.run.param[k].shape)) <= 1e-4, name
    assert t2.evaluate(vx, vy)[0] == want["best"]["acc"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_resume_from_checkpoint_is_bit_identical(K, tmp_path, dtype):
    from paper_2503_23186_amd.trainer import VitTrainer, step_lr
    net, inp, ds = _loop_case(dtype)
    nb = 24 // 4
    orders = WL.epoch_orders(67, 24, 4, 4)
    lrs = step_lr(0.05, nb, 4, milestones=[2])
    full = VitTrainer(net)
    full.load_state(inp["params"], inp["mom"])
    tx, ty = full.to_device(ds["train_x"], ds["train_y"])
    vx, vy = full.to_device(ds["val_x"], ds["val_y"])
    h_full = full.fit(tx, ty, vx, vy, orders, lrs, 0.9, 1e-3)
    a = VitTrainer(net)
    a.load_state(inp["params"], inp["mom"])
    h_a = a.fit(tx, ty, vx, vy, orders[:2], lrs, 0.9, 1e-3)
    ck = str(tmp_path / "mid.safetensors")
    a.save_checkpoint(ck)
    b = VitTrainer(net)
    b.load_checkpoint(ck)
    h_b = b.fit(tx, ty, vx, vy, orders[2:], lrs, 0.9, 1e-3)
    assert h_a + h_b == h_full
    for k in range(len(full.run.names)):
        assert torch.equal(full.run.param[k], b.run.param[k]) and torch.equal(full.run.mom[k], b.run.mom[k])
    # the per-call profile leaves the training state alone
    before = [t.clone() for t in b.run.param + b.run.mom]
    prof = b.profile(steps=2)
    assert len(prof) == b.run.n_calls and all(ms >= 0 for _, ms in prof)
    assert all(torch.equal(x, y) for x, y in zip(before, b.run.param + b.run.mom))
