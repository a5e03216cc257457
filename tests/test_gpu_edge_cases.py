"""GPU parity on the degenerate cases of the method: decisions taken exactly at their threshold
(argmax ties, ReLU at zero), logit rows without a finite maximum, labels outside the class range,
operands that are not aligned for the vector paths."""
import numpy as np
import pytest
import torch

from util import dev, dev_f32, host, max_rel_err, rep

pytestmark = pytest.mark.gpu

from oracle import ops as ref  # noqa: E402


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    from paper_2503_23186_amd import cnnk
    return cnnk


def ws_for(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0"), max(int(nbytes), 256)


def run_head(K, x, Wm, b, lab, dtype, backward=True, gx=None, gW=None):
    N, F = x.shape
    classes = Wm.shape[0]
    dt = K.BF16 if dtype == "bf16" else K.F32
    d = K.fc_desc(N, F, classes, dt)
    ws, nb = ws_for(K.cnnk_fc_workspace_bytes(d))
    gx = dev(x, dtype) if gx is None else gx
    gW = dev_f32(Wm) if gW is None else gW
    out = dict(loss=torch.zeros(1, device="cuda:0"), pred=torch.full((N,), -7, dtype=torch.int32, device="cuda:0"),
               probs=torch.zeros((N, classes), device="cuda:0"))
    if backward:
        out.update(dx=torch.zeros((N, F), dtype=gx.dtype, device="cuda:0"),
                   dW=torch.zeros((classes, F), device="cuda:0"), db=torch.zeros(classes, device="cuda:0"))
    K.cnnk_fc_softmax_xent(d, gx, gW, dev_f32(b), torch.from_numpy(np.asarray(lab, dtype=np.int32)).to("cuda:0"),
                           out["loss"], out["pred"], out["probs"], out.get("dx"), out.get("dW"), out.get("db"), ws, nb)
    torch.cuda.synchronize()
    return out


# F = 64, 640: vector path with the features in registers; 52: scalar path; 2056: vector gradients
# with the scalar logits loop
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("F", [64, 52, 640, 2056])
@pytest.mark.parametrize("classes", [100, 7])
def test_fc_argmax_ties_lowest_index_wins(K, F, classes, dtype):
    """Logits that are exact small integers (one-hot features times integer weights), so that ties
    are exact in every precision: all classes equal, maxima duplicated in the middle, at both ends,
    across the wavefronts that share a row."""
    rng = np.random.default_rng(61)
    N = 40
    x = np.zeros((N, F))
    feat = rng.integers(0, F, N)
    x[np.arange(N), feat] = 1.0
    Wm = rng.integers(-3, 4, (classes, F)).astype(np.float64)
    b = np.zeros(classes)
    # planted rows: feature column f decides the logits of the samples that select it
    f0, f1, f2, f3 = 0, 1, 2, 3
    x[:4] = 0.0
    x[0, f0] = x[1, f1] = x[2, f2] = x[3, f3] = 1.0
    Wm[:, f0] = 2.0                                        # every class ties: class 0
    Wm[:, f1] = -1.0; Wm[[classes - 1, classes // 2], f1] = 3.0      # two maxima: the lower index
    Wm[:, f2] = 0.0; Wm[classes - 1, f2] = 1.0             # a single maximum in the last class
    Wm[:, f3] = 1.0; Wm[0, f3] = 0.0                       # every class but the first ties: class 1
    lab = rng.integers(0, classes, N)
    r = ref.fc_softmax_xent(x, Wm, b, lab)
    assert r["pred"][0] == 0 and r["pred"][1] == classes // 2 and r["pred"][2] == classes - 1 and r["pred"][3] == 1
    out = run_head(K, x, Wm, b, lab, dtype)
    assert np.array_equal(out["pred"].cpu().numpy(), r["pred"])       # exact logits: every row compared
    assert abs(out["loss"].item() - r["loss"]) <= 1e-5 * abs(r["loss"])
    # all-zero weights: every row ties over all classes, the loss is ln(classes)
    out = run_head(K, x, np.zeros_like(Wm), b, lab, dtype)
    assert np.array_equal(out["pred"].cpu().numpy(), np.zeros(N, dtype=np.int32))
    assert abs(out["loss"].item() - np.log(classes)) <= 1e-6 * np.log(classes)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fc_rows_without_a_finite_maximum(K, dtype):
    """The class scan starts at class 0 and moves on a strictly greater logit only: rows of -inf,
    rows of NaN and rows whose first logit is NaN predict class 0; a NaN elsewhere is never greater
    and is skipped.  Same decisions as the oracle's scan on the same inputs."""
    rng = np.random.default_rng(62)
    N, F, classes = 12, 64, 100
    x = rep(rng.standard_normal((N, F)), dtype)
    Wm = (rng.standard_normal((classes, F)) / 8).astype(np.float32).astype(np.float64)
    lab = rng.integers(0, classes, N)
    with np.errstate(all="ignore"):
        # every logit -inf
        b = np.full(classes, -np.inf)
        r = ref.fc_softmax_xent(x, Wm, b, lab)
        out = run_head(K, x, Wm, b, lab, dtype, backward=False)
        assert np.array_equal(r["pred"], np.zeros(N, dtype=np.int32))
        assert np.array_equal(out["pred"].cpu().numpy(), r["pred"])
        # one sample's features NaN: that row predicts 0, the others are unaffected
        b = np.zeros(classes)
        xn = x.copy(); xn[5, :] = np.nan
        r = ref.fc_softmax_xent(xn, Wm, b, lab)
        out = run_head(K, xn, Wm, b, lab, dtype, backward=False)
        z = np.delete(x, 5, axis=0) @ Wm.T
        top2 = np.sort(z, axis=1)[:, -2:]
        assert np.all(top2[:, 1] - top2[:, 0] > 1e-4)            # the other rows have clear winners
        assert r["pred"][5] == 0 and np.array_equal(out["pred"].cpu().numpy(), r["pred"])
        assert np.isnan(out["loss"].item()) and np.isnan(r["loss"])
        # NaN in the first class only: class 0 everywhere; NaN in a later class only: skipped
        for j in (0, 37):
            Wn = Wm.copy(); Wn[j, :] = np.nan
            r = ref.fc_softmax_xent(x, Wn, b, lab)
            out = run_head(K, x, Wn, b, lab, dtype, backward=False)
            assert np.array_equal(out["pred"].cpu().numpy(), r["pred"])
            if j == 0:
                assert np.all(r["pred"] == 0)
            else:
                assert np.all(r["pred"] != j) and len(set(r["pred"].tolist())) > 1


def test_fc_label_outside_the_class_range(K):
    """The labels are device data: a label outside [0, classes) cannot be refused on the host (the
    oracle refuses it), so the sample's loss, and the mean, become NaN; predictions do not depend
    on the labels."""
    rng = np.random.default_rng(63)
    N, F, classes = 9, 64, 10
    x = rep(rng.standard_normal((N, F)), "f32")
    Wm = (rng.standard_normal((classes, F)) / 8).astype(np.float32).astype(np.float64)
    b = np.zeros(classes)
    lab = rng.integers(0, classes, N)
    good = ref.fc_softmax_xent(x, Wm, b, lab)
    for bad in (classes, -1, 1 << 20):
        lab2 = lab.copy(); lab2[4] = bad
        with pytest.raises(ValueError):
            ref.fc_softmax_xent(x, Wm, b, lab2)
        out = run_head(K, x, Wm, b, lab2, "f32")
        assert np.isnan(out["loss"].item())
        assert np.array_equal(out["pred"].cpu().numpy(), good["pred"])
        assert max_rel_err(host(out["probs"]), good["probs"]) <= 1e-5


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("F", [64, 2056])
def test_fc_operands_off_the_vector_alignment(K, F, dtype):
    """x or W starting off a 16-byte boundary must take the element-wise paths (same results)."""
    rng = np.random.default_rng(64)
    N, classes = 6, 10
    x = rep(rng.standard_normal((N, F)), dtype)
    Wm = (rng.standard_normal((classes, F)) / np.sqrt(F)).astype(np.float32).astype(np.float64)
    b = (0.1 * rng.standard_normal(classes)).astype(np.float32).astype(np.float64)
    lab = rng.integers(0, classes, N)
    r = ref.fc_softmax_xent(x, Wm, b, lab)
    for shift_x, shift_w in ((1, 0), (0, 1), (1, 1)):
        bx = torch.zeros(N * F + 8, dtype=dev(x, dtype).dtype, device="cuda:0")
        bw = torch.zeros(classes * F + 8, dtype=torch.float32, device="cuda:0")
        gx = bx[shift_x:shift_x + N * F]; gx.copy_(dev(x, dtype).reshape(-1))
        gW = bw[shift_w:shift_w + classes * F]; gW.copy_(dev_f32(Wm).reshape(-1))
        assert (gx.data_ptr() % 16 != 0) == bool(shift_x) and (gW.data_ptr() % 16 != 0) == bool(shift_w)
        out = run_head(K, x, Wm, b, lab, dtype, gx=gx, gW=gW)
        assert abs(out["loss"].item() - r["loss"]) <= 1e-5 * abs(r["loss"])
        assert max_rel_err(host(out["dW"]), r["dW"]) <= 1e-5 and max_rel_err(host(out["db"]), r["db"]) <= 1e-5
        assert max_rel_err(host(out["dx"]), r["dx"]) <= (4e-3 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("with_res", [False, True])
def test_relu_exactly_at_zero(K, with_res, dtype):
    """ReLU'(0) = 0 (the mask is y > 0, strict).  Channels hold the values {-a, 0, +a} with as many
    +a as -a, so the batch mean is exactly 0 in any precision and, with beta = 0 (and a zero
    residual there), a third of the pre-activations are exactly 0.  Those elements must give y = 0
    and pass no gradient: the residual gradient is compared bit for bit, dbeta and dgamma would
    move by O(1) if the mask were y >= 0."""
    N, H, W, C = 6, 4, 4, 16
    rng = np.random.default_rng(65)
    m = N * H * W
    x = np.empty((m, C))
    for c in range(C):
        a = 2.0 ** int(rng.integers(-2, 3))                     # exactly representable in bf16
        col = np.array([0.0, a, -a] * (m // 3))
        x[:, c] = rng.permutation(col)
    x = x.reshape(N, H, W, C)
    zero = x == 0.0
    gamma = (1 + 0.25 * rng.integers(-2, 3, C)).astype(np.float64)
    beta = np.zeros(C)
    res = None
    if with_res:
        res = rep(rng.standard_normal(x.shape), dtype)
        res[zero] = 0.0
    dy = rep(1.0 + rng.random(x.shape), dtype)               # positive: a wrong mask cannot cancel
    y_ref, mean_ref, invstd_ref = ref.bn_relu_fwd(x, gamma, beta, relu=True, residual=res)
    assert np.all(mean_ref == 0.0) and np.all(y_ref[zero] == 0.0)
    dt = K.BF16 if dtype == "bf16" else K.F32
    d = K.bn_desc(N, H, W, C, dt, 1)
    ws, nb = ws_for(K.cnnk_bn_workspace_bytes(d))
    gx, gg, gb = dev(x, dtype), dev_f32(gamma), dev_f32(beta)
    gres = dev(res, dtype) if with_res else None
    gy = torch.full(x.shape, 5.0, dtype=gx.dtype, device="cuda:0")
    gm = torch.empty(C, device="cuda:0"); gi = torch.empty(C, device="cuda:0")
    K.cnnk_bn_relu_fwd(d, gx, gres, gg, gb, gy, gm, gi, None, None, None, None, ws, nb)
    torch.cuda.synchronize()
    stor = 4e-3 if dtype == "bf16" else 1e-5
    assert np.all(host(gm) == 0.0)
    assert np.all(host(gy)[zero] == 0.0)
    assert max_rel_err(host(gy), y_ref) <= stor
    y_in = host(gy)                                          # the kernel's own stored output decides the mask
    dx_ref, dres_ref, dg_ref, db_ref = ref.bn_relu_bwd(dy, x, y_in, gamma, host(gm), host(gi), relu=True,
                                                       want_dres=with_res)
    variants = [gy] if with_res else [gy, None]              # None: mask recomputed from x
    for ymask in variants:
        gdx = torch.full(x.shape, 5.0, dtype=gx.dtype, device="cuda:0")
        gdr = torch.full(x.shape, 5.0, dtype=gx.dtype, device="cuda:0") if with_res else None
        gdg = torch.empty(C, device="cuda:0"); gdb = torch.empty(C, device="cuda:0")
        K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, ymask, gg, gb, gm, gi, gdx, gdr, 0, gdg, gdb, ws, nb)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdb), db_ref) <= 1e-5 and max_rel_err(host(gdg), dg_ref) <= 1e-4
        assert max_rel_err(host(gdx), dx_ref) <= stor
        if with_res:
            assert np.array_equal(host(gdr), dres_ref)
            assert np.all(host(gdr)[zero] == 0.0)
    # what a non-strict mask would have produced is far outside the tolerance (the test can fail)
    dz_wrong = dy * (y_in >= 0)
    assert abs(dz_wrong.reshape(-1, C).sum(0) - db_ref).max() > 0.2 * abs(db_ref).max()
