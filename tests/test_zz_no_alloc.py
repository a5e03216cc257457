"""The classifier-head entry point that allocates nothing (scratch in an array inside the library's
code object) against the workspace-taking entry point: same kernels, so the same bits; and against
the oracle.  Two calls in a row, the second on a smaller input, so that what the first call left
in the shared array cannot leak into the second."""
import numpy as np
import pytest
import torch

from util import dev, dev_f32, host, max_rel_err, rep

from oracle import ops as ref  # noqa: E402


def _outputs(N, F, classes, tdtype, poison):
    o = dict(loss=torch.full((1,), poison, device="cuda:0"),
             pred=torch.full((N,), -5, dtype=torch.int32, device="cuda:0"),
             probs=torch.full((N, classes), poison, device="cuda:0"),
             dx=torch.full((N, F), poison, dtype=tdtype, device="cuda:0"),
             dW=torch.full((classes, F), poison, device="cuda:0"),
             db=torch.full((classes,), poison, device="cuda:0"))
    return o


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_head_matches_the_workspace_head(dtype):
    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    from paper_2503_23186_amd import cnnk as K
    rng = np.random.default_rng(71)
    dt = K.BF16 if dtype == "bf16" else K.F32
    # the second case is smaller than the first in every dimension; the third is the benchmark's head
    for N, F, classes in [(96, 640, 100), (17, 52, 10), (256, 512, 100)]:
        x = rep(rng.standard_normal((N, F)), dtype)
        Wm = (rng.standard_normal((classes, F)) / np.sqrt(F)).astype(np.float32).astype(np.float64)
        b = (0.1 * rng.standard_normal(classes)).astype(np.float32).astype(np.float64)
        lab = rng.integers(0, classes, N).astype(np.int32)
        d = K.fc_desc(N, F, classes, dt)
        gx, gW, gb = dev(x, dtype), dev_f32(Wm), dev_f32(b)
        gl = torch.from_numpy(lab).to("cuda:0")
        a = _outputs(N, F, classes, gx.dtype, 3.0)
        s = _outputs(N, F, classes, gx.dtype, -4.0)
        nb = K.cnnk_fc_workspace_bytes(d)
        assert nb <= K.FC_STATIC_SCRATCH_BYTES
        ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda:0")
        K.cnnk_fc_softmax_xent(d, gx, gW, gb, gl, a["loss"], a["pred"], a["probs"], a["dx"], a["dW"], a["db"], ws, nb)
        K.cnnk_fc_softmax_xent_static(d, gx, gW, gb, gl, s["loss"], s["pred"], s["probs"], s["dx"], s["dW"], s["db"])
        torch.cuda.synchronize()
        for k in a:
            assert torch.equal(a[k], s[k]), (k, N, F, classes)
        r = ref.fc_softmax_xent(x, Wm, b, lab)
        assert abs(s["loss"].item() - r["loss"]) <= 1e-5 * abs(r["loss"])
        assert max_rel_err(host(s["probs"]), r["probs"]) <= 1e-5
        assert max_rel_err(host(s["dW"]), r["dW"]) <= 1e-5 and max_rel_err(host(s["db"]), r["db"]) <= 1e-5
        assert max_rel_err(host(s["dx"]), r["dx"]) <= (4e-3 if dtype == "bf16" else 1e-5)
        z = x @ Wm.T + b
        top2 = np.sort(z, axis=1)[:, -2:]
        safe = (top2[:, 1] - top2[:, 0]) > 1e-4
        assert np.array_equal(s["pred"].cpu().numpy()[safe], r["pred"][safe])
        # forward half only
        f = _outputs(N, F, classes, gx.dtype, 9.0)
        K.cnnk_fc_softmax_xent_static(d, gx, gW, gb, gl, f["loss"], f["pred"], f["probs"], None, None, None)
        torch.cuda.synchronize()
        assert torch.equal(f["loss"], a["loss"]) and torch.equal(f["pred"], a["pred"]) and torch.equal(f["probs"], a["probs"])


@pytest.mark.gpu
def test_static_scratch_head_refuses_what_does_not_fit():
    from paper_2503_23186_amd import cnnk as K
    d = K.fc_desc(4096, 64, 100, K.F32)        # 4096 * 101 floats > 1 MiB
    assert K.cnnk_fc_workspace_bytes(d) > K.FC_STATIC_SCRATCH_BYTES
    t = torch.zeros(8, device="cuda:0")
    with pytest.raises(K.CnnkError) as e:
        K.cnnk_fc_softmax_xent_static(d, t, t, t, t, t, t, None, None, None, None)
    assert e.value.status == 4
