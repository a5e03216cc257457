"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol that
include/cnnk.h declares, and rejects bad arguments on the host before launching anything."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def cnnk():
    lib_path = os.path.join(ROOT, "paper_2503_23186_amd", "libcnnk.so")
    if not os.path.exists(lib_path):
        from paper_2503_23186_amd.build import build
        build()
    from paper_2503_23186_amd import cnnk as mod
    return mod


def declared_functions(header="cnnk.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cnnk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(cnnk):
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(cnnk.lib, n), n
    assert sorted(cnnk.EXPORTS) == names
    assert "gfx950" in cnnk.version()


def test_every_symbol_of_the_transformer_header_is_exported(cnnk):
    from paper_2503_23186_amd import vit
    names = declared_functions("cnnk_vit.h")
    assert len(names) >= 15
    for n in names:
        assert hasattr(cnnk.lib, n), n
    assert sorted(vit.EXPORTS) == names
    assert C.sizeof(vit.LnDesc) == 24 and C.sizeof(vit.AttnDesc) == 20 and C.sizeof(vit.EmbedDesc) == 20
    assert C.sizeof(vit.VitDesc) == 40 and C.sizeof(vit.VitBuffers) == 152


def test_transformer_entry_points_reject_bad_arguments_on_the_host(cnnk):
    from paper_2503_23186_amd import vit
    ln = vit.ln_desc(8, 30, cnnk.F32)
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_layernorm_fwd(ln, 256, 256, 256, 256, 256)
    assert e.value.status == 3                              # C must be a multiple of 4
    ln = vit.ln_desc(8, 32, cnnk.F32)
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_layernorm_fwd(ln, 256, 256, 256, None, 256)
    assert e.value.status == 1
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_layernorm_bwd(ln, 256, 256, 256, 256, None, 256, 256, 256, None, 0)
    assert e.value.status == 4
    assert vit.cnnk_layernorm_workspace_bytes(ln) >= 2 * 32 * 4
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_bias_act_fwd(4, 12, cnnk.BF16, vit.ACT_NONE, 256, 256, None, None, 256)
    assert e.value.status == 3
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_bias_act_fwd(4, 16, cnnk.BF16, vit.ACT_GELU, 256, 256, 256, 256, 256)
    assert e.value.status == 3                              # no residual behind the activation
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_attention_fwd(vit.attn_desc(1, 197, 12, 48, cnnk.BF16), 256, 256, 256)
    assert e.value.status == 3
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_attention_fwd(vit.attn_desc(1, 0, 12, 64, cnnk.BF16), 256, 256, 256)
    assert e.value.status == 2
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_vit_patchify(vit.embed_desc(1, 30, 8, 64, cnnk.F32), 256, 256)
    assert e.value.status == 2                              # the image is not a whole number of patches
    d = vit.vit_desc(64, 224, 16, 768, 12, 12, 3072, 100, cnnk.BF16)
    assert vit.cnnk_vit_step_calls(d) == 3 + 12 * 7 + 2 + 2 + 12 * 15 + 2 + 1
    assert vit.cnnk_vit_step_call_name(d, 0) == "embed.patchify"
    assert vit.cnnk_vit_step_call_name(d, vit.cnnk_vit_step_calls(d) - 1) == "update"
    off, nb = vit.cnnk_vit_tensor(d, vit.TENSOR_IDS.index("QKV"), 3)
    assert nb == 64 * 197 * 2304 * 2 and off % 256 == 0
    assert vit.cnnk_vit_arena_bytes(d) > 12 * 2 * nb
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_vit_tensor(d, vit.TENSOR_IDS.index("QKV"), 12)
    assert e.value.status == 2
    bad = vit.vit_desc(64, 224, 16, 768, 10, 12, 3072, 100, cnnk.BF16)
    assert vit.cnnk_vit_arena_bytes(bad) == 0               # 768 / 10 heads
    b = vit.VitBuffers()
    with pytest.raises(cnnk.CnnkError) as e:
        vit.cnnk_vit_train_step(d, b, 0.1, 0.9, 0.0)
    assert e.value.status == 1


def test_struct_layouts_match_header(cnnk):
    assert C.sizeof(cnnk.ConvDesc) == 40 and C.sizeof(cnnk.BnDesc) == 32
    assert C.sizeof(cnnk.PoolDesc) == 24 and C.sizeof(cnnk.FcDesc) == 16
    assert C.sizeof(cnnk.Layer) == 24 + 40


def test_argument_errors_are_reported_before_any_launch(cnnk):
    d = cnnk.conv_desc(2, 8, 8, 16, 16, 3, 3, 1, 1, cnnk.BF16)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_conv2d_fwd(d, None, None, None)
    assert e.value.status == 1
    bad = cnnk.conv_desc(2, 8, 8, 16, 16, 5, 5, 1, 2, cnnk.BF16)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_conv2d_fwd(bad, 256, 256, 256)
    assert e.value.status == 3
    neg = cnnk.conv_desc(0, 8, 8, 16, 16, 3, 3, 1, 1, cnnk.BF16)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_conv2d_wgrad(neg, 256, 256, 256)
    assert e.value.status == 2
    # dgrad on the MFMA path needs its workspace
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_conv2d_dgrad(d, 256, 256, 256, 0, None, 0)
    assert e.value.status == 4
    assert cnnk.cnnk_conv2d_workspace_bytes(d, cnnk.PASS_DGRAD) >= 16 * 16 * 9 * 2
    bn = cnnk.bn_desc(2, 4, 4, 12, cnnk.F32, 1)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_bn_relu_fwd(bn, 256, None, 256, 256, 256, 256, 256, ws=256, ws_bytes=1 << 20)
    assert e.value.status == 3          # C must be a multiple of 8
    pool = cnnk.pool_desc(2, 5, 4, 8, cnnk.F32, cnnk.POOL_MAX2)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_pool_fwd(pool, 256, 256, 256)
    assert e.value.status == 2          # odd height
    fc = cnnk.fc_desc(4, 16, 100, cnnk.F32)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_fc_softmax_xent(fc, 256, 256, 256, 256, 256, 256, None, 256, 256, 256, None, 0)
    assert e.value.status == 4
    assert cnnk.status_string(4).startswith("workspace")
    # the allocation-free head refuses shapes beyond its fixed scratch, and bad arguments, on the host
    big = cnnk.fc_desc(4096, 64, 100, cnnk.F32)
    assert cnnk.cnnk_fc_workspace_bytes(big) > cnnk.FC_STATIC_SCRATCH_BYTES
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_fc_softmax_xent_static(big, 256, 256, 256, 256, 256, 256, None, None, None, None)
    assert e.value.status == 4
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_fc_softmax_xent_static(fc, 256, 256, 256, None, 256, 256, None, None, None, None)
    assert e.value.status == 1


def test_train_step_validates_the_layer_list(cnnk):
    import workloads as WL
    net = WL.mini_resnet()
    nl = len(net.layers)
    layers = (cnnk.Layer * nl)()
    # an all-zero list is a list of malformed convolutions
    assert cnnk.cnnk_train_step_workspace_bytes(layers, nl) == 0
    b = cnnk.Buffers()
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_train_step(layers, nl, b, 256, 0.1, 0.9, 0.0, 256, 256)
    assert e.value.status == 1


def test_train_step_checks_the_workspace_before_any_launch(cnnk):
    """Workspace too small, and the second stream without the doubled workspace: both are argument
    errors found on the host (no GPU needed; the fake pointers are never dereferenced)."""
    import ctypes as C
    import workloads as WL
    from paper_2503_23186_amd.runner import build_c_layers
    net = WL.mini_resnet(batch=4, dtype="bf16", widths=(64, 128))
    nl, ns, npar = len(net.layers), len(net.slots), len(net.params)
    layers = build_c_layers(net.layers, cnnk.BF16)
    need = cnnk.cnnk_train_step_workspace_bytes(layers, nl)
    assert need > 0
    fake = 4096

    def arr(n):
        a = (C.c_void_p * n)()
        for k in range(n):
            a[k] = fake
        return a

    keep = dict(act=arr(ns), dact=arr(ns), param=arr(npar), param_lp=arr(npar), grad=arr(npar), mom=arr(npar),
                bn_save=arr(nl), bn_running=arr(nl), pool_idx=arr(nl))
    b = cnnk.Buffers()
    b.n_slots, b.n_params = ns, npar
    for k, a in keep.items():
        setattr(b, k, C.cast(a, C.POINTER(C.c_void_p)))
    b.ws, b.ws_bytes = fake, need - 1
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_train_step(layers, nl, b, fake, 0.1, 0.9, 0.0, fake, fake)
    assert e.value.status == 4
    b.ws_bytes = need            # enough for one stream, not for two
    b.aux_stream, b.ev_fork, b.ev_join = fake, fake, fake
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_train_step(layers, nl, b, fake, 0.1, 0.9, 0.0, fake, fake)
    assert e.value.status == 4


def test_epoch_loop_entry_points_reject_bad_arguments_on_the_host(cnnk):
    """cnnk_bn_relu_infer, cnnk_count_correct and cnnk_eval_step validate before they launch."""
    import workloads as WL
    from paper_2503_23186_amd.runner import build_c_layers
    d = cnnk.bn_desc(2, 4, 4, 16, cnnk.F32, 1, 1e-5, 0.1)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_bn_relu_infer(d, 256, None, 256, 256, 256, None, 256)       # no running variance
    assert e.value.status == 1
    odd = cnnk.bn_desc(2, 4, 4, 12, cnnk.F32, 1, 1e-5, 0.1)                    # channels not in octets
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_bn_relu_infer(odd, 256, None, 256, 256, 256, 256, 256)
    assert e.value.status == 3
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_count_correct(0, 256, 256, 256)
    assert e.value.status == 2
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_count_correct(8, 256, None, 256)
    assert e.value.status == 1
    net = WL.mini_resnet()
    layers = build_c_layers(net.layers, cnnk.F32)
    b = cnnk.Buffers()
    with pytest.raises(cnnk.CnnkError) as e:                                   # no buffers at all
        cnnk.cnnk_eval_step(layers, len(net.layers), b, 256, 256, 256, None, 0)
    assert e.value.status == 1
    # forward-only classifier head: the three gradient outputs come together or not at all
    fd = cnnk.fc_desc(4, 16, 10, cnnk.F32)
    with pytest.raises(cnnk.CnnkError) as e:
        cnnk.cnnk_fc_softmax_xent(fd, 256, 256, 256, 256, 256, 256, None, 256, None, 256, 256, 1 << 20)
    assert e.value.status == 1
