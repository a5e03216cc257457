"""GPU parity of every cnnk entry point against the fp64 oracle on the same seeded inputs.
Sizes span several tiles and ragged tails; both storage modes."""
import numpy as np
import pytest
import torch

from util import TOL, dev, dev_f32, host, max_rel_err, rep

pytestmark = pytest.mark.gpu

from oracle import ops as ref  # noqa: E402


@pytest.fixture(scope="module")
def K():
    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    from paper_2503_23186_amd import cnnk
    return cnnk


def ws_for(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0"), max(int(nbytes), 256)


# N,H,W,Cin,Cout,R,stride : multi-tile + ragged M, ragged Cout tile, BK=16 path (Cin=16,24), strided,
# odd sizes, 1x1, the 3-channel stem (direct kernels), deep reduction.
CONV_SHAPES = [
    (3, 10, 10, 64, 64, 3, 1), (2, 16, 16, 32, 128, 3, 1), (4, 8, 8, 128, 72, 3, 1),
    (2, 16, 16, 64, 128, 3, 2), (3, 7, 9, 24, 40, 3, 2), (2, 12, 12, 16, 160, 3, 1),
    (2, 16, 16, 64, 128, 1, 2), (5, 8, 8, 256, 64, 1, 1), (2, 9, 9, 40, 24, 1, 2),
    (2, 32, 32, 3, 64, 3, 1), (9, 4, 4, 512, 512, 3, 1), (2, 32, 32, 64, 64, 3, 1),
    (130, 4, 4, 64, 8, 3, 1), (3, 9, 9, 3, 16, 3, 2), (2, 8, 8, 3, 24, 3, 1), (2, 8, 8, 2, 128, 3, 1),
    (2, 8, 8, 3, 16, 1, 1), (3, 33, 33, 3, 64, 3, 1),
    # channel counts that end in a ragged 64-channel tile of the 3x3 stride-1 weight-gradient kernel
    (2, 16, 16, 160, 160, 3, 1), (4, 8, 8, 96, 160, 3, 1), (2, 16, 16, 96, 224, 3, 1),
]


def conv_inputs(shape, dtype, seed):
    N, H, W, Cin, Cout, R, st = shape
    rng = np.random.default_rng(seed)
    pad = R // 2
    x = rep(rng.standard_normal((N, H, W, Cin)), dtype)
    w = rep(rng.standard_normal((Cout, R, R, Cin)) * np.sqrt(2.0 / (Cin * R * R)), dtype)
    Ho, Wo = ref.out_hw(H, W, R, R, st, pad)
    dy = rep(rng.standard_normal((N, Ho, Wo, Cout)), dtype)
    return x, w, dy, pad


@pytest.mark.parametrize("shape", [s for s in CONV_SHAPES if s[3] < 8])
def test_thin_input_fma_kernels(K, shape):
    """The direct (plain-FMA) kernels in bf16 storage for very thin inputs, which normally take the
    first-layer or the padded MFMA path."""
    K.cnnk_tune(8, -1)
    try:
        test_conv_fwd_dgrad_wgrad(K, shape, "bf16")
    finally:
        K.cnnk_tune(8, 0)


@pytest.mark.parametrize("shape", [s for s in CONV_SHAPES if s[3] == 3 and s[5] == 3 and s[6] == 1])
def test_first_layer_on_the_padded_input_path(K, shape):
    """3-channel 3x3 stride-1 layers normally take the dedicated first-layer kernels; the padded-input
    path behind them (used for other thin inputs) is kept covered for these shapes too."""
    K.cnnk_tune(11, -1)
    try:
        test_conv_fwd_dgrad_wgrad(K, shape, "bf16")
    finally:
        K.cnnk_tune(11, 0)


@pytest.mark.parametrize("tpb", [2, 3, 8])
@pytest.mark.parametrize("shape", [s for s in CONV_SHAPES if s[3] >= 8])
def test_gathered_gemm_kernels_with_several_tiles_per_workgroup(K, shape, tpb):
    """The gathered implicit-GEMM kernels walk several tiles per workgroup on large layers (the next
    tile's loads are in flight during the current tile's epilogue); forced here on small shapes so
    that tile borders, ragged last tiles and workgroups with fewer tiles than the others are hit.
    The LDS-patch kernels are switched off so that every 3x3 shape takes this path too."""
    K.cnnk_tune(14, tpb)
    K.cnnk_tune(4, -1)
    try:
        test_conv_fwd_dgrad_wgrad(K, shape, "bf16")
    finally:
        K.cnnk_tune(14, 0)
        K.cnnk_tune(4, 0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_fwd_dgrad_wgrad(K, shape, dtype):
    N, H, W, Cin, Cout, R, st = shape
    if dtype == "f32" and N * H * W * Cin * Cout > 3e8:
        pytest.skip("fp32 direct kernels: keep the case small")
    x, w, dy, pad = conv_inputs(shape, dtype, 11)
    dt = K.BF16 if dtype == "bf16" else K.F32
    d = K.conv_desc(N, H, W, Cin, Cout, R, R, st, pad, dt)
    out_tol = 4e-3 if dtype == "bf16" else 1e-5     # one storage rounding of the output
    acc_tol = 1e-4 if dtype == "bf16" else 1e-5     # fp32 outputs of fp32 accumulation
    gx, gw, gdy = dev(x, dtype), dev(w, dtype), dev(dy, dtype)
    # forward (+ channel statistics)
    y_ref = ref.conv2d_fwd(x, w, st, pad)
    gy = torch.full(y_ref.shape, 7.0, dtype=gx.dtype, device=gx.device)
    ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_FWD))
    if Cout % 8 == 0:
        s1 = torch.zeros(Cout, device=gx.device); s2 = torch.zeros(Cout, device=gx.device)
        K.cnnk_conv2d_fwd(d, gx, gw, gy, s1, s2, ws, nb)
    else:
        K.cnnk_conv2d_fwd(d, gx, gw, gy, None, None, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gy), y_ref) <= out_tol
    if Cout % 8 == 0:
        stat_tol = 2e-2 if dtype == "bf16" else 1e-4
        assert max_rel_err(host(s1), y_ref.reshape(-1, Cout).sum(0)) <= stat_tol
        assert max_rel_err(host(s2), (y_ref ** 2).reshape(-1, Cout).sum(0)) <= stat_tol
    # data gradient: overwrite, then accumulate
    dx_ref = ref.conv2d_dgrad(dy, w, x.shape, st, pad)
    gdx = torch.full(x.shape, 3.0, dtype=gx.dtype, device=gx.device)
    ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_DGRAD))
    K.cnnk_conv2d_dgrad(d, gdy, gw, gdx, 0, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdx), dx_ref) <= out_tol
    base = rep(np.random.default_rng(5).standard_normal(x.shape), dtype)
    gdx2 = dev(base, dtype)
    K.cnnk_conv2d_dgrad(d, gdy, gw, gdx2, 1, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdx2), dx_ref + base) <= 2 * out_tol
    # weight gradient
    dw_ref = ref.conv2d_wgrad(x, dy, w.shape, st, pad)
    gdw = torch.full(w.shape, 9.0, dtype=torch.float32, device=gx.device)
    ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_WGRAD))
    K.cnnk_conv2d_wgrad(d, gx, gdy, gdw, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdw), dw_ref) <= acc_tol


WG_SHAPES = [(4, 8, 8, 64, 128), (3, 16, 16, 64, 64), (2, 32, 32, 128, 64), (18, 4, 4, 64, 64), (5, 8, 8, 192, 64),
             (1, 32, 32, 64, 64)]


@pytest.mark.parametrize("target", [1, 2, 3, 4, 0])   # 2, 3: fewer partials than the reduce has thread groups
@pytest.mark.parametrize("shape", WG_SHAPES)
def test_conv_wgrad_patch_kernel(K, shape, target):
    """3x3 stride-1 weight gradient through the LDS-patch kernel (tiles loaded straight into LDS):
    one workgroup per output tile (plain stores), a few (partial sums), and the default split."""
    N, H, W, Cin, Cout = shape
    x, w, dy, pad = conv_inputs((N, H, W, Cin, Cout, 3, 1), "bf16", 17)
    d = K.conv_desc(N, H, W, Cin, Cout, 3, 3, 1, 1, K.BF16)
    K.cnnk_tune(6, target)
    try:
        dw_ref = ref.conv2d_wgrad(x, dy, w.shape, 1, 1)
        gdw = torch.full(w.shape, 9.0, dtype=torch.float32, device="cuda:0")
        ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_WGRAD))
        K.cnnk_conv2d_wgrad(d, dev(x, "bf16"), dev(dy, "bf16"), gdw, ws, nb)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdw), dw_ref) <= 1e-4
    finally:
        K.cnnk_tune(6, 0)


PATCH_TILES = [(256, 128), (256, 64), (128, 128), (128, 64)]
PATCH_SHAPES = [(4, 8, 8, 64, 128), (2, 16, 16, 32, 64), (2, 32, 32, 32, 64), (18, 4, 4, 64, 136),
                (5, 8, 8, 96, 72), (3, 16, 16, 64, 40), (1, 32, 32, 160, 32)]


def patch_case(K, shape, tune):
    """3x3 stride-1 forward (+ channel sums) and data gradient (overwrite and accumulate) under the
    given cnnk_tune overrides, every output element against the oracle."""
    N, H, W, Cin, Cout = shape
    x, w, dy, pad = conv_inputs((N, H, W, Cin, Cout, 3, 1), "bf16", 13)
    d = K.conv_desc(N, H, W, Cin, Cout, 3, 3, 1, 1, K.BF16)
    for k, v in tune.items():
        K.cnnk_tune(k, v)
    try:
        gx, gw, gdy = dev(x, "bf16"), dev(w, "bf16"), dev(dy, "bf16")
        y_ref = ref.conv2d_fwd(x, w, 1, 1)
        gy = torch.full(y_ref.shape, 7.0, dtype=gx.dtype, device=gx.device)
        ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_FWD))
        s1 = torch.zeros(Cout, device=gx.device); s2 = torch.zeros(Cout, device=gx.device)
        K.cnnk_conv2d_fwd(d, gx, gw, gy, s1, s2, ws, nb)
        torch.cuda.synchronize()
        assert max_rel_err(host(gy), y_ref) <= 4e-3
        assert max_rel_err(host(s1), y_ref.reshape(-1, Cout).sum(0)) <= 1e-4
        assert max_rel_err(host(s2), (y_ref ** 2).reshape(-1, Cout).sum(0)) <= 1e-4
        dx_ref = ref.conv2d_dgrad(dy, w, x.shape, 1, 1)
        base = rep(np.random.default_rng(5).standard_normal(x.shape), "bf16")
        ws, nb = ws_for(K.cnnk_conv2d_workspace_bytes(d, K.PASS_DGRAD))
        gdx = torch.full(x.shape, 3.0, dtype=gx.dtype, device=gx.device)
        K.cnnk_conv2d_dgrad(d, gdy, gw, gdx, 0, ws, nb)
        gdx2 = dev(base, "bf16")
        K.cnnk_conv2d_dgrad(d, gdy, gw, gdx2, 1, ws, nb)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdx), dx_ref) <= 4e-3
        assert max_rel_err(host(gdx2), dx_ref + base) <= 8e-3
    finally:
        for k in tune:
            K.cnnk_tune(k, 0)


@pytest.mark.parametrize("groups", [2, 1])
@pytest.mark.parametrize("tile", PATCH_TILES)
@pytest.mark.parametrize("shape", PATCH_SHAPES)
def test_conv_patch_kernels_every_tile(K, shape, tile, groups):
    """3x3 stride-1 forward / data gradient through each LDS-patch tile configuration.  On grids this
    small a workgroup splits the reduction over two groups of wavefronts when the number of 32-channel
    chunks is even (64 and 128 source channels here); groups = 1 keeps it to one group."""
    patch_case(K, shape, {4: tile[0], 5: tile[1], 13: 0 if groups == 2 else -1})


# (shape, (BM, BN), pixel tiles of the launch): bands of rows inside an image (row above / below
# the band changes from tile to tile), whole-image tiles, a ragged last tile of whole images, and
# channel counts that end in a ragged channel tile
PATCH_WALKS = [((8, 32, 32, 64, 64), (256, 64), 32), ((32, 8, 8, 128, 128), (256, 64), 8),
               ((32, 8, 8, 128, 128), (128, 128), 16), ((7, 8, 8, 64, 72), (128, 64), 4),
               ((7, 8, 8, 64, 72), (256, 64), 2), ((12, 16, 16, 32, 40), (128, 64), 24),
               ((58, 4, 4, 64, 136), (128, 128), 8), ((6, 16, 16, 96, 160), (256, 128), 6)]


@pytest.mark.parametrize("tpb", [2, 4, 8])
@pytest.mark.parametrize("shape,tile,mtiles", PATCH_WALKS)
def test_conv_patch_kernels_several_tiles_per_workgroup(K, shape, tile, mtiles, tpb):
    """A workgroup of the LDS-patch kernels walks several pixel tiles on large layers (the next
    tile's first patch chunk and weights are fetched under the last steps of the current tile, the
    accumulators are written out and cleared at the border).  The library picks that only for
    layers with at least 512 workgroups' worth of tiles; forced here on small shapes so that every
    output element, the channel sums and the accumulating data gradient are compared."""
    N, H, W, Cin, Cout = shape
    assert mtiles == -(-N * H * W // tile[0])
    if mtiles % tpb != 0:
        pytest.skip("the library ignores a walk length that does not divide the tile count")
    patch_case(K, shape, {4: tile[0], 5: tile[1], 13: tpb})


@pytest.mark.parametrize("shape", [(4, 8, 8, 64, 128), (18, 4, 4, 64, 136), (16, 4, 4, 64, 64)])
def test_conv_patch_kernels_without_the_pixel_permutation(K, shape):
    """Narrow images (W < 16) normally map GEMM rows to pixels through a permutation that keeps the
    LDS reads free of bank conflicts; with it switched off the results must not change."""
    patch_case(K, shape, {7: -1})


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape,relu,with_res", [((3, 9, 7, 64), True, False), ((2, 16, 16, 160), True, True),
                                                  ((5, 4, 4, 512), False, False), ((8, 32, 32, 16), True, False),
                                                  ((2, 3, 3, 2048), False, True), ((64, 8, 8, 24), True, True)])
def test_bn_relu_fwd_bwd(K, shape, relu, with_res, dtype):
    N, H, W, Cc = shape
    rng = np.random.default_rng(21)
    x = rep(0.7 + 1.3 * rng.standard_normal(shape), dtype)
    res = rep(rng.standard_normal(shape), dtype) if with_res else None
    gamma = (1 + 0.1 * rng.standard_normal(Cc)).astype(np.float32).astype(np.float64)
    beta = (0.1 * rng.standard_normal(Cc)).astype(np.float32).astype(np.float64)
    rm = rng.standard_normal(Cc).astype(np.float32).astype(np.float64)
    rv = (1 + rng.random(Cc)).astype(np.float32).astype(np.float64)
    rm_ref, rv_ref = rm.copy(), rv.copy()
    y_ref, mean_ref, invstd_ref = ref.bn_relu_fwd(x, gamma, beta, relu=relu, residual=res,
                                                  running_mean=rm_ref, running_var=rv_ref)
    dt = K.BF16 if dtype == "bf16" else K.F32
    d = K.bn_desc(N, H, W, Cc, dt, relu)
    ws, nb = ws_for(K.cnnk_bn_workspace_bytes(d))
    gx = dev(x, dtype); gres = dev(res, dtype) if with_res else None
    gg, gb = dev_f32(gamma), dev_f32(beta)
    gy = torch.zeros_like(gx)
    gmean = torch.zeros(Cc, device=gx.device); ginv = torch.zeros(Cc, device=gx.device)
    grm, grv = dev_f32(rm), dev_f32(rv)
    K.cnnk_bn_relu_fwd(d, gx, gres, gg, gb, gy, gmean, ginv, grm, grv, None, None, ws, nb)
    torch.cuda.synchronize()
    stor = 4e-3 if dtype == "bf16" else 1e-5
    assert max_rel_err(host(gmean), mean_ref) <= 1e-5
    assert max_rel_err(host(ginv), invstd_ref) <= 1e-5
    assert max_rel_err(host(grm), rm_ref) <= 1e-5 and max_rel_err(host(grv), rv_ref) <= 1e-5
    assert max_rel_err(host(gy), y_ref) <= stor
    # statistics handed in as sums (the path fed by the convolution's per-channel sums)
    s1 = dev_f32(x.reshape(-1, Cc).sum(0)); s2 = dev_f32((x ** 2).reshape(-1, Cc).sum(0))
    gy2 = torch.zeros_like(gx)
    K.cnnk_bn_relu_fwd(d, gx, gres, gg, gb, gy2, gmean, ginv, None, None, s1, s2, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gy2), y_ref) <= max(stor, 1e-4)
    # backward on the oracle's own y rounded to storage (mask decided on identical inputs)
    y_in = rep(y_ref, dtype)
    dy = rep(rng.standard_normal(shape), dtype)
    dx_ref, dres_ref, dg_ref, db_ref = ref.bn_relu_bwd(dy, x, y_in, gamma, mean_ref, invstd_ref, relu=relu,
                                                       want_dres=with_res)
    gdx = torch.zeros_like(gx); gdres = torch.zeros_like(gx) if with_res else None
    gdg = torch.zeros(Cc, device=gx.device); gdb = torch.zeros(Cc, device=gx.device)
    K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, dev(y_in, dtype), gg, gb, dev_f32(mean_ref), dev_f32(invstd_ref),
                       gdx, gdres, 0, gdg, gdb, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdg), dg_ref) <= 1e-4 and max_rel_err(host(gdb), db_ref) <= 1e-4
    assert max_rel_err(host(gdx), dx_ref) <= stor
    if with_res:
        assert np.array_equal(host(gdres), dres_ref)
    if relu and not with_res:
        # y withheld: the mask is recomputed from x with the forward's arithmetic, so it must equal
        # the mask of the kernel's own forward output for the statistics that forward saved
        K.cnnk_bn_relu_fwd(d, gx, None, gg, gb, gy, gmean, ginv, None, None, None, None, ws, nb)
        torch.cuda.synchronize()
        dx_r, _, dg_r, db_r = ref.bn_relu_bwd(dy, x, host(gy), gamma, host(gmean), host(ginv), relu=True,
                                              want_dres=False)
        gdx3 = torch.zeros_like(gx)
        K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, None, gg, gb, gmean, ginv, gdx3, None, 0, gdg, gdb, ws, nb)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdg), dg_r) <= 1e-4 and max_rel_err(host(gdb), db_r) <= 1e-4
        assert max_rel_err(host(gdx3), dx_r) <= stor
        # withheld y needs beta and no residual branch
        with pytest.raises(RuntimeError):
            K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, None, gg, None, gmean, ginv, gdx3, None, 0, gdg, gdb, ws, nb)
    # accumulate flags
    base = rep(rng.standard_normal(shape), dtype)
    gdx2 = dev(base, dtype); gdres2 = dev(base, dtype) if with_res else None
    K.cnnk_bn_relu_bwd(d, dev(dy, dtype), gx, dev(y_in, dtype), gg, gb, dev_f32(mean_ref), dev_f32(invstd_ref),
                       gdx2, gdres2, 3, gdg, gdb, ws, nb)
    torch.cuda.synchronize()
    assert max_rel_err(host(gdx2), dx_ref + base) <= 2 * stor
    if with_res:
        assert max_rel_err(host(gdres2), dres_ref + base) <= 2 * stor


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pool_fwd_bwd(K, dtype):
    rng = np.random.default_rng(31)
    dt = K.BF16 if dtype == "bf16" else K.F32
    for shape in [(3, 8, 6, 24), (2, 32, 32, 64), (1, 2, 2, 8)]:
        N, H, W, Cc = shape
        x = rep(rng.standard_normal(shape), dtype)
        x[0, 0:2, 0:2, 0] = 1.5      # a four-way tie and a two-way tie: first in scan order wins
        x[0, 0, 1, 1] = x[0, 1, 0, 1] = 9.0
        y_ref, am_ref = ref.pool_fwd(x, "max2")
        d = K.pool_desc(N, H, W, Cc, dt, K.POOL_MAX2)
        gy = torch.zeros(y_ref.shape, dtype=dev(x, dtype).dtype, device="cuda:0")
        gam = torch.full(y_ref.shape, 255, dtype=torch.uint8, device="cuda:0")
        K.cnnk_pool_fwd(d, dev(x, dtype), gy, gam)
        torch.cuda.synchronize()
        assert np.array_equal(host(gy), y_ref)
        assert np.array_equal(gam.cpu().numpy(), am_ref)          # index work: bit exact
        dy = rep(rng.standard_normal(y_ref.shape), dtype)
        dx_ref = ref.pool_bwd(dy, am_ref, shape, "max2")
        gdx = torch.full(shape, 5.0, dtype=gy.dtype, device="cuda:0")
        K.cnnk_pool_bwd(d, dev(dy, dtype), gam, gdx, 0)
        torch.cuda.synchronize()
        assert np.array_equal(host(gdx), dx_ref)
        base = rep(rng.standard_normal(shape), dtype)
        gdx2 = dev(base, dtype)
        K.cnnk_pool_bwd(d, dev(dy, dtype), gam, gdx2, 1)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdx2), dx_ref + base) <= (8e-3 if dtype == "bf16" else 1e-6)
        # global average pool
        g_ref, _ = ref.pool_fwd(x, "gap")
        dg = K.pool_desc(N, H, W, Cc, dt, K.POOL_GAP)
        gg = torch.zeros((N, 1, 1, Cc), dtype=gy.dtype, device="cuda:0")
        K.cnnk_pool_fwd(dg, dev(x, dtype), gg, None)
        torch.cuda.synchronize()
        assert max_rel_err(host(gg), g_ref) <= (4e-3 if dtype == "bf16" else 1e-6)
        dyg = rep(rng.standard_normal((N, 1, 1, Cc)), dtype)
        gdxg = torch.zeros(shape, dtype=gy.dtype, device="cuda:0")
        K.cnnk_pool_bwd(dg, dev(dyg, dtype), None, gdxg, 0)
        torch.cuda.synchronize()
        assert max_rel_err(host(gdxg), ref.pool_bwd(dyg, None, shape, "gap")) <= (4e-3 if dtype == "bf16" else 1e-6)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,F,classes", [(8, 16, 100), (256, 512, 100), (33, 640, 100), (5, 2048, 10), (7, 52, 10), (3, 1024, 7), (64, 1536, 100), (4, 2056, 5)])
def test_fc_softmax_xent(K, N, F, classes, dtype):
    rng = np.random.default_rng(41)
    x = rep(rng.standard_normal((N, F)), dtype)
    Wm = (rng.standard_normal((classes, F)) / np.sqrt(F)).astype(np.float32).astype(np.float64)
    b = (0.1 * rng.standard_normal(classes)).astype(np.float32).astype(np.float64)
    lab = rng.integers(0, classes, N).astype(np.int32)
    r = ref.fc_softmax_xent(x, Wm, b, lab)
    dt = K.BF16 if dtype == "bf16" else K.F32
    d = K.fc_desc(N, F, classes, dt)
    ws, nb = ws_for(K.cnnk_fc_workspace_bytes(d))
    gl = torch.zeros(1, device="cuda:0"); gp = torch.zeros(N, dtype=torch.int32, device="cuda:0")
    gpr = torch.zeros((N, classes), device="cuda:0")
    gdx = torch.zeros((N, F), dtype=dev(x, dtype).dtype, device="cuda:0")
    gdW = torch.zeros((classes, F), device="cuda:0"); gdb = torch.zeros(classes, device="cuda:0")
    K.cnnk_fc_softmax_xent(d, dev(x, dtype), dev_f32(Wm), dev_f32(b), torch.from_numpy(lab).to("cuda:0"),
                           gl, gp, gpr, gdx, gdW, gdb, ws, nb)
    torch.cuda.synchronize()
    assert abs(gl.item() - r["loss"]) <= 1e-5 * abs(r["loss"])
    # predicted class: exact wherever the oracle's top-2 margin exceeds fp32 logit error
    z = x @ Wm.T + b
    top2 = np.sort(z, axis=1)[:, -2:]
    safe = (top2[:, 1] - top2[:, 0]) > 1e-4
    assert safe.sum() >= N - 1
    assert np.array_equal(gp.cpu().numpy()[safe], r["pred"][safe])
    assert max_rel_err(host(gpr), r["probs"]) <= 1e-5
    assert max_rel_err(host(gdW), r["dW"]) <= 1e-5 and max_rel_err(host(gdb), r["db"]) <= 1e-5
    assert max_rel_err(host(gdx), r["dx"]) <= (4e-3 if dtype == "bf16" else 1e-5)


def test_sgd_add_route(K):
    rng = np.random.default_rng(51)
    for n in [1, 7, 1000, 4099, 1 << 20]:
        w = rng.standard_normal(n).astype(np.float32).astype(np.float64)
        v = rng.standard_normal(n).astype(np.float32).astype(np.float64)
        g = rng.standard_normal(n).astype(np.float32).astype(np.float64)
        w_ref, v_ref = w.copy(), v.copy()
        ref.sgd_momentum(w_ref, v_ref, g, 0.1, 0.9, 5e-4)
        gw, gv, gg = dev_f32(w), dev_f32(v), dev_f32(g)
        glp = torch.zeros(n, dtype=torch.bfloat16, device="cuda:0")
        K.cnnk_sgd_momentum(n, gw, gv, gg, glp, 0.1, 0.9, 5e-4)
        torch.cuda.synchronize()
        assert max_rel_err(host(gw), w_ref) <= 1e-6 and max_rel_err(host(gv), v_ref) <= 1e-6
        assert torch.equal(glp, gw.to(torch.bfloat16))            # RNE copy of the new weights
        for dtype in ("f32", "bf16"):
            dt = K.BF16 if dtype == "bf16" else K.F32
            a = rep(rng.standard_normal(n), dtype); b = rep(rng.standard_normal(n), dtype)
            gy = torch.zeros(n, dtype=dev(a, dtype).dtype, device="cuda:0")
            K.cnnk_add(n, dt, dev(a, dtype), dev(b, dtype), gy)
            gr = dev(b, dtype)
            K.cnnk_grad_route(n, dt, dev(a, dtype), gr, 1)
            gc = dev(b, dtype)
            K.cnnk_grad_route(n, dt, dev(a, dtype), gc, 0)
            torch.cuda.synchronize()
            tol = 4e-3 if dtype == "bf16" else 1e-6
            assert max_rel_err(host(gy), a + b) <= tol and max_rel_err(host(gr), a + b) <= tol
            assert np.array_equal(host(gc), a)


def test_sgd_unaligned_tensors(K):
    """Tensors that are not 16-byte aligned take the scalar path of the update kernel."""
    rng = np.random.default_rng(52)
    n = 9000
    w = rng.standard_normal(n + 1).astype(np.float32).astype(np.float64)
    v = rng.standard_normal(n + 1).astype(np.float32).astype(np.float64)
    g = rng.standard_normal(n + 1).astype(np.float32).astype(np.float64)
    w_ref, v_ref = w[1:].copy(), v[1:].copy()
    ref.sgd_momentum(w_ref, v_ref, g[1:], 0.1, 0.9, 5e-4)
    gw, gv, gg = dev_f32(w), dev_f32(v), dev_f32(g)
    K.cnnk_sgd_momentum(n, gw[1:], gv[1:], gg[1:], None, 0.1, 0.9, 5e-4)
    torch.cuda.synchronize()
    assert max_rel_err(host(gw[1:]), w_ref) <= 1e-6 and max_rel_err(host(gv[1:]), v_ref) <= 1e-6
    assert host(gw[:1])[0] == w[0] and host(gv[:1])[0] == v[0]
