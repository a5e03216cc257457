"""ctypes wrappers over libcnnk_ref.so (numpy float64 in, numpy float64 out).  Test infrastructure."""
from __future__ import annotations
import ctypes as C
import os
import numpy as np
from .build import build, LIB

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = C.CDLL(LIB)
        _lib.cnnk_ref_sgd_momentum.argtypes = [C.c_long, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_double, C.c_double, C.c_double]
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _chk(rc, name):
    if rc != 0:
        raise ValueError("%s failed with code %d" % (name, rc))


def out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv2d_fwd(x, w, stride, pad):
    x, w = _f64(x), _f64(w)
    N, H, W_, Cin = x.shape
    Cout, R, S, Cin2 = w.shape
    assert Cin == Cin2
    Ho, Wo = out_hw(H, W_, R, S, stride, pad)
    y = np.empty((N, Ho, Wo, Cout))
    _chk(lib().cnnk_ref_conv2d_fwd(N, H, W_, Cin, Cout, R, S, stride, pad, _p(x), _p(w), _p(y)), "conv2d_fwd")
    return y


def conv2d_dgrad(dy, w, x_shape, stride, pad):
    dy, w = _f64(dy), _f64(w)
    N, H, W_, Cin = x_shape
    Cout, R, S, _ = w.shape
    assert dy.shape == (N,) + out_hw(H, W_, R, S, stride, pad) + (Cout,)
    dx = np.empty((N, H, W_, Cin))
    _chk(lib().cnnk_ref_conv2d_dgrad(N, H, W_, Cin, Cout, R, S, stride, pad, _p(dy), _p(w), _p(dx)), "conv2d_dgrad")
    return dx


def conv2d_wgrad(x, dy, w_shape, stride, pad):
    x, dy = _f64(x), _f64(dy)
    N, H, W_, Cin = x.shape
    Cout, R, S, _ = w_shape
    assert dy.shape == (N,) + out_hw(H, W_, R, S, stride, pad) + (Cout,)
    dw = np.empty((Cout, R, S, Cin))
    _chk(lib().cnnk_ref_conv2d_wgrad(N, H, W_, Cin, Cout, R, S, stride, pad, _p(x), _p(dy), _p(dw)), "conv2d_wgrad")
    return dw


def bn_relu_fwd(x, gamma, beta, relu=True, residual=None, eps=1e-5, momentum=0.1,
                running_mean=None, running_var=None):
    """Returns y, save_mean, save_invstd; running_mean/var (float64 arrays) are updated in place."""
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, H, W_, Cc = x.shape
    residual = None if residual is None else _f64(residual)
    y = np.empty_like(x)
    mean = np.empty(Cc)
    invstd = np.empty(Cc)
    _chk(lib().cnnk_ref_bn_relu_fwd(N, H, W_, Cc, C.c_double(eps), C.c_double(momentum), int(relu),
                                    _p(x), _p(residual), _p(gamma), _p(beta), _p(y), _p(mean),
                                    _p(invstd), _p(running_mean), _p(running_var)), "bn_relu_fwd")
    return y, mean, invstd


def bn_relu_infer(x, gamma, beta, running_mean, running_var, relu=True, residual=None, eps=1e-5):
    """Inference-mode batch norm: running statistics instead of the batch's."""
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, H, W_, Cc = x.shape
    residual = None if residual is None else _f64(residual)
    y = np.empty_like(x)
    _chk(lib().cnnk_ref_bn_relu_infer(N, H, W_, Cc, C.c_double(eps), int(relu), _p(x), _p(residual),
                                      _p(gamma), _p(beta), _p(_f64(running_mean)), _p(_f64(running_var)),
                                      _p(y)), "bn_relu_infer")
    return y


def bn_relu_bwd(dy, x, y, gamma, mean, invstd, relu=True, want_dres=False):
    dy, x, y, gamma = _f64(dy), _f64(x), _f64(y), _f64(gamma)
    N, H, W_, Cc = x.shape
    dx = np.empty_like(x)
    dres = np.empty_like(x) if want_dres else None
    dg = np.empty(Cc)
    db = np.empty(Cc)
    _chk(lib().cnnk_ref_bn_relu_bwd(N, H, W_, Cc, int(relu), _p(dy), _p(x), _p(y), _p(gamma),
                                    _p(_f64(mean)), _p(_f64(invstd)), _p(dx), _p(dres), _p(dg), _p(db)),
         "bn_relu_bwd")
    return dx, dres, dg, db


def pool_fwd(x, mode):
    x = _f64(x)
    N, H, W_, Cc = x.shape
    if mode == "max2":
        y = np.empty((N, H // 2, W_ // 2, Cc))
        am = np.empty((N, H // 2, W_ // 2, Cc), dtype=np.uint8)
        _chk(lib().cnnk_ref_pool_fwd(N, H, W_, Cc, 0, _p(x), _p(y), _p(am)), "pool_fwd")
        return y, am
    y = np.empty((N, 1, 1, Cc))
    _chk(lib().cnnk_ref_pool_fwd(N, H, W_, Cc, 1, _p(x), _p(y), None), "pool_fwd")
    return y, None


def pool_bwd(dy, argmax, x_shape, mode):
    dy = _f64(dy)
    N, H, W_, Cc = x_shape
    dx = np.empty(x_shape)
    if mode == "max2":
        am = np.ascontiguousarray(argmax, dtype=np.uint8)
        _chk(lib().cnnk_ref_pool_bwd(N, H, W_, Cc, 0, _p(dy), _p(am), _p(dx)), "pool_bwd")
    else:
        _chk(lib().cnnk_ref_pool_bwd(N, H, W_, Cc, 1, _p(dy), None, _p(dx)), "pool_bwd")
    return dx


def fc_softmax_xent(x, W, b, labels):
    """Returns dict(loss, pred, probs, dx, dW, db)."""
    x, W, b = _f64(x), _f64(W), _f64(b)
    N, F = x.shape
    classes = W.shape[0]
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    loss = np.empty(1)
    pred = np.empty(N, dtype=np.int32)
    probs = np.empty((N, classes))
    dx = np.empty((N, F))
    dW = np.empty((classes, F))
    db = np.empty(classes)
    _chk(lib().cnnk_ref_fc_softmax_xent(N, F, classes, _p(x), _p(W), _p(b), _p(labels), _p(loss),
                                        _p(pred), _p(probs), _p(dx), _p(dW), _p(db)), "fc_softmax_xent")
    return dict(loss=float(loss[0]), pred=pred, probs=probs, dx=dx, dW=dW, db=db)


def sgd_momentum(w, v, g, lr, momentum, weight_decay=0.0):
    """In place on float64 contiguous w, v."""
    assert w.dtype == np.float64 and v.dtype == np.float64 and w.flags.c_contiguous and v.flags.c_contiguous
    g = _f64(g)
    _chk(lib().cnnk_ref_sgd_momentum(w.size, _p(w), _p(v), _p(g), lr, momentum, weight_decay), "sgd_momentum")


def round_bf16(a):
    """Return a copy of `a` with every value rounded to the nearest bfloat16 (ties to even)."""
    out = np.array(a, dtype=np.float64, copy=True, order="C")
    lib().cnnk_ref_round_bf16.argtypes = [C.c_long, C.c_void_p]
    _chk(lib().cnnk_ref_round_bf16(out.size, _p(out)), "round_bf16")
    return out


def num_threads():
    return lib().cnnk_ref_num_threads()
