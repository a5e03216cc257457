"""ctypes binding of libcnnk.so: same names as the C entry points, marshalling only.

Tensor arguments may be torch tensors (their data_ptr() is passed), integers (raw device
addresses) or None (NULL).  Every function returns nothing and raises CnnkError on a non-zero
status.  `stream` is a raw hipStream_t value (0 = default stream), e.g.
torch.cuda.current_stream().cuda_stream.
"""
from __future__ import annotations
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcnnk.so")

F32, BF16 = 0, 1
POOL_MAX2, POOL_GAP = 0, 1
PASS_FWD, PASS_DGRAD, PASS_WGRAD = 0, 1, 2
OP_CONV, OP_BN, OP_POOL, OP_ADD, OP_FC_LOSS = 0, 1, 2, 3, 4

EXPORTS = ["cnnk_status_string", "cnnk_version", "cnnk_tune", "cnnk_conv2d_workspace_bytes", "cnnk_conv2d_fwd",
           "cnnk_conv2d_dgrad", "cnnk_conv2d_wgrad", "cnnk_bn_workspace_bytes", "cnnk_bn_relu_fwd",
           "cnnk_bn_relu_infer", "cnnk_bn_relu_bwd", "cnnk_pool_fwd", "cnnk_pool_bwd", "cnnk_add", "cnnk_grad_route",
           "cnnk_fc_workspace_bytes", "cnnk_fc_softmax_xent", "cnnk_fc_softmax_xent_static", "cnnk_count_correct", "cnnk_sgd_momentum", "cnnk_round_bf16", "cnnk_gather_rows",
           "cnnk_train_step_workspace_bytes", "cnnk_train_step_event_groups", "cnnk_train_step",
           "cnnk_eval_step"]


class CnnkError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, status_string(status)))


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "H", "W", "Cin", "Cout", "R", "S", "stride", "pad", "dtype")]


class BnDesc(C.Structure):
    _fields_ = [("N", C.c_int), ("H", C.c_int), ("W", C.c_int), ("C", C.c_int), ("dtype", C.c_int),
                ("eps", C.c_float), ("momentum", C.c_float), ("relu", C.c_int)]


class PoolDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "H", "W", "C", "dtype", "mode")]


class FcDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "F", "classes", "dtype")]


class _DescUnion(C.Union):
    _fields_ = [("conv", ConvDesc), ("bn", BnDesc), ("pool", PoolDesc), ("fc", FcDesc)]


class Layer(C.Structure):
    _fields_ = [("op", C.c_int), ("in0", C.c_int), ("in1", C.c_int), ("out", C.c_int), ("p0", C.c_int),
                ("p1", C.c_int), ("d", _DescUnion)]


class Buffers(C.Structure):
    _fields_ = [("n_slots", C.c_int), ("n_params", C.c_int),
                ("act", C.POINTER(C.c_void_p)), ("dact", C.POINTER(C.c_void_p)),
                ("param", C.POINTER(C.c_void_p)), ("param_lp", C.POINTER(C.c_void_p)),
                ("grad", C.POINTER(C.c_void_p)), ("mom", C.POINTER(C.c_void_p)),
                ("bn_save", C.POINTER(C.c_void_p)), ("bn_running", C.POINTER(C.c_void_p)),
                ("pool_idx", C.POINTER(C.c_void_p)), ("probs", C.c_void_p),
                ("ws", C.c_void_p), ("ws_bytes", C.c_size_t),
                ("events", C.POINTER(C.c_void_p)), ("n_events", C.c_int),
                ("aux_stream", C.c_void_p), ("ev_fork", C.c_void_p), ("ev_join", C.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libcnnk.so is not built: run `python -m paper_2503_23186_amd.build` "
                           "(there is no CPU fallback)")
    # The buffers and streams handed to the library come from torch, so both must run on one HIP
    # runtime.  torch ships its own copy of libamdhip64 and the dynamic loader serves every later request
    # for that name with whichever copy came first: with the library loaded before torch its kernels
    # would be registered with another runtime than the one that owns the memory, and every launch fails.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, ci, cf, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    lib.cnnk_status_string.restype = C.c_char_p
    lib.cnnk_status_string.argtypes = [ci]
    lib.cnnk_version.restype = C.c_char_p
    lib.cnnk_tune.argtypes = [ci, ci]
    lib.cnnk_conv2d_workspace_bytes.restype = sz
    lib.cnnk_conv2d_workspace_bytes.argtypes = [C.POINTER(ConvDesc), ci]
    lib.cnnk_conv2d_fwd.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cnnk_conv2d_dgrad.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, ci, vp, sz, vp]
    lib.cnnk_conv2d_wgrad.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, sz, vp]
    lib.cnnk_bn_workspace_bytes.restype = sz
    lib.cnnk_bn_workspace_bytes.argtypes = [C.POINTER(BnDesc)]
    lib.cnnk_bn_relu_fwd.argtypes = [C.POINTER(BnDesc)] + [vp] * 11 + [vp, sz, vp]
    lib.cnnk_bn_relu_infer.argtypes = [C.POINTER(BnDesc)] + [vp] * 7 + [vp]
    lib.cnnk_bn_relu_bwd.argtypes = [C.POINTER(BnDesc)] + [vp] * 9 + [ci, vp, vp, vp, sz, vp]
    lib.cnnk_pool_fwd.argtypes = [C.POINTER(PoolDesc), vp, vp, vp, vp]
    lib.cnnk_pool_bwd.argtypes = [C.POINTER(PoolDesc), vp, vp, vp, ci, vp]
    lib.cnnk_add.argtypes = [sz, ci, vp, vp, vp, vp]
    lib.cnnk_grad_route.argtypes = [sz, ci, vp, vp, ci, vp]
    lib.cnnk_fc_workspace_bytes.restype = sz
    lib.cnnk_fc_workspace_bytes.argtypes = [C.POINTER(FcDesc)]
    lib.cnnk_fc_softmax_xent.argtypes = [C.POINTER(FcDesc)] + [vp] * 10 + [vp, sz, vp]
    lib.cnnk_fc_softmax_xent_static.argtypes = [C.POINTER(FcDesc)] + [vp] * 10 + [vp]
    lib.cnnk_count_correct.argtypes = [ci, vp, vp, vp, vp]
    lib.cnnk_sgd_momentum.argtypes = [sz, vp, vp, vp, vp, cf, cf, cf, vp]
    lib.cnnk_round_bf16.argtypes = [sz, vp, vp, vp]
    lib.cnnk_gather_rows.argtypes = [ci, C.c_longlong, sz, vp, vp, vp, vp, vp]
    lib.cnnk_train_step_workspace_bytes.restype = sz
    lib.cnnk_train_step_workspace_bytes.argtypes = [C.POINTER(Layer), ci]
    lib.cnnk_train_step_event_groups.argtypes = [ci]
    lib.cnnk_train_step.argtypes = [C.POINTER(Layer), ci, C.POINTER(Buffers), vp, cf, cf, cf, vp, vp, vp]
    lib.cnnk_eval_step.argtypes = [C.POINTER(Layer), ci, C.POINTER(Buffers), vp, vp, vp, vp, vp]
    return lib


lib = _load()


def ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(rc, where):
    if rc != 0:
        raise CnnkError(rc, where)


def status_string(status):
    return lib.cnnk_status_string(int(status)).decode()


def version():
    return lib.cnnk_version().decode()


def cnnk_tune(key, value):
    _check(lib.cnnk_tune(int(key), int(value)), "cnnk_tune")


def conv_desc(N, H, W, Cin, Cout, R, S, stride, pad, dtype):
    return ConvDesc(N, H, W, Cin, Cout, R, S, stride, pad, dtype)


def bn_desc(N, H, W, Cc, dtype, relu, eps=1e-5, momentum=0.1):
    return BnDesc(N, H, W, Cc, dtype, eps, momentum, int(relu))


def pool_desc(N, H, W, Cc, dtype, mode):
    return PoolDesc(N, H, W, Cc, dtype, mode)


def fc_desc(N, F, classes, dtype):
    return FcDesc(N, F, classes, dtype)


def cnnk_conv2d_workspace_bytes(d, pass_):
    return lib.cnnk_conv2d_workspace_bytes(C.byref(d), pass_)


def cnnk_conv2d_fwd(d, x, w, y, ch_sum=None, ch_sumsq=None, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_conv2d_fwd(C.byref(d), ptr(x), ptr(w), ptr(y), ptr(ch_sum), ptr(ch_sumsq), ptr(ws),
                               ws_bytes, stream), "cnnk_conv2d_fwd")


def cnnk_conv2d_dgrad(d, dy, w, dx, accumulate=0, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_conv2d_dgrad(C.byref(d), ptr(dy), ptr(w), ptr(dx), int(accumulate), ptr(ws), ws_bytes,
                                 stream), "cnnk_conv2d_dgrad")


def cnnk_conv2d_wgrad(d, x, dy, dw, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_conv2d_wgrad(C.byref(d), ptr(x), ptr(dy), ptr(dw), ptr(ws), ws_bytes, stream),
           "cnnk_conv2d_wgrad")


def cnnk_bn_workspace_bytes(d):
    return lib.cnnk_bn_workspace_bytes(C.byref(d))


def cnnk_bn_relu_fwd(d, x, residual, gamma, beta, y, save_mean, save_invstd, running_mean=None,
                     running_var=None, ch_sum=None, ch_sumsq=None, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_bn_relu_fwd(C.byref(d), ptr(x), ptr(residual), ptr(gamma), ptr(beta), ptr(y),
                                ptr(save_mean), ptr(save_invstd), ptr(running_mean), ptr(running_var),
                                ptr(ch_sum), ptr(ch_sumsq), ptr(ws), ws_bytes, stream), "cnnk_bn_relu_fwd")


def cnnk_bn_relu_infer(d, x, residual, gamma, beta, running_mean, running_var, y, stream=0):
    _check(lib.cnnk_bn_relu_infer(C.byref(d), ptr(x), ptr(residual), ptr(gamma), ptr(beta), ptr(running_mean),
                                  ptr(running_var), ptr(y), stream), "cnnk_bn_relu_infer")


def cnnk_bn_relu_bwd(d, dy, x, y, gamma, beta, save_mean, save_invstd, dx, dresidual, flags, dgamma, dbeta,
                     ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_bn_relu_bwd(C.byref(d), ptr(dy), ptr(x), ptr(y), ptr(gamma), ptr(beta), ptr(save_mean),
                                ptr(save_invstd), ptr(dx), ptr(dresidual), int(flags), ptr(dgamma),
                                ptr(dbeta), ptr(ws), ws_bytes, stream), "cnnk_bn_relu_bwd")


def cnnk_pool_fwd(d, x, y, argmax=None, stream=0):
    _check(lib.cnnk_pool_fwd(C.byref(d), ptr(x), ptr(y), ptr(argmax), stream), "cnnk_pool_fwd")


def cnnk_pool_bwd(d, dy, argmax, dx, accumulate=0, stream=0):
    _check(lib.cnnk_pool_bwd(C.byref(d), ptr(dy), ptr(argmax), ptr(dx), int(accumulate), stream),
           "cnnk_pool_bwd")


def cnnk_add(n, dtype, a, b, y, stream=0):
    _check(lib.cnnk_add(n, dtype, ptr(a), ptr(b), ptr(y), stream), "cnnk_add")


def cnnk_grad_route(n, dtype, src, dst, accumulate=0, stream=0):
    _check(lib.cnnk_grad_route(n, dtype, ptr(src), ptr(dst), int(accumulate), stream), "cnnk_grad_route")


def cnnk_fc_workspace_bytes(d):
    return lib.cnnk_fc_workspace_bytes(C.byref(d))


def cnnk_fc_softmax_xent(d, x, W, b, labels, loss, pred, probs, dx, dW, db, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_fc_softmax_xent(C.byref(d), ptr(x), ptr(W), ptr(b), ptr(labels), ptr(loss), ptr(pred),
                                    ptr(probs), ptr(dx), ptr(dW), ptr(db), ptr(ws), ws_bytes, stream),
           "cnnk_fc_softmax_xent")


FC_STATIC_SCRATCH_BYTES = 1 << 20


def cnnk_fc_softmax_xent_static(d, x, W, b, labels, loss, pred, probs, dx, dW, db, stream=0):
    _check(lib.cnnk_fc_softmax_xent_static(C.byref(d), ptr(x), ptr(W), ptr(b), ptr(labels), ptr(loss), ptr(pred),
                                           ptr(probs), ptr(dx), ptr(dW), ptr(db), stream),
           "cnnk_fc_softmax_xent_static")


def cnnk_count_correct(n, pred, labels, n_correct, stream=0):
    _check(lib.cnnk_count_correct(int(n), ptr(pred), ptr(labels), ptr(n_correct), stream), "cnnk_count_correct")


def cnnk_sgd_momentum(n, w, v, g, w_bf16, lr, momentum, weight_decay=0.0, stream=0):
    _check(lib.cnnk_sgd_momentum(n, ptr(w), ptr(v), ptr(g), ptr(w_bf16), lr, momentum, weight_decay, stream),
           "cnnk_sgd_momentum")


def cnnk_round_bf16(n, w, w_bf16, stream=0):
    _check(lib.cnnk_round_bf16(n, ptr(w), ptr(w_bf16), stream), "cnnk_round_bf16")


def cnnk_gather_rows(n_rows, n_src_rows, row_bytes, src, idx, dst, bad_index=None, stream=0):
    _check(lib.cnnk_gather_rows(int(n_rows), int(n_src_rows), int(row_bytes), ptr(src), ptr(idx), ptr(dst),
                                ptr(bad_index), stream), "cnnk_gather_rows")


def cnnk_train_step_workspace_bytes(layers, n_layers):
    return lib.cnnk_train_step_workspace_bytes(layers, n_layers)


def cnnk_train_step_event_groups(n_layers):
    return lib.cnnk_train_step_event_groups(n_layers)


def cnnk_train_step(layers, n_layers, buffers, labels, lr, momentum, weight_decay, loss, pred, stream=0):
    _check(lib.cnnk_train_step(layers, n_layers, C.byref(buffers), ptr(labels), lr, momentum, weight_decay,
                               ptr(loss), ptr(pred), stream), "cnnk_train_step")


def cnnk_eval_step(layers, n_layers, buffers, labels, loss, pred, n_correct=None, stream=0):
    _check(lib.cnnk_eval_step(layers, n_layers, C.byref(buffers), ptr(labels), ptr(loss), ptr(pred),
                              ptr(n_correct), stream), "cnnk_eval_step")


# ---- HIP runtime plumbing for callers that time launches with events (no arithmetic here) ----
_hip = None


def _hiprt():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        _hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        _hip.hipEventSynchronize.argtypes = [C.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
    return _hip


def hip_event_create():
    e = C.c_void_p()
    rc = _hiprt().hipEventCreate(C.byref(e))
    if rc != 0:
        raise RuntimeError("hipEventCreate failed: %d" % rc)
    return e.value


def hip_event_record(ev, stream=0):
    rc = _hiprt().hipEventRecord(ev, stream)
    if rc != 0:
        raise RuntimeError("hipEventRecord failed: %d" % rc)


def hip_event_synchronize(ev):
    rc = _hiprt().hipEventSynchronize(ev)
    if rc != 0:
        raise RuntimeError("hipEventSynchronize failed: %d" % rc)


def hip_event_elapsed_ms(start, stop):
    ms = C.c_float()
    rc = _hiprt().hipEventElapsedTime(C.byref(ms), start, stop)
    if rc != 0:
        raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
    return ms.value
