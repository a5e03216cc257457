"""Binding of include/cnnk_vit.h (argument marshalling only) and VitRunner: device buffers for
cnnk_vit_train_step.  Every step of the path runs inside libcnnk.so; torch provides device memory
and the stream handle.  There is no CPU fallback."""
from __future__ import annotations
import ctypes as C
import numpy as np
import torch
from . import cnnk
from .cnnk import lib, ptr, _check, F32, BF16

EXPORTS = ["cnnk_linear_workspace_bytes", "cnnk_linear_fwd", "cnnk_linear_dgrad", "cnnk_linear_wgrad", "cnnk_layernorm_fwd", "cnnk_layernorm_workspace_bytes", "cnnk_layernorm_bwd", "cnnk_bias_act_fwd",
           "cnnk_bias_act_workspace_bytes", "cnnk_bias_act_bwd", "cnnk_attention_fwd", "cnnk_attention_bwd",
           "cnnk_vit_patchify", "cnnk_vit_embed_fwd", "cnnk_vit_embed_bwd", "cnnk_vit_arena_bytes",
           "cnnk_vit_workspace_bytes", "cnnk_vit_tensor", "cnnk_vit_step_calls", "cnnk_vit_step_call_name",
           "cnnk_vit_train_step", "cnnk_vit_eval_step"]

ACT_NONE, ACT_GELU = 0, 1
TENSOR_IDS = ["PATCHES", "TOK", "H", "QKV", "O", "XMID", "H2", "U", "G", "XOUT", "F",
              "DTOK", "DH", "DQKV", "DO", "DXMID", "DH2", "DU", "DG", "DXOUT", "DF"]
BLOCK_PARAMS = ("g1", "b1", "Wqkv", "bqkv", "Wo", "bo", "g2", "b2", "W1", "c1", "W2", "c2")


class LnDesc(C.Structure):
    _fields_ = [("rows", C.c_int), ("C", C.c_int), ("dtype", C.c_int), ("eps", C.c_float), ("x_stride", C.c_longlong)]


class AttnDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("B", "T", "heads", "dh", "dtype")]


class EmbedDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("B", "image", "patch", "dim", "dtype")]


class VitDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("B", "image", "patch", "dim", "heads", "layers", "mlp", "classes", "dtype")] + \
               [("ln_eps", C.c_float)]


class VitBuffers(C.Structure):
    _fields_ = [("n_params", C.c_int), ("param", C.POINTER(C.c_void_p)), ("param_lp", C.POINTER(C.c_void_p)),
                ("grad", C.POINTER(C.c_void_p)), ("mom", C.POINTER(C.c_void_p)), ("x", C.c_void_p),
                ("labels", C.c_void_p), ("loss", C.c_void_p), ("pred", C.c_void_p), ("probs", C.c_void_p),
                ("arena", C.c_void_p), ("arena_bytes", C.c_size_t), ("ws", C.c_void_p), ("ws_bytes", C.c_size_t),
                ("events", C.POINTER(C.c_void_p)), ("n_events", C.c_int),
                ("aux_stream", C.c_void_p), ("ev_fork", C.c_void_p), ("ev_join", C.c_void_p)]


def _declare():
    vp, ci, cf, sz, ll = C.c_void_p, C.c_int, C.c_float, C.c_size_t, C.c_longlong
    lib.cnnk_layernorm_fwd.argtypes = [C.POINTER(LnDesc), vp, vp, vp, vp, vp, vp]
    lib.cnnk_layernorm_workspace_bytes.restype = sz
    lib.cnnk_layernorm_workspace_bytes.argtypes = [C.POINTER(LnDesc)]
    lib.cnnk_layernorm_bwd.argtypes = [C.POINTER(LnDesc)] + [vp] * 8 + [vp, sz, vp]
    lib.cnnk_bias_act_fwd.argtypes = [ll, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.cnnk_bias_act_workspace_bytes.restype = sz
    lib.cnnk_bias_act_workspace_bytes.argtypes = [ll, ci]
    lib.cnnk_bias_act_bwd.argtypes = [ll, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.cnnk_linear_workspace_bytes.restype = sz
    lib.cnnk_linear_workspace_bytes.argtypes = [ll, ci, ci, ci]
    lib.cnnk_linear_fwd.argtypes = [ll, ci, ci, ci, vp, vp, vp, vp, ci, vp, vp, vp, sz, vp]
    lib.cnnk_linear_dgrad.argtypes = [ll, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.cnnk_linear_wgrad.argtypes = [ll, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.cnnk_attention_fwd.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp]
    lib.cnnk_attention_bwd.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp]
    lib.cnnk_vit_patchify.argtypes = [C.POINTER(EmbedDesc), vp, vp, vp]
    lib.cnnk_vit_embed_fwd.argtypes = [C.POINTER(EmbedDesc), vp, vp, vp, vp, vp, vp]
    lib.cnnk_vit_embed_bwd.argtypes = [C.POINTER(EmbedDesc), vp, vp, vp, vp, vp, vp]
    lib.cnnk_vit_arena_bytes.restype = sz
    lib.cnnk_vit_arena_bytes.argtypes = [C.POINTER(VitDesc)]
    lib.cnnk_vit_workspace_bytes.restype = sz
    lib.cnnk_vit_workspace_bytes.argtypes = [C.POINTER(VitDesc)]
    lib.cnnk_vit_tensor.argtypes = [C.POINTER(VitDesc), ci, ci, C.POINTER(sz), C.POINTER(sz)]
    lib.cnnk_vit_step_calls.argtypes = [C.POINTER(VitDesc)]
    lib.cnnk_vit_step_call_name.argtypes = [C.POINTER(VitDesc), ci, C.c_char_p, ci]
    lib.cnnk_vit_train_step.argtypes = [C.POINTER(VitDesc), C.POINTER(VitBuffers), cf, cf, cf, vp]
    lib.cnnk_vit_eval_step.argtypes = [C.POINTER(VitDesc), C.POINTER(VitBuffers), vp, vp]


_declare()


def ln_desc(rows, Cc, dtype, eps=1e-6, x_stride=0):
    return LnDesc(rows, Cc, dtype, eps, x_stride)


def cnnk_layernorm_fwd(d, x, gamma, beta, y, stats, stream=0):
    _check(lib.cnnk_layernorm_fwd(C.byref(d), ptr(x), ptr(gamma), ptr(beta), ptr(y), ptr(stats), stream), "cnnk_layernorm_fwd")


def cnnk_layernorm_workspace_bytes(d):
    return int(lib.cnnk_layernorm_workspace_bytes(C.byref(d)))


def cnnk_layernorm_bwd(d, dy, x, gamma, stats, dres, dx, dgamma, dbeta, ws, ws_bytes, stream=0):
    _check(lib.cnnk_layernorm_bwd(C.byref(d), ptr(dy), ptr(x), ptr(gamma), ptr(stats), ptr(dres), ptr(dx), ptr(dgamma),
                                  ptr(dbeta), ptr(ws), ws_bytes, stream), "cnnk_layernorm_bwd")


def cnnk_bias_act_fwd(rows, Cc, dtype, act, z, bias, res, u, y, stream=0):
    _check(lib.cnnk_bias_act_fwd(rows, Cc, dtype, act, ptr(z), ptr(bias), ptr(res), ptr(u), ptr(y), stream), "cnnk_bias_act_fwd")


def cnnk_bias_act_workspace_bytes(rows, Cc):
    return int(lib.cnnk_bias_act_workspace_bytes(rows, Cc))


def cnnk_bias_act_bwd(rows, Cc, dtype, act, dy, u, dz, dbias, ws, ws_bytes, stream=0):
    _check(lib.cnnk_bias_act_bwd(rows, Cc, dtype, act, ptr(dy), ptr(u), ptr(dz), ptr(dbias), ptr(ws), ws_bytes, stream),
           "cnnk_bias_act_bwd")


def cnnk_linear_workspace_bytes(rows, K, N, dtype):
    return int(lib.cnnk_linear_workspace_bytes(rows, K, N, dtype))


def cnnk_linear_fwd(rows, K, N, dtype, x, w, bias, act, u, y, ws=None, ws_bytes=0, stream=0, res=None):
    _check(lib.cnnk_linear_fwd(rows, K, N, dtype, ptr(x), ptr(w), ptr(bias), ptr(res), act, ptr(u), ptr(y), ptr(ws), ws_bytes, stream),
           "cnnk_linear_fwd")


def cnnk_linear_dgrad(rows, K, N, dtype, dy, w, dx, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_linear_dgrad(rows, K, N, dtype, ptr(dy), ptr(w), ptr(dx), ptr(ws), ws_bytes, stream), "cnnk_linear_dgrad")


def cnnk_linear_wgrad(rows, K, N, dtype, x, dy, dw, ws=None, ws_bytes=0, stream=0):
    _check(lib.cnnk_linear_wgrad(rows, K, N, dtype, ptr(x), ptr(dy), ptr(dw), ptr(ws), ws_bytes, stream), "cnnk_linear_wgrad")


def attn_desc(B, T, heads, dh, dtype):
    return AttnDesc(B, T, heads, dh, dtype)


def cnnk_attention_fwd(d, qkv, o, lse, stream=0):
    _check(lib.cnnk_attention_fwd(C.byref(d), ptr(qkv), ptr(o), ptr(lse), stream), "cnnk_attention_fwd")


def cnnk_attention_bwd(d, qkv, o, d_o, lse, dqkv, stream=0):
    _check(lib.cnnk_attention_bwd(C.byref(d), ptr(qkv), ptr(o), ptr(d_o), ptr(lse), ptr(dqkv), stream), "cnnk_attention_bwd")


def embed_desc(B, image, patch, dim, dtype):
    return EmbedDesc(B, image, patch, dim, dtype)


def cnnk_vit_patchify(d, x, patches, stream=0):
    _check(lib.cnnk_vit_patchify(C.byref(d), ptr(x), ptr(patches), stream), "cnnk_vit_patchify")


def cnnk_vit_embed_fwd(d, z, be, cls, pos, tok, stream=0):
    _check(lib.cnnk_vit_embed_fwd(C.byref(d), ptr(z), ptr(be), ptr(cls), ptr(pos), ptr(tok), stream), "cnnk_vit_embed_fwd")


def cnnk_vit_embed_bwd(d, dtok, dz, dbe, dcls, dpos, stream=0):
    _check(lib.cnnk_vit_embed_bwd(C.byref(d), ptr(dtok), ptr(dz), ptr(dbe), ptr(dcls), ptr(dpos), stream), "cnnk_vit_embed_bwd")


def vit_desc(B, image, patch, dim, heads, layers, mlp, classes, dtype, ln_eps=1e-6):
    return VitDesc(B, image, patch, dim, heads, layers, mlp, classes, dtype, ln_eps)


def cnnk_vit_arena_bytes(d):
    return int(lib.cnnk_vit_arena_bytes(C.byref(d)))


def cnnk_vit_workspace_bytes(d):
    return int(lib.cnnk_vit_workspace_bytes(C.byref(d)))


def cnnk_vit_tensor(d, tensor_id, layer=0):
    off, nb = C.c_size_t(0), C.c_size_t(0)
    _check(lib.cnnk_vit_tensor(C.byref(d), tensor_id, layer, C.byref(off), C.byref(nb)), "cnnk_vit_tensor")
    return int(off.value), int(nb.value)


def cnnk_vit_step_calls(d):
    return int(lib.cnnk_vit_step_calls(C.byref(d)))


def cnnk_vit_step_call_name(d, i):
    buf = C.create_string_buffer(64)
    _check(lib.cnnk_vit_step_call_name(C.byref(d), i, buf, 64), "cnnk_vit_step_call_name")
    return buf.value.decode()


def cnnk_vit_train_step(d, buffers, lr, momentum, weight_decay, stream=0):
    _check(lib.cnnk_vit_train_step(C.byref(d), C.byref(buffers), lr, momentum, weight_decay, stream), "cnnk_vit_train_step")


def cnnk_vit_eval_step(d, buffers, n_correct=None, stream=0):
    _check(lib.cnnk_vit_eval_step(C.byref(d), C.byref(buffers), ptr(n_correct), stream), "cnnk_vit_eval_step")


def param_names(layers):
    names = ["We", "be", "cls", "pos"]
    for l in range(layers):
        names += ["%s.%d" % (n, l) for n in BLOCK_PARAMS]
    return names + ["gf", "bf", "Wh", "bh"]


class VitRunner:
    """Device buffers of one ViT training step.  net: a workloads.ViT-style description (batch, image,
    patch, dim, heads, layers, mlp, classes, dtype, param_table())."""

    def __init__(self, net, device="cuda:0", keep_probs=True, two_streams=True):
        self.net = net
        self.dev = torch.device(device)
        self.dt = BF16 if net.dtype == "bf16" else F32
        self.tdt = torch.bfloat16 if net.dtype == "bf16" else torch.float32
        self.desc = vit_desc(net.batch, net.image, net.patch, net.dim, net.heads, net.layers, net.mlp, net.classes, self.dt)
        table = net.param_table()
        self.names = [n for n, _, _ in table]
        assert self.names == param_names(net.layers)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.param = [torch.zeros(s, **f32) for _, s, _ in table]
        self.grad = [torch.zeros(s, **f32) for _, s, _ in table]
        self.mom = [torch.zeros(s, **f32) for _, s, _ in table]
        self.param_lp = [torch.zeros(s, dtype=torch.bfloat16, device=self.dev) if (k == "w" and net.dtype == "bf16") else None
                         for _, s, k in table]
        self.x = torch.zeros((net.batch, net.image, net.image, 3), dtype=self.tdt, device=self.dev)
        self.labels = torch.zeros(net.batch, dtype=torch.int32, device=self.dev)
        self.loss = torch.zeros(1, **f32)
        self.pred = torch.zeros(net.batch, dtype=torch.int32, device=self.dev)
        self.probs = torch.zeros((net.batch, net.classes), **f32) if keep_probs else None
        self.arena_bytes = cnnk_vit_arena_bytes(self.desc)
        self.ws_bytes = cnnk_vit_workspace_bytes(self.desc)
        if self.arena_bytes == 0:
            raise ValueError("unsupported ViT configuration")
        self.arena = torch.zeros(self.arena_bytes, dtype=torch.uint8, device=self.dev)
        self.ws = torch.zeros(max(self.ws_bytes, 256) * (2 if two_streams else 1), dtype=torch.uint8, device=self.dev)
        self.aux_stream = torch.cuda.Stream(device=self.dev) if two_streams else None
        n = len(table)
        arr = lambda ts: (C.c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])
        self._keep = [arr(self.param), arr(self.param_lp), arr(self.grad), arr(self.mom)]
        cast = lambda a: C.cast(a, C.POINTER(C.c_void_p))
        self.buffers = VitBuffers(n, cast(self._keep[0]), cast(self._keep[1]), cast(self._keep[2]), cast(self._keep[3]),
                                  self.x.data_ptr(), self.labels.data_ptr(), self.loss.data_ptr(), self.pred.data_ptr(),
                                  None if self.probs is None else self.probs.data_ptr(), self.arena.data_ptr(),
                                  self.arena_bytes, self.ws.data_ptr(), self.ws.numel(), None, 0,
                                  self.aux_stream.cuda_stream if two_streams else None,
                                  cnnk.hip_event_create() if two_streams else None,
                                  cnnk.hip_event_create() if two_streams else None)
        self.n_calls = cnnk_vit_step_calls(self.desc)
        self.call_names = [cnnk_vit_step_call_name(self.desc, i) for i in range(self.n_calls)]
        self._events = None

    # -- data in ------------------------------------------------------------------------------------
    def load(self, x, labels, params, mom):
        """Host arrays: x [B, H, W, 3], labels [B], params / mom {name: array}."""
        self.x.copy_(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.dev).to(self.tdt))
        self.labels.copy_(torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)))
        for k, name in enumerate(self.names):
            self.param[k].copy_(torch.from_numpy(np.ascontiguousarray(params[name], dtype=np.float32)))
            self.mom[k].copy_(torch.from_numpy(np.ascontiguousarray(mom[name], dtype=np.float32)))
        self.refresh_low_precision()
        torch.cuda.synchronize()

    def refresh_low_precision(self):
        s = torch.cuda.current_stream().cuda_stream
        for p, lp in zip(self.param, self.param_lp):
            if lp is not None:
                cnnk.cnnk_round_bf16(p.numel(), p, lp, s)

    # -- the step -------------------------------------------------------------------------------------
    def step(self, lr, momentum, weight_decay=0.0):
        cnnk_vit_train_step(self.desc, self.buffers, lr, momentum, weight_decay, torch.cuda.current_stream().cuda_stream)

    def enable_timing(self, on=True):
        if on and self._events is None:
            evs = [cnnk.hip_event_create() for _ in range(2 * self.n_calls)]
            self._events = evs
            self._ev_arr = (C.c_void_p * len(evs))(*evs)
        if on:
            self.buffers.events = C.cast(self._ev_arr, C.POINTER(C.c_void_p))
            self.buffers.n_events = 2 * self.n_calls
        else:
            self.buffers.events = None
            self.buffers.n_events = 0

    def call_times_ms(self):
        """Per-call times of the last timed step (after a device synchronisation)."""
        return [cnnk.hip_event_elapsed_ms(self._events[2 * i], self._events[2 * i + 1]) for i in range(self.n_calls)]

    # -- data out -----------------------------------------------------------------------------------
    def tensor(self, name, layer=0):
        """A view of an arena tensor (TENSOR_IDS) as a torch tensor of the storage dtype, flat."""
        off, nb = cnnk_vit_tensor(self.desc, TENSOR_IDS.index(name), layer)
        return self.arena[off:off + nb].view(self.tdt)
