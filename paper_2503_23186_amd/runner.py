"""StepRunner: device buffers (torch tensors) + the C layer list for cnnk_train_step.

The runner only allocates, copies and marshals; every step of the training path runs inside
libcnnk.so.  Layer records are plain dicts:
  conv(x,y,w,N,H,W,Cin,Cout,R,S,stride,pad)  bn(x,res,y,gamma,beta,N,H,W,C,relu)
  pool(x,y,mode,N,H,W,C)  add(a,b,y,N,H,W,C)  fc_loss(x,W,b,N,F,classes)
"""
from __future__ import annotations
import ctypes as C
import numpy as np
import torch
from . import cnnk

BN_EPS = 1e-5
BN_MOMENTUM = 0.1


def _numel(shape):
    n = 1
    for d in shape:
        n *= int(d)
    return n


def build_c_layers(layers, dt):
    """The layer list (dicts of workloads.nets.Net.layers) as the array of cnnk_layer structs that
    cnnk_train_step takes.  Marshalling only; needs no GPU."""
    nl = len(layers)
    arr = (cnnk.Layer * nl)()
    for i, L in enumerate(layers):
        cl = arr[i]
        cl.in0 = cl.in1 = cl.out = cl.p0 = cl.p1 = -1
        op = L["op"]
        if op == "conv":
            cl.op = cnnk.OP_CONV
            cl.in0, cl.out, cl.p0 = L["x"], L["y"], L["w"]
            cl.d.conv = cnnk.conv_desc(L["N"], L["H"], L["W"], L["Cin"], L["Cout"], L["R"], L["S"],
                                       L["stride"], L["pad"], dt)
        elif op == "bn":
            cl.op = cnnk.OP_BN
            cl.in0, cl.in1, cl.out, cl.p0, cl.p1 = L["x"], L["res"], L["y"], L["gamma"], L["beta"]
            cl.d.bn = cnnk.bn_desc(L["N"], L["H"], L["W"], L["C"], dt, L["relu"], BN_EPS, BN_MOMENTUM)
        elif op == "pool":
            cl.op = cnnk.OP_POOL
            cl.in0, cl.out = L["x"], L["y"]
            mode = cnnk.POOL_MAX2 if L["mode"] == "max2" else cnnk.POOL_GAP
            cl.d.pool = cnnk.pool_desc(L["N"], L["H"], L["W"], L["C"], dt, mode)
        elif op == "add":
            cl.op = cnnk.OP_ADD
            cl.in0, cl.in1, cl.out = L["a"], L["b"], L["y"]
            cl.d.pool = cnnk.pool_desc(L["N"], L["H"], L["W"], L["C"], dt, 0)
        elif op == "fc_loss":
            cl.op = cnnk.OP_FC_LOSS
            cl.in0, cl.p0, cl.p1 = L["x"], L["W"], L["b"]
            cl.d.fc = cnnk.fc_desc(L["N"], L["F"], L["classes"], dt)
        else:
            raise ValueError(op)
    return arr


class StepRunner:
    def __init__(self, layers, slot_shapes, param_shapes, dtype, device="cuda:0", keep_probs=True,
                 two_streams=True):
        """dtype: 'f32' or 'bf16' (storage mode of activations and conv weights)."""
        if not torch.cuda.is_available():
            raise RuntimeError("StepRunner needs a GPU: the HIP path has no CPU fallback")
        self.dev = torch.device(device)
        self.bf16 = dtype == "bf16"
        self.dt = cnnk.BF16 if self.bf16 else cnnk.F32
        self.tdt = torch.bfloat16 if self.bf16 else torch.float32
        self.layers = layers
        self.slot_shapes = [tuple(s) for s in slot_shapes]
        self.param_shapes = [tuple(s) for s in param_shapes]
        nl, ns, npar = len(layers), len(slot_shapes), len(param_shapes)
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=self.dev)
        self.act = [z(s, self.tdt) for s in self.slot_shapes]
        self.dact = [None] + [z(s, self.tdt) for s in self.slot_shapes[1:]]
        self.param = [z(s, torch.float32) for s in self.param_shapes]
        self.grad = [z(s, torch.float32) for s in self.param_shapes]
        self.mom = [z(s, torch.float32) for s in self.param_shapes]
        conv_params = {L["w"] for L in layers if L["op"] == "conv"}
        self.param_lp = [z(s, torch.bfloat16) if (self.bf16 and k in conv_params) else None
                         for k, s in enumerate(self.param_shapes)]
        self.bn_save = [None] * nl
        self.bn_running = [None] * nl
        self.pool_idx = [None] * nl
        self.c_layers = build_c_layers(layers, self.dt)
        self.N = self.slot_shapes[0][0]
        self.classes = None
        for i, L in enumerate(layers):
            if L["op"] == "bn":
                self.bn_save[i] = z((2, L["C"]), torch.float32)
                run = z((2, L["C"]), torch.float32)
                run[1].fill_(1.0)
                self.bn_running[i] = run
            elif L["op"] == "pool" and L["mode"] == "max2":
                self.pool_idx[i] = z((L["N"], L["H"] // 2, L["W"] // 2, L["C"]), torch.uint8)
            elif L["op"] == "fc_loss":
                self.classes = L["classes"]
        self.labels = z((self.N,), torch.int32)
        self.loss = z((1,), torch.float32)
        self.pred = z((self.N,), torch.int32)
        self.probs = z((self.N, self.classes), torch.float32) if keep_probs else None
        self.ws_bytes = int(cnnk.cnnk_train_step_workspace_bytes(self.c_layers, nl))
        self.ws = torch.empty(max(self.ws_bytes, 256) * (2 if two_streams else 1), dtype=torch.uint8,
                              device=self.dev)

        def parr(ts):
            a = (C.c_void_p * len(ts))()
            for k, t in enumerate(ts):
                a[k] = None if t is None else t.data_ptr()
            return a

        self._arrs = dict(act=parr(self.act), dact=parr(self.dact), param=parr(self.param),
                          param_lp=parr(self.param_lp), grad=parr(self.grad), mom=parr(self.mom),
                          bn_save=parr(self.bn_save), bn_running=parr(self.bn_running),
                          pool_idx=parr(self.pool_idx))
        b = cnnk.Buffers()
        b.n_slots, b.n_params = ns, npar
        for k, a in self._arrs.items():
            setattr(b, k, C.cast(a, C.POINTER(C.c_void_p)))
        b.probs = None if self.probs is None else self.probs.data_ptr()
        b.ws = self.ws.data_ptr()
        b.ws_bytes = self.ws.numel()
        b.events = None
        b.n_events = 0
        # second stream (default priority) + two events for the weight gradients
        self.aux_stream = torch.cuda.Stream(device=self.dev) if two_streams else None
        b.aux_stream = self.aux_stream.cuda_stream if two_streams else None
        b.ev_fork = cnnk.hip_event_create() if two_streams else None
        b.ev_join = cnnk.hip_event_create() if two_streams else None
        self.buffers = b
        self._events = None

    # -- host <-> device copies (not part of the timed path) -------------------------------
    def load(self, x, labels, params, mom):
        self.act[0].copy_(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.dev))
        self.labels.copy_(torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(self.dev))
        for k, (p, v) in enumerate(zip(params, mom)):
            self.param[k].copy_(torch.from_numpy(np.ascontiguousarray(p, dtype=np.float32)).to(self.dev))
            self.mom[k].copy_(torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(self.dev))
        self.refresh_low_precision()
        torch.cuda.synchronize()

    def refresh_low_precision(self):
        """bf16 copies of the convolution weights from the fp32 masters (the step's update kernel
        keeps them current afterwards)."""
        s = torch.cuda.current_stream().cuda_stream
        for k, lp in enumerate(self.param_lp):
            if lp is not None:
                cnnk.cnnk_round_bf16(lp.numel(), self.param[k], lp, s)

    def step(self, lr=0.1, momentum=0.9, weight_decay=0.0, stream=None):
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        cnnk.cnnk_train_step(self.c_layers, len(self.layers), self.buffers, self.labels, lr, momentum,
                             weight_decay, self.loss, self.pred, s)

    def enable_timing(self, on=True):
        """Have cnnk_train_step record a HIP event pair around each of its entry-point calls."""
        if on and self._events is None:
            n = 2 * cnnk.cnnk_train_step_event_groups(len(self.layers))
            self._events = (C.c_void_p * n)(*[cnnk.hip_event_create() for _ in range(n)])
        self.buffers.events = C.cast(self._events, C.POINTER(C.c_void_p)) if on else None
        self.buffers.n_events = len(self._events) if on else 0

    def group_times_ms(self):
        """Elapsed time of every group of the last timed step (call after a synchronise)."""
        ev = self._events
        return [cnnk.hip_event_elapsed_ms(ev[2 * g], ev[2 * g + 1]) for g in range(len(ev) // 2)]

    def group_table(self):
        """(group index, layer index, phase) in the order documented in cnnk.h."""
        n = len(self.layers)
        rows = [(i, i, "fwd") for i in range(n)]
        for i in range(n - 2, -1, -1):
            g0 = n + 2 * (n - 2 - i)
            conv = self.layers[i]["op"] == "conv"
            rows.append((g0, i, "wgrad" if conv else "bwd"))
            rows.append((g0 + 1, i, "dgrad" if conv else "none"))
        rows.append((3 * n - 2, -1, "update"))
        return rows

    @staticmethod
    def host(t):
        return None if t is None else t.detach().to("cpu").to(torch.float64).numpy()
