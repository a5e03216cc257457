"""Trainer: the single-device epoch loop of the paper's Algorithm 1 around cnnk_train_step.

Per epoch: one cnnk_train_step per mini-batch (forward, loss, backward, update), then the
validation metric with cnnk_eval_step (inference-mode batch norm) and "save checkpoint if the
validation metric improved".  Every multi-device line of the algorithm (distribute, synchronise
gradients, choose a strategy) has nothing to do on one device; `profile()` returns the measured
per-layer execution times that the algorithm's scheduler takes as t_comp.

Host logic only: the learning-rate schedules, the sample order, batching out of a device-resident
data set (a gather into the step's input buffer), the checkpoint file.  All arithmetic of the
training path runs inside libcnnk.so; there is no CPU fallback.

Checkpoint = one safetensors file: fp32 master parameters, momentum buffers, BN running
statistics, and the counters (epoch, step, best accuracy) as metadata strings.  Restoring it and
continuing gives bit-identical results to never having stopped.
"""
from __future__ import annotations
import math
import numpy as np
import torch
from safetensors.torch import save_file, safe_open

from . import cnnk
from .runner import StepRunner


# ---- learning-rate schedules: one value per step -------------------------------------------------
def constant_lr(base, total_steps):
    return [float(base)] * int(total_steps)


def step_lr(base, steps_per_epoch, epochs, milestones, gamma=0.1):
    """base * gamma^(number of milestones <= epoch), constant within an epoch."""
    out = []
    for e in range(int(epochs)):
        k = sum(1 for m in milestones if e >= m)
        out += [float(base) * float(gamma) ** k] * int(steps_per_epoch)
    return out


def cosine_lr(base, total_steps, warmup_steps=0, floor=0.0):
    """Linear warm-up from base/warmup_steps to base, then half a cosine down to `floor`."""
    out = []
    for k in range(int(total_steps)):
        if k < warmup_steps:
            out.append(float(base) * (k + 1) / warmup_steps)
        else:
            t = (k - warmup_steps) / max(1, total_steps - warmup_steps)
            out.append(float(floor) + 0.5 * (float(base) - float(floor)) * (1.0 + math.cos(math.pi * t)))
    return out


# ---- checkpoint file (CPU tensors in, CPU tensors out) -------------------------------------------
def write_checkpoint(path, tensors, meta):
    """tensors: {name: CPU tensor}; meta: {name: int | float | str} stored as strings."""
    save_file({k: v.contiguous() for k, v in tensors.items()}, path,
              metadata={k: repr(v) if isinstance(v, float) else str(v) for k, v in meta.items()})


def read_checkpoint(path):
    with safe_open(path, framework="pt", device="cpu") as f:
        meta = dict(f.metadata() or {})
        tensors = {k: f.get_tensor(k) for k in f.keys()}
    return tensors, meta


class Trainer:
    def __init__(self, net, device="cuda:0", two_streams=True):
        """net: a workloads-style description with .layers, .slots, .params, .dtype, .name."""
        self.net = net
        self.run = StepRunner(net.layers, net.slots, [p["shape"] for p in net.params], net.dtype, device=device,
                              keep_probs=False, two_streams=two_streams)
        self.batch = self.run.N
        self.n_correct = torch.zeros(1, dtype=torch.int32, device=self.run.dev)
        self.bad_index = torch.zeros(1, dtype=torch.int32, device=self.run.dev)   # set by a batch gather
        self.epoch = 0          # epochs completed
        self.step = 0           # steps completed
        self.best_acc = -1.0
        self.best_epoch = -1

    # -- state ------------------------------------------------------------------------------------
    def load_state(self, params, mom):
        """Initial parameters and momentum buffers (host arrays); running statistics start at (0, 1)."""
        r = self.run
        for k, (p, v) in enumerate(zip(params, mom)):
            r.param[k].copy_(torch.from_numpy(np.ascontiguousarray(p, dtype=np.float32)))
            r.mom[k].copy_(torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)))
        self._refresh_low_precision()
        for run in r.bn_running:
            if run is not None:
                run[0].zero_()
                run[1].fill_(1.0)
        torch.cuda.synchronize()

    def _refresh_low_precision(self):
        self.run.refresh_low_precision()

    def to_device(self, x, y):
        """A host data set (float NHWC, int labels) as device tensors of the storage dtype."""
        r = self.run
        xt = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(r.dev).to(r.tdt).contiguous()
        yt = torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(r.dev)
        return xt, yt

    # -- one mini-batch / one validation pass ---------------------------------------------------------
    def train_batch(self, x_all, y_all, idx, lr, momentum, weight_decay):
        r = self.run
        s = torch.cuda.current_stream().cuda_stream
        row_bytes = x_all[0].numel() * x_all.element_size()
        cnnk.cnnk_gather_rows(self.batch, x_all.shape[0], row_bytes, x_all, idx, r.act[0], self.bad_index, s)
        cnnk.cnnk_gather_rows(self.batch, y_all.shape[0], 4, y_all, idx, r.labels, self.bad_index, s)
        r.step(lr, momentum, weight_decay)
        self.step += 1

    def evaluate(self, x_all, y_all):
        """Inference-mode pass over x_all in batches.  Returns (accuracy, mean loss over batches)."""
        r = self.run
        n = x_all.shape[0]
        if n % self.batch:
            raise ValueError("validation set size must be a multiple of the batch size")
        self.n_correct.zero_()
        losses = torch.empty(n // self.batch, dtype=torch.float32, device=r.dev)
        s = torch.cuda.current_stream().cuda_stream
        for b in range(n // self.batch):
            r.act[0].copy_(x_all[b * self.batch:(b + 1) * self.batch])
            r.labels.copy_(y_all[b * self.batch:(b + 1) * self.batch])
            cnnk.cnnk_eval_step(r.c_layers, len(r.layers), r.buffers, r.labels, losses[b:b + 1], r.pred,
                                self.n_correct, s)
        torch.cuda.synchronize()
        return self.n_correct.item() / n, float(losses.double().mean().item())

    # -- the epoch loop ---------------------------------------------------------------------------------
    def fit(self, train_x, train_y, val_x, val_y, orders, lrs, momentum=0.9, weight_decay=0.0, ckpt_path=None):
        """orders: one index array per epoch still to run (whole mini-batches); lrs: the learning rate
        of every step, indexed by the global step counter (so a resumed run passes the same list).
        Returns [(mean train loss, validation accuracy, validation loss)] per epoch run."""
        r = self.run
        history = []
        for order in orders:
            idx_all = torch.from_numpy(np.ascontiguousarray(order, dtype=np.int64)).to(r.dev)
            nb = idx_all.numel() // self.batch
            if nb * self.batch != idx_all.numel():
                raise ValueError("an epoch's order must hold whole mini-batches")
            losses = torch.empty(nb, dtype=torch.float32, device=r.dev)
            for b in range(nb):
                self.train_batch(train_x, train_y, idx_all[b * self.batch:(b + 1) * self.batch], lrs[self.step],
                                 momentum, weight_decay)
                losses[b:b + 1].copy_(r.loss)
            if self.bad_index.item() != 0:
                raise ValueError("an epoch's order names a sample outside the training set")
            acc, vloss = self.evaluate(val_x, val_y)
            history.append((float(losses.double().mean().item()), acc, vloss))
            self.epoch += 1
            if acc > self.best_acc:
                self.best_acc, self.best_epoch = acc, self.epoch - 1
                if ckpt_path is not None:
                    self.save_checkpoint(ckpt_path)
        return history

    # -- checkpoint ---------------------------------------------------------------------------------------
    def save_checkpoint(self, path):
        r = self.run
        torch.cuda.synchronize()
        t = {}
        for k in range(len(r.param)):
            t["param.%d" % k] = r.param[k].cpu()
            t["mom.%d" % k] = r.mom[k].cpu()
        for i, run in enumerate(r.bn_running):
            if run is not None:
                t["bn_running.%d" % i] = run.cpu()
        write_checkpoint(path, t, dict(net=self.net.name, dtype=self.net.dtype, epoch=self.epoch, step=self.step,
                                       best_acc=float(self.best_acc), best_epoch=self.best_epoch))

    def load_checkpoint(self, path):
        r = self.run
        t, meta = read_checkpoint(path)
        if meta.get("net") != self.net.name or meta.get("dtype") != self.net.dtype:
            raise ValueError("checkpoint is for %s/%s" % (meta.get("net"), meta.get("dtype")))
        for k in range(len(r.param)):
            if tuple(t["param.%d" % k].shape) != tuple(r.param[k].shape):
                raise ValueError("checkpoint parameter %d has shape %s" % (k, tuple(t["param.%d" % k].shape)))
        for k in range(len(r.param)):
            r.param[k].copy_(t["param.%d" % k])
            r.mom[k].copy_(t["mom.%d" % k])
        for i, run in enumerate(r.bn_running):
            if run is not None:
                run.copy_(t["bn_running.%d" % i])
        self._refresh_low_precision()
        self.epoch, self.step = int(meta["epoch"]), int(meta["step"])
        self.best_acc, self.best_epoch = float(meta["best_acc"]), int(meta["best_epoch"])
        torch.cuda.synchronize()

    # -- per-layer execution times (the scheduler's t_comp) ------------------------------------------------
    def profile(self, steps=3):
        """Median per-call times (ms) of `steps` timed steps on whatever batch the input buffer holds,
        as [(layer index, phase, ms)].  The steps run with a zero learning rate, and the momentum
        buffers and running statistics are put back afterwards, so the training state is unchanged."""
        r = self.run
        keep_mom = [v.clone() for v in r.mom]
        keep_run = [None if t is None else t.clone() for t in r.bn_running]
        r.enable_timing(True)
        rows = r.group_table()
        acc = []
        for _ in range(steps):
            r.step(0.0, 0.0, 0.0)
            torch.cuda.synchronize()
            acc.append(r.group_times_ms())
        r.enable_timing(False)
        for v, k in zip(r.mom, keep_mom):
            v.copy_(k)
        for t, k in zip(r.bn_running, keep_run):
            if t is not None:
                t.copy_(k)
        torch.cuda.synchronize()
        med = np.median(np.asarray(acc), axis=0)
        return [(layer, phase, float(med[g])) for g, layer, phase in rows]


class VitTrainer:
    """The same epoch loop around cnnk_vit_train_step (the paper's second model family): one step per
    mini-batch, cnnk_vit_eval_step over the validation set, best-so-far checkpoint (fp32 masters,
    momentum buffers, counters).  net: a workloads.ViT-style description."""

    def __init__(self, net, device="cuda:0", two_streams=True):
        from .vit import VitRunner
        self.net = net
        self.run = VitRunner(net, device=device, keep_probs=False, two_streams=two_streams)
        self.batch = net.batch
        self.n_correct = torch.zeros(1, dtype=torch.int32, device=self.run.dev)
        self.bad_index = torch.zeros(1, dtype=torch.int32, device=self.run.dev)
        self.epoch = 0
        self.step = 0
        self.best_acc = -1.0
        self.best_epoch = -1

    def load_state(self, params, mom):
        """params / mom: {name: host array} in the names of VitRunner.names."""
        r = self.run
        for k, name in enumerate(r.names):
            r.param[k].copy_(torch.from_numpy(np.ascontiguousarray(params[name], dtype=np.float32)))
            r.mom[k].copy_(torch.from_numpy(np.ascontiguousarray(mom[name], dtype=np.float32)))
        r.refresh_low_precision()
        torch.cuda.synchronize()

    def to_device(self, x, y):
        r = self.run
        xt = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(r.dev).to(r.tdt).contiguous()
        yt = torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(r.dev)
        return xt, yt

    def train_batch(self, x_all, y_all, idx, lr, momentum, weight_decay):
        r = self.run
        s = torch.cuda.current_stream().cuda_stream
        row_bytes = x_all[0].numel() * x_all.element_size()
        cnnk.cnnk_gather_rows(self.batch, x_all.shape[0], row_bytes, x_all, idx, r.x, self.bad_index, s)
        cnnk.cnnk_gather_rows(self.batch, y_all.shape[0], 4, y_all, idx, r.labels, self.bad_index, s)
        r.step(lr, momentum, weight_decay)
        self.step += 1

    def evaluate(self, x_all, y_all):
        from .vit import cnnk_vit_eval_step
        r = self.run
        n = x_all.shape[0]
        if n % self.batch:
            raise ValueError("validation set size must be a multiple of the batch size")
        self.n_correct.zero_()
        losses = torch.empty(n // self.batch, dtype=torch.float32, device=r.dev)
        s = torch.cuda.current_stream().cuda_stream
        for b in range(n // self.batch):
            r.x.copy_(x_all[b * self.batch:(b + 1) * self.batch])
            r.labels.copy_(y_all[b * self.batch:(b + 1) * self.batch])
            cnnk_vit_eval_step(r.desc, r.buffers, self.n_correct, s)
            losses[b:b + 1].copy_(r.loss)
        torch.cuda.synchronize()
        return self.n_correct.item() / n, float(losses.double().mean().item())

    def fit(self, train_x, train_y, val_x, val_y, orders, lrs, momentum=0.9, weight_decay=0.0, ckpt_path=None):
        r = self.run
        history = []
        for order in orders:
            idx_all = torch.from_numpy(np.ascontiguousarray(order, dtype=np.int64)).to(r.dev)
            nb = idx_all.numel() // self.batch
            if nb * self.batch != idx_all.numel():
                raise ValueError("an epoch's order must hold whole mini-batches")
            losses = torch.empty(nb, dtype=torch.float32, device=r.dev)
            for b in range(nb):
                self.train_batch(train_x, train_y, idx_all[b * self.batch:(b + 1) * self.batch], lrs[self.step], momentum,
                                 weight_decay)
                losses[b:b + 1].copy_(r.loss)
            if self.bad_index.item() != 0:
                raise ValueError("an epoch's order names a sample outside the training set")
            acc, vloss = self.evaluate(val_x, val_y)
            history.append((float(losses.double().mean().item()), acc, vloss))
            self.epoch += 1
            if acc > self.best_acc:
                self.best_acc, self.best_epoch = acc, self.epoch - 1
                if ckpt_path is not None:
                    self.save_checkpoint(ckpt_path)
        return history

    def save_checkpoint(self, path):
        r = self.run
        torch.cuda.synchronize()
        t = {}
        for k, name in enumerate(r.names):
            t["param." + name] = r.param[k].cpu()
            t["mom." + name] = r.mom[k].cpu()
        write_checkpoint(path, t, dict(net=self.net.name, dtype=self.net.dtype, epoch=self.epoch, step=self.step,
                                       best_acc=float(self.best_acc), best_epoch=self.best_epoch))

    def load_checkpoint(self, path):
        r = self.run
        t, meta = read_checkpoint(path)
        if meta.get("net") != self.net.name or meta.get("dtype") != self.net.dtype:
            raise ValueError("checkpoint is for %s/%s" % (meta.get("net"), meta.get("dtype")))
        for k, name in enumerate(r.names):
            if tuple(t["param." + name].shape) != tuple(r.param[k].shape):
                raise ValueError("checkpoint parameter %s has shape %s" % (name, tuple(t["param." + name].shape)))
        for k, name in enumerate(r.names):
            r.param[k].copy_(t["param." + name])
            r.mom[k].copy_(t["mom." + name])
        r.refresh_low_precision()
        self.epoch, self.step = int(meta["epoch"]), int(meta["step"])
        self.best_acc, self.best_epoch = float(meta["best_acc"]), int(meta["best_epoch"])
        torch.cuda.synchronize()

    def profile(self, steps=3):
        """Median per-call times (ms) of `steps` timed steps as [(call name, ms)]; the steps run with a zero
        learning rate and the momentum buffers are put back afterwards."""
        r = self.run
        keep_mom = [v.clone() for v in r.mom]
        r.enable_timing(True)
        acc = []
        for _ in range(steps):
            r.step(0.0, 0.0, 0.0)
            torch.cuda.synchronize()
            acc.append(r.call_times_ms())
        r.enable_timing(False)
        for v, k in zip(r.mom, keep_mom):
            v.copy_(k)
        torch.cuda.synchronize()
        med = np.median(np.asarray(acc), axis=0)
        return list(zip(r.call_names, [float(x) for x in med]))
