"""Helpers shared by the GPU parity tests: host<->device conversion and the error metric."""
import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}      # max |gpu - ref| / max |ref| per tensor (spec bars)
DEV = "cuda:0"

from oracle.ensemble import (JITTER_REL, JITTER_SEEDS, SCALE_TO_EXACT, SCALE_TO_MEMBER,  # noqa: E402,F401
                             ensemble_bound)


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def dev(a, dtype="f32"):
    """numpy float64 -> device tensor of the storage dtype (values must already be representable)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(DEV).to(tdtype(dtype)).contiguous()


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def host(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def max_rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def rep(a, dtype):
    """Make host data representable in the storage dtype (so input quantisation is not an error source)."""
    from workloads import to_bf16_representable
    if dtype == "bf16":
        return to_bf16_representable(a)
    return np.asarray(a, dtype=np.float32).astype(np.float64)
