"""cnnk: one device's CNN training step on MI355X (gfx950) as hand-written HIP kernels.

`cnnk` is the thin ctypes binding over libcnnk.so (argument marshalling only); `runner`
allocates device buffers with torch and drives cnnk_train_step over a layer list.
There is no CPU fallback: importing `cnnk` raises if the library has not been built.
"""
from . import cnnk  # noqa: F401
from .runner import StepRunner  # noqa: F401
