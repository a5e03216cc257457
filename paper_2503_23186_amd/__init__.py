"""cnnk: one device's CNN training step on MI355X (gfx950) as hand-written HIP kernels.

`cnnk` is the thin ctypes binding over libcnnk.so (argument marshalling only); `runner`
allocates device buffers with torch and drives cnnk_train_step over a layer list; `trainer` is
the epoch loop around it; `vit` is the binding and runner of the Vision Transformer step
(include/cnnk_vit.h).  There is no CPU fallback: importing `cnnk` (directly, or through
StepRunner / Trainer) raises if the library has not been built.  The submodules are imported on
first use so that `python -m paper_2503_23186_amd.build` can run before a library exists.
"""
import importlib

_LAZY = {"cnnk": (".cnnk", None), "StepRunner": (".runner", "StepRunner"), "Trainer": (".trainer", "Trainer"),
         "vit": (".vit", None), "VitRunner": (".vit", "VitRunner"), "VitTrainer": (".trainer", "VitTrainer")}


def __getattr__(name):
    if name in _LAZY:
        mod, attr = _LAZY[name]
        m = importlib.import_module(mod, __name__)
        return m if attr is None else getattr(m, attr)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))
