"""fp64 CPU oracle of one CNN training step.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It shares no code with the HIP path and never imports it.  ops.py wraps the C library
(cnnk_ref.c, direct loops in double precision); step.py chains the operators over a layer
list by the chain rule (forward, loss, backward, SGD-momentum update); loop.py is the epoch loop
around it (mini-batches, validation in inference mode, best-so-far checkpoint); ensemble.py is the
ensemble of legal bf16 walks that grades a free-running bf16 step; vit.py is the training step of the
paper's second model family (a Vision Transformer) in numpy; asa_ref.py minimises the scheduler's
objective by enumeration.
"""
from . import ops
from .step import train_step, forward_loss, eval_forward, initial_running
from . import loop
from . import ensemble

__all__ = ["ops", "train_step", "forward_loss", "eval_forward", "initial_running", "loop", "ensemble"]
