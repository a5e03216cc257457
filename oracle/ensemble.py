"""Ensemble of equally legal bf16-storage walks of the oracle, and the acceptance bound built on
it.  Test infrastructure.

A free-running bf16 step and the float64 walk decide ReLU masks and pool winners on values that
differ by storage rounding, and a flipped decision moves a gradient by far more than the rounding
itself, whatever the implementation.  How far a correct bf16 implementation may lie from the
float64 walk, and from another correct one, is therefore measured on the oracle alone: walks with
bf16 stores that differ only in roundings which an fp32 accumulation could decide either way
(oracle.step.train_step, `jitter`).
"""
from __future__ import annotations
import numpy as np

# Amplitude of the perturbation that decides a rounding, relative to the tensor's rms.  An fp32
# accumulation of K products in K/16 matrix instructions makes K/16 roundings of relative size
# 2^-24 on a running sum of the output's own size: a random walk of sqrt(K/16) * 2^-24, i.e. 2^-20
# for the deepest reduction of the benchmark networks (K = 4608); doubled for the fp32 operations
# behind it (scale, shift, residual sum).
JITTER_REL = 2.0 ** -19
JITTER_SEEDS = (11, 12, 13)


# The amplitude above is a model: the implementation's own figure is taken to be known only to
# within a factor of two (r = its noise power over the model's, r <= 2).  The number of decisions
# that differ between two walks is proportional to the sum of their noise powers, and a distance
# grows like the square root of that number: against the float64 walk (no noise) an implementation
# may therefore lie sqrt(r) = sqrt(2) times as far as a member does, and from a member
# sqrt((r + 1) / 2) = sqrt(1.5) times as far as two members lie apart.
SCALE_TO_EXACT = 2.0 ** 0.5
SCALE_TO_MEMBER = 1.5 ** 0.5


def ensemble_bound(samples, tol, scale=1.0):
    """Acceptance bound for a figure of the implementation under test, given the same figure of the
    ensemble's members: `scale` times their mean (see above) plus three (sample) standard
    deviations, the usual band outside which a draw from the same distribution falls about once in
    a thousand, plus the bar `tol` that the figure has to meet when nothing is chaotic."""
    a = np.asarray(samples, dtype=np.float64)
    return float(scale * a.mean() + 3.0 * a.std(ddof=1) + tol)


def walks(step_fn):
    """The ensemble: step_fn(storage, jitter) -> result, called for the plain bf16-storage walk and
    once per seed."""
    return [step_fn("bf16", None)] + [step_fn("bf16", (s, JITTER_REL)) for s in JITTER_SEEDS]
