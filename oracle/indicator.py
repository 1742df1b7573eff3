"""CPU oracle, part 3: the inexactness controller (paper section 3.2.3).

TEST INFRASTRUCTURE ONLY; shares no code with the library.

The paper's procedure, step by step: the convergence factor of MGRIT iteration k is the ratio
of consecutive fine-level residual norms.  Every few batches (the period is a parameter; the
paper's example is 500) the number of iterations is doubled for one batch and the factor of
the final iteration is examined.  A factor above 1 means the iteration count is no longer
effective; the mitigation is either a higher iteration count or serial training.

Readings where the paper is silent (the same in the library, listed in the design notes):
batches are counted from 0 and batch b probes when b + 1 is a multiple of the period; "a higher
iteration count" is the doubled count the probe just ran, allowed while it stays within a
ceiling, serial beyond; the switch to serial is final; a non-finite residual fails the probe,
two vanished residuals pass it.

Pins (tests/test_indicator.py): hand-written scenarios; the factor of a scalar linear two-level
iteration against its closed form; a diverging and a converging MGRIT run of the oracle.
"""
from __future__ import annotations

import math
from typing import Sequence

SERIAL, MORE_ITERATIONS = 0, 1


def convergence_factors(resnorms: Sequence[float]):
    """||r^(k+1)|| / ||r^(k)|| for consecutive iterations."""
    return [b / a for a, b in zip(resnorms[:-1], resnorms[1:])]


class Controller:
    def __init__(self, iters, probe_every, mitigation=SERIAL, max_iters=0, threshold=1.0):
        self.iters, self.probe_every = iters, probe_every
        self.mitigation, self.max_iters, self.threshold = mitigation, max_iters, threshold
        self.batch, self.serial, self.failures, self.last_factor = 0, False, 0, None
        self._probe = False

    def begin_batch(self) -> int:
        """Iterations for the coming batch; 0 means serial propagation."""
        self._probe = False
        if self.serial:
            return 0
        if self.probe_every > 0 and (self.batch + 1) % self.probe_every == 0:
            self._probe = True
            return 2 * self.iters
        return self.iters

    def end_batch(self, resnorms: Sequence[float]) -> bool:
        """Feed the residual norms of the batch; True if the policy changed."""
        self.batch += 1
        probe, self._probe = self._probe, False
        if not probe or self.serial or len(resnorms) < 2:
            return False
        prev, last = float(resnorms[-2]), float(resnorms[-1])
        if not (math.isfinite(prev) and math.isfinite(last)):
            factor = math.inf
        elif prev == 0.0:
            factor = 0.0 if last == 0.0 else math.inf
        else:
            factor = last / prev
        self.last_factor = factor
        if not factor > self.threshold:
            return False
        self.failures += 1
        if self.mitigation == MORE_ITERATIONS and 2 * self.iters <= self.max_iters:
            self.iters *= 2
        else:
            self.serial = True
        return True
