"""Helpers shared by the GPU parity tests: move a seeded workload to the device, run the
oracle on the same inputs, compare."""
from __future__ import annotations

import numpy as np
import torch

from oracle import transformer_ode as tode
from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

TOL = {wls.DTYPE_F32: 1e-5, wls.DTYPE_BF16: 2e-2}   # normwise relative tolerance per dtype


def shape_of(wl, batch=None):
    return tode.Shape(wl.arch, wl.d_model, wl.n_heads, wl.batch if batch is None else batch, wl.seq,
                      wl.mem_seq, wl.ln_eps)


class DeviceModel:
    """Packed parameter blocks on the GPU plus the same parameters as named host arrays."""

    def __init__(self, wl, n_layers=None, weight_std=0.02, keep_host=True):
        self.wl = wl
        self.desc = mb.model_desc(wl)
        n_layers = wl.N if n_layers is None else n_layers
        self.host = []
        self.blocks = []
        for n in range(n_layers):
            p = wls.layer_params(wl, n, weight_std)
            self.blocks.append(mb.pack_theta(self.desc, p))
            self.host.append(p if keep_host else None)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def relerr(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def increment_tolerance(tol, ref, base, n_steps):
    """Bar for the error of (state - start value) relative to that increment.

    The state is stored in fp32, so each of the n_steps Euler updates rounds it by up to
    2^-24 |Z| per element no matter how accurate F is; these roundings add up like a random
    walk.  Relative to the (small) increment that floor is sqrt(n) 2^-24 |Z| / |dZ|; a factor
    4 covers the spread.  It is added to the dtype's relative tolerance."""
    ref = np.asarray(ref, np.float64)
    inc = np.linalg.norm(ref - base)
    if inc == 0.0:
        return float("inf")
    return tol + 4.0 * np.sqrt(max(n_steps, 1)) * 2.0 ** -24 * np.linalg.norm(ref) / inc


def assert_close(got, ref, base, tol, what, n_steps=1):
    """Normwise relative error on the value and on its increment over `base` (the state it
    started from): a few-percent error in F must not hide behind the O(1) state."""
    e_val = relerr(got, ref)
    e_inc = relerr(np.asarray(got, np.float64) - base, np.asarray(ref, np.float64) - base)
    tol_inc = increment_tolerance(tol, ref, base, n_steps)
    assert np.isfinite(np.asarray(got)).all(), f"{what}: non-finite values"
    assert e_val <= tol, f"{what}: value error {e_val:.3e} > {tol}"
    assert e_inc <= tol_inc, f"{what}: increment error {e_inc:.3e} > {tol_inc:.3e} (value error {e_val:.3e})"
    return e_val, e_inc


RESNORM_NOISE_FACTOR = 4.0


def resnorm_bounds(r, tol, inc_norm, inc_err):
    """Interval in which a computed residual norm may lie when the oracle's is r.

    The computed propagator differs from the exact one in two ways.  A systematic part (a slightly
    different F) scales the residual like the increments it is made of: relative `tol`, both ways.
    A noise part (operand rounding) is uncorrelated with the residual, so it adds in quadrature and
    in effect only raises the norm: got^2 ~ r^2 + n^2 (the cross term 2 r n cos(angle) is small in
    many dimensions: a tenth of n is granted downwards).  The size of n is tied to what the same run
    shows at the states: with `inc_err` the measured relative error of the total increment
    |w_N - w_0| = `inc_norm`, tests/test_oracle_resnorm_noise.py perturbs the oracle's steps with
    independent noise and finds n = 1.0 .. 1.3 times inc_err * inc_norm for every residual norm after
    the first (the noise that has piled up in the C-points is what the residual sees).  The library's
    rounding errors are not independent: a coarse step is evaluated twice at nearly equal inputs (for
    the right-hand side and in the solve) by the same deterministic kernel, so part of its error
    cancels in the correction and the final state comes out better than independent noise of the
    same size per step would leave it; measured ratios are 1.2 .. 1.3 for two-level FCF runs and up to
    2.9 for four-level F-relaxation.  RESNORM_NOISE_FACTOR = 4 covers that.
    The first residual norm is far above n, so its bar is in effect purely relative; late norms of a
    fast-converging run sink below n and are then only bounded by it."""
    n = RESNORM_NOISE_FACTOR * inc_err * inc_norm
    return max(0.0, r * (1.0 - tol) - 0.1 * n), float(np.sqrt((r * (1.0 + tol)) ** 2 + n * n))
