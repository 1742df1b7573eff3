"""How accurately can a residual norm be reproduced by an implementation whose layer steps are only
good to a relative tolerance?  (CPU only; backs the bar that the GPU parity tests put on the residual
norms, tests/gpu_util.py: resnorm_bounds.)

The oracle's propagator is perturbed: every evaluation's increment gets element-wise relative noise
of size eps, the kind of error that operand rounding causes.  Findings, asserted below:
  * the first residual norm hardly moves (the noise is uncorrelated with the residual and adds in
    quadrature: relative change ~ (noise / residual)^2 / 2);
  * the second residual norm of a converging run is small itself, and moves by an ABSOLUTE amount
    that scales with eps and with the total increment |w_N - w_0|, not with its own size: a purely
    relative bar on it would be wrong by an order of magnitude;
  * that amount is tied to the error the same perturbed run shows in its final state: with e_inc the
    relative error of the increment w_N - w_0, sqrt(got^2 - r^2) is 0.9 .. 1.3 times
    e_inc |w_N - w_0| -- which is what resnorm_bounds grants, with its margin."""
import numpy as np
import pytest

from oracle import mgrit as om, transformer_ode as tode
from paper_2601_09026_amd import workloads as wls

from gpu_util import RESNORM_NOISE_FACTOR, resnorm_bounds

CASES = {
    "encoder_fcf": (wls.named_workloads()["bert_base"].scaled(batch=1, seq=32, d_model=128, n_heads=2, d_ff=256,
                                                              N=32, h=1.0 / 32), "FCF"),
    "deep_narrow_f_3_levels": (wls.named_workloads()["mc_deep_narrow"].scaled(batch=1, seq=64, N=64, h=1.0 / 64,
                                                                             cf=4, levels=3), "F"),
}


@pytest.mark.parametrize("case", list(CASES))
def test_residual_norm_under_step_noise(case):
    wl, relax = CASES[case]
    sh = tode.Shape(wl.arch, wl.d_model, wl.n_heads, wl.batch, wl.seq, wl.mem_seq, wl.ln_eps)
    theta = [wls.layer_params(wl, n) for n in range(wl.N)]
    Z0 = wls.initial_state(wl)
    exact = om.forward_propagator(theta, wl.h, wl.cf, sh)
    Z, r, _ = om.mgrit_solve(exact, Z0, wl.N, wl.cf, wl.levels, 2, relax)
    inc = np.linalg.norm(Z[-1] - Z[0])
    assert r[1] < 0.05 * r[0]                                   # a converging run: the second norm is small
    shifts = {}
    for eps in (1e-3, 4e-3):
        rng = np.random.default_rng(7)

        def noisy(lvl, j, w):
            d = exact(lvl, j, w) - w
            return w + d * (1.0 + eps * rng.standard_normal(d.shape))

        Zn, rn, _ = om.mgrit_solve(noisy, Z0, wl.N, wl.cf, wl.levels, 2, relax)
        e_inc = np.linalg.norm((Zn[-1] - Z0) - (Z[-1] - Z0)) / inc
        # first norm: second-order small in the noise
        assert abs(rn[0] - r[0]) <= 0.1 * eps * r[0]
        # second norm: raised, by an amount of the order e_inc * |w_N - w_0| added in quadrature
        n2 = rn[1] ** 2 - r[1] ** 2
        assert n2 > 0
        n = np.sqrt(n2)
        assert 0.9 * e_inc * inc <= n <= 1.3 * e_inc * inc, (n, e_inc * inc)
        lo, hi = resnorm_bounds(r[1], 0.0, inc, e_inc)
        assert lo <= rn[1] <= hi
        shifts[eps] = n
        # ... far more than a bar relative to the norm itself would allow at the larger noise level
        if eps == 4e-3:
            assert rn[1] - r[1] > 0.3 * r[1]
    # linear in eps
    assert 3.0 < shifts[4e-3] / shifts[1e-3] < 5.0
    assert RESNORM_NOISE_FACTOR >= 1.3
