"""The inexactness controller (paper section 3.2.3): the oracle's policy against hand-written
scenarios and MGRIT runs with a known outcome, and the library's host-side implementation
against the oracle on forced residual sequences.  No GPU."""
import numpy as np
import pytest

from oracle import indicator as oind, mgrit as omgrit
from paper_2601_09026_amd import binding as mb


# ------------------------------------------------------------------ the oracle, pinned
def test_probe_schedule_and_doubling():
    c = oind.Controller(iters=2, probe_every=5)
    its = []
    for b in range(12):
        its.append(c.begin_batch())
        c.end_batch([1.0, 0.1, 0.01, 0.001][:its[-1]])
    # batches 4 and 9 (the 5th and 10th) run twice the iterations, nothing else changes
    assert its == [2, 2, 2, 2, 4, 2, 2, 2, 2, 4, 2, 2]
    assert not c.serial and c.failures == 0 and c.last_factor == pytest.approx(0.1)


def test_factor_above_one_switches_to_serial_for_good():
    c = oind.Controller(iters=1, probe_every=3)
    for b in range(2):
        assert c.begin_batch() == 1
        assert c.end_batch([5.0]) is False            # ordinary batches are never judged, whatever they show
    assert c.begin_batch() == 2
    assert c.end_batch([1.0, 1.25]) is True           # final-iteration factor 1.25 > 1
    assert c.serial and c.last_factor == pytest.approx(1.25) and c.failures == 1
    for b in range(7):
        assert c.begin_batch() == 0                   # serial from now on, no more probes
        assert c.end_batch([]) is False


def test_only_the_final_iterations_factor_counts():
    c = oind.Controller(iters=2, probe_every=1)
    assert c.begin_batch() == 4
    assert c.end_batch([1.0, 3.0, 2.0, 1.0]) is False     # grew first, but the last factor is 0.5
    assert c.begin_batch() == 4
    assert c.end_batch([1.0, 0.1, 0.01, 0.011]) is True   # shrank first, the last factor is 1.1
    assert c.serial


def test_more_iterations_until_the_ceiling_then_serial():
    c = oind.Controller(iters=1, probe_every=1, mitigation=oind.MORE_ITERATIONS, max_iters=4)
    assert c.begin_batch() == 2 and c.end_batch([1.0, 2.0]) and c.iters == 2 and not c.serial
    assert c.begin_batch() == 4 and c.end_batch([1.0, 1.0, 1.0, 1.5]) and c.iters == 4 and not c.serial
    assert c.begin_batch() == 8 and c.end_batch([1.0] * 7 + [0.9]) is False       # now effective
    assert c.begin_batch() == 8 and c.end_batch([1.0] * 7 + [1.01]) and c.serial  # 8 > ceiling: serial


def test_degenerate_residuals():
    c = oind.Controller(iters=1, probe_every=1)
    c.begin_batch(); assert c.end_batch([0.0, 0.0]) is False and c.last_factor == 0.0   # converged exactly
    c.begin_batch(); assert c.end_batch([1.0, float("nan")]) is True and c.serial       # blew up


@pytest.mark.parametrize("a,expect_serial", [(-0.5, False), (-30.0, True)])
def test_on_scalar_mgrit_runs(a, expect_serial):
    """Two-level F-relaxation on z' = a z with h = 0.1, cf = 4.  The C-point error is multiplied per
    iteration by a factor built from phi^cf - phi_c (fine minus coarse propagation over an interval):
    for a = -0.5 that difference is 0.004 and the iteration converges; for a = -30 it is 16 + 11 = 27
    (phi = -2, phi_c = -11) and the residual grows until the exactness front arrives.  The verdict of
    the controller on the oracle's own residual norms is pinned, and for the contracting case a bound
    on the first factor from the geometric series of the coarse propagation."""
    N, cf, h = 64, 4, 0.1
    step = omgrit.linear_propagator(a, h, cf)
    c = oind.Controller(iters=2, probe_every=1)
    it = c.begin_batch()
    _, res, _ = omgrit.mgrit_solve(step, np.array([1.0]), N, cf, 2, it, "F")
    c.end_batch(res)
    fac = oind.convergence_factors(res)
    assert c.last_factor == pytest.approx(fac[-1])
    assert c.serial is expect_serial
    if not expect_serial:
        assert all(f < 1 for f in fac)
        phi, phic = 1 + a * h, 1 + a * h * cf
        assert fac[0] < abs(phi ** cf - phic) / (1 - abs(phic)) + 1e-12


# ------------------------------------------------------------------ the library against the oracle
def drive(seed, iters, period, mitigation, max_iters, threshold, n_batches=60):
    rng = np.random.default_rng(seed)
    lib = mb.mgrit_indicator_init(iters, period, mitigation, max_iters, threshold)
    ora = oind.Controller(iters, period, mitigation, max_iters, threshold)
    for b in range(n_batches):
        a, o = mb.mgrit_indicator_begin_batch(lib), ora.begin_batch()
        assert a == o, (seed, b)
        # forced residual history: random factors around 1, sometimes degenerate
        res = np.cumprod(np.concatenate([[1.0], rng.uniform(0.3, 1.4, max(a - 1, 0))])).astype(np.float32)[:a]
        if a >= 2 and rng.random() < 0.05:
            res[-1] = np.float32("inf")
        if a >= 2 and rng.random() < 0.05:
            res[-2:] = 0.0
        ca, co = mb.mgrit_indicator_end_batch(lib, res), ora.end_batch([float(x) for x in res])
        assert bool(ca) == co, (seed, b)
        assert (lib.iters, bool(lib.serial), lib.failures, lib.batch) == (ora.iters, ora.serial, ora.failures, ora.batch)
        if ora.last_factor is not None:
            assert lib.last_factor == pytest.approx(ora.last_factor, rel=1e-6) or (
                np.isinf(lib.last_factor) and np.isinf(ora.last_factor))


@pytest.mark.parametrize("seed", range(12))
def test_library_policy_equals_oracle_on_forced_sequences(seed):
    drive(seed, iters=1 + seed % 3, period=1 + seed % 4, mitigation=seed % 2, max_iters=[0, 4, 16][seed % 3],
          threshold=[1.0, 0.9][seed % 2])


def test_library_rejects_bad_arguments():
    ind = mb.Indicator()
    L = mb.lib()
    assert L.mgrit_indicator_init(None, 1, 1, 0, 0, 1.0) == -1
    assert L.mgrit_indicator_init(ind, 0, 1, 0, 0, 1.0) == -1
    assert L.mgrit_indicator_init(ind, 1, -1, 0, 0, 1.0) == -1
    assert L.mgrit_indicator_init(ind, 1, 1, 7, 0, 1.0) == -1
    assert L.mgrit_indicator_init(ind, 1, 1, 0, 0, 0.0) == -1
    assert L.mgrit_indicator_init(ind, 1, 0, 0, 0, 1.0) == 0
    assert L.mgrit_indicator_begin_batch(None) == -1
    assert L.mgrit_indicator_end_batch(ind, None, 3) == -1
    # period 0: never probes
    for _ in range(5):
        assert mb.mgrit_indicator_begin_batch(ind) == 1
        assert mb.mgrit_indicator_end_batch(ind, [9.0]) == 0
