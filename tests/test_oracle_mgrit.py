"""Pins for the oracle's MGRIT driver (CPU only).

What the paper and the mathematics fix, independent of the oracle's own code:
* the exact solution of the level-0 system is serial forward propagation
  (Remark in section 3.2.1): one level or cf = 1 must equal the serial pass,
  and the serial solution must be a fixed point with zero residual;
* two-level MGRIT is exact on one more C-point per iteration with F-relaxation
  and on two more with FCF-relaxation (so it reproduces serial propagation after
  N/cf, resp. ceil(N/(2 cf)), iterations) -- and is NOT exact beyond that front;
* for the scalar linear problem dz/dt = a z every iterate has a closed form,
  computed below by a short scalar recurrence that never calls the oracle;
* the adjoint run obeys the same statements on the reversed index.
"""
import math

import numpy as np
import pytest

from oracle import mgrit, transformer_ode as tode
from paper_2601_09026_amd import workloads as wls


def tiny(arch=wls.ARCH_ENCODER, N=16, cf=4, levels=2, d=16, H=2, f=32, B=1, S=4, std=0.5, h=None,
         seed=21):
    h = 1.0 / N if h is None else h
    wl = wls.Workload("t", arch, d, H, f, B, S, 3 if arch == wls.ARCH_CROSS else 0,
                      N, h, cf, levels, 1, wls.DTYPE_F32, seed)
    sh = tode.Shape(arch, d, H, B, S, wl.mem_seq)
    th = [wls.layer_params(wl, n, weight_std=std) for n in range(N)]
    return wl, sh, th


def relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ------------------------------------------------------------------ limits
@pytest.mark.parametrize("levels,cf", [(1, 4), (2, 1), (3, 1)])
def test_single_level_or_cf1_is_serial(levels, cf):
    wl, sh, th = tiny(h=1.0)
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh)
    W, res, _ = mgrit.mgrit_forward(Z0, th, wl.h, cf, levels, 3, sh)
    assert max(np.abs(a - b).max() for a, b in zip(W, ser)) == 0.0


def test_serial_forward_is_the_plain_recursion():
    """Z_{n+1} = Z_n + h F(Z_n, theta_n), written out here without the oracle's driver."""
    wl, sh, th = tiny(N=5, h=0.7)
    Z = wls.initial_state(wl).astype(np.float64)
    ser = mgrit.serial_forward(Z, th, wl.h, sh)
    for n in range(5):
        assert np.array_equal(ser[n], Z)
        Z = Z + wl.h * tode.F(Z, th[n], sh)
    assert np.array_equal(ser[5], Z)


# ------------------------------------------------------------------ exactness front
@pytest.mark.parametrize("relax,speed", [("F", 1), ("FCF", 2)])
@pytest.mark.parametrize("arch", [wls.ARCH_ENCODER, wls.ARCH_CAUSAL])
def test_two_level_exactness_front(relax, speed, arch):
    wl, sh, th = tiny(arch=arch, N=24, cf=3, h=1.0, std=0.4)   # h = 1: the paper's own setting
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh)
    M = wl.N // wl.cf
    scale = np.abs(ser[-1]).max()
    for it in range(1, M // speed + 1):
        W, res, _ = mgrit.mgrit_forward(Z0, th, wl.h, wl.cf, 2, it, sh, relax=relax)
        front = min(M, speed * it)
        # every point up to the front C-point (and the F-points that follow it) is exact
        last_exact = min(wl.N, front * wl.cf + wl.cf - 1)
        for n in range(last_exact + 1):
            assert np.abs(W[n] - ser[n]).max() < 1e-11 * scale, (it, n)
        # beyond the front it is a genuine, inexact iterate
        if front + 1 <= M:
            assert np.abs(W[(front + 1) * wl.cf] - ser[(front + 1) * wl.cf]).max() > 1e-6, it
    W, res, _ = mgrit.mgrit_forward(Z0, th, wl.h, wl.cf, 2, math.ceil(M / speed), sh, relax=relax)
    assert max(np.abs(a - b).max() for a, b in zip(W, ser)) < 1e-11 * scale


def test_benchmark_config_1_is_exact_after_two_fcf_iterations():
    """M = 4 coarse intervals, FCF, 2 iterations: the front covers everything."""
    wl = wls.named_workloads()["tiny_encoder"]
    sh = tode.Shape(wl.arch, wl.d_model, wl.n_heads, wl.batch, wl.seq)
    th = [wls.layer_params(wl, n) for n in range(wl.N)]
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh)
    W, res, counts = mgrit.mgrit_forward(Z0, th, wl.h, wl.cf, wl.levels, wl.iters, sh)
    assert max(np.abs(a - b).max() for a, b in zip(W, ser)) < 1e-12
    assert len(res) == 2 and res[1] < res[0]
    lamN = wls.terminal_adjoint(wl)
    sa = mgrit.serial_adjoint(lamN, ser, th, wl.h, sh)
    la, ares, _ = mgrit.mgrit_adjoint(lamN, ser, th, wl.h, wl.cf, wl.levels, wl.iters, sh)
    assert max(np.abs(a - b).max() for a, b in zip(la, sa)) < 1e-12


# ------------------------------------------------------------------ fixed point
@pytest.mark.parametrize("levels", [2, 3])
@pytest.mark.parametrize("relax", ["F", "FCF"])
def test_serial_solution_is_a_fixed_point(levels, relax):
    wl, sh, th = tiny(N=16, cf=2, levels=levels, h=1.0)
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh)
    W, res, _ = mgrit.mgrit_forward(Z0, th, wl.h, wl.cf, levels, 2, sh, relax=relax, init=ser)
    scale = np.abs(ser[-1]).max()
    assert all(r < 1e-11 * scale for r in res)
    assert max(np.abs(a - b).max() for a, b in zip(W, ser)) < 1e-11 * scale


@pytest.mark.parametrize("levels,cf,N", [(3, 2, 16), (3, 4, 32), (4, 2, 16)])
def test_multilevel_converges_to_serial(levels, cf, N):
    wl, sh, th = tiny(N=N, cf=cf, levels=levels, h=1.0, std=0.3)
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh)
    errs, allres = [], None
    for it in (1, 2, 4, N // cf):
        W, res, _ = mgrit.mgrit_forward(Z0, th, wl.h, cf, levels, it, sh)
        errs.append(relerr(W[-1], ser[-1]))
        allres = res
    assert errs[0] > 1e-8            # a genuine iterate first
    assert errs[-1] < 1e-10          # converged
    assert errs[2] < errs[0]
    assert allres[-1] < 1e-9 * allres[0]


# ------------------------------------------------------------------ scalar linear closed forms
def scalar_two_level(a, h, cf, N, iters, relax, z0=1.0):
    """Closed-form two-level iterates for dz/dt = a z, C-point values only.

    phi = 1 + h a (fine step), phic = 1 + cf h a (coarse step).  With u the old
    C-point values: F-relaxation makes the residual at C-point k equal to
    phi^cf u_{k-1} - u_k, so the coarse solve gives
        v_k = phic v_{k-1} + (phi^cf - phic) u_{k-1};
    FCF first replaces u_k by phi^cf u_{k-1} (all k at once), then does the same.
    Residual norms are those of the relaxed values.
    """
    phi, phic = 1.0 + h * a, 1.0 + cf * h * a
    M = N // cf
    u = [z0] * (M + 1)
    res = []
    for _ in range(iters):
        if relax == "FCF":
            u = [u[0]] + [phi ** cf * u[k - 1] for k in range(1, M + 1)]
        r = [phi ** cf * u[k - 1] - u[k] for k in range(1, M + 1)]
        res.append(math.sqrt(sum(x * x for x in r)))
        v = [u[0]]
        for k in range(1, M + 1):
            v.append(phic * v[k - 1] + (phi ** cf - phic) * u[k - 1])
        u = v
    return u, res


@pytest.mark.parametrize("relax", ["F", "FCF"])
@pytest.mark.parametrize("a", [-1.5, 0.8])
def test_scalar_linear_two_level_closed_form(relax, a):
    N, cf, h = 12, 3, 0.25
    for iters in (1, 2, 3):
        u, res = scalar_two_level(a, h, cf, N, iters, relax, z0=2.0)
        W, r, _ = mgrit.mgrit_solve(mgrit.linear_propagator(a, h, cf), np.array([2.0]), N, cf, 2,
                                    iters, relax)
        for k in range(N // cf + 1):
            assert abs(W[k * cf][0] - u[k]) < 1e-13 * max(1.0, abs(u[k]))
            for i in range(1, cf):       # F-points follow their C-point
                if k * cf + i <= N:
                    assert abs(W[k * cf + i][0] - (1 + h * a) ** i * u[k]) < 1e-13 * max(1.0, abs(u[k]))
        assert np.allclose(r, res, rtol=1e-11, atol=1e-13)


def test_scalar_linear_limit_is_the_stability_function_power():
    a, h, cf, N = -0.9, 0.1, 2, 16
    for levels in (2, 3, 4):
        W, _, _ = mgrit.mgrit_solve(mgrit.linear_propagator(a, h, cf), np.array([1.0]), N, cf, levels,
                                    N, "FCF")
        for n in range(N + 1):
            assert abs(W[n][0] - (1 + h * a) ** n) < 1e-13


def test_three_level_scalar_first_iterate():
    """One FCF V-cycle of three-level MGRIT for dz/dt = a z, worked out by hand below.

    Level 1 is itself the two-level method applied to the level-1 equation
    v_k = phi1 v_{k-1} + g_k, where g is the full-approximation right-hand side.
    """
    a, h, cf, N, z0 = 0.6, 0.2, 2, 8, 1.0
    phi0, phi1, phi2 = 1 + h * a, 1 + 2 * h * a, 1 + 4 * h * a
    M0, M1 = 4, 2
    # level 0: FCF from the constant guess
    u = [z0] + [phi0 ** 2 * z0] * M0           # C-relaxed C-points (F-points were phi0*z0)
    r0 = [phi0 ** 2 * u[k - 1] - u[k] for k in range(1, M0 + 1)]
    g1 = [0.0] + [u[k] - phi1 * u[k - 1] + r0[k - 1] for k in range(1, M0 + 1)]
    # level 1 (points v_0..v_4 = u): FCF with right-hand side g1, cf = 2
    v = list(u)
    for k in range(M1):                         # F-relax
        v[2 * k + 1] = phi1 * v[2 * k] + g1[2 * k + 1]
    c = {2 * k: phi1 * v[2 * k - 1] + g1[2 * k] for k in range(1, M1 + 1)}
    for n, x in c.items():                      # C-relax
        v[n] = x
    for k in range(M1):                         # F-relax
        v[2 * k + 1] = phi1 * v[2 * k] + g1[2 * k + 1]
    r1 = [phi1 * v[2 * k - 1] + g1[2 * k] - v[2 * k] for k in range(1, M1 + 1)]
    what = [v[0], v[2], v[4]]
    g2 = [0.0] + [what[k] - phi2 * what[k - 1] + r1[k - 1] for k in range(1, M1 + 1)]
    x = [what[0]]
    for k in range(1, M1 + 1):                  # coarsest: serial
        x.append(phi2 * x[k - 1] + g2[k])
    for k in range(1, M1 + 1):                  # correct level 1, interpolate
        v[2 * k] += x[k] - what[k]
    for k in range(M1):
        v[2 * k + 1] = phi1 * v[2 * k] + g1[2 * k + 1]
    # correct level 0 C-points: u_k += v_k - u_k  =>  u = v
    W, res, counts = mgrit.mgrit_solve(mgrit.linear_propagator(a, h, cf), np.array([z0]), N, cf, 3, 1,
                                       "FCF")
    for k in range(M0 + 1):
        assert abs(W[2 * k][0] - v[k]) < 1e-14
    assert abs(res[0] - math.sqrt(sum(t * t for t in r0))) < 1e-14
    # evaluation counts: level 0: F(4) C(4) F(4) resid(4) interp(4) = 20; level 1: rhs 4 + F2 C2 F2
    # resid 2 interp 2 = 14; level 2: rhs 2 + solve 2 = 4
    assert counts == [20, 14, 4]


def test_two_level_evaluation_counts():
    wl, sh, th = tiny(N=16, cf=4)
    _, _, counts = mgrit.mgrit_forward(wls.initial_state(wl), th, wl.h, 4, 2, 2, sh)
    # per iteration, level 0: F 12 + C 4 + F 12 + residual 4 + interpolation 12; level 1: rhs 4 + solve 4
    assert counts == [2 * 44, 2 * 8]


# ------------------------------------------------------------------ adjoint
@pytest.mark.parametrize("relax,speed", [("F", 1), ("FCF", 2)])
def test_adjoint_exactness_front_and_limit(relax, speed):
    wl, sh, th = tiny(arch=wls.ARCH_CAUSAL, N=12, cf=3, h=1.0, std=0.4)
    Z = mgrit.serial_forward(wls.initial_state(wl), th, wl.h, sh)
    lamN = wls.terminal_adjoint(wl)
    ser = mgrit.serial_adjoint(lamN, Z, th, wl.h, sh)
    assert np.array_equal(ser[wl.N], lamN.astype(np.float64))
    M = wl.N // wl.cf
    scale = np.abs(ser[0]).max()
    for it in range(1, M // speed + 1):
        lam, res, _ = mgrit.mgrit_adjoint(lamN, Z, th, wl.h, wl.cf, 2, it, sh, relax=relax)
        front = min(M, speed * it)
        for m in range(min(wl.N, front * wl.cf + wl.cf - 1) + 1):      # reversed index
            assert np.abs(lam[wl.N - m] - ser[wl.N - m]).max() < 1e-11 * scale, (it, m)
        if front + 1 <= M:
            n = wl.N - (front + 1) * wl.cf
            assert np.abs(lam[n] - ser[n]).max() > 1e-7
    lam1, _, _ = mgrit.mgrit_adjoint(lamN, Z, th, wl.h, wl.cf, 1, 1, sh)
    assert max(np.abs(a - b).max() for a, b in zip(lam1, ser)) == 0.0


def test_adjoint_serial_is_the_gradient_of_the_serial_forward():
    """lambda_0 = d<C, Z_N>/dZ_0: directional finite differences through the serial pass."""
    wl, sh, th = tiny(N=6, h=0.5, std=0.4)
    Z0 = wls.initial_state(wl).astype(np.float64)
    C = wls.terminal_adjoint(wl).astype(np.float64)
    Z = mgrit.serial_forward(Z0, th, wl.h, sh)
    lam = mgrit.serial_adjoint(C, Z, th, wl.h, sh)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for _ in range(4):
        v = rng.standard_normal(Z0.shape)
        Lp = (C * mgrit.serial_forward(Z0 + eps * v, th, wl.h, sh)[-1]).sum()
        Lm = (C * mgrit.serial_forward(Z0 - eps * v, th, wl.h, sh)[-1]).sum()
        fd = (Lp - Lm) / (2 * eps)
        assert abs(fd - (lam[0] * v).sum()) < 1e-7 * max(1.0, abs(fd))
    # and the gradient at an interior layer: perturb Z_3, propagate layers 3..5
    v = rng.standard_normal(Z0.shape)
    def tail(z):
        for n in range(3, 6):
            z = tode.phi(z, th[n], wl.h, sh)
        return (C * z).sum()
    fd = (tail(Z[3] + eps * v) - tail(Z[3] - eps * v)) / (2 * eps)
    assert abs(fd - (lam[3] * v).sum()) < 1e-7 * max(1.0, abs(fd))


def test_adjoint_coarse_step_is_transpose_of_coarse_forward_step():
    """<mu, dPhi^1_j(Z) v> = <Psi^1(mu) , v> for the coarse propagators (injected theta, step cf h)."""
    wl, sh, th = tiny(N=8, cf=4, h=0.25, std=0.4)
    Z = mgrit.serial_forward(wls.initial_state(wl), th, wl.h, sh)
    fwd = mgrit.forward_propagator(th, wl.h, wl.cf, sh)
    adj = mgrit.adjoint_propagator(th, Z, wl.h, wl.cf, sh)
    rng = np.random.default_rng(1)
    mu, v = rng.standard_normal(Z[0].shape), rng.standard_normal(Z[0].shape)
    eps = 1e-6
    # coarse forward step j=1 starts at layer n=4; its transpose is the reversed-index step
    # landing on n=4: N - (j'+1)*cf = 4  =>  j' = 0
    Jv = (fwd(1, 1, Z[4] + eps * v) - fwd(1, 1, Z[4] - eps * v)) / (2 * eps)
    assert abs((mu * Jv).sum() - (adj(1, 0, mu) * v).sum()) < 1e-7 * abs((mu * Jv).sum())


# ------------------------------------------------------------------ coarse-level operators
def test_coarse_forward_step_uses_step_cf_pow_l_h_and_the_injected_layer():
    """Section 3.2.1: level l has the step size cf^l h, and a coarse step takes the parameters of
    the fine layer it starts at ("injected weights"): Phi^l_j(w) = w + cf^l h F(w; theta_{j cf^l}).
    Written out here with the layer function and explicit integers (cf = 4: cf^2 = 16 differs
    from 2 cf = 8, so a product in place of the power fails too)."""
    wl, sh, th = tiny(N=32, cf=4, h=0.125, std=0.4)
    w = wls.initial_state(wl).astype(np.float64)
    step = mgrit.forward_propagator(th, 0.125, 4, sh)
    #            level, j, fine layer, step size
    for lvl, j, layer, hstep in [(0, 5, 5, 0.125), (1, 0, 0, 0.5), (1, 3, 12, 0.5), (1, 7, 28, 0.5),
                                 (2, 0, 0, 2.0), (2, 1, 16, 2.0)]:
        want = w + hstep * tode.F(w, th[layer], sh)
        assert np.abs(step(lvl, j, w) - want).max() < 1e-13 * np.abs(want).max(), (lvl, j)
        # the neighbouring layers and the fine step size give something else
        assert np.abs(step(lvl, j, w) - (w + hstep * tode.F(w, th[layer + 1], sh))).max() > 1e-4
        if lvl:
            assert np.abs(step(lvl, j, w) - (w + 0.125 * tode.F(w, th[layer], sh))).max() > 1e-4


def test_coarse_adjoint_step_uses_step_cf_pow_l_h_and_lands_on_the_injected_layer():
    """Section 3.2.2: the adjoint runs the same grid backwards.  The level-l step from reversed
    point j to j+1 is the transpose of the forward coarse step that starts at layer
    n = N - (j+1) cf^l: mu + cf^l h (dF/dZ(Z_n; theta_n))^T mu."""
    wl, sh, th = tiny(arch=wls.ARCH_CAUSAL, N=32, cf=4, h=0.125, std=0.4)
    Z = mgrit.serial_forward(wls.initial_state(wl), th, 0.125, sh)
    mu = wls.terminal_adjoint(wl).astype(np.float64)
    step = mgrit.adjoint_propagator(th, Z, 0.125, 4, sh)
    for lvl, j, layer, hstep in [(0, 0, 31, 0.125), (0, 9, 22, 0.125), (1, 0, 28, 0.5), (1, 2, 20, 0.5),
                                 (1, 7, 0, 0.5), (2, 0, 16, 2.0), (2, 1, 0, 2.0)]:
        dX, _ = tode.F_vjp(Z[layer], th[layer], mu, sh)
        want = mu + hstep * dX
        assert np.abs(step(lvl, j, mu) - want).max() < 1e-13 * np.abs(want).max(), (lvl, j)
        near = layer - 1 if layer else layer + 1
        other, _ = tode.F_vjp(Z[near], th[near], mu, sh)
        assert np.abs(step(lvl, j, mu) - (mu + hstep * other)).max() > 1e-5
        if lvl:
            assert np.abs(step(lvl, j, mu) - (mu + 0.125 * dX)).max() > 1e-5


def test_stacked_coarse_steps_use_step_cf_pow_l_h_and_the_layer_they_start_at():
    """The same two statements for the stacked encoder-decoder grid (section 3.1, eq.
    "fp_transformer"): a coarse step takes type, parameters and step size cf^l h of the fine layer
    n it starts at: an encoder step on X below N_enc, a decoder step on Y (memory = the X part of
    its input) from there on; its transpose also adds the memory cotangent to the X part."""
    cf, h, n_enc, n_dec = 4, 0.125, 8, 24
    enc = wls.Workload("e", wls.ARCH_ENCODER, 16, 2, 32, 1, 4, 0, n_enc, h, cf, 3, 1, wls.DTYPE_F32, 31)
    dec = wls.Workload("d", wls.ARCH_CROSS, 16, 2, 32, 1, 3, 4, n_dec, h, cf, 3, 1, wls.DTYPE_F32, 32)
    sw = wls.StackedWorkload("s", enc, dec)
    she, shd = tode.Shape(enc.arch, 16, 2, 1, 4), tode.Shape(dec.arch, 16, 2, 1, 3, 4)
    th = [wls.stacked_layer_params(sw, n, 0.4) for n in range(sw.N)]
    w = wls.stacked_initial_state(sw).astype(np.float64)
    X, Y = w[:4], w[4:]
    fwd = mgrit.stacked_forward_propagator(th, n_enc, h, cf, she, shd)
    for lvl, j, layer, hstep in [(1, 1, 4, 0.5), (1, 2, 8, 0.5), (1, 5, 20, 0.5), (2, 0, 0, 2.0), (2, 1, 16, 2.0)]:
        if layer < n_enc:
            want = np.concatenate([X + hstep * tode.F(X, th[layer], she), Y])
        else:
            want = np.concatenate([X, Y + hstep * tode.F(Y, th[layer], shd, X)])
        assert np.abs(fwd(lvl, j, w) - want).max() < 1e-13 * np.abs(want).max(), (lvl, j)
    Z = mgrit.stacked_serial_forward(w, th, n_enc, h, she, shd)
    mu = wls.stacked_terminal_adjoint(sw).astype(np.float64)
    mx, my = mu[:4], mu[4:]
    adj = mgrit.stacked_adjoint_propagator(th, Z, n_enc, h, cf, she, shd)
    for lvl, j, layer, hstep in [(1, 0, 28, 0.5), (1, 4, 12, 0.5), (1, 5, 8, 0.5), (1, 6, 4, 0.5),
                                 (2, 0, 16, 2.0), (2, 1, 0, 2.0)]:
        Xn, Yn = Z[layer][:4], Z[layer][4:]
        if layer < n_enc:
            dX, _ = tode.F_vjp(Xn, th[layer], mx, she)
            want = np.concatenate([mx + hstep * dX, my])
        else:
            dY, dE = tode.F_vjp(Yn, th[layer], my, shd, Xn)
            want = np.concatenate([mx + hstep * dE, my + hstep * dY])
        assert np.abs(adj(lvl, j, mu) - want).max() < 1e-13 * np.abs(want).max(), (lvl, j)


def test_two_level_first_iterate_written_out_from_the_layer_function():
    """Fig. 2 / section 3.2.1 for two levels with F-relaxation, in the form the error equation
    takes once r and the injected values are substituted: with u the C-point values before the
    cycle (all equal to Z_0 here),
        v_k = Phi_c,k-1(v_{k-1}) + Phi_{k cf - 1} o .. o Phi_{(k-1) cf}(u_{k-1}) - Phi_c,k-1(u_{k-1}),
    Phi_n(w) = w + h F(w; theta_n) the fine steps and Phi_c,k(w) = w + cf h F(w; theta_{k cf}) the
    coarse one -- layer-dependent theta, so a wrong layer index or step size on the coarse level
    changes v.  Nothing of the oracle's driver or propagators is used to build the expected values."""
    cf, h = 4, 0.5
    wl, sh, th = tiny(N=16, cf=cf, h=h, std=0.4)
    Z0 = wls.initial_state(wl).astype(np.float64)
    M = wl.N // cf
    u = [Z0.copy() for _ in range(M + 1)]
    v = [Z0.copy()]
    for k in range(1, M + 1):
        fine = u[k - 1]
        for n in range((k - 1) * cf, k * cf):
            fine = fine + h * tode.F(fine, th[n], sh)
        coarse_v = v[k - 1] + cf * h * tode.F(v[k - 1], th[(k - 1) * cf], sh)
        coarse_u = u[k - 1] + cf * h * tode.F(u[k - 1], th[(k - 1) * cf], sh)
        v.append(coarse_v + fine - coarse_u)
    W, res, _ = mgrit.mgrit_forward(Z0, th, h, cf, 2, 1, sh, relax="F")
    scale = np.abs(v[-1]).max()
    for k in range(M + 1):
        assert np.abs(W[k * cf] - v[k]).max() < 1e-12 * scale, k
    # the second C-point is a genuine inexact iterate: it is not what serial propagation gives
    ser = mgrit.serial_forward(Z0, th, h, sh)
    assert np.abs(v[2] - ser[2 * cf]).max() > 1e-3 * scale
    # F-points follow their corrected C-point by fine steps (interpolation)
    z = v[2]
    for i in range(1, cf):
        z = z + h * tode.F(z, th[2 * cf + i - 1], sh)
        assert np.abs(W[2 * cf + i] - z).max() < 1e-12 * scale


def test_two_level_first_adjoint_iterate_written_out_from_the_layer_vjp():
    """The same cycle for the adjoint (section 3.2.2) on the reversed index m = N - n, mu_m =
    lambda_{N-m}: the fine step from m to m+1 is mu + h J(Z_n; theta_n)^T mu with n = N - 1 - m, the
    coarse step from coarse point k-1 to k is mu + cf h J(Z_n; theta_n)^T mu with n = N - k cf."""
    cf, h = 4, 0.5
    wl, sh, th = tiny(arch=wls.ARCH_CAUSAL, N=16, cf=cf, h=h, std=0.4)
    N, M = wl.N, wl.N // cf
    Z = mgrit.serial_forward(wls.initial_state(wl), th, h, sh)
    lamN = wls.terminal_adjoint(wl).astype(np.float64)

    def jt(n, mu):
        return tode.F_vjp(Z[n], th[n], mu, sh)[0]

    u = [lamN.copy() for _ in range(M + 1)]
    v = [lamN.copy()]
    for k in range(1, M + 1):
        fine = u[k - 1]
        for m in range((k - 1) * cf, k * cf):
            fine = fine + h * jt(N - 1 - m, fine)
        n_c = N - k * cf
        v.append(v[k - 1] + cf * h * jt(n_c, v[k - 1]) + fine - (u[k - 1] + cf * h * jt(n_c, u[k - 1])))
    lam, _, _ = mgrit.mgrit_adjoint(lamN, Z, th, h, cf, 2, 1, sh, relax="F")
    scale = np.abs(v[-1]).max()
    for k in range(M + 1):
        assert np.abs(lam[N - k * cf] - v[k]).max() < 1e-12 * scale, k
    ser = mgrit.serial_adjoint(lamN, Z, th, h, sh)
    assert np.abs(v[2] - ser[N - 2 * cf]).max() > 1e-4 * scale


def test_cross_attention_decoder_mgrit_runs_and_converges():
    wl, sh, th = tiny(arch=wls.ARCH_CROSS, N=8, cf=2, h=1.0, std=0.3)
    mem = wls.cross_memory(wl)
    Z0 = wls.initial_state(wl)
    ser = mgrit.serial_forward(Z0, th, wl.h, sh, mem)
    W1, r1, _ = mgrit.mgrit_forward(Z0, th, wl.h, 2, 2, 1, sh, mem)
    W2, r2, _ = mgrit.mgrit_forward(Z0, th, wl.h, 2, 2, 2, sh, mem)
    assert relerr(W1[-1], ser[-1]) > 1e-8
    assert max(np.abs(a - b).max() for a, b in zip(W2, ser)) < 1e-11 * np.abs(ser[-1]).max()


def test_coarse_level_is_first_order_approximation():
    """Remark of section 3.2.1: level l+1 approximates level l to O(h).

    Halving h (same weights reused as a function of time) should roughly halve the gap between
    the coarse-grid and fine-grid solutions at the final time.
    """
    d, H, f, B, S = 16, 2, 32, 1, 4
    gaps = []
    base = wls.Workload("t", wls.ARCH_ENCODER, d, H, f, B, S, 0, 1, 1.0, 2, 1, 0, wls.DTYPE_F32, 5)
    th1 = wls.layer_params(base, 0, weight_std=0.4)
    sh = tode.Shape(wls.ARCH_ENCODER, d, H, B, S)
    Z0 = wls.initial_state(base)
    for N in (8, 16, 32):
        h = 1.0 / N
        th = [th1] * N                                    # theta constant in time
        fine = mgrit.serial_forward(Z0, th, h, sh)[-1]
        coarse = mgrit.serial_forward(Z0, th[: N // 2], 2 * h, sh)[-1]
        gaps.append(np.linalg.norm(fine - coarse))
    assert 1.6 < gaps[0] / gaps[1] < 2.4 and 1.6 < gaps[1] / gaps[2] < 2.4


def test_parameter_gradients_are_the_gradient_of_the_serial_network():
    """dtheta_n = d<C, Z_N>/dtheta_n: central finite differences through the serial forward pass in
    single entries of several layers' parameters, and exact linearity in the terminal adjoint."""
    wl, sh, th = tiny(N=5, h=0.5, std=0.4)
    Z0 = wls.initial_state(wl).astype(np.float64)
    C = wls.terminal_adjoint(wl).astype(np.float64)
    Z = mgrit.serial_forward(Z0, th, wl.h, sh)
    lam = mgrit.serial_adjoint(C, Z, th, wl.h, sh)
    grads = mgrit.parameter_gradients(lam, Z, th, wl.h, sh)
    assert len(grads) == wl.N
    rng = np.random.default_rng(5)
    eps = 1e-6
    for n in (0, 2, 4):
        for name, shape in wls.param_shapes(wl).items():
            idx = tuple(int(rng.integers(0, s)) for s in shape)
            def loss(delta):
                t = [dict(x) for x in th]
                w = np.array(t[n][name], dtype=np.float64)
                w[idx] += delta
                t[n][name] = w
                return (C * mgrit.serial_forward(Z0, t, wl.h, sh)[-1]).sum()
            fd = (loss(eps) - loss(-eps)) / (2 * eps)
            assert abs(fd - grads[n][name][idx]) < 2e-6 * max(1.0, abs(fd)), (n, name, idx)
    lam2 = mgrit.serial_adjoint(-3.0 * C, Z, th, wl.h, sh)
    g2 = mgrit.parameter_gradients(lam2, Z, th, wl.h, sh)
    for name in grads[1]:
        assert np.allclose(g2[1][name], -3.0 * grads[1][name], rtol=1e-12, atol=1e-14)


def test_decoder_memory_and_parameter_gradients_by_finite_differences():
    """Cross-attention decoder: dL/dE (sum of one term per layer) and the cross-attention parameters'
    gradients equal central finite differences of <C, Y_N> through the serial decoder network."""
    wl, sh, th = tiny(arch=wls.ARCH_CROSS, N=4, h=0.5, std=0.4, B=2)
    Y0 = wls.initial_state(wl).astype(np.float64)
    C = wls.terminal_adjoint(wl).astype(np.float64)
    E = wls.cross_memory(wl).astype(np.float64)
    Y = mgrit.serial_forward(Y0, th, wl.h, sh, E)
    lam = mgrit.serial_adjoint(C, Y, th, wl.h, sh, E)
    dE = mgrit.memory_gradient(lam, Y, th, wl.h, sh, E)
    grads = mgrit.parameter_gradients(lam, Y, th, wl.h, sh, E)
    rng = np.random.default_rng(8)
    eps = 1e-6
    for _ in range(4):
        v = rng.standard_normal(E.shape)
        fd = ((C * mgrit.serial_forward(Y0, th, wl.h, sh, E + eps * v)[-1]).sum() -
              (C * mgrit.serial_forward(Y0, th, wl.h, sh, E - eps * v)[-1]).sum()) / (2 * eps)
        assert abs(fd - (dE * v).sum()) < 1e-7 * max(1.0, abs(fd))
    for n in (0, 3):
        for name in ("Wkv_c", "bkv_c", "Wq_c", "bq_c", "Wo_c", "bo_c", "ln3_g", "ln3_b"):
            shape = wls.param_shapes(wl)[name]
            idx = tuple(int(rng.integers(0, s)) for s in shape)
            def loss(delta):
                t = [dict(x) for x in th]
                w = np.array(t[n][name], dtype=np.float64)
                w[idx] += delta
                t[n][name] = w
                return (C * mgrit.serial_forward(Y0, t, wl.h, sh, E)[-1]).sum()
            fd = (loss(eps) - loss(-eps)) / (2 * eps)
            assert abs(fd - grads[n][name][idx]) < 2e-6 * max(1.0, abs(fd)), (n, name, idx)


def test_buffered_network_reduces_to_per_layer_step_sizes():
    """With a serial middle the buffered network is the plain recursion with step 1 on the open and
    close layers and h in between; with MGRIT in the middle, enough iterations reproduce it; and its
    adjoint is the gradient of that network (finite differences)."""
    wl, sh, th = tiny(N=12, cf=2, h=0.25, std=0.4)
    no, nc, hb = 2, 2, 1.0
    Z0 = wls.initial_state(wl).astype(np.float64)
    C = wls.terminal_adjoint(wl).astype(np.float64)
    steps = [hb] * no + [wl.h] * (wl.N - no - nc) + [hb] * nc
    def plain(z0):
        Z = [z0]
        for n, hs in enumerate(steps):
            Z.append(tode.phi(Z[-1], th[n], hs, sh))
        return Z
    ref = plain(Z0)
    Z, res = mgrit.buffered_forward(Z0, th, wl.h, 2, 1, 1, sh, no, nc, hb)
    assert len(Z) == wl.N + 1 and res == []
    for a, b in zip(Z, ref):
        assert np.allclose(a, b, rtol=0, atol=1e-13)
    Zm, res = mgrit.buffered_forward(Z0, th, wl.h, 2, 2, 4, sh, no, nc, hb)      # M = 4 intervals: exact after 4
    assert len(res) == 4
    assert np.allclose(Zm[-1], ref[-1], rtol=0, atol=1e-12)
    Zi, _ = mgrit.buffered_forward(Z0, th, wl.h, 2, 2, 1, sh, no, nc, hb)        # one iteration: inexact middle ...
    assert np.abs(Zi[-1] - ref[-1]).max() > 1e-6
    assert np.allclose(Zi[no], ref[no], rtol=0, atol=1e-13)                      # ... but exact open layers
    lam, _ = mgrit.buffered_adjoint(C, ref, th, wl.h, 2, 2, 4, sh, no, nc, hb)
    assert len(lam) == wl.N + 1
    rng = np.random.default_rng(2)
    eps = 1e-6
    for _ in range(3):
        v = rng.standard_normal(Z0.shape)
        fd = ((C * plain(Z0 + eps * v)[-1]).sum() - (C * plain(Z0 - eps * v)[-1]).sum()) / (2 * eps)
        assert abs(fd - (lam[0] * v).sum()) < 1e-7 * max(1.0, abs(fd))


# ------------------------------------------------------------------ stacked encoder-decoder grid
def stacked_tiny(n_enc=6, n_dec=6, cf=2, levels=2, d=16, H=2, f=32, B=2, Sx=5, Sy=4, std=0.5, h=0.5):
    enc = wls.Workload("e", wls.ARCH_ENCODER, d, H, f, B, Sx, 0, n_enc, h, cf, levels, 1, wls.DTYPE_F32, 51)
    dec = wls.Workload("d", wls.ARCH_CROSS, d, H, f, B, Sy, Sx, n_dec, h, cf, levels, 1, wls.DTYPE_F32, 52)
    sw = wls.StackedWorkload("s", enc, dec)
    she = tode.Shape(enc.arch, d, H, B, Sx, 0)
    shd = tode.Shape(dec.arch, d, H, B, Sy, Sx)
    th = [wls.stacked_layer_params(sw, n, std) for n in range(sw.N)]
    return sw, she, shd, th


def test_stacked_serial_forward_is_encoder_then_decoder():
    """Eq. "fp_transformer": X is frozen after the last encoder step and Y before it, so the
    serial stacked pass is the encoder stack followed by the decoder stack that attends to the
    encoder's output.  The two stacks are run here by the single-network functions."""
    sw, she, shd, th = stacked_tiny()
    Z0 = wls.stacked_initial_state(sw)
    Z = mgrit.stacked_serial_forward(Z0, th, sw.n_enc, sw.dec.h, she, shd)
    tx = sw.enc.tokens
    X = mgrit.serial_forward(Z0[:tx], th[:sw.n_enc], sw.dec.h, she)
    Y = mgrit.serial_forward(Z0[tx:], th[sw.n_enc:], sw.dec.h, shd, X[-1])
    for n in range(sw.N + 1):
        assert np.array_equal(Z[n][:tx], X[min(n, sw.n_enc)])
        assert np.array_equal(Z[n][tx:], Y[max(n - sw.n_enc, 0)])


def test_stacked_serial_adjoint_is_the_gradient_of_the_stacked_network():
    """lambda_0 = d<C, Z_N>/dZ_0 by central differences, for perturbations of source and target
    embeddings: the source direction only reaches the loss through every decoder layer's
    cross-attention, so it checks the memory cotangent that the decoder steps add to lambda_X."""
    sw, she, shd, th = stacked_tiny(n_enc=3, n_dec=3)
    Z0 = wls.stacked_initial_state(sw).astype(np.float64)
    C = wls.stacked_terminal_adjoint(sw).astype(np.float64)
    C[:sw.enc.tokens] *= 0.3          # the final X enters the loss too, with another weight
    Z = mgrit.stacked_serial_forward(Z0, th, sw.n_enc, sw.dec.h, she, shd)
    lam = mgrit.stacked_serial_adjoint(C, Z, th, sw.n_enc, sw.dec.h, she, shd)
    rng = np.random.default_rng(3)
    for part in ("x", "y", "both"):
        D = rng.standard_normal(Z0.shape)
        if part == "x":
            D[sw.enc.tokens:] = 0.0
        if part == "y":
            D[:sw.enc.tokens] = 0.0
        eps = 1e-6
        Lp = np.sum(C * mgrit.stacked_serial_forward(Z0 + eps * D, th, sw.n_enc, sw.dec.h, she, shd)[-1])
        Lm = np.sum(C * mgrit.stacked_serial_forward(Z0 - eps * D, th, sw.n_enc, sw.dec.h, she, shd)[-1])
        fd = (Lp - Lm) / (2 * eps)
        assert abs(fd - np.sum(lam[0] * D)) <= 1e-7 * max(1.0, abs(fd)), (part, fd, np.sum(lam[0] * D))


def test_stacked_adjoint_handover_is_terminal_plus_memory_gradient():
    """At the encoder's end lambda_X equals its terminal value plus the decoder's gradient with
    respect to its memory (one term per decoder layer), and lambda_Y does not change over the
    encoder steps."""
    sw, she, shd, th = stacked_tiny(n_enc=4, n_dec=5)
    Z0 = wls.stacked_initial_state(sw)
    C = wls.stacked_terminal_adjoint(sw).astype(np.float64)
    Z = mgrit.stacked_serial_forward(Z0, th, sw.n_enc, sw.dec.h, she, shd)
    lam = mgrit.stacked_serial_adjoint(C, Z, th, sw.n_enc, sw.dec.h, she, shd)
    tx = sw.enc.tokens
    Y = [z[tx:] for z in Z[sw.n_enc:]]
    lamY = mgrit.serial_adjoint(C[tx:], Y, th[sw.n_enc:], sw.dec.h, shd, Z[-1][:tx])
    dE = mgrit.memory_gradient(lamY, Y, th[sw.n_enc:], sw.dec.h, shd, Z[-1][:tx])
    assert relerr(lam[sw.n_enc][:tx], C[:tx] + dE) < 1e-13
    for n in range(sw.n_enc + 1):
        assert np.array_equal(lam[n][tx:], lam[sw.n_enc][tx:])
    assert relerr(lam[sw.n_enc][tx:], lamY[0]) < 1e-13


@pytest.mark.parametrize("relax,speed", [("F", 1), ("FCF", 2)])
def test_stacked_mgrit_exactness_front_and_limit(relax, speed):
    """Two-level MGRIT on the stacked grid: exact on `speed` more C-points per iteration, across
    the encoder/decoder switch (n_enc = 5 is not a C-point), and equal to the serial pass after
    enough iterations; forward and adjoint."""
    sw, she, shd, th = stacked_tiny(n_enc=5, n_dec=7, cf=2, levels=2)
    Z0 = wls.stacked_initial_state(sw)
    C = wls.stacked_terminal_adjoint(sw)
    ser = mgrit.stacked_serial_forward(Z0, th, sw.n_enc, sw.dec.h, she, shd)
    lser = mgrit.stacked_serial_adjoint(C, ser, th, sw.n_enc, sw.dec.h, she, shd)
    M = sw.N // 2
    for it in (1, 2, 3):
        W, res, _ = mgrit.stacked_mgrit_forward(Z0, th, sw.n_enc, sw.dec.h, 2, 2, it, she, shd, relax)
        lam, lres, _ = mgrit.stacked_mgrit_adjoint(C, ser, th, sw.n_enc, sw.dec.h, 2, 2, it, she, shd, relax)
        front = min(speed * it, M)
        for k in range(front + 1):
            assert relerr(W[2 * k], ser[2 * k]) < 1e-12
            assert relerr(lam[sw.N - 2 * k], lser[sw.N - 2 * k]) < 1e-12
        if front < M:
            assert relerr(W[-1], ser[-1]) > 1e-8
            assert relerr(lam[0], lser[0]) > 1e-8
    W, res, _ = mgrit.stacked_mgrit_forward(Z0, th, sw.n_enc, sw.dec.h, 2, 2, M, she, shd, relax)
    assert max(relerr(a, b) for a, b in zip(W, ser)) < 1e-12


def test_stacked_parameter_gradients_by_finite_differences():
    """One encoder matrix (reaches the loss only through the decoder's memory), one decoder
    cross-attention matrix and one decoder LayerNorm gain."""
    sw, she, shd, th = stacked_tiny(n_enc=3, n_dec=3)
    Z0 = wls.stacked_initial_state(sw)
    C = wls.stacked_terminal_adjoint(sw).astype(np.float64)
    C[:sw.enc.tokens] = 0.0           # loss on the decoder output only
    Z = mgrit.stacked_serial_forward(Z0, th, sw.n_enc, sw.dec.h, she, shd)
    lam = mgrit.stacked_serial_adjoint(C, Z, th, sw.n_enc, sw.dec.h, she, shd)
    g = mgrit.stacked_parameter_gradients(lam, Z, th, sw.n_enc, sw.dec.h, she, shd)
    rng = np.random.default_rng(5)
    for n, name in ((1, "W1"), (4, "Wkv_c"), (5, "ln3_g"), (0, "bqkv")):
        D = rng.standard_normal(th[n][name].shape)
        vals = []
        for sgn in (+1, -1):
            th2 = [dict(t) for t in th]
            th2[n][name] = th[n][name].astype(np.float64) + sgn * 1e-6 * D
            vals.append(np.sum(C * mgrit.stacked_serial_forward(Z0, th2, sw.n_enc, sw.dec.h, she, shd)[-1]))
        fd = (vals[0] - vals[1]) / 2e-6
        assert abs(fd - np.sum(g[n][name] * D)) <= 2e-7 * max(1.0, abs(fd)), (n, name, fd, np.sum(g[n][name] * D))
