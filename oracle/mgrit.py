"""CPU oracle, part 2: serial propagation and MGRIT over the layer axis.

TEST INFRASTRUCTURE ONLY (see transformer_ode.py).  float64, plain loops, every
level has its own arrays; nothing is fused, aliased or skipped.

MGRIT is an iteration: its limit is serial propagation, its nu-th iterate is
not.  So this file holds both the definition (serial_*) and the algorithm
taken step by step in the paper's order (section 3.2, the two-level box of
Fig. 2, the V-cycle paragraph, and FCF-relaxation of Appendix A / Algorithm 1).

Level l (l = 0 .. L-1) has N_l = N / cf^l steps of size cf^l * h and the level
equation  w_j = Phi^l_{j-1}(w_{j-1}) + g_j,  j = 1..N_l,  w_0 = the initial
value; on level 0 g == 0 and the equation is serial propagation written as the
block-bidiagonal system A_0 W_0 = G_0.  C-points of a level are the indices
k*cf, the others are F-points.

One V-cycle on level l < L-1:
  1. relaxation: F-relaxation (cf-1 steps from every C-point, all intervals
     independent), and for FCF also C-relaxation (one step into every C-point)
     followed by F-relaxation again;
  2. residual of the level equation at the C-points, r_k = Phi(w_{k cf - 1})
     + g_{k cf} - w_{k cf}; it is zero at F-points after F-relaxation; on
     level 0 its 2-norm is recorded (the convergence indicator is the ratio of
     consecutive norms);
  3. restriction by injection: coarse unknowns = the C-point values; because
     the operator is nonlinear the coarse error equation A_1 e_1 = r_1 is posed
     in full-approximation form: solve  v_k = Phi^{l+1}_{k-1}(v_{k-1}) + g^{l+1}_k
     with  g^{l+1}_k = what_k - Phi^{l+1}_{k-1}(what_{k-1}) + r_k  (what = injected
     values) -- for a linear F this is exactly A_1 e_1 = r_1 with e = v - what;
  4. coarse solve: serially on the coarsest level, else recursively a V-cycle;
  5. correction w_{k cf} += v_k - what_k, then F-relaxation so that the
     F-points follow the corrected C-points ("interpolation").

A coarse step that starts at coarse point j of level l uses the parameters of
the fine layer j*cf^l (theta is a function of time sampled at t_n) and the step
size cf^l * h.

The adjoint problem is the same algorithm on the reversed index m = N - n with
mu_m = lambda_{N-m}: the level-l step from m=j to j+1 is
mu + cf^l h J(Z_n; theta_n)^T mu with n = N - (j+1) cf^l, i.e. the transpose of
the coarse forward step that starts at layer n.

Pins (tests/test_oracle_mgrit.py): one level or cf = 1 == serial; exactness
front of two-level MGRIT (k C-points per F-iteration, 2k per FCF-iteration);
serial solution is a fixed point with zero residual; closed-form recurrences
for a scalar linear F; three-level fixed point and limit; the coarse-level steps
(step size cf^l h, parameters and linearisation point of the fine layer the step starts at,
levels 1 and 2, forward, adjoint and stacked) against the layer function with explicit
integers, and the first two-level iterate v_k = Phi_c(v_{k-1}) + Phi^cf(u_{k-1}) - Phi_c(u_{k-1})
written out from the layer function alone (forward and adjoint).  Stacked
encoder-decoder grid: serial pass == encoder stack then decoder stack run by
the single-network functions; lambda_0 and parameter gradients against central
differences of the stacked network; the hand-over lambda_X(N_enc) == terminal
value + the decoder's memory gradient; exactness front across the switch.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from . import transformer_ode as tode

# A propagator is step(level, j, w) -> Phi^level_j(w): the step that starts at
# point j of that level (without the right-hand side g).
Propagator = Callable[[int, int, np.ndarray], np.ndarray]


def serial_solve(step: Propagator, w0: np.ndarray, N: int) -> List[np.ndarray]:
    """w_{n+1} = Phi^0_n(w_n), n = 0..N-1.  Returns [w_0 .. w_N]."""
    W = [np.array(w0, dtype=np.float64)]
    for n in range(N):
        W.append(step(0, n, W[n]))
    return W


def _f_relax(step, lvl, W, g, cf, M):
    for k in range(M):                         # parallel-for over coarse intervals
        n = cf * k
        for i in range(cf - 1):
            W[n + i + 1] = step(lvl, n + i, W[n + i]) + g[n + i + 1]


def _c_relax(step, lvl, W, g, cf, M):
    new = {}
    for k in range(1, M + 1):                  # parallel-for: reads only F-points
        n = cf * k
        new[n] = step(lvl, n - 1, W[n - 1]) + g[n]
    for n, v in new.items():
        W[n] = v


def _vcycle(step, lvl, W, g, cf, levels, relax, resnorms, counts):
    N_l = len(W) - 1
    if lvl == levels - 1:                      # coarsest level: serial solve
        for j in range(1, N_l + 1):
            W[j] = step(lvl, j - 1, W[j - 1]) + g[j]
        counts[lvl] += N_l
        return
    M = N_l // cf
    _f_relax(step, lvl, W, g, cf, M)
    counts[lvl] += M * (cf - 1)
    if relax == "FCF":
        _c_relax(step, lvl, W, g, cf, M)
        _f_relax(step, lvl, W, g, cf, M)
        counts[lvl] += M * cf
    # residual at the C-points
    r = [None] * (M + 1)
    for k in range(1, M + 1):
        n = cf * k
        r[k] = step(lvl, n - 1, W[n - 1]) + g[n] - W[n]
    counts[lvl] += M
    if lvl == 0:
        resnorms.append(float(np.sqrt(sum(float(np.sum(rk * rk)) for rk in r[1:]))))
    # restriction by injection + FAS right-hand side
    Wc = [W[cf * k].copy() for k in range(M + 1)]
    What = [w.copy() for w in Wc]
    gc = [np.zeros_like(W[0]) for _ in range(M + 1)]
    for k in range(1, M + 1):
        gc[k] = What[k] - step(lvl + 1, k - 1, What[k - 1]) + r[k]
    counts[lvl + 1] += M
    _vcycle(step, lvl + 1, Wc, gc, cf, levels, relax, resnorms, counts)
    # correction at the C-points, then interpolation by F-relaxation
    for k in range(1, M + 1):
        W[cf * k] = W[cf * k] + (Wc[k] - What[k])
    _f_relax(step, lvl, W, g, cf, M)
    counts[lvl] += M * (cf - 1)


def mgrit_solve(step: Propagator, w0: np.ndarray, N: int, cf: int, levels: int, iters: int,
                relax: str = "FCF", init: Optional[Sequence[np.ndarray]] = None
                ) -> Tuple[List[np.ndarray], List[float], List[int]]:
    """`iters` V-cycles of `levels`-level MGRIT for w_{n+1} = Phi_n(w_n).

    Initial guess: w0 copied into every point (only the C-point values matter,
    the first F-relaxation overwrites the F-points), or `init` (N+1 states).
    Returns (states [w_0..w_N], residual norms per iteration, step
    evaluations per level).
    """
    assert relax in ("F", "FCF")
    assert cf >= 1 and levels >= 1 and iters >= 0
    if levels == 1 or cf == 1:
        W = serial_solve(step, w0, N)
        return W, [], [N]
    assert N % (cf ** (levels - 1)) == 0, "N must be divisible by cf^(levels-1)"
    w0 = np.array(w0, dtype=np.float64)
    if init is None:
        W = [w0.copy() for _ in range(N + 1)]
    else:
        assert len(init) == N + 1
        W = [np.array(x, dtype=np.float64) for x in init]
        W[0] = w0.copy()
    g = [np.zeros_like(w0) for _ in range(N + 1)]
    resnorms: List[float] = []
    counts = [0] * levels
    for _ in range(iters):
        _vcycle(step, 0, W, g, cf, levels, relax, resnorms, counts)
    return W, resnorms, counts


# ----------------------------------------------------------------------------
# propagators
# ----------------------------------------------------------------------------
def forward_propagator(theta: Sequence[dict], h: float, cf: int, sh: tode.Shape,
                       mem=None) -> Propagator:
    """Phi^l_j(w) = w + cf^l h F(w; theta_{j cf^l})."""
    def step(lvl, j, w):
        s = cf ** lvl
        return tode.phi(w, theta[j * s], s * h, sh, mem)
    return step


def adjoint_propagator(theta: Sequence[dict], Z: Sequence[np.ndarray], h: float, cf: int,
                       sh: tode.Shape, mem=None) -> Propagator:
    """Step of the reversed-index adjoint system, linearised at the stored states Z_n."""
    N = len(Z) - 1

    def step(lvl, j, mu):
        s = cf ** lvl
        n = N - (j + 1) * s
        return tode.psi(mu, Z[n], theta[n], s * h, sh, mem)
    return step


def linear_propagator(a: float, h: float, cf: int) -> Propagator:
    """Toy problem dz/dt = a z: Phi^l(w) = (1 + cf^l h a) w (same at every point)."""
    def step(lvl, j, w):
        return (1.0 + (cf ** lvl) * h * a) * w
    return step


# ----------------------------------------------------------------------------
# the four entry points the HIP library is compared with
# ----------------------------------------------------------------------------
def serial_forward(Z0, theta, h, sh, mem=None):
    return serial_solve(forward_propagator(theta, h, 1, sh, mem), Z0, len(theta))


def mgrit_forward(Z0, theta, h, cf, levels, iters, sh, mem=None, relax="FCF", init=None):
    """Returns (Z_0..Z_N, residual norms, evaluation counts per level)."""
    return mgrit_solve(forward_propagator(theta, h, cf, sh, mem), Z0, len(theta),
                       cf, levels, iters, relax, init)


def serial_adjoint(lamN, Z, theta, h, sh, mem=None):
    """lambda_n for n = 0..N (index n, not the reversed index)."""
    N = len(theta)
    mu = serial_solve(adjoint_propagator(theta, Z, h, 1, sh, mem), lamN, N)
    return mu[::-1]


def parameter_gradients(lam, Z, theta, h, sh, mem=None):
    """dtheta_n = h * (dF/dtheta_n (Z_n))^T lambda_{n+1} for n = 0..N-1 (paper section 3.1: with
    lambda the adjoint states of the Euler network, this is the gradient of the loss with respect
    to layer n's parameters; with MGRIT's inexact Z and lambda it is the paper's inexact
    gradient).  lam and Z are indexed by n = 0..N.  Returns a list of dicts shaped like theta."""
    out = []
    for n, th in enumerate(theta):
        g = tode.F_param_vjp(Z[n], th, lam[n + 1], sh, mem)
        out.append({k: h * v for k, v in g.items()})
    return out


def memory_gradient(lam, Z, theta, h, sh, mem):
    """dL/dE = sum over layers of h * (dF_dec/dE (Y_n))^T lambda_{n+1}: the encoder output E enters
    every decoder layer's cross-attention, so its gradient collects one term per layer."""
    out = np.zeros_like(np.asarray(mem, dtype=np.float64))
    for n, th in enumerate(theta):
        _, dE = tode.F_vjp(Z[n], th, lam[n + 1], sh, mem)
        out += h * dE
    return out


def mgrit_adjoint(lamN, Z, theta, h, cf, levels, iters, sh, mem=None, relax="FCF", init=None):
    """Returns (lambda_0..lambda_N, residual norms, evaluation counts per level)."""
    N = len(theta)
    if init is not None:
        init = list(init)[::-1]
    mu, res, counts = mgrit_solve(adjoint_propagator(theta, Z, h, cf, sh, mem), lamN, N,
                                  cf, levels, iters, relax, init)
    return mu[::-1], res, counts


# ----------------------------------------------------------------------------
# buffer layers (paper appendix "Buffer layers"): the first n_open and last n_close layers are
# propagated serially with their own step size (1 in the paper), the layers in between by MGRIT
# ----------------------------------------------------------------------------
def buffered_forward(Z0, theta, h, cf, levels, iters, sh, n_open, n_close, h_buffer, mem=None, relax="FCF"):
    """States after every layer of the whole network (n_open + N + n_close + 1 of them) and the
    residual norms of the MGRIT part."""
    N = len(theta) - n_open - n_close
    Z = serial_forward(Z0, theta[:n_open], h_buffer, sh, mem) if n_open else [np.asarray(Z0, dtype=np.float64)]
    mid, res, _ = mgrit_forward(Z[-1], theta[n_open:n_open + N], h, cf, levels, iters, sh, mem, relax)
    Z = Z + mid[1:]
    if n_close:
        Z = Z + serial_forward(Z[-1], theta[n_open + N:], h_buffer, sh, mem)[1:]
    return Z, res


def buffered_adjoint(lamN, Z, theta, h, cf, levels, iters, sh, n_open, n_close, h_buffer, mem=None, relax="FCF"):
    """Adjoint states lambda_n, n = 0..n_open+N+n_close, and the MGRIT part's residual norms."""
    N = len(theta) - n_open - n_close
    a, b = n_open, n_open + N
    tail = serial_adjoint(lamN, Z[b:], theta[b:], h_buffer, sh, mem) if n_close else [np.asarray(lamN, np.float64)]
    mid, res, _ = mgrit_adjoint(tail[0], Z[a:b + 1], theta[a:b], h, cf, levels, iters, sh, mem, relax)
    head = serial_adjoint(mid[0], Z[:a + 1], theta[:a], h_buffer, sh, mem) if n_open else [mid[0]]
    return head[:-1] + mid + tail[1:], res


# ----------------------------------------------------------------------------
# stacked encoder-decoder system (paper section 3.1, eq. "fp_transformer"): one state
# Z_n = [X_n ; Y_n] on one time axis of N = N_enc + N_dec steps.  For n < N_enc the encoder layer
# advances X and leaves Y alone; from N_enc on the decoder layer advances Y, reading the X part
# of the same state as its cross-attention memory, and leaves X alone.  Rows of a state array:
# the B*S_x encoder tokens first, then the B*S_y decoder tokens.
# ----------------------------------------------------------------------------
def _split_xy(w, sh_enc: tode.Shape):
    tx = sh_enc.batch * sh_enc.seq
    w = np.asarray(w, dtype=np.float64)
    return w[:tx], w[tx:]


def stacked_forward_propagator(theta: Sequence[dict], n_enc: int, h: float, cf: int, sh_enc: tode.Shape,
                               sh_dec: tode.Shape) -> Propagator:
    """Phi^l_j([X;Y]) = [X;Y] + cf^l h F(t_n, [X;Y]), n = j cf^l: the piecewise F of the stacked
    system, taken at the step's starting time like theta."""
    def step(lvl, j, w):
        s = cf ** lvl
        n = j * s
        X, Y = _split_xy(w, sh_enc)
        if n < n_enc:
            return np.concatenate([tode.phi(X, theta[n], s * h, sh_enc), Y])
        return np.concatenate([X, tode.phi(Y, theta[n], s * h, sh_dec, X)])
    return step


def stacked_adjoint_propagator(theta: Sequence[dict], Z: Sequence[np.ndarray], n_enc: int, h: float, cf: int,
                               sh_enc: tode.Shape, sh_dec: tode.Shape) -> Propagator:
    """Transpose of the stacked step that starts at layer n = N - (j+1) cf^l, linearised at Z_n.
    A decoder step depends on X through the cross-attention memory, so its transpose adds the
    memory cotangent to the X part of the adjoint state."""
    N = len(Z) - 1

    def step(lvl, j, mu):
        s = cf ** lvl
        n = N - (j + 1) * s
        mx, my = _split_xy(mu, sh_enc)
        Xn, Yn = _split_xy(Z[n], sh_enc)
        if n < n_enc:
            return np.concatenate([tode.psi(mx, Xn, theta[n], s * h, sh_enc), my])
        dY, dX = tode.F_vjp(Yn, theta[n], my, sh_dec, Xn)
        return np.concatenate([mx + s * h * dX, my + s * h * dY])
    return step


def stacked_serial_forward(Z0, theta, n_enc, h, sh_enc, sh_dec):
    return serial_solve(stacked_forward_propagator(theta, n_enc, h, 1, sh_enc, sh_dec), Z0, len(theta))


def stacked_mgrit_forward(Z0, theta, n_enc, h, cf, levels, iters, sh_enc, sh_dec, relax="FCF"):
    """Returns (Z_0..Z_N, residual norms, evaluation counts per level)."""
    return mgrit_solve(stacked_forward_propagator(theta, n_enc, h, cf, sh_enc, sh_dec), Z0, len(theta),
                       cf, levels, iters, relax, None)


def stacked_serial_adjoint(lamN, Z, theta, n_enc, h, sh_enc, sh_dec):
    mu = serial_solve(stacked_adjoint_propagator(theta, Z, n_enc, h, 1, sh_enc, sh_dec), lamN, len(theta))
    return mu[::-1]


def stacked_mgrit_adjoint(lamN, Z, theta, n_enc, h, cf, levels, iters, sh_enc, sh_dec, relax="FCF"):
    """Returns (lambda_0..lambda_N, residual norms, evaluation counts per level)."""
    mu, res, counts = mgrit_solve(stacked_adjoint_propagator(theta, Z, n_enc, h, cf, sh_enc, sh_dec), lamN,
                                  len(theta), cf, levels, iters, relax, None)
    return mu[::-1], res, counts


def stacked_parameter_gradients(lam, Z, theta, n_enc, h, sh_enc, sh_dec):
    """dtheta_n = h (dF/dtheta_n (t_n, Z_n))^T lambda_{n+1}: an encoder layer sees the X parts, a
    decoder layer the Y parts with the X part of Z_n as memory."""
    out = []
    for n, th in enumerate(theta):
        lx, ly = _split_xy(lam[n + 1], sh_enc)
        Xn, Yn = _split_xy(Z[n], sh_enc)
        g = tode.F_param_vjp(Xn, th, lx, sh_enc) if n < n_enc else tode.F_param_vjp(Yn, th, ly, sh_dec, Xn)
        out.append({k: h * v for k, v in g.items()})
    return out
