"""CPU oracle, part 1: the layer step of the neural-ODE transformer and its adjoint.

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, no blocking, no fusion, no
code shared with the HIP library.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this.

What is written out here (paper section 3.1):

* encoder step (eq. "encoder"):  X_{n+1} = X_n + h * F_enc(X_n),
      F_enc(X) = phi1(X) + phi2(X + phi1(X)),
      phi1 = SA o LN,  phi2 = MLP o LN  (pre-layer-norm);
  the inner residual X + phi1(X) is NOT scaled by h, only the outer update is.
* decoder-only step: the same with a causal mask in the attention.
* encoder-decoder decoder step (eq. "decoder"):
      Ybar = phi1(Y) + phi3(Y + phi1(Y), E),   phi3 = CA o LN  (cross-attention on
      the encoder output E),  F_dec = Ybar + phi2(Y + Ybar).
* the discrete adjoint of the forward-Euler step (eq. "tdp", right):
      lambda_n = lambda_{n+1} + h * (dF/dZ (Z_n))^T lambda_{n+1},
  the reading under which lambda_n is exactly the back-propagated gradient.

Choices the paper leaves open (same on both sides, listed in the design notes):
LayerNorm eps = 1e-5 with biased variance, exact erf GELU, a bias on every
projection, attention scale 1/sqrt(d_head), LayerNorm of phi3 acts on the
decoder stream only (the encoder output is used as it is).

Parameters arrive as a dict of named float arrays with ``W`` stored
``[out_features, in_features]`` (``y = x @ W.T + b``); ``Wqkv`` rows are
Q | K | V, head j owning rows j*d_h .. (j+1)*d_h of each third.

Pins (tests/test_oracle_*.py): h=1 step == torch's pre-LN encoder / decoder
layer in fp64; VJP == torch.autograd on an independent torch forward; central
finite differences; <c, J v> == <J^T c, v>; zero weights => F == 0; parameter
cotangents == torch.autograd with respect to torch's own block parameters and
central finite differences in single parameter entries.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
from scipy.special import erf

ARCH_ENCODER, ARCH_CAUSAL, ARCH_CROSS = 0, 1, 2


@dataclass(frozen=True)
class Shape:
    arch: int
    d_model: int
    n_heads: int
    batch: int
    seq: int
    mem_seq: int = 0
    ln_eps: float = 1e-5


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------
# building blocks, forward
# ----------------------------------------------------------------------------
def layer_norm(x, gamma, beta, eps):
    """Per token over the feature axis; biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_prime(z):
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def _split_heads(x, B, S, H):
    """[B*S, H*dh] -> [B, H, S, dh]"""
    dh = x.shape[1] // H
    return x.reshape(B, S, H, dh).transpose(0, 2, 1, 3)


def _merge_heads(x):
    """[B, H, S, dh] -> [B*S, H*dh]"""
    B, H, S, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, H * dh)


def attention_probs(q, k, causal):
    """softmax over keys of q k^T / sqrt(d_h); q [B,H,Sq,dh], k [B,H,Sk,dh]."""
    dh = q.shape[-1]
    a = np.matmul(q, k.transpose(0, 1, 3, 2)) / np.sqrt(dh)
    if causal:
        Sq, Sk = a.shape[-2:]
        a = np.where(np.arange(Sk)[None, :] > np.arange(Sq)[:, None], -np.inf, a)
    a = a - a.max(axis=-1, keepdims=True)
    e = np.exp(a)
    return e / e.sum(axis=-1, keepdims=True)


def self_attention(u, th, sh: Shape, causal):
    d, H, B, S = sh.d_model, sh.n_heads, sh.batch, sh.seq
    qkv = u @ _f64(th["Wqkv"]).T + _f64(th["bqkv"])
    q = _split_heads(qkv[:, 0:d], B, S, H)
    k = _split_heads(qkv[:, d:2 * d], B, S, H)
    v = _split_heads(qkv[:, 2 * d:3 * d], B, S, H)
    p = attention_probs(q, k, causal)
    o = _merge_heads(np.matmul(p, v))
    return o @ _f64(th["Wo"]).T + _f64(th["bo"])


def cross_attention(u, mem, th, sh: Shape):
    d, H, B, S, Sm = sh.d_model, sh.n_heads, sh.batch, sh.seq, sh.mem_seq
    q = _split_heads(u @ _f64(th["Wq_c"]).T + _f64(th["bq_c"]), B, S, H)
    kv = mem @ _f64(th["Wkv_c"]).T + _f64(th["bkv_c"])
    k = _split_heads(kv[:, 0:d], B, Sm, H)
    v = _split_heads(kv[:, d:2 * d], B, Sm, H)
    p = attention_probs(q, k, causal=False)
    o = _merge_heads(np.matmul(p, v))
    return o @ _f64(th["Wo_c"]).T + _f64(th["bo_c"])


def mlp(u, th):
    return gelu(u @ _f64(th["W1"]).T + _f64(th["b1"])) @ _f64(th["W2"]).T + _f64(th["b2"])


def F(X, th: Dict[str, np.ndarray], sh: Shape, mem: Optional[np.ndarray] = None):
    """Right-hand side of the layer ODE at state X ([batch*seq, d])."""
    X = _f64(X)
    eps = sh.ln_eps
    causal = sh.arch != ARCH_ENCODER
    s = self_attention(layer_norm(X, _f64(th["ln1_g"]), _f64(th["ln1_b"]), eps), th, sh, causal)
    if sh.arch == ARCH_CROSS:
        c = cross_attention(layer_norm(X + s, _f64(th["ln3_g"]), _f64(th["ln3_b"]), eps),
                            _f64(mem), th, sh)
        ybar = s + c
    else:
        ybar = s
    m = mlp(layer_norm(X + ybar, _f64(th["ln2_g"]), _f64(th["ln2_b"]), eps), th)
    return ybar + m


def phi(X, th, hstep, sh: Shape, mem=None):
    """One forward-Euler layer step of size hstep."""
    X = _f64(X)
    return X + hstep * F(X, th, sh, mem)


# ----------------------------------------------------------------------------
# vector-Jacobian products (reverse mode written out by hand)
# ----------------------------------------------------------------------------
def _layer_norm_vjp(dy, x, gamma, eps):
    d = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    dxhat = dy * gamma
    return rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                   - xhat * (dxhat * xhat).sum(axis=-1, keepdims=True) / d)


def _attention_core_vjp(do, q, k, v, causal):
    """Cotangents of q, k, v for o = softmax(q k^T / sqrt(dh)) v, all [B,H,S,dh]."""
    dh = q.shape[-1]
    p = attention_probs(q, k, causal)
    dv = np.matmul(p.transpose(0, 1, 3, 2), do)
    dp = np.matmul(do, v.transpose(0, 1, 3, 2))
    da = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = np.matmul(da, k) / np.sqrt(dh)
    dk = np.matmul(da.transpose(0, 1, 3, 2), q) / np.sqrt(dh)
    return dq, dk, dv


def _self_attention_vjp(ds, u, th, sh: Shape, causal):
    """Cotangent of u for s = SA(u)."""
    d, H, B, S = sh.d_model, sh.n_heads, sh.batch, sh.seq
    Wqkv = _f64(th["Wqkv"])
    qkv = u @ Wqkv.T + _f64(th["bqkv"])
    q = _split_heads(qkv[:, 0:d], B, S, H)
    k = _split_heads(qkv[:, d:2 * d], B, S, H)
    v = _split_heads(qkv[:, 2 * d:3 * d], B, S, H)
    do = _split_heads(ds @ _f64(th["Wo"]), B, S, H)
    dq, dk, dv = _attention_core_vjp(do, q, k, v, causal)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)
    return dqkv @ Wqkv


def _cross_attention_vjp(dc, u, mem, th, sh: Shape):
    """Cotangents (du, dmem) for c = CA(u, mem)."""
    d, H, B, S, Sm = sh.d_model, sh.n_heads, sh.batch, sh.seq, sh.mem_seq
    Wq, Wkv = _f64(th["Wq_c"]), _f64(th["Wkv_c"])
    q = _split_heads(u @ Wq.T + _f64(th["bq_c"]), B, S, H)
    kv = mem @ Wkv.T + _f64(th["bkv_c"])
    k = _split_heads(kv[:, 0:d], B, Sm, H)
    v = _split_heads(kv[:, d:2 * d], B, Sm, H)
    do = _split_heads(dc @ _f64(th["Wo_c"]), B, S, H)
    dq, dk, dv = _attention_core_vjp(do, q, k, v, causal=False)
    du = _merge_heads(dq) @ Wq
    dkv = np.concatenate([_merge_heads(dk), _merge_heads(dv)], axis=1)
    return du, dkv @ Wkv


def _mlp_vjp(dm, u, th):
    W1, W2 = _f64(th["W1"]), _f64(th["W2"])
    z = u @ W1.T + _f64(th["b1"])
    dz = (dm @ W2) * gelu_prime(z)
    return dz @ W1


def F_vjp(X, th, c, sh: Shape, mem=None):
    """(dF/dX)^T c at state X; for the cross-attention arch also (dF/dE)^T c.

    Returns (dX, dE) with dE None unless arch == ARCH_CROSS.
    """
    X, c = _f64(X), _f64(c)
    eps = sh.ln_eps
    causal = sh.arch != ARCH_ENCODER
    g1, b1 = _f64(th["ln1_g"]), _f64(th["ln1_b"])
    g2, b2 = _f64(th["ln2_g"]), _f64(th["ln2_b"])
    # forward quantities that the reverse sweep linearises about
    u1 = layer_norm(X, g1, b1, eps)
    s = self_attention(u1, th, sh, causal)
    if sh.arch == ARCH_CROSS:
        g3, b3 = _f64(th["ln3_g"]), _f64(th["ln3_b"])
        mem = _f64(mem)
        x3 = X + s
        u3 = layer_norm(x3, g3, b3, eps)
        ybar = s + cross_attention(u3, mem, th, sh)
    else:
        ybar = s
    x2 = X + ybar
    u2 = layer_norm(x2, g2, b2, eps)
    # F = ybar + m,  m = MLP(LN2(x2)),  x2 = X + ybar
    dx2 = _layer_norm_vjp(_mlp_vjp(c, u2, th), x2, g2, eps)
    dybar = c + dx2
    dX = dx2.copy()
    dE = None
    if sh.arch == ARCH_CROSS:
        # ybar = s + CA(LN3(x3), E),  x3 = X + s
        du3, dE = _cross_attention_vjp(dybar, u3, mem, th, sh)
        dx3 = _layer_norm_vjp(du3, x3, g3, eps)
        dX += dx3
        ds = dybar + dx3
    else:
        ds = dybar
    du1 = _self_attention_vjp(ds, u1, th, sh, causal)
    dX += _layer_norm_vjp(du1, X, g1, eps)
    return dX, dE


def _layer_norm_param_vjp(dy, x, eps):
    """Cotangents (dgamma, dbeta) of y = LN(x) * gamma + beta: sums over tokens."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    xhat = (x - mu) / np.sqrt(var + eps)
    return (dy * xhat).sum(axis=0), dy.sum(axis=0)


def F_param_vjp(X, th, c, sh: Shape, mem=None):
    """(dF/dtheta)^T c at state X: one array per parameter of the block, shaped like it.

    With c = lambda_{n+1} and X = Z_n this is, up to the factor h, the gradient of the loss with
    respect to layer n's parameters (paper section 3.1: the adjoint variable is the
    back-propagated gradient; theta enters the step only through h * F).  Every linear map
    y = u W^T + b contributes dW = dy^T u and db = sum over tokens of dy; LayerNorm contributes
    sums of dy * xhat and dy.  Written out operator by operator, no reuse of F_vjp.
    """
    X, c = _f64(X), _f64(c)
    eps = sh.ln_eps
    d, H, B, S = sh.d_model, sh.n_heads, sh.batch, sh.seq
    causal = sh.arch != ARCH_ENCODER
    g1, b1 = _f64(th["ln1_g"]), _f64(th["ln1_b"])
    g2, b2 = _f64(th["ln2_g"]), _f64(th["ln2_b"])
    Wqkv, Wo, W1, W2 = _f64(th["Wqkv"]), _f64(th["Wo"]), _f64(th["W1"]), _f64(th["W2"])
    out = {}
    # forward quantities
    u1 = layer_norm(X, g1, b1, eps)
    qkv = u1 @ Wqkv.T + _f64(th["bqkv"])
    q = _split_heads(qkv[:, 0:d], B, S, H)
    k = _split_heads(qkv[:, d:2 * d], B, S, H)
    v = _split_heads(qkv[:, 2 * d:3 * d], B, S, H)
    o = _merge_heads(attention_probs(q, k, causal) @ v)
    s = o @ Wo.T + _f64(th["bo"])
    if sh.arch == ARCH_CROSS:
        g3, b3 = _f64(th["ln3_g"]), _f64(th["ln3_b"])
        Wq, Wkv, Woc = _f64(th["Wq_c"]), _f64(th["Wkv_c"]), _f64(th["Wo_c"])
        mem = _f64(mem)
        Sm = sh.mem_seq
        x3 = X + s
        u3 = layer_norm(x3, g3, b3, eps)
        qc = _split_heads(u3 @ Wq.T + _f64(th["bq_c"]), B, S, H)
        kvc = mem @ Wkv.T + _f64(th["bkv_c"])
        kc = _split_heads(kvc[:, 0:d], B, Sm, H)
        vc = _split_heads(kvc[:, d:2 * d], B, Sm, H)
        oc = _merge_heads(attention_probs(qc, kc, False) @ vc)
        ybar = s + oc @ Woc.T + _f64(th["bo_c"])
    else:
        ybar = s
    x2 = X + ybar
    u2 = layer_norm(x2, g2, b2, eps)
    z = u2 @ W1.T + _f64(th["b1"])
    a = gelu(z)
    # F = ybar + m,  m = a W2^T + b2
    out["W2"], out["b2"] = c.T @ a, c.sum(axis=0)
    dz = (c @ W2) * gelu_prime(z)
    out["W1"], out["b1"] = dz.T @ u2, dz.sum(axis=0)
    du2 = dz @ W1
    out["ln2_g"], out["ln2_b"] = _layer_norm_param_vjp(du2, x2, eps)
    dybar = c + _layer_norm_vjp(du2, x2, g2, eps)
    if sh.arch == ARCH_CROSS:
        out["Wo_c"], out["bo_c"] = dybar.T @ oc, dybar.sum(axis=0)
        doc = _split_heads(dybar @ Woc, B, S, H)
        dqc, dkc, dvc = _attention_core_vjp(doc, qc, kc, vc, causal=False)
        dqc = _merge_heads(dqc)
        dkvc = np.concatenate([_merge_heads(dkc), _merge_heads(dvc)], axis=1)
        out["Wq_c"], out["bq_c"] = dqc.T @ u3, dqc.sum(axis=0)
        out["Wkv_c"], out["bkv_c"] = dkvc.T @ mem, dkvc.sum(axis=0)
        du3 = dqc @ Wq
        out["ln3_g"], out["ln3_b"] = _layer_norm_param_vjp(du3, x3, eps)
        ds = dybar + _layer_norm_vjp(du3, x3, g3, eps)
    else:
        ds = dybar
    out["Wo"], out["bo"] = ds.T @ o, ds.sum(axis=0)
    do = _split_heads(ds @ Wo, B, S, H)
    dq, dk, dv = _attention_core_vjp(do, q, k, v, causal)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)
    out["Wqkv"], out["bqkv"] = dqkv.T @ u1, dqkv.sum(axis=0)
    du1 = dqkv @ Wqkv
    out["ln1_g"], out["ln1_b"] = _layer_norm_param_vjp(du1, X, eps)
    return out


def psi(lam, Z, th, hstep, sh: Shape, mem=None):
    """Adjoint of one forward-Euler step linearised at Z: lam + hstep * J(Z)^T lam."""
    lam = _f64(lam)
    dX, _ = F_vjp(Z, th, lam, sh, mem)
    return lam + hstep * dX
