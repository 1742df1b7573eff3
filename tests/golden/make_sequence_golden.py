#!/usr/bin/env python3
"""Writes tests/golden/<workload>_seq<b>.npz: the CPU oracle's complete MGRIT iterate (forward and
adjoint) for ONE sequence of a full-size benchmark configuration, computed by the oracle ONLY
(nothing from the HIP library is used).

Sequences are independent through the whole method (attention never crosses a sequence), so the
oracle's run on one sequence alone is what the full-batch run holds in that sequence's rows.  The
three-level forward and adjoint iteration of the deepest configurations (gpt2_small, mc_deep_narrow)
takes the oracle a quarter of an hour per sequence, too long for a test, which is why its result
is stored.  Stored, all float32:

  points        the level-0 C-points n = 0, cf, 2 cf, .. N (they include the C-points of every
                coarser level), where relaxation, FAS right-hand side, coarse solve and
                correction of all levels leave their mark
  tokens        the sampled token rows of the sequence
  Z, lam        [points, tokens, d]: Z_n and lambda_n at those points and tokens
  Z_inc_norm, lam_inc_norm
                [N+1]: |Z_n - Z_0| and |lambda_n - lambda_N| over the whole sequence, every n
  Z_norm, lam_norm
                [N+1]: |Z_n|, |lambda_n| over the whole sequence

The adjoint is linearised about the oracle's own forward iterate (sec. 3.2.2).  Usage, from the
repository root:

    python tests/golden/make_sequence_golden.py [workload [sequence]]     (default gpt2_small 5)
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import mgrit as omgrit, transformer_ode as tode          # noqa: E402
from paper_2601_09026_amd import workloads as wls                     # noqa: E402


def sample_tokens(seq):
    """16 token rows spread over the sequence, both ends and both sides of the 128-row tile edges."""
    want = [0, 1, 7, 31, 64, 100, 127, 128, 200, 255, 256, 300, 383, 384, 450, seq - 1]
    return np.array(sorted({min(t, seq - 1) for t in want}), dtype=np.int64)


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "gpt2_small"
    b = int(sys.argv[2]) if len(sys.argv) > 2 else 5
    wl = wls.named_workloads()[name]
    assert wl.mem_seq == 0 and 0 <= b < wl.batch
    sh = tode.Shape(wl.arch, wl.d_model, wl.n_heads, 1, wl.seq, 0, wl.ln_eps)
    th = [wls.layer_params(wl, n) for n in range(wl.N)]
    rows = slice(b * wl.seq, (b + 1) * wl.seq)
    Z0 = wls.initial_state(wl)[rows]
    lamN = wls.terminal_adjoint(wl)[rows]
    relax = "FCF" if wl.relax else "F"
    t = time.time()
    Z, rf, _ = omgrit.mgrit_forward(Z0, th, wl.h, wl.cf, wl.levels, wl.iters, sh, None, relax)
    print(name, "sequence", b, "forward", rf, f"{time.time() - t:.0f}s", flush=True)
    t = time.time()
    lam, ra, _ = omgrit.mgrit_adjoint(lamN, Z, th, wl.h, wl.cf, wl.levels, wl.iters, sh, None, relax)
    print(name, "sequence", b, "adjoint", ra, f"{time.time() - t:.0f}s", flush=True)
    points = np.arange(0, wl.N + 1, wl.cf)
    tokens = sample_tokens(wl.seq)
    out = os.path.join(ROOT, "tests", "golden", f"{name}_seq{b}.npz")
    np.savez_compressed(
        out, points=points, tokens=tokens, sequence=np.int64(b),
        Z=np.stack([Z[n][tokens] for n in points]).astype(np.float32),
        lam=np.stack([lam[n][tokens] for n in points]).astype(np.float32),
        Z_inc_norm=np.array([np.linalg.norm(Z[n] - Z[0]) for n in range(wl.N + 1)]),
        lam_inc_norm=np.array([np.linalg.norm(lam[n] - lam[wl.N]) for n in range(wl.N + 1)]),
        Z_norm=np.array([np.linalg.norm(Z[n]) for n in range(wl.N + 1)]),
        lam_norm=np.array([np.linalg.norm(lam[n]) for n in range(wl.N + 1)]),
        forward_resnorm=np.array(rf), adjoint_resnorm=np.array(ra))
    print("wrote", out, os.path.getsize(out), "bytes")


if __name__ == "__main__":
    main()
