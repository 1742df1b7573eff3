#!/usr/bin/env python3
"""Writes tests/golden/resnorms.json: the residual-norm histories of the full-size benchmark
configurations, computed by the CPU oracle ONLY (nothing from the HIP library is used).

The residual norm is a sum over the whole batch, so unlike the states it cannot be checked
sequence by sequence at test time; the full-batch oracle run takes minutes per workload on a
few cores, which is why its (tiny) result is stored.  Usage, from the repository root:

    python tests/golden/make_resnorm_golden.py [workload ...]

Existing entries of other workloads are kept.  Inputs come from the seeded generators in
paper_2601_09026_amd/workloads.py (shapes and MGRIT settings of the five configurations).
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import mgrit as omgrit, transformer_ode as tode          # noqa: E402
from paper_2601_09026_amd import workloads as wls                     # noqa: E402

OUT = os.path.join(ROOT, "tests", "golden", "resnorms.json")


def run(name, memory=None):
    wl = wls.named_workloads()[name]
    sh = tode.Shape(wl.arch, wl.d_model, wl.n_heads, wl.batch, wl.seq, wl.mem_seq, wl.ln_eps)
    th = [wls.layer_params(wl, n) for n in range(wl.N)]
    Z0 = wls.initial_state(wl)
    relax = "FCF" if wl.relax else "F"
    t = time.time()
    Z, rf, counts = omgrit.mgrit_forward(Z0, th, wl.h, wl.cf, wl.levels, wl.iters, sh, memory, relax)
    entry = {"forward": rf, "forward_evaluations": counts, "forward_seconds": time.time() - t,
             "Z_N_norm": float(np.linalg.norm(Z[-1])), "increment_norm": float(np.linalg.norm(Z[-1] - Z[0]))}
    print(name, "forward", rf, f"{entry['forward_seconds']:.0f}s", flush=True)
    if True:
        t = time.time()
        lam, ra, _ = omgrit.mgrit_adjoint(wls.terminal_adjoint(wl), Z, th, wl.h, wl.cf, wl.levels, wl.iters, sh,
                                          memory, relax)
        entry.update({"adjoint": ra, "adjoint_seconds": time.time() - t,
                      "lambda_0_norm": float(np.linalg.norm(lam[0])),
                      "adjoint_increment_norm": float(np.linalg.norm(lam[0] - lam[-1]))})
        print(name, "adjoint", ra, f"{entry['adjoint_seconds']:.0f}s", flush=True)
    return entry, Z[-1]


def run_stacked(name):
    """The stacked encoder-decoder grid (one MGRIT over encoder layers followed by decoder layers)."""
    sw = wls.stacked_workloads()[name]
    e, d = sw.enc, sw.dec
    she = tode.Shape(e.arch, e.d_model, e.n_heads, e.batch, e.seq, 0, e.ln_eps)
    shd = tode.Shape(d.arch, d.d_model, d.n_heads, d.batch, d.seq, d.mem_seq, d.ln_eps)
    th = [wls.stacked_layer_params(sw, n) for n in range(sw.N)]
    relax = "FCF" if d.relax else "F"
    Z0 = wls.stacked_initial_state(sw)
    t = time.time()
    Z, rf, counts = omgrit.stacked_mgrit_forward(Z0, th, sw.n_enc, d.h, d.cf, d.levels, d.iters, she, shd, relax)
    entry = {"forward": rf, "forward_evaluations": counts, "forward_seconds": time.time() - t,
             "Z_N_norm": float(np.linalg.norm(Z[-1])), "increment_norm": float(np.linalg.norm(Z[-1] - Z[0]))}
    print(name, "forward", rf, f"{entry['forward_seconds']:.0f}s", flush=True)
    t = time.time()
    lam, ra, _ = omgrit.stacked_mgrit_adjoint(wls.stacked_terminal_adjoint(sw), Z, th, sw.n_enc, d.h, d.cf,
                                              d.levels, d.iters, she, shd, relax)
    entry.update({"adjoint": ra, "adjoint_seconds": time.time() - t,
                  "lambda_0_norm": float(np.linalg.norm(lam[0])),
                  "adjoint_increment_norm": float(np.linalg.norm(lam[0] - lam[-1]))})
    print(name, "adjoint", ra, f"{entry['adjoint_seconds']:.0f}s", flush=True)
    return entry


def main():
    names = sys.argv[1:] or ["tiny_encoder", "mt_encoder", "mt_decoder", "vit_small", "bert_base", "gpt2_small"]
    data = json.load(open(OUT)) if os.path.exists(OUT) else {}
    enc_out = None
    for name in names:
        memory = None
        if name in wls.stacked_workloads():
            data[name] = run_stacked(name)
            with open(OUT, "w") as f:
                json.dump(data, f, indent=1, sort_keys=True)
            continue
        if name == "mt_decoder":
            if enc_out is None:
                _, enc_out = run("mt_encoder")
            memory = enc_out.astype(np.float32)        # the decoder consumes the encoder's output
        entry, zn = run(name, memory)
        if name == "mt_encoder":
            enc_out = zn
        data[name] = entry
        with open(OUT, "w") as f:
            json.dump(data, f, indent=1, sort_keys=True)
    print("wrote", OUT)


if __name__ == "__main__":
    main()
