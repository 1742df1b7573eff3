"""GPU parity of the stacked encoder-decoder grid (paper section 3.1, eq. "fp_transformer":
one MGRIT grid over encoder layers followed by decoder layers, state [X ; Y]) against the CPU
oracle: states, adjoint states (the decoder steps add the memory cotangent to lambda_X),
residual norms and parameter gradients.  Both sides linearise the adjoint about the GPU's own
forward iterate."""
import numpy as np
import pytest
import torch

from oracle import mgrit as omgrit, transformer_ode as tode
from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import TOL, dev, relerr
from test_gpu_mgrit import check_resnorms, check_states
from test_gpu_param_grads import compare_layer

pytestmark = pytest.mark.gpu


def stacked(dtype=wls.DTYPE_F32, n_enc=8, n_dec=8, cf=4, levels=2, iters=2, h=1.0, d=64, H=4, f=128, B=2,
            Sx=24, Sy=20, relax=1, seed=61):
    enc = wls.Workload("enc", wls.ARCH_ENCODER, d, H, f, B, Sx, 0, n_enc, h, cf, levels, iters, dtype, seed,
                       relax=relax)
    dec = wls.Workload("dec", wls.ARCH_CROSS, d, H, f, B, Sy, Sx, n_dec, h, cf, levels, iters, dtype, seed + 1,
                       relax=relax)
    return wls.StackedWorkload("stacked", enc, dec)


def grad_blocks(sw, desc_e, desc_d):
    out = []
    for n in range(sw.N):
        nbytes = mb.grad_layout(desc_e if n < sw.n_enc else desc_d).block_bytes
        out.append(torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8))
    return out


def run_case(sw, weight_std=0.08, grads=False, max_groups=0, lanes=2):
    e, d = sw.enc, sw.dec
    print(f"[case] stacked dtype={d.dtype} d={d.d_model} B={d.batch} Sx={e.seq} Sy={d.seq} n_enc={sw.n_enc} "
          f"N={sw.N} cf={d.cf} L={d.levels} it={d.iters} relax={d.relax} grads={grads} mg={max_groups} "
          f"lanes={lanes}", flush=True)
    mb.mgrit_set_max_groups_per_launch(max_groups)
    mb.mgrit_set_lanes(lanes)
    try:
        desc_d = mb.model_desc(d)
        desc_e = mb.encoder_desc(desc_d)
        host = [wls.stacked_layer_params(sw, n, weight_std) for n in range(sw.N)]
        blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, host[n]) for n in range(sw.N)]
        she = tode.Shape(e.arch, e.d_model, e.n_heads, e.batch, e.seq, 0, e.ln_eps)
        shd = tode.Shape(d.arch, d.d_model, d.n_heads, d.batch, d.seq, d.mem_seq, d.ln_eps)
        tol = TOL[d.dtype]
        relax = "FCF" if d.relax else "F"
        opts = mb.mgrit_opts(sw.N, d.h, d.cf, d.levels, d.iters, d.relax)
        Z0 = wls.stacked_initial_state(sw)
        Zg, rg = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, dev(Z0), blocks)
        torch.cuda.synchronize()
        Zr, rr, _ = omgrit.stacked_mgrit_forward(Z0, host, sw.n_enc, d.h, d.cf, d.levels, d.iters, she, shd, relax)
        _, einc = check_states(Zg, Zr, tol, "Z")
        check_resnorms(rg, rr, tol, Zr, einc)
        # the parts a step leaves alone are copied exactly
        tx = e.tokens
        if d.levels == 1 or d.cf == 1:
            assert torch.equal(Zg[sw.N, :tx], Zg[sw.n_enc, :tx]) and torch.equal(Zg[0, tx:], Zg[sw.n_enc, tx:])

        lamN = wls.stacked_terminal_adjoint(sw)
        gb = grad_blocks(sw, desc_e, desc_d) if grads else None
        lg, ag = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Zg, blocks, dev(lamN), dtheta=gb)
        torch.cuda.synchronize()
        Zlin = list(Zg.cpu().numpy().astype(np.float64))
        lr, ar, _ = omgrit.stacked_mgrit_adjoint(lamN, Zlin, host, sw.n_enc, d.h, d.cf, d.levels, d.iters, she, shd,
                                                 relax)
        _, einc = check_states(lg, lr, tol, "lambda")
        check_resnorms(ag, ar, tol, lr[::-1], einc)
        # the X part carries the memory cotangent: checked on its own so that the larger Y part cannot hide it
        lx_g = lg[:, :tx].cpu().numpy().astype(np.float64)
        for n in (0, sw.n_enc):
            ref = lr[n][:tx]
            inc = np.linalg.norm(ref - lamN[:tx])
            err = np.linalg.norm(lx_g[n] - ref)
            assert err <= tol * max(inc, 1e-30) + 1e-6 * np.linalg.norm(ref), (n, err, inc)
        if grads:
            lg2, _ = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Zg, blocks, dev(lamN))
            torch.cuda.synchronize()
            assert torch.equal(lg, lg2)
            ref = omgrit.stacked_parameter_gradients(lr, Zlin, host, sw.n_enc, d.h, she, shd)
            worst = 0.0
            for n in range(sw.N):
                got = mb.unpack_grad(desc_e if n < sw.n_enc else desc_d, gb[n])
                worst = max(worst, compare_layer(got, ref[n], tol, f"layer {n}"))
            print(f"  worst relative gradient error over all parameters and layers: {worst:.2e} (bar {tol})")
    finally:
        mb.mgrit_set_max_groups_per_launch(0)
        mb.mgrit_set_lanes(2)


@pytest.mark.parametrize("relax", [1, 0])
def test_two_level_fp32(relax):
    run_case(stacked(relax=relax))


def test_switch_inside_a_coarse_interval_three_levels_fp32():
    """n_enc = 6 is neither a C-point of level 0 (cf = 2: it is) nor of level 1 (multiples of 4):
    a coarse step that starts at layer 4 is an encoder step of size 4 h."""
    run_case(stacked(n_enc=6, n_dec=10, cf=2, levels=3), grads=True)


def test_unaligned_switch_chunked_single_lane_fp32():
    run_case(stacked(n_enc=5, n_dec=11, cf=4, levels=2), max_groups=3, lanes=1, grads=True)


def test_serial_limit_fp32():
    run_case(stacked(n_enc=3, n_dec=4, cf=4, levels=1, iters=1), grads=True)


def test_parameter_gradients_fp32():
    run_case(stacked(n_enc=4, n_dec=4, cf=4, levels=2), grads=True)


def test_two_level_bf16_with_gradients():
    run_case(stacked(dtype=wls.DTYPE_BF16, d=256, H=4, f=512, B=2, Sx=50, Sy=40, h=0.25, n_enc=8, n_dec=8),
             weight_std=0.05, grads=True)


def test_mt_shape_reduced_bf16():
    """Model shape of the translation configuration (d = 512, 8 heads, f = 2048, 64-token sentences),
    4 sentence pairs, 8 + 8 layers."""
    sw = wls.stacked_workloads()["mt_stacked"]
    sw = wls.StackedWorkload("mt_small", sw.enc.scaled(batch=4, N=8, h=1.0 / 16), sw.dec.scaled(batch=4, N=8, h=1.0 / 16))
    run_case(sw, weight_std=0.02, grads=True)


def test_full_size_mt_stacked_sampled_sentence_pairs():
    """The translation configuration on one grid at its full size (64 sentence pairs, 32 + 32 layers), in
    the launch configuration bench.py times.  Sentence pairs are independent through the whole method, so
    the oracle recomputes sampled pairs alone (the complete MGRIT iteration, forward and adjoint) and every
    state of those pairs is compared.  The residual norms couple the batch: they are compared with the values
    the oracle computed offline for the full batch (tests/golden/resnorms.json, written by
    tests/golden/make_resnorm_golden.py from the oracle only)."""
    from gpu_util import increment_tolerance
    from test_gpu_full_size import check_norms, golden
    sw = wls.stacked_workloads()["mt_stacked"]
    e, d = sw.enc, sw.dec
    print(f"[case] full size mt_stacked: B={d.batch} Sx={e.seq} Sy={d.seq} d={d.d_model} N={sw.N} cf={d.cf} "
          f"L={d.levels} it={d.iters}", flush=True)
    desc_d = mb.model_desc(d)
    desc_e = mb.encoder_desc(desc_d)
    host = [wls.stacked_layer_params(sw, n) for n in range(sw.N)]
    blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, host[n]) for n in range(sw.N)]
    tol = TOL[d.dtype]
    opts = mb.mgrit_opts(sw.N, d.h, d.cf, d.levels, d.iters, d.relax)
    Z0 = wls.stacked_initial_state(sw)
    lamN = wls.stacked_terminal_adjoint(sw)
    Zg, rg = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, dev(Z0), blocks)
    lg, ag = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Zg, blocks, dev(lamN))
    torch.cuda.synchronize()
    she = tode.Shape(e.arch, e.d_model, e.n_heads, 1, e.seq, 0, e.ln_eps)
    shd = tode.Shape(d.arch, d.d_model, d.n_heads, 1, d.seq, d.mem_seq, d.ln_eps)
    tx = e.tokens
    einc = {"Z": 0.0, "lambda": 0.0}
    for b in (7, 62):
        rows = np.concatenate([np.arange(b * e.seq, (b + 1) * e.seq), tx + np.arange(b * d.seq, (b + 1) * d.seq)])
        Zr, _, _ = omgrit.stacked_mgrit_forward(Z0[rows], host, sw.n_enc, d.h, d.cf, d.levels, d.iters, she, shd)
        got = Zg[:, rows, :].cpu().numpy().astype(np.float64)
        lr, _, _ = omgrit.stacked_mgrit_adjoint(lamN[rows], list(got), host, sw.n_enc, d.h, d.cf, d.levels, d.iters,
                                                she, shd)
        lgot = lg[:, rows, :].cpu().numpy().astype(np.float64)
        for what, g, r, base_row, far in (("Z", got, Zr, 0, sw.N), ("lambda", lgot, lr, sw.N, 0)):
            for n in range(sw.N + 1):
                err = relerr(g[n], r[n])
                assert err <= tol, f"{what}(pair {b})[{n}]: value error {err:.3e} > {tol}"
            # increments over the start value, for the encoder rows and the decoder rows separately
            for part, sl in (("X", slice(0, e.seq)), ("Y", slice(e.seq, None))):
                for n in (far, sw.n_enc):
                    base = r[base_row][sl]
                    if np.linalg.norm(r[n][sl] - base) > 0:
                        err = relerr(g[n][sl] - base, r[n][sl] - base)
                        bar = increment_tolerance(tol, r[n][sl], base, abs(n - base_row))
                        print(f"  {what}_{part}(pair {b})[{n}] increment err {err:.2e} (bar {bar:.2e})")
                        assert err <= bar, f"{what}_{part}(pair {b})[{n}]: increment error {err:.3e} > {bar:.3e}"
                        einc[what] = max(einc[what], err)
    for norms in (rg.cpu().numpy(), ag.cpu().numpy()):
        assert np.isfinite(norms).all() and all(norms[i + 1] < norms[i] for i in range(d.iters - 1)), norms
    gold = golden("mt_stacked")
    check_norms("forward", rg.cpu().numpy(), gold["forward"], tol, gold["increment_norm"], einc["Z"])
    check_norms("adjoint", ag.cpu().numpy(), gold["adjoint"], tol, gold["adjoint_increment_norm"], einc["lambda"])


def test_overlapped_coarse_solve_is_bit_identical_on_the_stacked_grid():
    """Coarse steps of both kinds (encoder, then decoder) hand finished intervals to the helper lane:
    same states, adjoint states and norms as the sequential order, bit for bit."""
    sw = stacked(dtype=wls.DTYPE_BF16, d=128, H=2, f=256, n_enc=12, n_dec=20, cf=4, levels=2, h=0.5)
    d = sw.dec
    desc_d = mb.model_desc(d)
    desc_e = mb.encoder_desc(desc_d)
    blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, wls.stacked_layer_params(sw, n, 0.05))
              for n in range(sw.N)]
    opts = mb.mgrit_opts(sw.N, d.h, d.cf, d.levels, d.iters, d.relax)
    Z0, lamN = dev(wls.stacked_initial_state(sw)), dev(wls.stacked_terminal_adjoint(sw))
    out = []
    try:
        for on in (1, 0):
            mb.lib().mgrit_debug_pipeline_coarse_solve(on)
            Z, rz = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, Z0, blocks)
            lam, rl = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Z, blocks, lamN)
            torch.cuda.synchronize()
            out.append((Z, rz, lam, rl))
    finally:
        mb.lib().mgrit_debug_pipeline_coarse_solve(1)
    for x, y in zip(out[0], out[1]):
        assert torch.equal(x, y)


def test_overlapped_coarse_solve_with_many_hand_overs_on_the_stacked_grid():
    """36 intervals handed over one at a time (the pool of 16 hand-over events wraps around; the
    right-hand sides are formed in one sweep): bit-identical to the sequential order."""
    sw = stacked(dtype=wls.DTYPE_BF16, d=128, H=2, f=256, B=1, Sx=24, Sy=20, n_enc=60, n_dec=84, cf=4, levels=2, h=0.1)
    d = sw.dec
    print(f"[case] stacked, many hand-overs: N={sw.N} n_enc={sw.n_enc}", flush=True)
    desc_d = mb.model_desc(d)
    desc_e = mb.encoder_desc(desc_d)
    blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, wls.stacked_layer_params(sw, n, 0.05))
              for n in range(sw.N)]
    opts = mb.mgrit_opts(sw.N, d.h, d.cf, d.levels, d.iters, d.relax)
    Z0, lamN = dev(wls.stacked_initial_state(sw)), dev(wls.stacked_terminal_adjoint(sw))
    out = []
    try:
        for on in (1, 0):
            mb.lib().mgrit_debug_pipeline_coarse_solve(on)
            mb.lib().mgrit_debug_pipeline_chunk(1 if on else 0)
            Z, rz = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, Z0, blocks)
            lam, rl = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Z, blocks, lamN)
            torch.cuda.synchronize()
            out.append((Z, rz, lam, rl))
    finally:
        mb.lib().mgrit_debug_pipeline_coarse_solve(1)
        mb.lib().mgrit_debug_pipeline_chunk(0)
    assert torch.isfinite(out[0][0]).all() and torch.isfinite(out[0][2]).all()
    for x, y in zip(out[0], out[1]):
        assert torch.equal(x, y)
