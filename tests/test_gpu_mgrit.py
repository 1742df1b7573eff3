"""GPU parity of mgrit_forward / mgrit_adjoint against the CPU oracle's MGRIT, all states and
residual norms, on the same seeded inputs.

Small cases cover genuine (inexact) iterates: two and three levels, F and FCF relaxation, one
to three V-cycles, an initial guess supplied by the caller, serial limits.  The benchmark
configurations are run at their own model shape with the batch cut to what the oracle
finishes in seconds (sequences are independent, so a batch subset is exact, except for the
residual norm, which is a sum over the batch and is compared on the same subset)."""
import numpy as np
import pytest
import torch

from oracle import mgrit as omgrit
from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import TOL, DeviceModel, dev, increment_tolerance, relerr, resnorm_bounds, shape_of

pytestmark = pytest.mark.gpu


def check_states(got_all, ref_list, tol, what):
    """Every state against the oracle's (normwise relative error), and the increments over the start
    value at the far end and in the middle.  Returns (worst value error, worst increment error)."""
    ref = np.stack(ref_list)
    got = got_all.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite"
    base = ref[0] if what.startswith("Z") else ref[-1]
    worst, worst_inc = 0.0, 0.0
    for n in range(ref.shape[0]):
        e = relerr(got[n], ref[n])
        assert e <= tol, f"{what}[{n}]: value error {e:.3e} > {tol}"
        worst = max(worst, e)
    # increments over the start value, at the far end and in the middle
    for n in ([ref.shape[0] - 1, ref.shape[0] // 2] if what.startswith("Z") else [0, ref.shape[0] // 2]):
        if np.linalg.norm(ref[n] - base) > 0:
            e = relerr(got[n] - base, ref[n] - base)
            steps = n if what.startswith("Z") else ref.shape[0] - 1 - n
            tol_inc = increment_tolerance(tol, ref[n], base, steps)
            assert e <= tol_inc, f"{what}[{n}]: increment error {e:.3e} > {tol_inc:.3e}"
            print(f"  {what}[{n}] value err {relerr(got[n], ref[n]):.2e} increment err {e:.2e} (bar {tol_inc:.2e})")
            worst_inc = max(worst_inc, e)
    return worst, worst_inc


def check_resnorms(got, ref, tol, states, inc_err):
    """Residual norms of the GPU run against the oracle's.  `states`: the oracle's states, first to
    last in the direction of the solve; `inc_err`: the relative error of the GPU's increments measured
    against the oracle in this same run (check_states).  The interval comes from resnorm_bounds:
    relative `tol`, widened upwards by the noise the measured increment error implies, added in
    quadrature; the convergence factors (ratios of consecutive norms, sec. 3.2.3) follow from the norms
    and are printed."""
    got = got.cpu().numpy().astype(np.float64)
    inc = float(np.linalg.norm(np.asarray(states[-1], np.float64) - np.asarray(states[0], np.float64)))
    noise = inc_err * inc
    for i, r in enumerate(ref):
        lo, hi = resnorm_bounds(r, tol, inc, inc_err)
        print(f"  resnorm[{i}]: {got[i]:.6g} vs oracle {r:.6g} (allowed {lo:.6g} .. {hi:.6g}; noise level {noise:.3g})")
        assert lo <= got[i] <= hi, f"resnorm[{i}]: {got[i]} vs {r}, allowed {lo} .. {hi}"
        if i > 0:
            print(f"  convergence factor {i}: {got[i] / got[i - 1]:.5g} vs oracle {r / ref[i - 1]:.5g}")


def run_case(wl, weight_std=0.02, relax="FCF", adjoint=False, init_from_serial=False, max_groups=0):
    print(f"[case] mgrit {wl.name} arch={wl.arch} dtype={wl.dtype} d={wl.d_model} B={wl.batch} S={wl.seq} "
          f"N={wl.N} cf={wl.cf} L={wl.levels} it={wl.iters} relax={relax} adj={adjoint} "
          f"init={init_from_serial} mg={max_groups}", flush=True)
    mb.mgrit_set_max_groups_per_launch(max_groups)
    try:
        dm = DeviceModel(wl, weight_std=weight_std)
        sh = shape_of(wl)
        tol = TOL[wl.dtype]
        Z0 = wls.initial_state(wl)
        mem = wls.cross_memory(wl)
        opts = mb.mgrit_opts(wl.N, wl.h, wl.cf, wl.levels, wl.iters, 1 if relax == "FCF" else 0,
                             1 if init_from_serial else 0)
        init = omgrit.serial_forward(Z0, dm.host, wl.h, sh, mem) if init_from_serial else None
        Z_all = None
        if init_from_serial:
            Z_all = dev(np.stack(init))
        Zg, rg = mb.mgrit_forward(dm.desc, opts, dev(Z0), dm.blocks, memory=None if mem is None else dev(mem),
                                  Z_all=Z_all)
        torch.cuda.synchronize()
        Zr, rr, counts = omgrit.mgrit_forward(Z0, dm.host, wl.h, wl.cf, wl.levels, wl.iters, sh, mem,
                                              relax=relax, init=init)
        _, einc = check_states(Zg, Zr, tol, "Z")
        check_resnorms(rg, rr, tol, Zr, einc)
        if adjoint:
            lamN = wls.terminal_adjoint(wl)
            # linearise both sides about the same states: the GPU's own forward result
            Zlin = Zg.cpu().numpy()
            lg, arg = mb.mgrit_adjoint(dm.desc, opts, Zg, dm.blocks, dev(lamN),
                                       memory=None if mem is None else dev(mem))
            torch.cuda.synchronize()
            lr, arr, _ = omgrit.mgrit_adjoint(lamN, list(Zlin), dm.host, wl.h, wl.cf, wl.levels, wl.iters,
                                              sh, mem, relax=relax)
            _, einc = check_states(lg, lr, tol, "lambda")
            check_resnorms(arg, arr, tol, lr[::-1], einc)
        return Zg, Zr, rr
    finally:
        mb.mgrit_set_max_groups_per_launch(0)


def tiny(arch=wls.ARCH_ENCODER, dtype=wls.DTYPE_F32, N=32, cf=4, levels=2, iters=1, h=1.0, d=64, H=4, f=128,
         B=2, S=24, seed=41):
    return wls.Workload("tiny", arch, d, H, f, B, S, 20 if arch == wls.ARCH_CROSS else 0, N, h, cf, levels,
                        iters, dtype, seed)


# ----------------------------------------------------------------- genuine iterates, fp32
@pytest.mark.parametrize("relax", ["F", "FCF"])
@pytest.mark.parametrize("iters", [1, 2])
def test_two_level_inexact_iterates_fp32(relax, iters):
    # h = 1 (the paper's setting) and stronger weights: iterates differ visibly from serial
    wl = tiny(iters=iters)
    Zg, Zr, rr = run_case(wl, weight_std=0.08, relax=relax, adjoint=True)
    ser = omgrit.serial_forward(wls.initial_state(wl), DeviceModel(wl, weight_std=0.08).host, wl.h,
                                shape_of(wl))
    assert relerr(Zr[-1], ser[-1]) > 1e-4, "case is not a genuine inexact iterate"


# (the ends of the paper's parameter study, Table 2: coarsening factors 2 to 16, 2 to 5 levels)
@pytest.mark.parametrize("levels,cf,N", [(3, 2, 16), (3, 4, 32), (4, 2, 16), (5, 2, 32), (2, 16, 32)])
def test_multilevel_vcycles_fp32(levels, cf, N):
    run_case(tiny(arch=wls.ARCH_CAUSAL, N=N, cf=cf, levels=levels, iters=2), weight_std=0.08, adjoint=True)


@pytest.mark.parametrize("levels", [2, 3])
def test_cross_attention_decoder_forward_and_adjoint_fp32(levels):
    run_case(tiny(arch=wls.ARCH_CROSS, N=16, cf=2 if levels == 3 else 4, levels=levels, iters=2), weight_std=0.08,
             adjoint=True)


@pytest.mark.parametrize("levels,cf", [(1, 4), (2, 1)])
def test_serial_limits(levels, cf):
    wl = tiny(N=8, cf=cf, levels=levels, iters=3)
    Zg, Zr, rr = run_case(wl, weight_std=0.08, adjoint=True)
    assert rr == []


def test_serial_solution_is_a_fixed_point_on_the_gpu():
    wl = tiny(N=16, cf=4, levels=2, iters=1)
    Zg, Zr, rr = run_case(wl, weight_std=0.08, init_from_serial=True)


def test_sweeps_split_into_launch_chunks():
    run_case(tiny(N=32, cf=4, levels=2, iters=1), weight_std=0.08, adjoint=True, max_groups=3)


def test_zero_iterations_are_refused_unless_serial():
    """Without a V-cycle the F-points would never be written: refused before anything is enqueued."""
    wl = tiny(N=8, cf=4, levels=2, iters=0)
    dm = DeviceModel(wl)
    Z0 = dev(wls.initial_state(wl))
    with pytest.raises(mb.MgritError) as e:
        mb.mgrit_forward(dm.desc, mb.mgrit_opts(8, 1.0, 4, 2, 0), Z0, dm.blocks)
    assert e.value.status == mb.MGRIT_INVALID_ARG
    Zg, _ = mb.mgrit_forward(dm.desc, mb.mgrit_opts(8, 1.0, 4, 1, 0), Z0, dm.blocks)     # serial: iters unused
    torch.cuda.synchronize()
    assert torch.isfinite(Zg).all()


def test_run_to_run_bit_identical():
    wl = tiny(arch=wls.ARCH_CAUSAL, dtype=wls.DTYPE_BF16, N=16, cf=4, levels=2, iters=2, d=128, f=256)
    dm = DeviceModel(wl, weight_std=0.05)
    Z0 = dev(wls.initial_state(wl))
    opts = mb.mgrit_opts(16, 1.0, 4, 2, 2)
    a, ra = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks)
    b, rb = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(ra, rb)


@pytest.mark.parametrize("levels,cf,N", [(2, 4, 32), (3, 2, 16), (2, 4, 12)])
def test_overlapped_coarse_solve_is_bit_identical_to_the_sequential_order(levels, cf, N):
    """The serial coarse solve hands finished intervals to the helper lane, which F-relaxes them while
    the remaining coarse steps run: the same kernels on the same data as one after the other, so every
    state, adjoint state and residual norm must agree bit for bit (M = 8, 4 and 3 intervals on the level
    above the coarsest; 3 is not a multiple of the launch chunk)."""
    wl = tiny(arch=wls.ARCH_CAUSAL, dtype=wls.DTYPE_BF16, N=N, cf=cf, levels=levels, iters=2, d=128, f=256)
    dm = DeviceModel(wl, weight_std=0.05)
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))
    opts = mb.mgrit_opts(N, 1.0, cf, levels, 2)
    out = []
    try:
        for on in (1, 0, 1):
            mb.lib().mgrit_debug_pipeline_coarse_solve(on)
            Z, rz = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks)
            lam, rl = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN)
            torch.cuda.synchronize()
            out.append((Z, rz, lam, rl))
    finally:
        mb.lib().mgrit_debug_pipeline_coarse_solve(1)
    for a, b in ((out[0], out[1]), (out[0], out[2])):
        for x, y in zip(a, b):
            assert torch.equal(x, y)


@pytest.mark.parametrize("chunk", [1, 3])
def test_overlapped_coarse_solve_with_many_hand_overs_is_bit_identical(chunk):
    """40 intervals handed over one at a time: 39 hand-overs go through the pool of 16 events, which
    wraps around, and with more than 16 chunks the right-hand sides are formed in one sweep instead of
    chunk by chunk; 3 at a time gives 14 chunks with a ragged last one (right-hand sides chunk by
    chunk).  Forward and adjoint against the sequential order, bit for bit."""
    N, cf = 160, 4
    wl = tiny(arch=wls.ARCH_CAUSAL, dtype=wls.DTYPE_BF16, N=N, cf=cf, levels=2, iters=2, d=128, f=256, B=1, S=40)
    print(f"[case] many hand-overs: N={N} cf={cf} chunk={chunk}", flush=True)
    dm = DeviceModel(wl, weight_std=0.05, keep_host=False)
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))
    opts = mb.mgrit_opts(N, 0.1, cf, 2, 2)
    out = []
    try:
        for on in (1, 0):
            mb.lib().mgrit_debug_pipeline_coarse_solve(on)
            mb.lib().mgrit_debug_pipeline_chunk(chunk if on else 0)
            Z, rz = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks)
            lam, rl = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN)
            torch.cuda.synchronize()
            out.append((Z, rz, lam, rl))
    finally:
        mb.lib().mgrit_debug_pipeline_coarse_solve(1)
        mb.lib().mgrit_debug_pipeline_chunk(0)
    assert torch.isfinite(out[0][0]).all() and torch.isfinite(out[0][2]).all()
    for x, y in zip(out[0], out[1]):
        assert torch.equal(x, y)


# ----------------------------------------------------------------- benchmark configurations
def test_config1_tiny_encoder_full():
    wl = wls.named_workloads()["tiny_encoder"]
    Zg, Zr, rr = run_case(wl, adjoint=True)
    # M = 4, FCF, 2 iterations: the exactness front covers everything -> equals serial propagation
    ser = omgrit.serial_forward(wls.initial_state(wl), DeviceModel(wl).host, wl.h, shape_of(wl))
    assert relerr(Zg[-1].cpu().numpy(), ser[-1]) < 1e-5


def test_config2_bert_shape_reduced_batch():
    run_case(wls.named_workloads()["bert_base"].scaled(batch=2))


def test_config3_gpt2_shape_reduced():
    # model shape, causal mask, three levels and cf as configured; depth and batch reduced
    run_case(wls.named_workloads()["gpt2_small"].scaled(batch=1, N=16, h=1.0 / 16), adjoint=True)


def test_config4_vit_shape_reduced_batch():
    run_case(wls.named_workloads()["vit_small"].scaled(batch=2))


def test_config5_mt_encoder_decoder_reduced_batch():
    """Encoder MGRIT, then decoder MGRIT consuming the encoder output as cross-attention memory."""
    enc = wls.named_workloads()["mt_encoder"].scaled(batch=2)
    dec = wls.named_workloads()["mt_decoder"].scaled(batch=2)
    Zg, Zr, _ = run_case(enc)
    # the decoder of each side consumes that side's own encoder output
    tol = TOL[dec.dtype]
    dm = DeviceModel(dec)
    sh = shape_of(dec)
    Y0 = wls.initial_state(dec)
    opts = mb.mgrit_opts(dec.N, dec.h, dec.cf, dec.levels, dec.iters)
    Yg, rg = mb.mgrit_forward(dm.desc, opts, dev(Y0), dm.blocks, memory=Zg[-1].contiguous())
    torch.cuda.synchronize()
    Yr, rr, _ = omgrit.mgrit_forward(Y0, dm.host, dec.h, dec.cf, dec.levels, dec.iters, sh, Zr[-1])
    _, einc = check_states(Yg, Yr, tol, "Z")
    check_resnorms(rg, rr, tol, Yr, einc)
    # decoder adjoint, both sides linearised about the GPU's decoder states and encoder output
    lamN = wls.terminal_adjoint(dec)
    lg, ag = mb.mgrit_adjoint(dm.desc, opts, Yg, dm.blocks, dev(lamN), memory=Zg[-1].contiguous())
    torch.cuda.synchronize()
    lr, ar, _ = omgrit.mgrit_adjoint(lamN, list(Yg.cpu().numpy()), dm.host, dec.h, dec.cf, dec.levels, dec.iters,
                                     sh, Zg[-1].cpu().numpy())
    _, einc = check_states(lg, lr, tol, "lambda")
    check_resnorms(ag, ar, tol, lr[::-1], einc)


# ----------------------------------------------------------------- deep-narrow shape of the scaling study
@pytest.mark.parametrize("levels,cf,N", [(4, 2, 32), (3, 4, 64)])
def test_deep_narrow_shape_reduced_f_relaxation(levels, cf, N):
    """One head of width 128 (the generic attention kernels), F-relaxation, three and four levels;
    sequence length and batch cut to what the oracle finishes in seconds."""
    wl = wls.named_workloads()["mc_deep_narrow"].scaled(batch=2, seq=192, N=N, h=1.0 / N, cf=cf, levels=levels)
    run_case(wl, relax="F", adjoint=True)


def test_measured_ceilings_are_plausible():
    """The two ceiling measurements run and land between a tenth of and the whole datasheet figure
    (2.5 PFLOP/s dense bf16 MFMA, 8 TB/s HBM)."""
    print("[case] measured ceilings", flush=True)
    a = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    tf = mb.mgrit_measure_mfma_ceiling(b, 2000)
    gbs = mb.mgrit_measure_copy_ceiling(a, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert 250.0 < tf < 2500.0, tf
    assert 800.0 < gbs < 8000.0, gbs
