"""mgrit_forward_linearising + mgrit_adjoint_linearised against the plain mgrit_forward + mgrit_adjoint:
the forward solve's closing relaxation leaves the block internals of the layers it steps through in the
adjoint's workspace, the adjoint evaluates only the others.  Same kernels' arithmetic on the same data, so
Z, lambda, residual norms, parameter gradients and the memory gradient must agree bit for bit.  All three
block types, two and three levels, F and FCF relaxation, a serial run, one and two lanes, with and without
gradients; the stacked encoder-decoder grid (switch layer aligned with the intervals and inside one); buffer
layers; and the argument checks of the entry points."""
import pytest
import torch

from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import DeviceModel, dev

pytestmark = pytest.mark.gpu


def grad_blocks(desc, n):
    nbytes = mb.grad_layout(desc).block_bytes
    return [torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8)
            for _ in range(n)]


def poisoned(nbytes):
    """A workspace full of NaN patterns: an entry of the cache that nobody wrote would show in lambda."""
    return torch.full(((max(nbytes, 256) + 3) // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8)


@pytest.mark.parametrize("arch,dtype,levels,cf,N,relax,lanes,mg,grads", [
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 2, 4, 16, 1, 2, 0, False),
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 2, 4, 16, 1, 2, 0, True),
    (wls.ARCH_CAUSAL, wls.DTYPE_BF16, 3, 2, 16, 1, 2, 3, True),
    (wls.ARCH_CAUSAL, wls.DTYPE_BF16, 3, 4, 32, 0, 2, 2, False),
    (wls.ARCH_CROSS, wls.DTYPE_BF16, 2, 4, 16, 1, 2, 0, True),
    (wls.ARCH_CROSS, wls.DTYPE_BF16, 2, 2, 8, 0, 1, 0, False),
    (wls.ARCH_CAUSAL, wls.DTYPE_F32, 2, 4, 8, 1, 1, 0, True),
    (wls.ARCH_ENCODER, wls.DTYPE_F32, 2, 2, 8, 1, 2, 0, False),
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 1, 4, 5, 1, 2, 0, True),
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 2, 4, 40, 1, 2, 1, False)])
def test_linearising_pair_equals_plain_pair(arch, dtype, levels, cf, N, relax, lanes, mg, grads):
    wl = wls.Workload("t", arch, 128, 2, 256, 2, 40, 24 if arch == wls.ARCH_CROSS else 0, N, 0.5, cf, levels, 2,
                      dtype, 91, relax=relax)
    print(f"[case] linearising arch={arch} dtype={dtype} L={levels} cf={cf} N={N} relax={relax} lanes={lanes} "
          f"mg={mg} grads={grads}", flush=True)
    dm = DeviceModel(wl, weight_std=0.05, keep_host=False)
    opts = mb.mgrit_opts(N, wl.h, cf, levels, 2, relax)
    mem = wls.cross_memory(wl)
    mem = None if mem is None else dev(mem)
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))
    mb.mgrit_set_lanes(lanes)
    mb.mgrit_set_max_groups_per_launch(mg)
    try:
        def adjoint(Z, ws, linearised):
            gb = grad_blocks(dm.desc, N) if grads else None
            dmem = torch.full_like(mem, float("nan")) if (grads and mem is not None) else None
            lam, res = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN, memory=mem, dtheta=gb, dmemory=dmem,
                                        workspace=ws, linearised=linearised)
            torch.cuda.synchronize()
            return [lam, res] + (gb or []) + ([dmem] if dmem is not None else [])

        need = mb.mgrit_workspace_bytes(dm.desc, opts, 2 if grads else 1)
        Zp, rp = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, memory=mem)
        plain = [Zp, rp] + adjoint(Zp, poisoned(need), False)
        for rep in range(2):                                  # the second time over a workspace already used
            ws = poisoned(need) if rep == 0 else ws
            Zl, rl = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, memory=mem, adjoint_workspace=ws,
                                      with_gradients=grads)
            shared = [Zl, rl] + adjoint(Zl, ws, True)
            assert len(shared) == len(plain)
            for i, (x, y) in enumerate(zip(plain, shared)):
                assert torch.equal(x, y), f"output {i} differs (repetition {rep})"
        for x in plain:
            assert torch.isfinite(x.float() if x.dtype != torch.uint8 else x.view(torch.float32)).all()
    finally:
        mb.mgrit_set_lanes(2)
        mb.mgrit_set_max_groups_per_launch(0)


def test_linearising_entry_points_check_their_arguments():
    wl = wls.Workload("t", wls.ARCH_ENCODER, 128, 2, 256, 2, 40, 0, 8, 0.5, 4, 2, 2, wls.DTYPE_BF16, 92)
    print("[case] linearising: argument checks", flush=True)
    dm = DeviceModel(wl, weight_std=0.05, keep_host=False)
    opts = mb.mgrit_opts(8, wl.h, 4, 2, 2)
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))
    need1, need2 = mb.mgrit_workspace_bytes(dm.desc, opts, 1), mb.mgrit_workspace_bytes(dm.desc, opts, 2)
    assert need2 > need1
    small = torch.empty(need1, dtype=torch.uint8, device="cuda")
    with pytest.raises(mb.MgritError) as e:                   # a gradient run needs the larger adjoint workspace
        mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, adjoint_workspace=small, with_gradients=True)
    assert e.value.status == mb.MGRIT_WORKSPACE_TOO_SMALL
    mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, adjoint_workspace=small, with_gradients=False)
    torch.cuda.synchronize()
    try:                                                      # without the N-layer cache there is nothing to share
        mb.mgrit_set_adjoint_cache(False)
        ws = torch.empty(need2, dtype=torch.uint8, device="cuda")
        with pytest.raises(mb.MgritError) as e:
            mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, adjoint_workspace=ws)
        assert e.value.status == mb.MGRIT_INVALID_ARG
        Z, _ = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks)
        with pytest.raises(mb.MgritError) as e:
            mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN, workspace=ws, linearised=True)
        assert e.value.status == mb.MGRIT_INVALID_ARG
    finally:
        mb.mgrit_set_adjoint_cache(True)
    torch.cuda.synchronize()


@pytest.mark.parametrize("n_enc,n_dec,cf,levels,relax,dtype,lanes,mg,grads", [
    (8, 8, 4, 2, 1, wls.DTYPE_BF16, 2, 0, False),
    (6, 10, 4, 2, 1, wls.DTYPE_BF16, 2, 0, True),           # the decoder starts inside a coarse interval
    (3, 13, 4, 3, 0, wls.DTYPE_BF16, 2, 2, True),           # no encoder layer is left to the adjoint's own pass
    (10, 6, 2, 2, 1, wls.DTYPE_F32, 1, 3, False),
    (5, 4, 4, 1, 1, wls.DTYPE_BF16, 2, 0, True)])           # serial run: the forward solve leaves every layer
def test_linearising_pair_equals_plain_pair_on_the_stacked_grid(n_enc, n_dec, cf, levels, relax, dtype, lanes, mg,
                                                                grads):
    enc = wls.Workload("enc", wls.ARCH_ENCODER, 128, 2, 256, 2, 24, 0, n_enc, 0.5, cf, levels, 2, dtype, 93,
                       relax=relax)
    dec = wls.Workload("dec", wls.ARCH_CROSS, 128, 2, 256, 2, 20, 24, n_dec, 0.5, cf, levels, 2, dtype, 94,
                       relax=relax)
    sw = wls.StackedWorkload("stacked", enc, dec)
    print(f"[case] linearising, stacked grid n_enc={n_enc} n_dec={n_dec} cf={cf} L={levels} relax={relax} "
          f"dtype={dtype} lanes={lanes} mg={mg} grads={grads}", flush=True)
    desc_d = mb.model_desc(dec)
    desc_e = mb.encoder_desc(desc_d)
    blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, wls.stacked_layer_params(sw, n, 0.05))
              for n in range(sw.N)]
    opts = mb.mgrit_opts(sw.N, dec.h, cf, levels, 2, relax)
    Z0, lamN = dev(wls.stacked_initial_state(sw)), dev(wls.stacked_terminal_adjoint(sw))
    mb.mgrit_set_lanes(lanes)
    mb.mgrit_set_max_groups_per_launch(mg)
    try:
        def adjoint(Z, ws, linearised):
            gb = None
            if grads:
                gb = [torch.full((mb.grad_layout(desc_e if n < sw.n_enc else desc_d).block_bytes // 4,), float("nan"),
                                 dtype=torch.float32, device="cuda").view(torch.uint8) for n in range(sw.N)]
            lam, res = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Z, blocks, lamN, dtheta=gb, workspace=ws,
                                                linearised=linearised)
            torch.cuda.synchronize()
            return [lam, res] + (gb or [])

        need = mb.mgrit_stacked_workspace_bytes(desc_d, opts, sw.n_enc, 2 if grads else 1)
        Zp, rp = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, Z0, blocks)
        plain = [Zp, rp] + adjoint(Zp, poisoned(need), False)
        ws = poisoned(need)
        for rep in range(2):
            Zl, rl = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, Z0, blocks, adjoint_workspace=ws,
                                              with_gradients=grads)
            shared = [Zl, rl] + adjoint(Zl, ws, True)
            for i, (x, y) in enumerate(zip(plain, shared)):
                assert torch.equal(x, y), f"output {i} differs (repetition {rep})"
        for x in plain:
            assert torch.isfinite(x.float() if x.dtype != torch.uint8 else x.view(torch.float32)).all()
    finally:
        mb.mgrit_set_lanes(2)
        mb.mgrit_set_max_groups_per_launch(0)


@pytest.mark.parametrize("arch,n_open,n_close,grads", [(wls.ARCH_CAUSAL, 2, 2, True), (wls.ARCH_ENCODER, 0, 3, False),
                                                       (wls.ARCH_CROSS, 1, 0, False)])
def test_linearising_pair_equals_plain_pair_with_buffer_layers(arch, n_open, n_close, grads):
    wl = wls.Workload("t", arch, 128, 2, 256, 2, 40, 24 if arch == wls.ARCH_CROSS else 0, 8, 0.25, 4, 2, 2,
                      wls.DTYPE_BF16, 95)
    print(f"[case] linearising, buffer layers arch={arch} open={n_open} close={n_close} grads={grads}", flush=True)
    n = n_open + 8 + n_close
    dm = DeviceModel(wl, n_layers=n, weight_std=0.05, keep_host=False)
    opts = mb.mgrit_opts(8, wl.h, 4, 2, 2)
    buf = mb.BufferOpts(n_open, n_close, 1.0)
    mem = wls.cross_memory(wl)
    mem = None if mem is None else dev(mem)
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))

    def adjoint(Z, ws, linearised):
        gb = grad_blocks(dm.desc, n) if grads else None
        lam, res = mb.mgrit_adjoint_buffered(dm.desc, opts, buf, Z, dm.blocks, lamN, memory=mem, dtheta=gb,
                                             workspace=ws, linearised=linearised)
        torch.cuda.synchronize()
        return [lam, res] + (gb or [])

    Zp, rp = mb.mgrit_forward_buffered(dm.desc, opts, buf, Z0, dm.blocks, memory=mem)
    plain = [Zp, rp] + adjoint(Zp, None, False)
    need = mb.mgrit_buffered_linearised_workspace_bytes(dm.desc, opts, buf, grads)
    assert need >= mb.mgrit_buffered_workspace_bytes(dm.desc, opts, buf, 2 if grads else 1)
    ws = poisoned(need)
    for rep in range(2):
        Zl, rl = mb.mgrit_forward_buffered(dm.desc, opts, buf, Z0, dm.blocks, memory=mem, adjoint_workspace=ws,
                                           with_gradients=grads)
        shared = [Zl, rl] + adjoint(Zl, ws, True)
        for i, (x, y) in enumerate(zip(plain, shared)):
            assert torch.equal(x, y), f"output {i} differs (repetition {rep})"
    for x in plain:
        assert torch.isfinite(x.float() if x.dtype != torch.uint8 else x.view(torch.float32)).all()
    with pytest.raises(mb.MgritError) as e:                   # one region per segment: the shared size is too small
        small = torch.empty(max(need - 256, 256), dtype=torch.uint8, device="cuda")
        mb.mgrit_forward_buffered(dm.desc, opts, buf, Z0, dm.blocks, memory=mem, adjoint_workspace=small,
                                  with_gradients=grads)
    assert e.value.status == mb.MGRIT_WORKSPACE_TOO_SMALL
