"""The adjoint without its N-layer linearisation cache (mgrit_set_adjoint_cache(0): every launch chunk
recomputes the block internals of its own layers): identical results, bit for bit, to the cached run --
the same kernels on the same data -- with a workspace smaller by the cache.  All three block types,
three levels, parameter gradients and the memory gradient, the stacked grid, buffer layers."""
import numpy as np
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


def both_modes(run):
    out = []
    try:
        for cache in (True, False, True):
            mb.mgrit_set_adjoint_cache(cache)
            out.append(run())
            torch.cuda.synchronize()
    finally:
        mb.mgrit_set_adjoint_cache(True)
    for other in out[1:]:
        for x, y in zip(out[0], other):
            assert torch.equal(x, y)
    for x in out[0]:
        assert torch.isfinite(x.float() if x.dtype != torch.uint8 else x.view(torch.float32)).all()


@pytest.mark.parametrize("arch,dtype,levels,cf,N,lanes,mg", [
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 2, 4, 16, 2, 0), (wls.ARCH_CAUSAL, wls.DTYPE_BF16, 3, 2, 16, 2, 3),
    (wls.ARCH_CROSS, wls.DTYPE_BF16, 2, 4, 16, 2, 0), (wls.ARCH_CAUSAL, wls.DTYPE_F32, 2, 4, 8, 1, 0),
    (wls.ARCH_ENCODER, wls.DTYPE_BF16, 1, 4, 5, 2, 0)])
def test_recompute_equals_cached(arch, dtype, levels, cf, N, lanes, mg):
    wl = wls.Workload("t", arch, 128, 2, 256, 2, 40, 24 if arch == wls.ARCH_CROSS else 0, N, 0.5, cf, levels, 2,
                      dtype, 83)
    print(f"[case] recompute arch={arch} dtype={dtype} L={levels} cf={cf} N={N} lanes={lanes} mg={mg}", flush=True)
    dm = DeviceModel(wl, weight_std=0.05, keep_host=False)
    opts = mb.mgrit_opts(N, wl.h, cf, levels, 2)
    mem = wls.cross_memory(wl)
    mem = None if mem is None else dev(mem)
    Z, _ = mb.mgrit_forward(dm.desc, opts, dev(wls.initial_state(wl)), dm.blocks, memory=mem)
    lamN = dev(wls.terminal_adjoint(wl))
    mb.mgrit_set_lanes(lanes)
    mb.mgrit_set_max_groups_per_launch(mg)
    try:
        sizes = []
        for cache in (True, False):
            mb.mgrit_set_adjoint_cache(cache)
            sizes.append((mb.mgrit_workspace_bytes(dm.desc, opts, 1), mb.mgrit_workspace_bytes(dm.desc, opts, 2)))
        mb.mgrit_set_adjoint_cache(True)
        if N > 8:
            assert sizes[1][0] < sizes[0][0] and sizes[1][1] < sizes[0][1], sizes

        def run():
            gb = grad_blocks(dm.desc, N)
            dmem = torch.full_like(mem, float("nan")) if mem is not None else None
            lam, res = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN, memory=mem, dtheta=gb, dmemory=dmem)
            lam2, res2 = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN, memory=mem)
            return [lam, res, lam2, res2] + gb + ([dmem] if dmem is not None else [])
        both_modes(run)
    finally:
        mb.mgrit_set_lanes(2)
        mb.mgrit_set_max_groups_per_launch(0)


def test_recompute_equals_cached_on_the_stacked_grid():
    enc = wls.Workload("enc", wls.ARCH_ENCODER, 128, 2, 256, 2, 24, 0, 6, 0.5, 4, 2, 2, wls.DTYPE_BF16, 84)
    dec = wls.Workload("dec", wls.ARCH_CROSS, 128, 2, 256, 2, 20, 24, 10, 0.5, 4, 2, 2, wls.DTYPE_BF16, 85)
    sw = wls.StackedWorkload("stacked", enc, dec)
    print(f"[case] recompute, stacked grid N={sw.N} n_enc={sw.n_enc}", flush=True)
    desc_d = mb.model_desc(dec)
    desc_e = mb.encoder_desc(desc_d)
    blocks = [mb.pack_theta(desc_e if n < sw.n_enc else desc_d, wls.stacked_layer_params(sw, n, 0.05))
              for n in range(sw.N)]
    opts = mb.mgrit_opts(sw.N, dec.h, dec.cf, dec.levels, dec.iters, dec.relax)
    Z, _ = mb.mgrit_forward_stacked(desc_d, opts, sw.n_enc, dev(wls.stacked_initial_state(sw)), blocks)
    lamN = dev(wls.stacked_terminal_adjoint(sw))

    def run():
        gb = [torch.full((mb.grad_layout(desc_e if n < sw.n_enc else desc_d).block_bytes // 4,), float("nan"),
                         dtype=torch.float32, device="cuda").view(torch.uint8) for n in range(sw.N)]
        lam, res = mb.mgrit_adjoint_stacked(desc_d, opts, sw.n_enc, Z, blocks, lamN, dtheta=gb)
        return [lam, res] + gb
    both_modes(run)


def test_recompute_equals_cached_with_buffer_layers():
    wl = wls.Workload("t", wls.ARCH_CAUSAL, 128, 2, 256, 2, 40, 0, 8, 0.25, 4, 2, 2, wls.DTYPE_BF16, 86)
    print("[case] recompute, buffer layers", flush=True)
    dm = DeviceModel(wl, n_layers=12, weight_std=0.05, keep_host=False)
    opts = mb.mgrit_opts(8, wl.h, 4, 2, 2)
    buf = mb.BufferOpts(2, 2, 1.0)
    Z, _ = mb.mgrit_forward_buffered(dm.desc, opts, buf, dev(wls.initial_state(wl)), dm.blocks)
    lamN = dev(wls.terminal_adjoint(wl))

    def run():
        lam, res = mb.mgrit_adjoint_buffered(dm.desc, opts, buf, Z, dm.blocks, lamN)
        return [lam, res]
    both_modes(run)
