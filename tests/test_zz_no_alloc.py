"""layer_step_batched_static -- the batched layer step on the library's own fixed scratch array, for
callers that cannot allocate -- against layer_step_batched on a caller workspace: forward and
adjoint, two calls in a row on the same GPU with the second one smaller (it finds the first call's
leftovers in the scratch array), bit for bit against the single-lane run of the existing entry
point and within the dtype's tolerance against its default (two-lane) run.  Sizes beyond the
array are refused before anything is enqueued."""
import numpy as np
import pytest
import torch

from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import TOL, DeviceModel, dev, relerr

pytestmark = pytest.mark.gpu


def case(arch, dtype, d, H, f, B, S, Sm, G, seed):
    wl = wls.Workload("t", arch, d, H, f, B, S, Sm if arch == wls.ARCH_CROSS else 0, 4, 0.25, 2, 2, 1, dtype, seed)
    dm = DeviceModel(wl, n_layers=G, weight_std=0.05, keep_host=False)
    rng = np.random.default_rng(seed)
    T = wl.tokens
    ins = [dev(rng.standard_normal((T, d))) for _ in range(G)]
    lin = [dev(rng.standard_normal((T, d))) for _ in range(G)]
    rhs = [dev(0.1 * rng.standard_normal((T, d))) for _ in range(G)]
    mem = wls.cross_memory(wl)
    return wl, dm, ins, lin, rhs, None if mem is None else dev(mem)


def run_pair(arch, dtype, d, H, f, B, S, Sm, G, seed, adjoint):
    wl, dm, ins, lin, rhs, mem = case(arch, dtype, d, H, f, B, S, Sm, G, seed)
    need = mb.mgrit_layer_step_static_bytes(dm.desc, adjoint, G)
    print(f"[case] static scratch arch={arch} dtype={dtype} d={d} B={B} S={S} G={G} adjoint={adjoint} "
          f"needs {need} of {mb.STATIC_SCRATCH_BYTES} bytes", flush=True)
    assert 0 < need <= mb.STATIC_SCRATCH_BYTES
    kw = dict(rhs=rhs, memory=mem, lin_state=lin if adjoint else None)
    got = [torch.full_like(t, float("nan")) for t in ins]
    mb.layer_step_batched_static(dm.desc, adjoint, ins, got, dm.blocks, 0.37, **kw)
    torch.cuda.synchronize()
    two_lane = [torch.full_like(t, float("nan")) for t in ins]
    mb.layer_step_batched(dm.desc, adjoint, ins, two_lane, dm.blocks, 0.37, **kw)
    torch.cuda.synchronize()
    one_lane = [torch.full_like(t, float("nan")) for t in ins]
    mb.mgrit_set_lanes(1)
    try:
        mb.layer_step_batched(dm.desc, adjoint, ins, one_lane, dm.blocks, 0.37, **kw)
        torch.cuda.synchronize()
    finally:
        mb.mgrit_set_lanes(2)
    for g in range(G):
        assert torch.isfinite(got[g]).all()
        assert torch.equal(got[g], one_lane[g]), f"group {g}: differs from the workspace entry point"
        base = (ins[g] + rhs[g]).double().cpu().numpy()
        e = relerr(got[g].double().cpu().numpy() - base, two_lane[g].double().cpu().numpy() - base)
        assert e <= TOL[dtype], f"group {g}: increment differs from the two-lane run by {e:.2e}"


@pytest.mark.parametrize("adjoint", [False, True])
def test_two_calls_in_a_row_second_smaller(adjoint):
    # bf16 causal, several GEMM tiles with a ragged tail, 5 groups (launch chunks of 4 + 1 or 5) ...
    run_pair(wls.ARCH_CAUSAL, wls.DTYPE_BF16, 256, 4, 512, 3, 50, 0, 5, 71, adjoint)
    # ... then a smaller problem of another block type and dtype on the same scratch array
    run_pair(wls.ARCH_CROSS, wls.DTYPE_F32, 64, 4, 128, 2, 20, 12, 2, 72, adjoint)
    # and the first size again: what the small call left behind must not matter either
    run_pair(wls.ARCH_CAUSAL, wls.DTYPE_BF16, 256, 4, 512, 3, 50, 0, 5, 71, adjoint)


def test_sizes_beyond_the_array_are_refused():
    wl = wls.named_workloads()["bert_base"]
    desc = mb.model_desc(wl)
    assert mb.mgrit_layer_step_static_bytes(desc, False, 6) > mb.STATIC_SCRATCH_BYTES
    x = torch.zeros((wl.tokens, wl.d_model), device="cuda")
    out = torch.full_like(x, 7.0)
    blk = torch.zeros(mb.mgrit_theta_layout(desc).block_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(mb.MgritError) as e:
        mb.layer_step_batched_static(desc, False, [x] * 6, [out] * 6, [blk] * 6, 0.1)
    assert e.value.status == mb.MGRIT_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


def test_one_full_size_step_of_every_benchmark_shape_fits():
    for wl in wls.named_workloads().values():
        desc = mb.model_desc(wl)
        for adjoint in (False, True):
            assert 0 < mb.mgrit_layer_step_static_bytes(desc, adjoint, 1) <= mb.STATIC_SCRATCH_BYTES, wl.name


@pytest.mark.parametrize("adjoint", [False, True])
def test_one_full_size_bert_step(adjoint):
    """One interval at the BERT shape (66 / 170 MiB of scratch), then a small call after it."""
    wl = wls.named_workloads()["bert_base"]
    run_pair(wl.arch, wl.dtype, wl.d_model, wl.n_heads, wl.d_ff, wl.batch, wl.seq, 0, 1, 73, adjoint)
    run_pair(wls.ARCH_ENCODER, wls.DTYPE_BF16, 128, 2, 256, 2, 40, 0, 3, 74, adjoint)
