"""A whole forward + adjoint step can be captured into a HIP graph by the caller (the library only
enqueues kernels, device-to-device copies and its fork/join events on the streams involved) and
replayed: every replay, with eager work and synchronisations between them, reproduces the eager
result bit for bit."""
import pytest
import torch

from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import DeviceModel, dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("grads", [False, True])
@pytest.mark.parametrize("dtype", [wls.DTYPE_F32, wls.DTYPE_BF16])
def test_captured_step_replays_bit_identically(dtype, grads):
    wl = wls.Workload("cap", wls.ARCH_CAUSAL, 128, 2, 256, 2, 32, 0, 16, 1.0 / 16, 4, 2, 2, dtype, 51)
    print(f"[case] graph capture dtype={dtype} grads={grads}", flush=True)
    dm = DeviceModel(wl, weight_std=0.05)
    opts = mb.mgrit_opts(wl.N, wl.h, wl.cf, wl.levels, wl.iters)
    T, d = wl.tokens, wl.d_model
    Z0, lamN = dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))
    Z_all = torch.empty((wl.N + 1, T, d), device="cuda")
    lam_all = torch.empty_like(Z_all)
    rf, ra = torch.zeros(2, device="cuda"), torch.zeros(2, device="cuda")
    ws = torch.empty(max(mb.mgrit_workspace_bytes(dm.desc, opts, 0),
                         mb.mgrit_workspace_bytes(dm.desc, opts, 2 if grads else 1)),
                     dtype=torch.uint8, device="cuda")
    # parameter gradients: emitted by the closing relaxation and by the pass over the remaining layers
    gblocks = None
    if grads:
        nbytes = mb.grad_layout(dm.desc).block_bytes
        gblocks = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(wl.N)]

    def step():
        s = torch.cuda.current_stream()
        mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, Z_all=Z_all, resnorm=rf, workspace=ws, stream=s)
        mb.mgrit_adjoint(dm.desc, opts, Z_all, dm.blocks, lamN, lambda_all=lam_all, resnorm=ra, workspace=ws, stream=s,
                         dtheta=gblocks)

    step()
    torch.cuda.synchronize()
    outs = [Z_all, lam_all, rf, ra] + (gblocks or [])
    want = [t.clone() for t in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()
    for i in range(3):
        for t in outs:
            t.fill_(i + 1)                           # eager work between replays; results must not survive
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), f"replay {i}"
