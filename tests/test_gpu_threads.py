"""Two host threads call the library at the same time, each on its own stream with its own buffers:
the entry points serialise while they enqueue (the helper lane of the two-lane mode exists once per
device), and both calls give the results of the same calls made one after the other, bit for bit."""
import threading

import pytest
import torch

from paper_2601_09026_amd import binding as mb
from paper_2601_09026_amd import workloads as wls

from gpu_util import DeviceModel, dev

pytestmark = pytest.mark.gpu


def test_concurrent_calls_from_two_host_threads():
    print("[case] two host threads, two streams", flush=True)
    wls_ = [wls.Workload("a", wls.ARCH_CAUSAL, 128, 2, 256, 2, 40, 0, 32, 0.1, 4, 2, 2, wls.DTYPE_BF16, 91),
            wls.Workload("b", wls.ARCH_ENCODER, 256, 4, 512, 3, 50, 0, 16, 0.2, 2, 3, 2, wls.DTYPE_BF16, 92)]
    jobs = []
    for wl in wls_:
        dm = DeviceModel(wl, weight_std=0.05, keep_host=False)
        opts = mb.mgrit_opts(wl.N, wl.h, wl.cf, wl.levels, wl.iters)
        jobs.append((dm, opts, dev(wls.initial_state(wl)), dev(wls.terminal_adjoint(wl))))

    def run(job, stream):
        dm, opts, Z0, lamN = job
        with torch.cuda.stream(stream):
            Z, rz = mb.mgrit_forward(dm.desc, opts, Z0, dm.blocks, stream=stream)
            lam, rl = mb.mgrit_adjoint(dm.desc, opts, Z, dm.blocks, lamN, stream=stream)
        return [Z, rz, lam, rl]

    torch.cuda.synchronize()
    ref = [run(j, torch.cuda.current_stream()) for j in jobs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        got = [None, None]
        errors = []

        def worker(i):
            try:
                torch.cuda.set_device(0)
                for _ in range(2):                  # several calls per thread, so that the enqueues interleave
                    got[i] = run(jobs[i], streams[i])
            except Exception as e:                  # noqa: BLE001
                errors.append(e)
        threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        assert not errors, errors
        for g, r in zip(got, ref):
            for x, y in zip(g, r):
                assert torch.equal(x, y), f"repetition {rep}"
