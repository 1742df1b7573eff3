#!/usr/bin/env python3
"""Benchmark of the MGRIT hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
mgrit_forward followed by mgrit_adjoint (linearised about the forward result) at the named
workload; the default is the largest benchmark configuration that runs forward + adjoint, the
GPT-2-small shape (causal, 128 layers, three levels).  The headline value is layer-steps*tokens/s = (Phi + Psi evaluations enqueued on
all levels) x (batch*seq) / wall time, with all inputs resident in HBM before the timed
region.  The pair of calls is mgrit_forward_linearising + mgrit_adjoint_linearised (the forward
solve's closing relaxation leaves the internals of the layers it steps through to the adjoint; results
identical to the plain pair, --plain-pair); what is left of the adjoint's linearisation pass is timed
but not counted as evaluations.

Prints ONE JSON line: metric, value, timing, the workload in `config`, `roofline` of the dominant
kernel and `cpu_baseline` (the oracle timed on the host).  Everything runs on one GPU;
--gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
from ctypes import byref as C_byref

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2_small",
                    help="tiny_encoder | bert_base | gpt2_small | vit_small | mt_encoder | mt_decoder | "
                         "mc_deep_narrow | mt_stacked (encoder and decoder on one grid)")
    ap.add_argument("--no-adjoint", action="store_true", help="time mgrit_forward only")
    ap.add_argument("--layers", type=int, default=0, help="parameter study: override N (h becomes 1/N)")
    ap.add_argument("--cf", type=int, default=0, help="parameter study: override the coarsening factor")
    ap.add_argument("--levels", type=int, default=0, help="parameter study: override the number of levels")
    ap.add_argument("--iters", type=int, default=0, help="parameter study: override the number of cycles")
    ap.add_argument("--seq", type=int, default=0, help="parameter study: override the sequence length")
    ap.add_argument("--batch", type=int, default=0, help="parameter study: override the batch size")
    ap.add_argument("--max-groups", type=int, default=0, help="groups per kernel launch (0 = library default)")
    ap.add_argument("--lanes", type=int, default=0, help="1 = single stream, 2 = two lanes (0 = library default)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one step captured into a HIP graph instead of eager launches")
    ap.add_argument("--gemm-tile", type=int, default=0, help="tuning: force a GEMM tile configuration (0 = by shape)")
    ap.add_argument("--param-grads", action="store_true",
                    help="also produce the parameter gradients in every step (not part of the headline metric: "
                         "the line then says so in `metric` and in config.param_grads)")
    ap.add_argument("--attn-wide", type=int, default=-1,
                    help="tuning: mask of d_head=128 attention kernels with 256-row blocks (1 fwd, 2 dQ, 4 dK/dV)")
    ap.add_argument("--pipe-chunk", type=int, default=0, help="tuning: intervals per hand-over of the coarse solve")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="tuning: serial coarse solve and the following F-relaxation one after the other")
    ap.add_argument("--plain-pair", action="store_true",
                    help="mgrit_forward + mgrit_adjoint instead of mgrit_forward_linearising + "
                         "mgrit_adjoint_linearised (the adjoint then evaluates the internals of all N layers itself)")
    ap.add_argument("--no-adjoint-cache", action="store_true",
                    help="adjoint without the N-layer linearisation cache (recomputed per launch chunk)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not record per-kernel HIP events in the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0,
                    help="budget of the oracle timing sample (half at all host threads, half at one)")
    ap.add_argument("--breakdown", action="store_true", help="print a per-kernel-class table to stderr")
    return ap.parse_args()


def oracle_sample(wl, n_phi, n_psi, budget_s, max_pairs):
    """Layer steps of the fp64 numpy oracle (as it stands) at the workload's full shape for about
    budget_s seconds; the per-step times are weighted by the evaluation counts of one bench step."""
    from oracle import transformer_ode as tode
    from paper_2601_09026_amd import workloads as wls
    sh = tode.Shape(wl.arch, wl.d_model, wl.n_heads, wl.batch, wl.seq, wl.mem_seq, wl.ln_eps)
    th = wls.layer_params(wl, 0)
    Z = wls.initial_state(wl).astype(np.float64)
    lam = wls.terminal_adjoint(wl).astype(np.float64)
    mem = wls.cross_memory(wl)
    t_phi, t_psi, n1, n2 = 0.0, 0.0, 0, 0
    t0 = time.perf_counter()
    while True:
        t = time.perf_counter(); Z = tode.phi(Z, th, wl.h, sh, mem); t_phi += time.perf_counter() - t; n1 += 1
        if n_psi:
            t = time.perf_counter(); lam = tode.psi(lam, Z, th, wl.h, sh, mem); t_psi += time.perf_counter() - t
            n2 += 1
        if time.perf_counter() - t0 > budget_s or n1 >= max_pairs:
            break
    est = n_phi * (t_phi / n1) + (n_psi * (t_psi / n2) if n2 else 0.0)
    return {"value": (n_phi + n_psi) * wl.tokens / est, "n_forward": n1, "n_adjoint": n2,
            "s_per_forward_step": t_phi / n1, "s_per_adjoint_step": (t_psi / n2) if n2 else None}


def cpu_baseline(wl, n_phi, n_psi, budget_s):
    """The oracle timed on the host: at all the threads its BLAS uses (the headline `value`, `cores`) and
    at one thread (`single_thread`), each on a bounded sample of the same workload."""
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    full = oracle_sample(wl, n_phi, n_psi, budget_s / 2, 64)
    out = {"value": full["value"], "unit": "layer-steps*tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{full['n_forward']} forward + {full['n_adjoint']} adjoint layer steps of the fp64 numpy oracle at "
                     f"the full {wl.name} shape (T={wl.tokens}); per-step times weighted by the step's "
                     f"{n_phi} forward / {n_psi} adjoint evaluations",
           "s_per_forward_step": full["s_per_forward_step"], "s_per_adjoint_step": full["s_per_adjoint_step"]}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            one = oracle_sample(wl, n_phi, n_psi, budget_s / 2, 8)
        out["single_thread"] = {"value": one["value"], "unit": "layer-steps*tokens/s", "cores": 1,
                                "sample": f"{one['n_forward']} forward + {one['n_adjoint']} adjoint layer steps, same shape",
                                "s_per_forward_step": one["s_per_forward_step"],
                                "s_per_adjoint_step": one["s_per_adjoint_step"]}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2601_09026_amd import binding as mb
    from paper_2601_09026_amd import workloads as wls

    sw = wls.stacked_workloads().get(args.workload)        # encoder + decoder on one grid, or None
    wl = sw.dec.scaled(name=sw.name, N=sw.N) if sw else wls.named_workloads()[args.workload]
    overridden = bool(args.layers or args.cf or args.levels or args.iters or args.seq or args.batch)
    if overridden:
        if sw:
            print("bench.py: the parameter-study overrides apply to the single-network workloads", file=sys.stderr)
            sys.exit(2)
        n_layers = args.layers or wl.N
        wl = wl.scaled(N=n_layers, h=1.0 / n_layers, cf=args.cf or wl.cf, levels=args.levels or wl.levels,
                       iters=args.iters or wl.iters, seq=args.seq or wl.seq, batch=args.batch or wl.batch)
    adjoint = not args.no_adjoint
    torch.cuda.set_device(0)
    if args.max_groups:
        mb.mgrit_set_max_groups_per_launch(args.max_groups)
    if args.lanes:
        mb.mgrit_set_lanes(args.lanes)
    if args.attn_wide >= 0:
        mb.lib().mgrit_debug_attention_wide_blocks(args.attn_wide)
    if args.pipe_chunk:
        mb.lib().mgrit_debug_pipeline_chunk(args.pipe_chunk)
    if args.no_pipeline:
        mb.lib().mgrit_debug_pipeline_coarse_solve(0)
    if args.gemm_tile:
        mb.lib().mgrit_debug_gemm_tile_config(args.gemm_tile)
    if args.no_adjoint_cache:
        mb.mgrit_set_adjoint_cache(False)
    desc = mb.model_desc(wl)
    opts = mb.mgrit_opts(wl.N, wl.h, wl.cf, wl.levels, wl.iters, wl.relax)
    # stacked grid: a state holds the encoder's and the decoder's tokens, an evaluation advances one
    # of the two parts (equally many tokens in this workload), which is what the metric counts
    T, d = (sw.tokens if sw else wl.tokens), wl.d_model
    if sw:
        assert sw.enc.tokens == sw.dec.tokens
    T_eval = wl.tokens

    # inputs resident in HBM before anything is timed
    if sw:
        desc_e = mb.encoder_desc(desc)
        theta = [mb.pack_theta(desc_e if n < sw.n_enc else desc, wls.stacked_layer_params(sw, n)) for n in range(sw.N)]
        Z0 = torch.from_numpy(wls.stacked_initial_state(sw)).cuda()
        lamN = torch.from_numpy(wls.stacked_terminal_adjoint(sw)).cuda()
    else:
        theta = [mb.pack_theta(desc, wls.layer_params(wl, n)) for n in range(wl.N)]
        Z0 = torch.from_numpy(wls.initial_state(wl)).cuda()
        lamN = torch.from_numpy(wls.terminal_adjoint(wl)).cuda()
    mem = None if sw else wls.cross_memory(wl)
    mem = None if mem is None else torch.from_numpy(mem).cuda()
    Z_all = torch.empty((wl.N + 1, T, d), dtype=torch.float32, device="cuda")
    lam_all = torch.empty_like(Z_all) if adjoint else None
    res_f = torch.zeros(max(wl.iters, 1), dtype=torch.float32, device="cuda")
    res_a = torch.zeros(max(wl.iters, 1), dtype=torch.float32, device="cuda")
    grads = None
    if args.param_grads:
        if not adjoint or (wl.arch == wls.ARCH_CROSS and not sw):
            print("bench.py: --param-grads needs the adjoint and an encoder or causal workload", file=sys.stderr)
            sys.exit(2)
        gbytes = [mb.grad_layout(desc_e if sw and n < sw.n_enc else desc).block_bytes for n in range(wl.N)]
        grads = [torch.empty(b, dtype=torch.uint8, device="cuda") for b in gbytes]
    if sw:
        ws_bytes = max(mb.mgrit_stacked_workspace_bytes(desc, opts, sw.n_enc, 0),
                       mb.mgrit_stacked_workspace_bytes(desc, opts, sw.n_enc, 2 if grads else 1) if adjoint else 0, 256)
    else:
        ws_bytes = max(mb.mgrit_workspace_bytes(desc, opts, 0),
                       mb.mgrit_workspace_bytes(desc, opts, 2 if grads else 1) if adjoint else 0, 256)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    # the linearising pair: the forward solve writes into the adjoint's workspace, so it needs one of its own
    shared = adjoint and not args.plain_pair and not args.no_adjoint_cache
    ws_fwd = ws
    if shared:
        fwd_bytes = mb.mgrit_stacked_workspace_bytes(desc, opts, sw.n_enc, 0) if sw else mb.mgrit_workspace_bytes(desc, opts, 0)
        ws_fwd = torch.empty(max(fwd_bytes, 256), dtype=torch.uint8, device="cuda")
        ws_bytes += ws_fwd.numel()
    n_phi = mb.mgrit_step_evaluations(opts)
    n_psi = n_phi if adjoint else 0
    stream = torch.cuda.current_stream()

    def step_stacked(stream):
        mb.mgrit_forward_stacked(desc, opts, sw.n_enc, Z0, theta, Z_all=Z_all, resnorm=res_f, workspace=ws_fwd,
                                 stream=stream, adjoint_workspace=ws if shared else None,
                                 with_gradients=bool(grads))
        if adjoint:
            mb.mgrit_adjoint_stacked(desc, opts, sw.n_enc, Z_all, theta, lamN, dtheta=grads, lambda_all=lam_all,
                                     resnorm=res_a, workspace=ws, stream=stream, linearised=shared)

    def step(stream=stream):
        if sw:
            return step_stacked(stream)
        mb.mgrit_forward(desc, opts, Z0, theta, memory=mem, Z_all=Z_all, resnorm=res_f, workspace=ws_fwd,
                         stream=stream, adjoint_workspace=ws if shared else None, with_gradients=bool(grads))
        if adjoint:
            mb.mgrit_adjoint(desc, opts, Z_all, theta, lamN, memory=mem, lambda_all=lam_all, resnorm=res_a,
                             workspace=ws, stream=stream, dtheta=grads, linearised=shared)

    # --graph: the caller captures one step (kernels, copies and the library's fork/join events)
    # into a HIP graph and replays it; what the launch-bound small workloads gain from that
    timed_step = step
    if args.graph:
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(torch.cuda.current_stream())
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    # timed region: exactly K steps, nothing else enqueued, no instrumentation beyond one event per step
    # boundary on the caller's stream (the library joins its helper lane back into that stream before a
    # call returns, so consecutive events bracket a whole step)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        timed_step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = (n_phi + n_psi) * T_eval / (ms_per_step * 1e-3)
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] +
                                                                          step_ms[len(step_ms) // 2])

    # second pass over the same K steps with a HIP event pair around every kernel launch (recorded
    # by the library on the launch stream).  Recording ~2500 event pairs per step costs several
    # percent of wall time, which is why it is kept out of the pass that `value` comes from.  The
    # kernels are timed on a single lane: with two lanes kernels of different chunks share the
    # GPU and a launch's duration no longer measures that kernel alone.
    events = not args.no_kernel_events
    totals = {}
    events_ms_per_step = None
    if events:
        mb.mgrit_set_lanes(1)
        mb.mgrit_profile_enable(200000)
        step()
        torch.cuda.synchronize()
        per_step = sum(v["launches"] for v in mb.mgrit_profile_read().values())
        mb.mgrit_profile_enable(per_step * args.steps + 64)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            step()
        torch.cuda.synchronize()
        events_ms_per_step = (time.perf_counter() - t2) * 1e3 / args.steps
        fold(mb, totals)
        mb.mgrit_profile_enable(0)
        mb.mgrit_set_lanes(args.lanes or 2)

    # roofline of the dominant kernel: the MFMA grouped GEMM (all epilogues together)
    roofline = None
    if totals:
        gemm = [v for k, v in totals.items() if k.startswith("gemm_mfma")]
        if gemm:
            fl = sum(v["flops"] for v in gemm); ms = sum(v["ms"] for v in gemm); n = sum(v["launches"] for v in gemm)
            ach = fl / (ms * 1e-3) / 1e12
            roofline = {"bound": "mfma", "kernel": "gemm_mfma_kernel (grouped projection GEMMs, all epilogues)",
                        "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": ach / PEAK_BF16_TFLOPS, "traffic": None if overridden else measured_traffic(wl, adjoint),
                        "launches_per_step": n / args.steps, "avg_launch_us": ms * 1e3 / n,
                        "flop_per_launch": fl / n,
                        "algorithmic_bytes_per_launch": sum(v["bytes"] for v in gemm) / n,
                        "share_of_instrumented_step_time": ms / args.steps / events_ms_per_step,
                        "instrumented_ms_per_step": events_ms_per_step,
                        # the launches over several groups (relaxation sweeps) and the single-group ones
                        # of the serial coarse chain, each by epilogue
                        "by_class": {k: {"TFLOPs": v["flops"] / (v["ms"] * 1e-3) / 1e12,
                                         "launches_per_step": v["launches"] / args.steps,
                                         "avg_launch_us": v["ms"] * 1e3 / v["launches"]}
                                     for k, v in sorted(totals.items()) if k.startswith("gemm_mfma") and v["ms"] > 0}}
            for part, pre in (("sweeps", "gemm_mfma_"), ("coarse_chain", "gemm_mfma_single_")):
                sel = [v for k, v in totals.items()
                       if k.startswith(pre) and (part == "coarse_chain" or not k.startswith("gemm_mfma_single_"))]
                if sel and sum(v["ms"] for v in sel) > 0:
                    p_ach = sum(v["flops"] for v in sel) / (sum(v["ms"] for v in sel) * 1e-3) / 1e12
                    roofline[part] = {"achieved": p_ach, "frac": p_ach / PEAK_BF16_TFLOPS,
                                      "launches_per_step": sum(v["launches"] for v in sel) / args.steps,
                                      "ms_per_step": sum(v["ms"] for v in sel) / args.steps}
        else:
            gen = totals.get("gemm_generic")
            if gen:
                ach = gen["flops"] / (gen["ms"] * 1e-3) / 1e12
                roofline = {"bound": "alu", "kernel": "gemm_f32_mfma_kernel (fp32 MFMA 32x32x2; odd shapes on the FMA kernel)", "achieved": ach,
                            "peak": 157.3, "unit": "TFLOP/s", "frac": ach / 157.3, "traffic": None,
                            "avg_launch_us": gen["ms"] * 1e3 / gen["launches"]}
        # long sequences with few features (the deep-narrow workload): the fused attention kernels
        # outweigh the GEMMs and are the dominant kernel instead (algorithmic flops: 2 products
        # forward, 5 backward; the two-pass backward recomputes two of them)
        att = [totals[k] for k in ("attn_fwd", "attn_bwd") if k in totals]
        if att and roofline is not None and roofline["bound"] == "mfma" and wl.d_model // wl.n_heads in (64, 128):
            a_ms = sum(v["ms"] for v in att)
            if a_ms > sum(v["ms"] for v in gemm):
                a_fl = sum(v["flops"] for v in att); a_n = sum(v["launches"] for v in att)
                ach = a_fl / (a_ms * 1e-3) / 1e12
                roofline = {"bound": "mfma", "kernel": "attn_fwd_mfma_kernel + attn_bwd_*_mfma_kernel (fused softmax attention)",
                            "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                            "launches_per_step": a_n / args.steps, "avg_launch_us": a_ms * 1e3 / a_n,
                            "flop_per_launch": a_fl / a_n,
                            "algorithmic_bytes_per_launch": sum(v["bytes"] for v in att) / a_n,
                            "share_of_instrumented_step_time": a_ms / args.steps / events_ms_per_step,
                            "instrumented_ms_per_step": events_ms_per_step,
                            "grouped_gemm_TFLOPs": roofline["achieved"]}
        hbm = {}
        # an event pair adds a few microseconds to the launch it brackets (reported, not subtracted: the
        # rates below are lower bounds; a kernel trace of the same launches gives the durations proper)
        bracket_us = mb.mgrit_measure_event_bracket(stream)
        # LayerNorm: the launches over several groups (relaxation sweeps: tens of MB, beyond the caches
        # between producer and consumer) and the single-group ones of the coarse chain apart
        for k in ("ln_fwd", "ln_vjp", "ln_fwd_single", "ln_vjp_single", "elementwise"):
            if k in totals and totals[k]["ms"] > 0:
                gbs = totals[k]["bytes"] / (totals[k]["ms"] * 1e-3) / 1e9
                hbm[k] = {"achieved_GBs": gbs, "frac_of_8TBs": gbs / PEAK_HBM_GBS,
                          "avg_launch_us": totals[k]["ms"] * 1e3 / totals[k]["launches"]}
        if roofline is not None:
            roofline["hbm_bound_kernels"] = hbm
            roofline["event_bracket_us"] = bracket_us
            # what this machine reaches: a register-resident MFMA loop and a 1 GiB streaming copy, so that
            # the fractions can be read against the achievable as well as against the datasheet
            a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
            b = torch.empty_like(a)
            a.fill_(1.0)
            mfma_c = mb.mgrit_measure_mfma_ceiling(b, 20000, stream)
            copy_c = mb.mgrit_measure_copy_ceiling(a, b, stream)
            del a, b
            roofline["measured_ceilings"] = {"mfma_bf16_TFLOPs": mfma_c, "copy_GBs": copy_c}
            if roofline["bound"] == "mfma":
                roofline["frac_of_measured_ceiling"] = roofline["achieved"] / mfma_c
            for v in hbm.values():
                v["frac_of_copy"] = v["achieved_GBs"] / copy_c
    if args.breakdown and totals:
        print(f"{'class':28s} {'launches/step':>13s} {'ms/step':>9s} {'TFLOP/s':>9s} {'GB/s':>9s}", file=sys.stderr)
        for k, v in sorted(totals.items(), key=lambda kv: -kv[1]["ms"]):
            ms = v["ms"] / args.steps
            print(f"{k:28s} {v['launches'] / args.steps:13.1f} {ms:9.3f} "
                  f"{v['flops'] / (v['ms'] * 1e-3) / 1e12:9.1f} {v['bytes'] / (v['ms'] * 1e-3) / 1e9:9.0f}",
                  file=sys.stderr)
        print(f"{'wall, this pass (1 lane)':28s} {'':13s} {events_ms_per_step:9.3f}", file=sys.stderr)
        print(f"{'wall, timed pass':28s} {'':13s} {ms_per_step:9.3f}", file=sys.stderr)

    out = {
        "metric": ("MGRIT fwd+adjoint+param-grads layer-steps*tokens/sec" if grads else
                   "MGRIT fwd+adjoint layer-steps*tokens/sec" if adjoint else "MGRIT fwd layer-steps*tokens/sec"),
        "value": value, "unit": "layer-steps*tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step,
        # each step also timed on the stream by an event pair: median, fastest and slowest step, and the
        # metric at the median (`value` itself is K steps over the wall clock between two synchronisations)
        "step_ms_by_events": {"median": median_ms, "min": step_ms[0], "max": step_ms[-1],
                              "value_at_median": (n_phi + n_psi) * T_eval / (median_ms * 1e-3)},
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.dtype == wls.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "d_model": wl.d_model, "n_heads": wl.n_heads, "d_ff": wl.d_ff,
                   "batch": wl.batch, "seq": wl.seq, "N": wl.N, "h": wl.h, "cf": wl.cf, "levels": wl.levels,
                   "iters": wl.iters, "relax": "FCF" if wl.relax else "F", "adjoint": adjoint,
                   "phi_evaluations": n_phi, "psi_evaluations": n_psi,
                   # dependent chain of batched sweeps per solve, against the N steps of serial propagation
                   "dependent_sweeps_per_solve": mb.mgrit_step_depth(opts), "serial_depth": wl.N,
                   "max_groups_per_launch": args.max_groups or mb.lib().mgrit_default_groups_per_launch(
                       C_byref(desc), max(wl.N // wl.cf, 1)), "lanes": args.lanes or 2,
                   "param_grads": bool(grads), "launch": "hip graph replay" if args.graph else "eager",
                   "adjoint_cache": not args.no_adjoint_cache, "workspace_bytes": int(ws_bytes),
                   "linearisation": "left by the forward solve's closing relaxation" if shared
                   else "the adjoint's own pass over all layers",
                   **({"stacked": True, "n_enc": sw.n_enc, "src_seq": sw.enc.seq} if sw else {})},
        "residual_norms": {"forward": [float(x) for x in res_f.cpu()[:wl.iters]],
                           "adjoint": [float(x) for x in res_a.cpu()[:wl.iters]] if adjoint else None},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        if sw:
            # about half of the evaluations are encoder steps, half decoder steps (n_enc = N / 2)
            ce = cpu_baseline(sw.enc, n_phi // 2, n_psi // 2, args.cpu_seconds / 2)
            cd = cpu_baseline(sw.dec, n_phi - n_phi // 2, n_psi - n_psi // 2, args.cpu_seconds / 2)
            work_e = (n_phi // 2 + n_psi // 2) * sw.enc.tokens
            work_d = (n_phi + n_psi) * T_eval - work_e
            cd["value"] = (work_e + work_d) / (work_e / ce["value"] + work_d / cd["value"])
            cd["sample"] = "encoder half: " + ce["sample"] + "; decoder half: " + cd["sample"]
            out["cpu_baseline"] = cd
        else:
            out["cpu_baseline"] = cpu_baseline(wl, n_phi, n_psi, args.cpu_seconds)
        out["gpu_over_cpu"] = value / out["cpu_baseline"]["value"]
    print(json.dumps(out))


def measured_traffic(wl, adjoint):
    """HBM bytes per grouped-GEMM launch (FETCH_SIZE + WRITE_SIZE, scaled by what the same counters
    read for a plain copy) from the committed rocprofv3 --pmc summary of this workload, or None when
    no summary covers it.  Counters cannot be read from inside this process."""
    if not adjoint:
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"{wl.name}_fwd_adjoint_pmc_summary.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_gemm_launch:"):
            return float(line.split(":")[1])
    return None


def fold(mb, totals):
    """Add the event pool's per-class totals to `totals` and reset the pool."""
    for k, v in mb.mgrit_profile_read().items():
        t = totals.setdefault(k, {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
        for f in ("ms", "flops", "bytes", "launches"):
            t[f] += v[f]
        if v.get("overflow"):
            t["overflow"] = True
    mb.mgrit_profile_reset()


if __name__ == "__main__":
    main()
