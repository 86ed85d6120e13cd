#!/usr/bin/env python3
"""Benchmark of the EF-compress hot path (Algorithm 4 of arxiv 1905.10936) on one MI355X.

One "step" = ef_worker_step for all M workers + ef_server_step + ef_apply over
one batch of synthetic gradients that are already resident in HBM.  Prints ONE
JSON line: throughput in Gelem/s counted as (M+1)*d elements through a
compressor per step, the HBM roofline of the dominant kernel (measured with
HIP events on the launch stream), and the CPU oracle timed on a bounded sample
of the same workload on this host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import ef_workloads as wl  # noqa: E402
import paper_1905_10936_amd as ef  # noqa: E402
from paper_1905_10936_amd import bench_probe  # noqa: E402

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE, scaled by a torch add kernel of known size run
# in the same process): see profiles/ef_step_flat_2p28.md.  None where not measured.
MEASURED_TRAFFIC_BYTES = {("flat_2p28", "direct"): 43318642898,        # ef::k_worker_uniform_direct<true>
                          ("flat_2p28", "persistent"): 43296770554}    # ef::k_worker_uniform<true>


def algorithmic_bytes(d, B, M, variant="sgdm"):
    """Bytes the method itself must move per element of d (fp32 state read
    once and written once, sign bits, scales)."""
    state = 12.0 if variant == "sgd" else 20.0              # g,e in, e out (+ m in, m out with momentum)
    worker = M * (state * d + d / 8.0 + 4.0 * B)            # + signs, scales
    server = 8.0 * d + (M + 1) * d / 8.0 + 4.0 * B * (M + 1)
    apply_ = (16.0 if variant == "wd" else 8.0) * d + d / 8.0 + 4.0 * B   # x (+ decay momentum) in and out
    return worker, server, apply_


def cpu_baseline(w, grads0, n_blocks, steps):
    """The oracle, as it stands, on the first n_blocks blocks of the workload
    (the method is block-separable), single thread."""
    import oracle
    offs = w.offsets[:n_blocks + 1].copy()
    ds = int(offs[-1])
    M = w.M
    g = np.ascontiguousarray(grads0[:, :ds].cpu().numpy())
    m = np.zeros((M, ds), np.float32)
    e = np.zeros((M, ds), np.float32)
    te = np.zeros(ds, np.float32)
    x = np.zeros(ds, np.float32)
    first = oracle.step(g, m, e, te, x, offs, np.float32(w.mu), np.float32(0.0), np.float32(w.eta))
    t0 = time.perf_counter()
    for _ in range(steps):
        oracle.step(g, m, e, te, x, offs, np.float32(w.mu), np.float32(w.eta), np.float32(w.eta))
    dt = (time.perf_counter() - t0) / steps
    return (M + 1) * ds / dt / 1e9, ds, first


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="flat_2p28", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--grad-sets", type=int, default=0, help="distinct gradient sets kept in HBM (0 = auto)")
    ap.add_argument("--cpu-blocks", type=int, default=0, help="blocks in the CPU oracle sample (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--fuse-limit", type=int, default=-1, help="override the plan's one-pass block limit")
    ap.add_argument("--spin-limit", type=int, default=-1, help="override the plan's wait budget")
    ap.add_argument("--persistent", type=int, default=-1, help="1/0: force the persistent worker kernel on/off")
    ap.add_argument("--lazy", action="store_true",
                    help="deferred residual correction for blocks beyond the one-pass limit (ef_plan_set_lazy)")
    ap.add_argument("--no-deferred", action="store_true",
                    help="skip the extra leg that times the same steps in the deferred-correction mode")
    ap.add_argument("--variant", default="sgdm", choices=["sgdm", "sgd", "fused", "wd"],
                    help="sgdm: Algorithm 4 (the default, the metric's configuration); sgd: Algorithm 3 worker "
                         "without a momentum buffer; fused: one message per worker (Section 4.2); wd: parameter "
                         "update with weight decay (Appendix A)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a captured HIP graph of the step (one graph per resident gradient set) "
                         "instead of eager calls; per-call times then come from an untimed eager pass")
    ap.add_argument("--calib", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB elementwise kernel (known size) for counter calibration")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs M simulated workers and the server on ONE GPU; "
              "--gpus N with N > 1 is not supported (no collectives are part of it).", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = wl.get(args.workload)
    d, B, M = w.d, w.B, w.M
    W = (d + 63) // 64
    plan = ef.ef_plan_create(w.offsets, M)
    if args.fuse_limit >= 0 or args.spin_limit >= 0:
        plan.tune(args.fuse_limit, args.spin_limit)
    if args.persistent >= 0:
        plan.set_persistent(args.persistent)
    if args.lazy:
        plan.set_lazy(True)

    # gradient sets resident in HBM, cycled over the steps
    n_sets = args.grad_sets or max(1, min(args.steps + args.warmup, int(64e9 // (4.0 * d * M)), 4))
    ds = (d + 3) // 4 * 4           # row stride in elements: the ABI wants a multiple of 4
    grads = torch.zeros((n_sets, M, ds), dtype=torch.float32, device=dev)
    for s in range(n_sets):
        for i in range(M):
            w.grad(s, i, device=dev, out=grads[s, i, :d])
    mom = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    err = torch.zeros((M, ds), dtype=torch.float32, device=dev)
    te = torch.zeros(d, dtype=torch.float32, device=dev)
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
    wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
    ss = torch.zeros(W, dtype=torch.int64, device=dev)
    sc = torch.zeros(B, dtype=torch.float32, device=dev)
    variant = args.variant
    if variant == "fused":
        pb = ef.ef_payload_bytes(plan)
        wmsg = torch.zeros((M, pb), dtype=torch.uint8, device=dev)
        smsg = torch.zeros(pb, dtype=torch.uint8, device=dev)
    if variant == "wd":
        decay_mom = torch.zeros(d, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    state = {"eta_prev": 0.0, "t": 0}

    def step(ev=None):
        g = grads[state["t"] % n_sets]
        if ev:
            ev[0].record(stream)
        if variant == "fused":
            ef.ef_worker_step_fused(plan, g, mom, err, w.mu, state["eta_prev"], w.eta, wmsg)
        elif variant == "sgd":
            ef.ef_worker_step_sgd(plan, g, err, state["eta_prev"], w.eta, ws, wc)
        else:
            ef.ef_worker_step(plan, g, mom, err, w.mu, state["eta_prev"], w.eta, ws, wc)
        if ev:
            ev[1].record(stream)
        if variant == "fused":
            ef.ef_server_step_fused(plan, M, wmsg, te, state["eta_prev"], w.eta, smsg)
        else:
            ef.ef_server_step(plan, M, ws, wc, te, state["eta_prev"], w.eta, ss, sc)
        if ev:
            ev[2].record(stream)
        if variant == "fused":
            ef.ef_apply_fused(plan, x, smsg, w.eta)
        elif variant == "wd":
            ef.ef_apply_wd(plan, x, decay_mom, ss, sc, w.eta, w.mu, 5e-4)
        else:
            ef.ef_apply(plan, x, ss, sc, w.eta)
        if ev:
            ev[3].record(stream)
        state["eta_prev"] = w.eta
        state["t"] += 1

    if args.calib:
        # known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE: reads 2^28 floats, writes 2^28 floats
        ca = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        cb = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        for _ in range(3):
            torch.add(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb

    first_payload = None
    for k in range(args.warmup):
        step()
        if k == 0:
            torch.cuda.synchronize()
            if variant in ("sgdm", "wd"):
                first_payload = (ws.cpu().numpy().view(np.uint64).copy(), ss.cpu().numpy().view(np.uint64).copy())
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    if args.graph:
        # per-call breakdown from an eager pass, then the timed region replays captured graphs
        for k in range(args.steps):
            step(events[k])
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graphs = []
        for s_ in range(n_sets):
            state["t"] = s_
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                step()
            graphs.append(gr)
        torch.cuda.synchronize()
        for k in range(max(args.warmup, 1)):
            graphs[k % n_sets].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graphs[k % n_sets].replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(events[k])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    fuse_limit_used = plan.fuse_limit
    # untimed diagnostic: one more worker and server call, asking each how many tiles left the one-pass route
    g = grads[state["t"] % n_sets]
    ef.ef_worker_step(plan, g, mom, err, w.mu, w.eta, w.eta, ws, wc)
    fb_worker = plan.last_fallbacks()
    ef.ef_server_step(plan, M, ws, wc, te, w.eta, w.eta, ss, sc)
    fb_server = plan.last_fallbacks()

    t_worker = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    t_server = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    t_apply = float(np.mean([e[2].elapsed_time(e[3]) for e in events]))
    bw, bs, ba = algorithmic_bytes(d, B, M, variant)
    step_bytes = bw + bs + ba
    achieved = bw / (t_worker * 1e-3) / 1e9

    # beside the headline (not part of `value`): the same steps with the deferred residual correction on
    deferred = None
    if not args.lazy and not args.graph and not args.no_deferred:
        plan.set_lazy(True)
        for k in range(max(args.warmup, 1)):
            step()
        ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(ev2[k])
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) * 1e3 / args.steps
        ef.ef_flush(plan, err, te)
        torch.cuda.synchronize()
        plan.set_lazy(False)
        tw2 = float(np.mean([e[0].elapsed_time(e[1]) for e in ev2]))
        deferred = {
            "ms_per_step": round(ms2, 4), "value": round((M + 1) * d / (ms2 * 1e-3) / 1e9, 3), "unit": "Gelem/s",
            "per_call_ms": {"ef_worker_step": round(tw2, 4),
                            "ef_server_step": round(float(np.mean([e[1].elapsed_time(e[2]) for e in ev2])), 4),
                            "ef_apply": round(float(np.mean([e[2].elapsed_time(e[3]) for e in ev2])), 4)},
            "worker_hbm_frac": round(bw / (tw2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "what": "ef_plan_set_lazy(1): e <- p - Delta of blocks beyond the one-pass limit is formed when the next "
                    "call loads the buffer (same bits), so no workgroup waits for a scale; same steps, same inputs, "
                    "timed after the headline run"}

    # untimed: the practical ceiling of the worker's access pattern on this machine (a bare stream of
    # the same reads and writes over the same buffers; the state is not needed any more)
    ceiling = ceiling_ticketed = ceiling_grouped = None
    if variant != "sgd" and M * ds >= 4096:
        torch.cuda.synchronize()
        p_ms, p_bytes = bench_probe.ef_stream_probe(grads[0].view(-1), mom.view(-1), err.view(-1), repeats=3)
        ceiling_ticketed = p_bytes / (p_ms * 1e-3) / 1e9
        p_ms, p_bytes = bench_probe.ef_stream_probe_grouped(grads[0].view(-1), mom.view(-1), err.view(-1), group=16, repeats=3)
        ceiling_grouped = p_bytes / (p_ms * 1e-3) / 1e9
        ceiling = max(ceiling_ticketed, ceiling_grouped)

    value = (M + 1) * d / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "EF-compress step Gelem/s (worker+server, M workers) and % of HBM roofline",
        "value": round(value, 3),
        "unit": "Gelem/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": dict(w.describe(), variant=variant, launch="hip graph replay" if args.graph else "eager calls",
                       deferred_residual_correction=bool(plan.lazy),
                       grad_sets_in_hbm=n_sets, elements_counted="(M+1)*d per step",
                       d_per_step_Gelem_s=round(d / (ms_per_step * 1e-3) / 1e9, 3)),
        "roofline": {
            "bound": "hbm",
            "kernel": ("ef::k_worker_uniform<true> (persistent)" if plan.persistent else "ef::k_worker_uniform_direct<true>") +
                      ", all M workers in one launch; timed as the whole ef_worker_step call (its mixed-tile and "
                      "list kernels included)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, "persistent" if plan.persistent else "direct"))
            if variant == "sgdm" and not plan.lazy else None,
            "algorithmic_bytes_per_launch": bw,
            "ms_per_launch": round(t_worker, 4),
            "practical_ceiling": None if ceiling is None else {
                "achieved": round(ceiling, 1), "unit": "GB/s", "frac_of_peak": round(ceiling / HBM_PEAK_GBS, 4),
                "worker_vs_ceiling": round(achieved / ceiling, 4),
                "unsynchronised_ticketed": round(ceiling_ticketed, 1),
                "in_step_groups_of_16": round(ceiling_grouped, 1),
                "what": "best of two bare 3-read/2-write fp32 streams over the same buffers and tiles, no compression "
                        "(measured in this run, untimed part): ef_stream_probe (tiles by ticket, workgroups not "
                        "synchronised) and ef_stream_probe_grouped (one workgroup per tile, the third array written "
                        "in step by groups of 16 tiles, as the worker kernel writes its residual)"},
        },
        "per_call_ms": {"ef_worker_step": round(t_worker, 4), "ef_server_step": round(t_server, 4),
                        "ef_apply": round(t_apply, 4)},
        "step_hbm_frac_algorithmic": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "worker_fuse_limit_tiles": fuse_limit_used,
        "deferred_correction_mode": deferred,
        "run_time_fallbacks": {"worker_parked_tiles": fb_worker[0], "worker_late_blocks": fb_worker[1],
                               "server_parked_tiles": fb_server[0], "server_late_blocks": fb_server[1]},
    }

    if not args.no_cpu and variant in ("sgdm", "wd"):
        # bounded sample: a prefix of blocks sized for roughly 10-30 s of single-thread work
        avg_block = d / B
        n_blocks = args.cpu_blocks or int(max(1, min(B, round(5e7 / avg_block))))
        cpu_steps = 2
        g0 = grads[0]
        cpu_val, ds, first = cpu_baseline(w, g0, n_blocks, cpu_steps)
        # the oracle's first step on the sample must reproduce the GPU's first payload there
        check = None
        if first_payload is not None and args.warmup >= 1:
            nw = ds // 64
            check = bool(np.array_equal(first[0][:, :nw], first_payload[0][:, :nw]) and
                         np.array_equal(first[2][:nw], first_payload[1][:nw]))
        out["cpu_baseline"] = {
            "value": round(cpu_val, 4), "unit": "Gelem/s", "cores": 1, "kind": "oracle",
            "sample": "first %d blocks (%d elements) of the same workload, all M=%d workers + server + apply, "
                      "%d steps after one warm-up, single thread; host has %d logical cores"
                      % (n_blocks, ds, M, cpu_steps, os.cpu_count()),
            "first_step_signs_match_gpu": check,
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
