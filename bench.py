#!/usr/bin/env python3
"""Benchmark of the EF-compress hot path (Algorithm 4 of arxiv 1905.10936) on one MI355X.

One "step" = ef_worker_step for all M workers + ef_server_step + ef_apply over
one batch of synthetic gradients that are already resident in HBM.  Prints ONE
JSON line: throughput in Gelem/s counted as (M+1)*d elements through a
compressor per step, the HBM roofline of the dominant kernel (measured with
HIP events on the launch stream), the other benchmark configurations timed the
same way (`other_workloads`), and the CPU oracle timed on a bounded sample of
the headline workload on this host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import glob
import json
import os
import re
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
TILE = 4096                     # elements a workgroup takes at a time (only used to name the dominant kernel's share)

# The benchmark configurations besides the headline one, timed after it (`other_workloads`).
OTHER_WORKLOADS = ("resnet20_like", "resnet50_like", "skewed_blocks", "transformer_like")


def algorithmic_bytes(d, B, M, variant="sgdm"):
    """Bytes the method itself must move per step (fp32 state read once and
    written once, sign bits, scales): worker call, server call, apply call."""
    state = 12.0 if variant == "sgd" else 20.0              # g,e in, e out (+ m in, m out with momentum)
    worker = M * (state * d + d / 8.0 + 4.0 * B)            # + signs, scales
    server = 8.0 * d + (M + 1) * d / 8.0 + 4.0 * B * (M + 1)
    apply_ = (16.0 if variant == "wd" else 8.0) * d + d / 8.0 + 4.0 * B   # x (+ decay momentum) in and out
    return worker, server, apply_


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from rocprofv3's FETCH_SIZE / WRITE_SIZE
    counters, as recorded in a summary under profiles/ (a line `traffic-json: {...}` written by
    bench_profile.py; each record names the commit it was measured at).  None if no summary has a
    record for this kernel on this workload: the figure is never a constant of this file."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for m in re.finditer(r"traffic-json:\s*(\{.*\})", open(path).read()):
            try:
                rec = json.loads(m.group(1))
            except ValueError:
                continue
            if rec.get("workload") == workload and rec.get("mode", "default") == "default" and kernel in rec.get("kernels", {}):
                k = rec["kernels"][kernel]
                return {"bytes_per_launch": k["traffic_bytes"], "ratio_to_algorithmic": k.get("ratio"),
                        "measured_at_commit": rec.get("commit"), "summary": os.path.relpath(path, ROOT)}
    return None


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


class Run:
    """Device state of one workload and the step over it."""

    def __init__(self, w, variant, n_sets, dev):
        self.w, self.variant, self.dev = w, variant, dev
        d, B, M = w.d, w.B, w.M
        W = (d + 63) // 64
        self.plan = ef.ef_plan_create(w.offsets, M)
        self.n_sets = n_sets
        ds = (d + 3) // 4 * 4           # row stride in elements: the ABI wants a multiple of 4
        self.ds = ds
        self.grads = torch.zeros((n_sets, M, ds), dtype=torch.float32, device=dev)
        for s in range(n_sets):
            for i in range(M):
                w.grad(s, i, device=dev, out=self.grads[s, i, :d])
        self.mom = torch.zeros((M, ds), dtype=torch.float32, device=dev)
        self.err = torch.zeros((M, ds), dtype=torch.float32, device=dev)
        self.te = torch.zeros(d, dtype=torch.float32, device=dev)
        self.x = torch.zeros(d, dtype=torch.float32, device=dev)
        self.ws = torch.zeros((M, W), dtype=torch.int64, device=dev)
        self.wc = torch.zeros((M, B), dtype=torch.float32, device=dev)
        self.ss = torch.zeros(W, dtype=torch.int64, device=dev)
        self.sc = torch.zeros(B, dtype=torch.float32, device=dev)
        if variant == "fused":
            pb = ef.ef_payload_bytes(self.plan)
            self.wmsg = torch.zeros((M, pb), dtype=torch.uint8, device=dev)
            self.smsg = torch.zeros(pb, dtype=torch.uint8, device=dev)
        if variant == "wd":
            self.decay_mom = torch.zeros(d, dtype=torch.float32, device=dev)
        if variant == "quality":
            self.quality = torch.zeros((M, 2), dtype=torch.float64, device=dev)
        torch.cuda.synchronize()
        self.stream = torch.cuda.current_stream()
        self.eta_prev, self.t = 0.0, 0
        self.held = None            # ef_state: m, e, e~ held by the library (the deferred leg)

    def timed_with_held_state(self, steps, warmup):
        """The same steps with m, e and e~ held by the library (ef_state_create): every call then runs
        in the deferred-correction mode.  The held state starts from zero, as Algorithm 4 does."""
        self.held = ef.ef_state_create(self.plan, self.w.M)
        self.eta_prev = 0.0
        ms, calls, _ = self.timed(steps, warmup)
        self.held.close()
        self.held = None
        return ms, calls

    def step(self, ev=None):
        w, plan, variant, M = self.w, self.plan, self.variant, self.w.M
        g = self.grads[self.t % self.n_sets]
        if ev:
            ev[0].record(self.stream)
        if self.held is not None:
            ef.ef_worker_step_state(plan, self.held, g, w.mu, self.eta_prev, w.eta, self.ws, self.wc)
            if ev:
                ev[1].record(self.stream)
            ef.ef_server_step_state(plan, self.held, M, self.ws, self.wc, self.eta_prev, w.eta, self.ss, self.sc)
            if ev:
                ev[2].record(self.stream)
            ef.ef_apply(plan, self.x, self.ss, self.sc, w.eta)
            if ev:
                ev[3].record(self.stream)
            self.eta_prev = w.eta
            self.t += 1
            return
        if variant == "fused":
            ef.ef_worker_step_fused(plan, g, self.mom, self.err, w.mu, self.eta_prev, w.eta, self.wmsg)
        elif variant == "sgd":
            ef.ef_worker_step_sgd(plan, g, self.err, self.eta_prev, w.eta, self.ws, self.wc)
        elif variant == "quality":
            ef.ef_worker_step_quality(plan, g, self.mom, self.err, w.mu, self.eta_prev, w.eta, self.ws, self.wc, self.quality)
        else:
            ef.ef_worker_step(plan, g, self.mom, self.err, w.mu, self.eta_prev, w.eta, self.ws, self.wc)
        if ev:
            ev[1].record(self.stream)
        if variant == "fused":
            ef.ef_server_step_fused(plan, M, self.wmsg, self.te, self.eta_prev, w.eta, self.smsg)
        else:
            ef.ef_server_step(plan, M, self.ws, self.wc, self.te, self.eta_prev, w.eta, self.ss, self.sc)
        if ev:
            ev[2].record(self.stream)
        if variant == "fused":
            ef.ef_apply_fused(plan, self.x, self.smsg, w.eta)
        elif variant == "wd":
            ef.ef_apply_wd(plan, self.x, self.decay_mom, self.ss, self.sc, w.eta, w.mu, 5e-4)
        else:
            ef.ef_apply(plan, self.x, self.ss, self.sc, w.eta)
        if ev:
            ev[3].record(self.stream)
        self.eta_prev = w.eta
        self.t += 1

    def timed(self, steps, warmup, first_payload=False):
        """`warmup` untimed steps, then exactly `steps` timed ones.  Returns (ms per step by the host
        clock around the synchronised region, mean ms of the three calls by HIP events, first payload)."""
        payload = None
        for k in range(warmup):
            self.step()
            if k == 0 and first_payload:
                torch.cuda.synchronize()
                payload = (self.ws.cpu().numpy().view(np.uint64).copy(), self.ss.cpu().numpy().view(np.uint64).copy())
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(events[k])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        calls = [float(np.mean([e[q].elapsed_time(e[q + 1]) for e in events])) for q in range(3)]
        return ms, calls, payload

    def worker_kernel(self):
        w = self.w
        mixed = bool(np.any(w.offsets[1:] % TILE != 0))
        mom = "false" if self.variant == "sgd" else "true"
        if self.variant == "quality":
            return "ef::k_worker_tiles<true, true, true>"
        if self.plan.persistent and self.variant != "sgd":
            return "ef::k_worker_uniform<%s>" % mom
        return "ef::k_worker_tiles<%s, %s, false>" % (mom, "true" if mixed else "false")

    def close(self):
        self.plan.close()


def summary_of(run, ms, calls, variant):
    """Figures of one timed run that the headline and the other workloads share."""
    w = run.w
    d, B, M = w.d, w.B, w.M
    bw, bs, ba = algorithmic_bytes(d, B, M, variant)
    t_worker, t_server, t_apply = calls
    return {
        "ms_per_step": round(ms, 4),
        "value": round((M + 1) * d / (ms * 1e-3) / 1e9, 3), "unit": "Gelem/s",
        "per_call_ms": {"ef_worker_step": round(t_worker, 4), "ef_server_step": round(t_server, 4),
                        "ef_apply": round(t_apply, 4)},
        "step_hbm_frac_algorithmic": round((bw + bs + ba) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "per_call_hbm_frac": {"ef_worker_step": round(bw / (t_worker * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                              "ef_server_step": round(bs / (t_server * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                              "ef_apply": round(ba / (t_apply * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "dominant_kernel": run.worker_kernel(),
    }


def other_workload(name, dev, steps, warmup):
    """One of the other benchmark configurations: default plan settings, eager calls, one gradient
    set resident, timed like the headline run (a few steps; the headline figure is not affected)."""
    w = wl.get(name)
    run = Run(w, "sgdm", 1, dev)
    ms, calls, _ = run.timed(steps, warmup)
    out = dict(summary_of(run, ms, calls, "sgdm"), d=w.d, B=w.B, M=w.M, steps=steps, warmup=warmup,
               worker_fuse_limit_tiles=run.plan.fuse_limit)
    if ms < 0.2:
        # launch-bound layouts: the same step as one captured HIP graph, replayed (untimed capture, wall clock
        # around the replays)
        side = torch.cuda.Stream()
        gr = torch.cuda.CUDAGraph()
        run.t = 0
        with torch.cuda.graph(gr, stream=side):
            run.step()
        torch.cuda.synchronize()
        reps = max(steps, 50)
        for _ in range(5):
            gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            gr.replay()
        torch.cuda.synchronize()
        out["hip_graph_replay"] = {"ms_per_step": round((time.perf_counter() - t0) * 1e3 / reps, 4), "replays": reps}
        del gr
    ms2, calls2 = run.timed_with_held_state(steps, max(warmup, 1))
    out["held_state_mode"] = {"ms_per_step": round(ms2, 4),
                                       "per_call_ms": {"ef_worker_step": round(calls2[0], 4),
                                                       "ef_server_step": round(calls2[1], 4),
                                                       "ef_apply": round(calls2[2], 4)}}
    run.close()
    del run
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="flat_2p28", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--grad-sets", type=int, default=0, help="distinct gradient sets kept in HBM (0 = auto)")
    ap.add_argument("--cpu-blocks", type=int, default=0, help="blocks in the CPU oracle sample (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-others", action="store_true", help="skip the other benchmark configurations")
    ap.add_argument("--fuse-limit", type=int, default=-1, help="override the plan's one-pass block limit")
    ap.add_argument("--spin-limit", type=int, default=-1, help="override the plan's wait budget")
    ap.add_argument("--persistent", type=int, default=-1, help="1/0: force the persistent worker kernel on/off")
    ap.add_argument("--lazy", action="store_true",
                    help="deferred residual correction for blocks beyond the one-pass limit (ef_plan_set_lazy)")
    ap.add_argument("--no-deferred", action="store_true",
                    help="skip the extra leg that times the same steps in the deferred-correction mode")
    ap.add_argument("--variant", default="sgdm", choices=["sgdm", "sgd", "fused", "wd", "quality"],
                    help="sgdm: Algorithm 4 (the default, the metric's configuration); sgd: Algorithm 3 worker "
                         "without a momentum buffer; fused: one message per worker (Section 4.2); wd: parameter "
                         "update with weight decay (Appendix A); quality: worker call that also reports phi and "
                         "delta of p (ef_worker_step_quality), plus one untimed ef_compressor_quality pass")
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
    variant = args.variant
    # gradient sets resident in HBM, cycled over the steps
    n_sets = args.grad_sets or max(1, min(args.steps + args.warmup, int(64e9 // (4.0 * d * M)), 4))
    run = Run(w, variant, n_sets, dev)
    plan = run.plan
    if args.fuse_limit >= 0 or args.spin_limit >= 0:
        plan.tune(args.fuse_limit, args.spin_limit)
    if args.persistent >= 0:
        plan.set_persistent(args.persistent)
    if args.lazy:
        plan.set_lazy(True)

    if args.calib:
        # known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE: reads 2^28 floats, writes 2^28 floats
        ca = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        cb = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        for _ in range(3):
            torch.add(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb

    if args.graph:
        # per-call breakdown from an eager pass, then the timed region replays captured graphs
        _, calls, first_payload = run.timed(args.steps, args.warmup, first_payload=variant in ("sgdm", "wd"))
        side = torch.cuda.Stream()
        graphs = []
        for s_ in range(n_sets):
            run.t = s_
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                run.step()
            graphs.append(gr)
        torch.cuda.synchronize()
        for k in range(max(args.warmup, 1)):
            graphs[k % n_sets].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graphs[k % n_sets].replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    else:
        ms_per_step, calls, first_payload = run.timed(args.steps, args.warmup, first_payload=variant in ("sgdm", "wd"))

    if variant == "quality":
        # untimed: the stand-alone diagnostics pass over the gradients, so that its kernels show in a trace
        ef.ef_compressor_quality(plan, run.grads[0], run.quality)
    fuse_limit_used = plan.fuse_limit
    # untimed diagnostic: one more worker and server call, asking each how many tiles left the one-pass route
    g = run.grads[run.t % n_sets]
    ef.ef_worker_step(plan, g, run.mom, run.err, w.mu, w.eta, w.eta, run.ws, run.wc)
    fb_worker = plan.last_fallbacks()
    ef.ef_server_step(plan, M, run.ws, run.wc, run.te, w.eta, w.eta, run.ss, run.sc)
    fb_server = plan.last_fallbacks()

    head = summary_of(run, ms_per_step, calls, variant)
    t_worker = calls[0]
    bw, _, _ = algorithmic_bytes(d, B, M, variant)
    achieved = bw / (t_worker * 1e-3) / 1e9

    # beside the headline (not part of `value`): the same steps with m, e and e~ held by the library
    deferred = None
    if not args.lazy and not args.graph and not args.no_deferred and variant == "sgdm":
        ms2, calls2 = run.timed_with_held_state(args.steps, max(args.warmup, 1))
        deferred = {
            "ms_per_step": round(ms2, 4), "value": round((M + 1) * d / (ms2 * 1e-3) / 1e9, 3), "unit": "Gelem/s",
            "per_call_ms": {"ef_worker_step_state": round(calls2[0], 4), "ef_server_step_state": round(calls2[1], 4),
                            "ef_apply": round(calls2[2], 4)},
            "worker_hbm_frac": round(bw / (calls2[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "what": "ef_state_create + ef_worker_step_state / ef_server_step_state: the library holds m, e and e~, so "
                    "e <- p - Delta of blocks beyond the one-pass limit can be formed when the next call loads the "
                    "buffer (same bits) and no workgroup waits for a large block's scale; same gradients, same "
                    "payloads and parameters, timed after the headline run"}

    # untimed: the practical ceiling of the worker's access pattern on this machine (a bare stream of
    # the same reads and writes over the same buffers; the state is not needed any more)
    ceiling = ceiling_ticketed = ceiling_grouped = None
    if variant != "sgd" and M * run.ds >= 4096:
        torch.cuda.synchronize()
        bufs = (run.grads[0].view(-1), run.mom.view(-1), run.err.view(-1))
        p_ms, p_bytes = bench_probe.ef_stream_probe(*bufs, repeats=3)
        ceiling_ticketed = p_bytes / (p_ms * 1e-3) / 1e9
        p_ms, p_bytes = bench_probe.ef_stream_probe_grouped(*bufs, group=16, repeats=3)
        ceiling_grouped = p_bytes / (p_ms * 1e-3) / 1e9
        ceiling = max(ceiling_ticketed, ceiling_grouped)

    kernel = head["dominant_kernel"]
    out = {
        "metric": "EF-compress step Gelem/s (worker+server, M workers) and % of HBM roofline",
        "value": head["value"],
        "unit": "Gelem/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": dict({k: v for k, v in w.describe().items() if k != "steps"},
                       steps_of_the_configuration=w.steps, variant=variant,
                       launch="hip graph replay" if args.graph else "eager calls",
                       deferred_residual_correction=bool(plan.lazy),
                       grad_sets_in_hbm=n_sets, elements_counted="(M+1)*d per step",
                       d_per_step_Gelem_s=round(d / (ms_per_step * 1e-3) / 1e9, 3)),
        "roofline": {
            "bound": "hbm",
            "kernel": kernel + ", all M workers in one launch; timed as the whole ef_worker_step call (the short "
                               "kernel that ends the call included)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": (measured_traffic(args.workload, kernel) or {}).get("bytes_per_launch")
            if variant == "sgdm" and not plan.lazy else None,
            "traffic_source": measured_traffic(args.workload, kernel) if variant == "sgdm" and not plan.lazy else None,
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
        "per_call_ms": head["per_call_ms"],
        "per_call_hbm_frac": head["per_call_hbm_frac"],
        "step_hbm_frac_algorithmic": head["step_hbm_frac_algorithmic"],
        "worker_fuse_limit_tiles": fuse_limit_used,
        "held_state_mode": deferred,
        "run_time_fallbacks": {"worker_parked_tiles": fb_worker[0], "worker_late_blocks": fb_worker[1],
                               "server_parked_tiles": fb_server[0], "server_late_blocks": fb_server[1]},
    }

    cpu = None
    if not args.no_cpu and variant in ("sgdm", "wd"):
        # bounded sample: a prefix of blocks sized for roughly 10-30 s of single-thread work
        avg_block = d / B
        n_blocks = args.cpu_blocks or int(max(1, min(B, round(5e7 / avg_block))))
        cpu_steps = 2
        cpu_val, ds, first = cpu_baseline(w, run.grads[0], n_blocks, cpu_steps)
        # the oracle's first step on the sample must reproduce the GPU's first payload there
        check = None
        if first_payload is not None and args.warmup >= 1:
            nw = ds // 64
            check = bool(np.array_equal(first[0][:, :nw], first_payload[0][:, :nw]) and
                         np.array_equal(first[2][:nw], first_payload[1][:nw]))
        cpu = {
            "value": round(cpu_val, 4), "unit": "Gelem/s", "cores": 1, "kind": "oracle",
            "sample": "first %d blocks (%d elements) of the same workload, all M=%d workers + server + apply, "
                      "%d steps after one warm-up, single thread; host has %d logical cores"
                      % (n_blocks, ds, M, cpu_steps, os.cpu_count()),
            "first_step_signs_match_gpu": check,
        }

    # the other benchmark configurations, after the headline run has given its memory back
    run.close()
    del run, plan, g
    torch.cuda.empty_cache()
    if not args.no_others and variant == "sgdm" and not args.lazy and not args.graph and args.workload == "flat_2p28":
        out["other_workloads"] = {name: other_workload(name, dev, 5, 2) for name in OTHER_WORKLOADS}
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
