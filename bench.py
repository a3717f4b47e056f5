#!/usr/bin/env python3
"""Benchmark of the sharded weight-update hot path on one MI355X.

Headline workload (the configuration the metric is quoted on): BERT-large-shaped, 398 float32
variables, 336 226 108 parameters, LAMB, 8 replicas; this GPU plays replica 0 and owns a packed
shard of S = 42 028 272 slots.  One step is one pass of the whole path over synthetic inputs
already resident in HBM:

    shard_format(full gradient tensors -> g[S])                          stage 1
    shard_update_lamb(w, g, m, v; other replicas' sums given)            stage 2 (3 kernels)
    unshard_format(gathered[N][S] -> full float32 weight tensors)        stage 3

The cross-replica collectives are not part of the path: the gathered buffer's other rows and the
other replicas' sums of squares are synthetic inputs.  `value` is the number of real parameters
in the shard divided by the time of one step.  Per-kernel durations come from HIP events the
library records on the launch stream (shard_profile_*), in a separate instrumented pass.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# algorithmic bytes per shard slot (float32 = 4 B), per kernel
BYTES_PER_SLOT = {
    "format": 8,       # read 4 + write 4
    "lamb_p1": 24,     # read g, w, m, v; write m, v
    "lamb_p2": 16,     # read w, m, v; write w
    "adam": 28,        # read g, w, m, v; write w, m, v
    "momentum": 20,    # read g, w, m; write w, m
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="bert_large")
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--replica-id", type=int, default=0)
    ap.add_argument("--chunk", type=int, default=0, help="chunk_elems of the plan (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--table", default=None, help="also time every config x stage and write a JSON table here")
    ap.add_argument("--stage", default=None,
                    help="instead of the headline step, run ONE stage of --config at --replicas for --steps launches "
                         "(adam | momentum | lars | lamb | adafactor | shard_format | unshard_format | shard_format_all | "
                         "adam_full_grads | momentum_full_grads | lamb_full_grads | lars_full_grads | "
                         "adam_step | momentum_step | lars_step | lamb_step = format g + update + unshard w | unshard_format_bf16 | "
                         "unshard_format_f32_to_bf16 | shard_format_bf16_to_f32 | lamb_step_bf16 | lamb_fused_step_bf16 | "
                         "adam_shape_probe = the flat Adam update in every launch shape | copy_order_probe = both orders of the "
                         "whole-model copies on tensors placed at several distances) "
                         "and print its HIP-event timing: the command to put under rocprofv3 for that kernel")
    ap.add_argument("--separate-tensors", action="store_true",
                    help="with --stage: every full tensor is an allocation of its own from torch's caching allocator "
                         "(how a framework holds its parameters; equal-sized tensors then sit a power of two apart) "
                         "instead of a slice of one flat buffer")
    ap.add_argument("--copy-order", default="auto", choices=["auto", "by_replica", "by_variable"],
                    help="with --stage: shard_plan_set_copy_walk before anything runs")
    ap.add_argument("--graph", action="store_true",
                    help="with --stage: also record the stage in a HIP graph (stream capture) and time its replays "
                         "beside the eager launches")
    ap.add_argument("--cold", action="store_true",
                    help="with --stage: flush the memory-side cache (a 1 GiB copy) before every launch of the stage")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first run one plain device copy of 1 GiB (2^28 float32), so that a rocprofv3 --pmc run "
                         "has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def _device_normal(n, std, gen, torch):
    return torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, std, generator=gen)


def _settle_copy(torch, su, plan, copy, gathered, full):
    """Has the library measure its two orders of a whole-model copy on these tensors (a set-up call that runs the
    copy and waits) before anything is timed; returns the order it fixed and the two times in ms per launch."""
    walk, (by_replica_ms, by_variable_ms) = su.shard_plan_tune_copy_walk(plan, copy, gathered, full)
    torch.cuda.synchronize()
    return {"walk": walk, "timed_ms_by_replica": round(by_replica_ms, 4), "timed_ms_by_variable": round(by_variable_ms, 4)}


def sources_sha16():
    """First 16 hex digits of the SHA-256 over the library's sources (csrc/ and include/, by name): what a
    counter summary under profiles/ is tied to, so that a figure measured on other kernels is not reported."""
    import hashlib
    h = hashlib.sha256()
    for d in (os.path.join(ROOT, "paper_2004_13336_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(d)):
            if name.endswith((".hip", ".cpp", ".hpp", ".h")):
                h.update(name.encode())
                h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def _median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def _time_stage(torch, su, plan, fn, kernels, warmup, iters):
    """One stage (one or several kernels), three ways, all on the stream the library launches on:
      median_us  median over `iters` calls, each bracketed by an event pair of its own;
      region_us  `iters` calls back to back inside ONE event pair, per call (how the headline step is timed;
                 for several kernels in a row this is what their sum really takes);
      kernel_us  per-kernel averages from the library's own event pairs, a breakdown (each pair adds a few
                 microseconds of its own, so their sum exceeds region_us)."""
    for t in range(1, 1 + max(warmup, 1)):
        fn(t)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(pairs):
        a.record(); fn(100 + i); b.record()
    torch.cuda.synchronize()
    median_us = 1e3 * _median([a.elapsed_time(b) for a, b in pairs])
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(iters):
        fn(1000 + i)
    b.record()
    torch.cuda.synchronize()
    region_us = 1e3 * a.elapsed_time(b) / iters
    su.shard_profile_reset(plan); su.shard_profile_enable(plan, True)
    for i in range(iters):
        fn(2000 + i)
    torch.cuda.synchronize()
    per = {}
    for k in kernels:
        n, ms = su.shard_profile_read(plan, k)
        per[k] = round(1e3 * ms / max(n, 1) * (n / iters if n else 0), 2)      # per call of the stage
    su.shard_profile_enable(plan, False)
    return {"median_us": round(median_us, 2), "region_us": round(region_us, 2), "kernel_us": per}


def _time_region(torch, fn, steps):
    """Milliseconds per call of fn over `steps` back-to-back calls, bracketed by synchronisation."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


class Workbench:
    """Device state of one replica of one configuration."""

    def __init__(self, cfg, N, r, chunk, torch, su, want_full=True, separate=False, copy_order="auto"):
        self.cfg, self.N, self.r, self.torch, self.su = cfg, N, r, torch, su
        self.plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8, None, chunk))
        su.shard_plan_set_copy_walk(self.plan, copy_order)
        S = self.plan.S
        self.S = S
        self.real = sum(self.plan.real_count(r))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(cfg.seed)
        self.gen = gen
        # the gathered [N][S] buffer; row r is this replica's weight shard, updated in place
        self.gathered = None
        if want_full:                      # rows on 128-byte boundaries
            self.gathered = su.gathered_empty(self.plan).normal_(0.0, cfg.weight_std, generator=gen)
        self.w = self.gathered[r] if want_full else _device_normal(S, cfg.weight_std, gen, torch)
        self.g = torch.zeros(S, dtype=torch.float32, device="cuda")
        self.m = torch.zeros(S, dtype=torch.float32, device="cuda")
        self.v = torch.zeros(S, dtype=torch.float32, device="cuda")
        self.w16 = None
        self.full_g = self.full_w = None
        if want_full:
            flat_g = _device_normal(cfg.total, cfg.grad_std, gen, torch)
            flat_w = torch.empty(cfg.total, dtype=torch.float32, device="cuda")
            self.full_g, self.full_w, pos = [], [], 0
            for n in cfg.numel:
                if separate:
                    self.full_g.append(flat_g[pos:pos + n].clone())
                    self.full_w.append(torch.empty(n, dtype=torch.float32, device="cuda"))
                else:
                    self.full_g.append(flat_g[pos:pos + n])
                    self.full_w.append(flat_w[pos:pos + n])
                pos += n
            self.full_g = su.FullTensors(self.plan, self.full_g)      # marshalled once, reused every step
            self.full_w = su.FullTensors(self.plan, self.full_w)
            su.shard_format(self.plan, r, self.full_g, self.g)
        else:
            self.g.normal_(0.0, cfg.grad_std, generator=gen)
        self.other = torch.zeros((self.plan.V, 2), dtype=torch.float32, device="cuda")
        self.local = torch.zeros((self.plan.V, 2), dtype=torch.float32, device="cuda")
        self.step = 0

    def hp(self):
        import numpy as np
        return {k: float(np.float32(v)) for k, v in self.cfg.hyper.items()}

    def settle_copies(self, format_all=False):
        """shard_plan_tune_copy_walk for the copies that are about to be timed, on the real buffers."""
        su, plan = self.su, self.plan
        if self.full_w is None:
            return {}
        out = {"unshard_format": _settle_copy(self.torch, su, plan, "unshard_format", self.gathered, self.full_w)}
        if format_all:
            out["shard_format_all"] = _settle_copy(self.torch, su, plan, "shard_format_all", self.gathered, self.full_g)
            self.gathered.normal_(0.0, self.cfg.weight_std, generator=self.gen)    # weights again, not gradients
        return out

    def free(self):
        self.plan.free()


def headline(args, torch, su, cfgs):
    cfg = [c for c in cfgs if c.name == args.config][0]
    N, r = args.replicas, args.replica_id
    wb = Workbench(cfg, N, r, args.chunk, torch, su)
    hp = wb.hp()
    plan = wb.plan
    if cfg.optimizer != "lamb":
        raise SystemExit("the headline step is the LAMB configuration; use --table for the others")
    # clean padding in this replica's weight row, then pre-warm m and v by two steps so no lane
    # works on all-zero state; the other replicas' sums are (N-1) copies of this replica's
    for t in wb.full_w.tensors:
        t.normal_(0.0, cfg.weight_std, generator=wb.gen)
    su.shard_format(plan, r, wb.full_w, wb.w)
    su.shard_update_lamb_partials(plan, r, wb.w, wb.g, wb.m, wb.v, hp, 1, wb.local)
    wb.m.zero_(); wb.v.zero_()
    wb.other.copy_(wb.local * float(N - 1))
    state = {"t": 0}

    def one_step():
        state["t"] += 1
        su.shard_format(plan, r, wb.full_g, wb.g)
        su.shard_update_lamb(plan, r, wb.w, wb.g, wb.m, wb.v, hp, state["t"], other_replicas_sumsq=wb.other)
        su.unshard_format(plan, wb.gathered, wb.full_w)

    unshard_walk = wb.settle_copies()["unshard_format"]
    for _ in range(max(args.warmup, 2)):
        one_step()
    ms_step, wall_ms = _time_region(torch, one_step, args.steps)
    # the same K steps once more, each inside an event pair of its own: the median beside the mean
    step_pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in step_pairs:
        a.record(); one_step(); b.record()
    torch.cuda.synchronize()
    median_ms_step = _median([a.elapsed_time(b) for a, b in step_pairs])

    # instrumented pass: the same K steps with an event pair around every kernel
    su.shard_profile_reset(plan)
    su.shard_profile_enable(plan, True)
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    kern = {}
    for name in ("format", "lamb_p1", "norm_reduce", "lamb_p2", "unshard", "ptr_table"):
        n, ms = su.shard_profile_read(plan, name)
        if n:
            kern[name] = {"launches": n, "avg_us": 1e3 * ms / n}
    su.shard_profile_enable(plan, False)

    S = wb.S
    alg_bytes = {
        "format": BYTES_PER_SLOT["format"] * S,
        "lamb_p1": BYTES_PER_SLOT["lamb_p1"] * S,
        "lamb_p2": BYTES_PER_SLOT["lamb_p2"] * S,
        "unshard": 4 * N * S + 4 * cfg.total,
    }
    rooflines = {}
    for name, b in alg_bytes.items():
        if name in kern:
            gbs = b / (kern[name]["avg_us"] * 1e-6) / 1e9
            rooflines[name] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": round(gbs / HBM_PEAK_GBS, 4), "avg_us": round(kern[name]["avg_us"], 2),
                               "bytes": b}
    dominant = max(rooflines, key=lambda k: rooflines[k]["avg_us"])
    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command, kept as a summary
    # under profiles/ ("traffic <kernel> <bytes>" lines) together with the hash of the library sources it was
    # measured on.  Counters cannot be read inside this run, so the figure is only reported while that hash is the
    # hash of the sources in this tree; otherwise traffic is null and traffic_source says why.
    traffic, traffic_source = None, None
    roof = dict(rooflines[dominant])
    roof["kernel"] = dominant + "_kernel"
    if dominant == "unshard" and unshard_walk["walk"] == "by_variable":
        roof["kernel"] = "unshard_flat_kernel"       # the copy was tuned onto its other order: another kernel
    tname = "bench_%s_lamb_n%d_hbm_traffic.txt" % (cfg.name, N)
    tpath = os.path.join(ROOT, "profiles", tname)
    if os.path.exists(tpath):
        measured_on, found = None, None
        for line in open(tpath):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic" and parts[1] == roof["kernel"]:
                found = int(parts[2])
            if len(parts) == 2 and parts[0] == "sources_sha16":
                measured_on = parts[1]
        current = sources_sha16()
        fresh = measured_on == current
        traffic = found if fresh else None
        traffic_source = {"file": "profiles/" + tname, "measured_on_sources_sha16": measured_on,
                          "this_build_sources_sha16": current,
                          "note": "measured by rocprofv3 --pmc in a separate run of this command; reported only while "
                                  "the library sources are the ones it was measured on" +
                                  ("" if fresh else " (they are not: traffic withheld)")}
    roof["traffic"] = traffic
    roof["traffic_source"] = traffic_source
    lamb_us = sum(kern[k]["avg_us"] for k in ("lamb_p1", "norm_reduce", "lamb_p2") if k in kern)
    update_only = {
        "kernels_us": round(lamb_us, 2),
        "params_per_s": wb.real / (lamb_us * 1e-6),
        "GBps": round(40 * S / (lamb_us * 1e-6) / 1e9, 1),
        "frac_of_hbm_peak": round(40 * S / (lamb_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
    }
    # the practical ceiling, measured in this same run on this same GPU: a plain copy (no table, no padding)
    # that moves as many bytes as unshard_format does
    half = (4 * N * S + 4 * cfg.total) // 2 // 16 * 16
    ca = torch.empty(half, dtype=torch.uint8, device="cuda"); cb = torch.empty(half, dtype=torch.uint8, device="cuda")
    ca.zero_()
    for _ in range(3):
        su.shard_profile_plain_copy(plan, cb, ca)
    su.shard_profile_reset(plan); su.shard_profile_enable(plan, True)
    for _ in range(20):
        su.shard_profile_plain_copy(plan, cb, ca)
    torch.cuda.synchronize()
    n_copy, ms_copy = su.shard_profile_read(plan, "plain_copy")
    su.shard_profile_enable(plan, False)
    copy_us = 1e3 * ms_copy / n_copy
    plain_copy = {"bytes": 2 * half, "avg_us": round(copy_us, 2), "GBps": round(2 * half / (copy_us * 1e-6) / 1e9, 1),
                  "frac_of_hbm_peak": round(2 * half / (copy_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                  "what": "plain device copy of the bytes unshard_format moves (one 128-bit access per thread, "
                          "non-temporal): the practical ceiling on this GPU, same run"}
    del ca, cb

    # The same step as the paper runs it (Section 4.2, all-gather in bfloat16): the float32 update also
    # emits bf16(w') into this replica's row of a bfloat16 gathered buffer, and unshard_format restores
    # bfloat16 tensors for the forward pass.  Reported beside the float32 headline, never as `value`.
    g16 = su.gathered_empty(plan, dtype=torch.bfloat16).normal_(0.0, cfg.weight_std, generator=wb.gen)
    flat16 = torch.empty(cfg.total, dtype=torch.bfloat16, device="cuda")
    full16, pos = [], 0
    for n in cfg.numel:
        full16.append(flat16[pos:pos + n])
        pos += n
    full16 = su.FullTensors(plan, full16)

    def one_step_bf16():
        state["t"] += 1
        su.shard_format(plan, r, wb.full_g, wb.g)
        su.shard_update_lamb(plan, r, wb.w, wb.g, wb.m, wb.v, hp, state["t"], other_replicas_sumsq=wb.other,
                             w_bf16_out=g16[r])
        su.unshard_format(plan, g16, full16)

    _settle_copy(torch, su, plan, "unshard_format", g16, full16)
    for _ in range(3):
        one_step_bf16()
    ms16, _ = _time_region(torch, one_step_bf16, args.steps)
    bf16_gather = {"ms_per_step": round(ms16, 5), "params_per_s": wb.real / (ms16 * 1e-3),
                   "what": "float32 LAMB update that also writes bf16(w'), bfloat16 gathered buffer and full tensors"}

    # both at once: gradient read in place from the full tensors, weights gathered in bfloat16
    def one_step_fused_bf16():
        state["t"] += 1
        su.shard_update_lamb_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v, hp, state["t"],
                                        other_replicas_sumsq=wb.other, w_bf16_out=g16[r])
        su.unshard_format(plan, g16, full16)

    for _ in range(3):
        one_step_fused_bf16()
    msfb, _ = _time_region(torch, one_step_fused_bf16, args.steps)
    fused_bf16 = {"ms_per_step": round(msfb, 5), "params_per_s": wb.real / (msfb * 1e-3),
                  "what": "shard_update_lamb_full_grads that also writes bf16(w') + bfloat16 unshard_format"}
    del g16, flat16, full16

    # The same float32 step with the formatting of the gradient fused into the update (Section 5.1): phase 1
    # reads replica r's pieces of the full gradients in place and no shard gradient is written.  Same
    # result bit for bit; reported beside the headline, never as `value`.
    def one_step_fused():
        state["t"] += 1
        su.shard_update_lamb_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v, hp, state["t"],
                                        other_replicas_sumsq=wb.other)
        su.unshard_format(plan, wb.gathered, wb.full_w)

    for _ in range(3):
        one_step_fused()
    msf, _ = _time_region(torch, one_step_fused, args.steps)
    fused_format = {"ms_per_step": round(msf, 5), "params_per_s": wb.real / (msf * 1e-3),
                    "what": "shard_update_lamb_full_grads (gradient read in place from the full tensors, no "
                            "shard_format launch) + unshard_format(w)"}

    out = {
        "metric": "shard weight-update params/s (340M LAMB, N=8, one replica's shard)",
        "value": wb.real / (ms_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5),
        "median_ms_per_step": round(median_ms_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s fp32 LAMB N=%d r=%d: shard_format(g) + shard_update_lamb + unshard_format(w)"
                               % (cfg.name, N, r),
                   "variables": plan.V, "params": cfg.total, "shard_slots": S, "shard_params": wb.real,
                   "chunk_elems": plan.chunk_elems, "unshard_order": unshard_walk},
        "roofline": roof,
        "kernels": rooflines,
        "update_only": update_only,
        "plain_copy": plain_copy,
        "bf16_gather": bf16_gather,
        "fused_format": fused_format,
        "fused_format_bf16_gather": fused_bf16,
        "wall_ms_per_step": round(wall_ms, 5),
    }
    wb.free()
    return out


def cpu_baseline(cfg, N, r):
    """The oracle, as it stands, on one step of the same workload; numpy runs single-threaded."""
    import numpy as np
    import oracle
    from workloads import normal_f32
    hp = {k: float(np.float32(v)) for k, v in cfg.hyper.items()}
    plan = oracle.make_plan(cfg.numel, N, 8)
    gs = [normal_f32(cfg.seed, i, "g", n, cfg.grad_std, 1) for i, n in enumerate(cfg.numel)]
    gathered = np.zeros((N, plan.S), np.float32)
    gathered[r] = oracle.shard_format(plan, r, [normal_f32(cfg.seed, i, "w", n, cfg.weight_std)
                                                for i, n in enumerate(cfg.numel)])
    m = np.zeros(plan.S, np.float32); v = np.zeros(plan.S, np.float32)
    real = sum(plan.real_count(i, r) for i in range(plan.V))
    steps, t0 = 0, time.perf_counter()
    while True:                                   # whole steps until about 12 s of CPU work are done
        steps += 1
        g = oracle.shard_format(plan, r, gs)
        m, v, u, part = oracle.lamb_shard_partials(plan, r, gathered[r], g, m, v, hp, steps)
        gathered[r] = oracle.lamb_shard_apply(plan, gathered[r], u, part * N, hp)
        full = oracle.unshard_format(plan, gathered)
        assert len(full) == plan.V
        dt = time.perf_counter() - t0
        if dt >= 12.0 or steps >= 64:
            break
    return {"value": real * steps / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": "%d steps of the same workload (%s N=%d r=%d, all %d variables: format g, LAMB on the shard, "
                      "unformat the whole model) in %.1f s" % (steps, cfg.name, N, r, plan.V, dt),
            "seconds": round(dt, 2)}


def _cpu_worker(job):
    """One worker of the all-cores baseline: whole steps of the same oracle on a subset of the variables."""
    name, N, r, indices, seconds = job
    import numpy as np
    import oracle
    from workloads import CONFIGS, normal_f32
    cfg = [c for c in CONFIGS if c.name == name][0]
    hp = {k: float(np.float32(v)) for k, v in cfg.hyper.items()}
    numel = [cfg.numel[i] for i in indices]
    plan = oracle.make_plan(numel, N, 8)
    gs = [normal_f32(cfg.seed, i, "g", cfg.numel[i], cfg.grad_std, 1) for i in indices]
    gathered = np.zeros((N, plan.S), np.float32)
    gathered[r] = oracle.shard_format(plan, r, [normal_f32(cfg.seed, i, "w", cfg.numel[i], cfg.weight_std) for i in indices])
    m = np.zeros(plan.S, np.float32); v = np.zeros(plan.S, np.float32)
    steps, t0 = 0, time.perf_counter()
    while True:
        steps += 1
        g = oracle.shard_format(plan, r, gs)
        m, v, u, part = oracle.lamb_shard_partials(plan, r, gathered[r], g, m, v, hp, steps)
        gathered[r] = oracle.lamb_shard_apply(plan, gathered[r], u, part * N, hp)
        oracle.unshard_format(plan, gathered)
        dt = time.perf_counter() - t0
        if dt >= seconds or steps >= 64:
            break
    return steps / dt


def cpu_baseline_all_cores(cfg, N, r, workers):
    """The same oracle with the variables dealt out to `workers` processes (every variable is independent
    of the others in this path); a whole step is done when the slowest worker is, so the rate is the
    shard's parameters times the lowest steps/s.  Must run before this process touches the GPU."""
    import multiprocessing as mp
    import oracle
    order = sorted(range(len(cfg.numel)), key=lambda i: -cfg.numel[i])
    groups, load = [[] for _ in range(workers)], [0] * workers
    for i in order:                                   # largest first onto the least loaded worker
        k = load.index(min(load))
        groups[k].append(i)
        load[k] += cfg.numel[i]
    groups = [sorted(g) for g in groups if g]
    plan = oracle.make_plan(cfg.numel, N, 8)
    real = sum(plan.real_count(i, r) for i in range(plan.V))
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(len(groups)) as pool:
        rates = pool.map(_cpu_worker, [(cfg.name, N, r, g, 10.0) for g in groups])
    dt = time.perf_counter() - t0
    return {"value": real * min(rates), "unit": "params/s", "cores": len(groups), "kind": "oracle",
            "sample": "the same whole steps with the %d variables dealt out to %d processes (numpy itself is "
                      "single-threaded), about 10 s each; rate = shard parameters x the slowest process's steps/s"
                      % (plan.V, len(groups)), "seconds": round(dt, 2)}


def table(args, torch, su, cfgs, path):
    """Every config x stage; written as JSON.  "us" is the time of one call of the stage with 50 calls back to back
    inside one event pair after 10 warm-up calls (several kernels in a row are timed together, as they run);
    "median_us" the median of 50 calls timed one by one; "kernel_us" the per-kernel breakdown."""
    rows = []
    for cfg in cfgs:
        # N = 1 is the replicated update the paper compares against (every replica updates the whole
        # model); where a configuration does not list it, only its update stage is timed
        for N in sorted(set(cfg.replicas) | {1}):
            r = 0
            big = cfg.total > 1_000_000_000
            extra = N not in cfg.replicas
            wb = Workbench(cfg, N, r, args.chunk, torch, su, want_full=not ((big and N == 1) or extra))
            plan, hp, S = wb.plan, wb.hp(), wb.S
            if cfg.mixed_bf16:
                wb.w16 = torch.zeros(S, dtype=torch.bfloat16, device="cuda")
            stages = []
            if cfg.optimizer == "adam":
                stages.append(("adam", lambda t: su.shard_update_adam(plan, r, wb.w, wb.g, wb.m, wb.v, hp, t,
                                                                      w_bf16_out=wb.w16),
                               ["adam"], (30 if cfg.mixed_bf16 else 28) * S))
            elif cfg.optimizer == "momentum":
                stages.append(("momentum", lambda t: su.shard_update_momentum(plan, r, wb.w, wb.g, wb.m, hp),
                               ["momentum"], 20 * S))
                lars_hp = dict(hp, trust_coeff=0.001, eps=0.0)     # the paper's optimizer for this model
                stages.append(("lars", lambda t: su.shard_update_lars(plan, r, wb.w, wb.g, wb.m, lars_hp,
                                                                      other_replicas_sumsq=wb.other),
                               ["lars_p1", "norm_reduce", "lars_p2"], 28 * S))
            else:
                stages.append(("lamb", lambda t: su.shard_update_lamb(plan, r, wb.w, wb.g, wb.m, wb.v, hp, t,
                                                                      other_replicas_sumsq=wb.other),
                               ["lamb_p1", "norm_reduce", "lamb_p2"], 40 * S))
            if wb.full_g is not None:
                # the same update with the gradient read in place from the full tensors (no shard_format)
                if cfg.optimizer == "adam":
                    stages.append(("adam_full_grads",
                                   lambda t: su.shard_update_adam_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v, hp, t,
                                                                             w_bf16_out=wb.w16),
                                   ["adam"], (30 if cfg.mixed_bf16 else 28) * S))
                elif cfg.optimizer == "momentum":
                    stages.append(("momentum_full_grads",
                                   lambda t: su.shard_update_momentum_full_grads(plan, r, wb.w, wb.full_g, wb.m, hp),
                                   ["momentum"], 20 * S))
                    stages.append(("lars_full_grads",
                                   lambda t: su.shard_update_lars_full_grads(plan, r, wb.w, wb.full_g, wb.m, lars_hp,
                                                                             other_replicas_sumsq=wb.other),
                                   ["lars_p1", "norm_reduce", "lars_p2"], 28 * S))
                else:
                    stages.append(("lamb_full_grads",
                                   lambda t: su.shard_update_lamb_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v, hp, t,
                                                                             other_replicas_sumsq=wb.other),
                                   ["lamb_p1", "norm_reduce", "lamb_p2"], 40 * S))
                stages.append(("shard_format", lambda t: su.shard_format(plan, r, wb.full_g, wb.g), ["format"], 8 * S))
                stages.append(("unshard_format", lambda t: su.unshard_format(plan, wb.gathered, wb.full_w),
                               ["unshard"], 4 * N * S + 4 * cfg.total))
                stages.append(("shard_format_all", lambda t: su.shard_format_all(plan, wb.full_g, wb.gathered),
                               ["format"], 4 * N * S + 4 * cfg.total))
                # the whole step of the configuration's optimizer: kernels timed one by one but run back to back in
                # a loop, so what one kernel leaves in the caches for the next to pay is inside the sum
                opt_name, opt_fn, opt_kernels, opt_bytes = stages[0]

                def whole_step(t, update=opt_fn):
                    su.shard_format(plan, r, wb.full_g, wb.g)
                    update(t)
                    su.unshard_format(plan, wb.gathered, wb.full_w)
                stages.append(("step: format + %s + unshard" % opt_name, whole_step, ["format"] + opt_kernels + ["unshard"],
                               8 * S + opt_bytes + 4 * N * S + 4 * cfg.total))
            copy_orders = wb.settle_copies(format_all=True)
            for name, fn, kernels, nbytes in stages:
                tm = _time_stage(torch, su, plan, fn, kernels, 10, 50)
                us = tm["region_us"]
                rows.append({"config": cfg.name, "N": N, "stage": name + (" (replicated)" if extra else ""), "S": S,
                             "us": us, "median_us": tm["median_us"], "kernel_us": tm["kernel_us"],
                             "params_per_s": wb.real / (us * 1e-6), "GBps": round(nbytes / (us * 1e-6) / 1e9, 1),
                             "frac_hbm_peak": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                             "cache_resident": nbytes < 256e6})
                if name in copy_orders:
                    rows[-1]["order"] = copy_orders[name]["walk"]
                print("table:", rows[-1], file=sys.stderr, flush=True)
            wb.free()
            del wb
            torch.cuda.empty_cache()
            if all(len(s) <= 2 for s in cfg.shapes) and cfg.total < 1_000_000_000 and not extra:
                rows.append(_adafactor_row(cfg, N, torch, su))
                print("table:", rows[-1], file=sys.stderr, flush=True)
    with open(path, "w") as f:
        json.dump(rows, f, indent=1)


def one_stage(args, torch, su, cfgs):
    """One stage of one configuration, --warmup + --steps launches; a small JSON line of its own."""
    cfg = [c for c in cfgs if c.name == args.config][0]
    N, r, name = args.replicas, args.replica_id, args.stage
    if name == "adafactor":
        row = _adafactor_row(cfg, N, torch, su, warmup=args.warmup, iters=args.steps)
        print(json.dumps(row))
        return
    if name == "adam_shape_probe":
        _adam_shape_probe(args, cfg, N, r, torch, su)
        return
    if name == "copy_order_probe":
        _copy_order_probe(args, N, torch, su)
        return
    bf16_names = ("unshard_format_bf16", "unshard_format_f32_to_bf16", "shard_format_bf16_to_f32", "lamb_step_bf16",
                  "lamb_fused_step_bf16")
    needs_full = (name in ("shard_format", "unshard_format", "shard_format_all") + bf16_names
                  or name.endswith("_full_grads")
                  or name.endswith("_step"))
    wb = Workbench(cfg, N, r, args.chunk, torch, su, want_full=needs_full, separate=args.separate_tensors,
                   copy_order=args.copy_order)
    plan, S = wb.plan, wb.S
    hp = wb.hp()
    adam_hp = hp if cfg.optimizer == "adam" else {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0}
    lamb_hp = hp if cfg.optimizer == "lamb" else {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01}
    mom_hp = hp if cfg.optimizer == "momentum" else {"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5}
    lars_hp = dict(mom_hp, trust_coeff=0.001, eps=0.0)
    if cfg.mixed_bf16:
        wb.w16 = torch.zeros(S, dtype=torch.bfloat16, device="cuda")
    stages = {
        "adam": (lambda t: su.shard_update_adam(plan, r, wb.w, wb.g, wb.m, wb.v, adam_hp, t, w_bf16_out=wb.w16),
                 ["adam"], (30 if cfg.mixed_bf16 else 28) * S),
        "momentum": (lambda t: su.shard_update_momentum(plan, r, wb.w, wb.g, wb.m, mom_hp), ["momentum"], 20 * S),
        "lars": (lambda t: su.shard_update_lars(plan, r, wb.w, wb.g, wb.m, lars_hp, other_replicas_sumsq=wb.other),
                 ["lars_p1", "norm_reduce", "lars_p2"], 28 * S),
        "lamb": (lambda t: su.shard_update_lamb(plan, r, wb.w, wb.g, wb.m, wb.v, lamb_hp, t, other_replicas_sumsq=wb.other),
                 ["lamb_p1", "norm_reduce", "lamb_p2"], 40 * S),
    }
    if needs_full:
        # the updates that read the gradient in place from the full tensors: the bytes of the plain update
        stages["adam_full_grads"] = (lambda t: su.shard_update_adam_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v,
                                                                                adam_hp, t, w_bf16_out=wb.w16),
                                     ["adam"], (30 if cfg.mixed_bf16 else 28) * S)
        stages["momentum_full_grads"] = (lambda t: su.shard_update_momentum_full_grads(plan, r, wb.w, wb.full_g, wb.m,
                                                                                        mom_hp), ["momentum"], 20 * S)
        stages["lamb_full_grads"] = (lambda t: su.shard_update_lamb_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v,
                                                                                lamb_hp, t,
                                                                                other_replicas_sumsq=wb.other),
                                     ["lamb_p1", "norm_reduce", "lamb_p2"], 40 * S)
        stages["lars_full_grads"] = (lambda t: su.shard_update_lars_full_grads(plan, r, wb.w, wb.full_g, wb.m, lars_hp,
                                                                                other_replicas_sumsq=wb.other),
                                     ["lars_p1", "norm_reduce", "lars_p2"], 28 * S)
        # whole steps (format g, update, unshard w) of each optimizer: what a cache policy costs or gains
        # the kernel AFTER it only shows in such a sum
        step_bytes = 8 * S + 4 * N * S + 4 * cfg.total

        def _step(update):
            def run(t):
                su.shard_format(plan, r, wb.full_g, wb.g)
                update(t)
                su.unshard_format(plan, wb.gathered, wb.full_w)
            return run
        for opt in ("adam", "momentum", "lars", "lamb"):
            fn0, ks, nb = stages[opt]
            stages[opt + "_step"] = (_step(fn0), ["format"] + ks + ["unshard"], nb + step_bytes)
        stages["shard_format"] = (lambda t: su.shard_format(plan, r, wb.full_g, wb.g), ["format"], 8 * S)
        stages["unshard_format"] = (lambda t: su.unshard_format(plan, wb.gathered, wb.full_w), ["unshard"],
                                    4 * N * S + 4 * cfg.total)
        stages["shard_format_all"] = (lambda t: su.shard_format_all(plan, wb.full_g, wb.gathered), ["format"],
                                      4 * N * S + 4 * cfg.total)
        if name in bf16_names:                                  # the all-gather in bfloat16 (Section 4.2)
            g16 = su.gathered_empty(plan, dtype=torch.bfloat16).normal_(0.0, cfg.weight_std)
            flat16 = torch.empty(cfg.total, dtype=torch.bfloat16, device="cuda").normal_(0.0, cfg.grad_std)
            full16, pos = [], 0
            for n in cfg.numel:
                full16.append(flat16[pos:pos + n]); pos += n
            full16 = su.FullTensors(plan, full16)
            model16 = 2 * N * S + 2 * cfg.total
            stages["unshard_format_bf16"] = (lambda t: su.unshard_format(plan, g16, full16), ["unshard"], model16)
            # the converting copies: float32 gathered rows -> bfloat16 tensors, bfloat16 gradients -> float32 shard
            stages["unshard_format_f32_to_bf16"] = (lambda t: su.unshard_format(plan, wb.gathered, full16), ["unshard"],
                                                    4 * N * S + 2 * cfg.total)
            stages["shard_format_bf16_to_f32"] = (lambda t: su.shard_format(plan, r, full16, wb.g), ["format"], 6 * S)

            # the step as the paper runs it: float32 update that also emits bf16(w'), bfloat16 gather buffer and tensors
            def lamb_step_bf16(t):
                su.shard_format(plan, r, wb.full_g, wb.g)
                su.shard_update_lamb(plan, r, wb.w, wb.g, wb.m, wb.v, lamb_hp, t, other_replicas_sumsq=wb.other,
                                     w_bf16_out=g16[r])
                su.unshard_format(plan, g16, full16)

            def lamb_fused_step_bf16(t):
                su.shard_update_lamb_full_grads(plan, r, wb.w, wb.full_g, wb.m, wb.v, lamb_hp, t,
                                                other_replicas_sumsq=wb.other, w_bf16_out=g16[r])
                su.unshard_format(plan, g16, full16)
            stages["lamb_step_bf16"] = (lamb_step_bf16, ["format", "lamb_p1", "norm_reduce", "lamb_p2", "unshard"],
                                        8 * S + 42 * S + model16)
            stages["lamb_fused_step_bf16"] = (lamb_fused_step_bf16, ["lamb_p1", "norm_reduce", "lamb_p2", "unshard"],
                                              42 * S + model16)
    if name not in stages:
        raise SystemExit("unknown --stage %s" % name)
    fn, kernels, nbytes = stages[name]
    copy_orders = wb.settle_copies(format_all=name == "shard_format_all") if needs_full else {}
    if name in bf16_names and name != "shard_format_bf16_to_f32":
        src = wb.gathered if name == "unshard_format_f32_to_bf16" else g16
        copy_orders = {"unshard_format": _settle_copy(torch, su, plan, "unshard_format", src, full16)}
    # --cold: a 1 GiB device copy between launches of the stage, so that nothing of the previous launch is
    # left in the 256 MB memory-side cache (between two real steps a forward and a backward pass run); the
    # event pairs time the library's kernels only
    spill = torch.empty((2, 1 << 28), dtype=torch.float32, device="cuda") if args.cold else None
    if spill is None:
        tm = _time_stage(torch, su, plan, fn, kernels, args.warmup, args.steps)
        per, us, median_us = tm["kernel_us"], tm["region_us"], tm["median_us"]
    else:
        # cold: only the library's own event pairs see the kernels without the spill
        for t in range(1, 1 + max(args.warmup, 1)):
            fn(t)
        su.shard_profile_reset(plan); su.shard_profile_enable(plan, True)
        for t in range(100, 100 + args.steps):
            spill[1].copy_(spill[0])
            fn(t)
        torch.cuda.synchronize()
        per = {}
        for k in kernels:
            n, ms = su.shard_profile_read(plan, k)
            per[k] = round(1e3 * ms / args.steps, 2)
        us, median_us = sum(per.values()), None
    extra = {}
    if args.graph and spill is None:
        # the same stage recorded once with stream capture and replayed: what launching costs beyond the kernels
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            fn(5000)                              # the lists of tensors become resident on this stream's device
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            fn(5001)
        torch.cuda.synchronize()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize(); a.record()
        for _ in range(args.steps):
            graph.replay()
        b.record(); torch.cuda.synchronize()
        extra["graph_replay_us"] = round(1e3 * a.elapsed_time(b) / args.steps, 2)
        del graph
    if name.startswith(("unshard_format", "shard_format_all")) and spill is None:
        # the practical ceiling for this copy: a plain device copy of the same number of bytes, same run
        half = nbytes // 2 // 16 * 16
        ca = torch.empty(half, dtype=torch.uint8, device="cuda").zero_(); cb = torch.empty(half, dtype=torch.uint8, device="cuda")
        tm_copy = _time_stage(torch, su, plan, lambda t: su.shard_profile_plain_copy(plan, cb, ca), ["plain_copy"],
                              args.warmup, args.steps)
        extra["plain_copy_same_bytes_us"] = tm_copy["region_us"]
    print(json.dumps({"config": cfg.name, "N": N, "stage": name, "S": S, "launches": args.steps, "kernel_us": per,
                      "total_us": round(us, 2), "median_us": median_us, **extra,
                      "timing": "sum of per-kernel event pairs" if args.cold else "region: calls back to back in one event pair",
                      "bytes": nbytes, "GBps": round(nbytes / (us * 1e-6) / 1e9, 1),
                      "frac_hbm_peak": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "cold": bool(args.cold),
                      "separate_tensors": bool(args.separate_tensors), "copy_orders": copy_orders}))
    wb.free()


def _copy_order_probe(args, N, torch, su):
    """Where the caller's tensors lie decides which order of a whole-model copy is faster.  A uniform model of 320
    float32 matrices of 1024 x 1024 (2.69 GB moved per copy at N = 8), each tensor a fixed distance after the
    previous one; for four distances: unshard_format and shard_format_all with the order forced either way, and
    what shard_plan_tune_copy_walk settles on.  --config is ignored."""
    V, n = 320, 1024 * 1024
    rows = []
    for skew_bytes in (0, 256, 4096, 16384):
        skew = skew_bytes // 4
        flat = torch.empty(V * (n + skew) + 64, dtype=torch.float32, device="cuda").normal_(0, 1e-3)
        row = {"distance": "4 MiB + %d B" % skew_bytes}
        for order in ("by_replica", "by_variable", "auto"):
            plan = su.shard_plan_bind(su.shard_plan([n] * V, N, 8))
            su.shard_plan_set_copy_walk(plan, order)
            full = su.FullTensors(plan, [flat[i * (n + skew): i * (n + skew) + n] for i in range(V)])
            gathered = su.gathered_empty(plan).normal_(0, 0.02)
            for copy, fn, k in (("unshard_format", lambda t: su.unshard_format(plan, gathered, full), "unshard"),
                                ("shard_format_all", lambda t: su.shard_format_all(plan, full, gathered), "format")):
                picked = None
                if order == "auto":
                    picked = su.shard_plan_tune_copy_walk(plan, copy, gathered, full)[0]
                tm = _time_stage(torch, su, plan, fn, [k], args.warmup, args.steps)
                row["%s %s" % (copy, "tuned" if order == "auto" else order)] = tm["region_us"]
                if picked:
                    row["%s tuned picks" % copy] = picked
            plan.free()
            del full, gathered
        rows.append(row)
        print("spacing:", row, file=sys.stderr, flush=True)
        del flat
        torch.cuda.empty_cache()
    print(json.dumps({"stage": "copy_order_probe", "N": N, "model": "320 float32 matrices of 1024 x 1024", "launches": args.steps,
                      "rows": rows}))


def _adam_shape_probe(args, cfg, N, r, torch, su):
    """The measurement behind the library's choice of launch shape: the flat Adam update of this shard in every
    shape shard_profile_adam_shape offers (threads per workgroup x workgroups resident per CU), each timed as
    --steps launches back to back, then the shape the library itself picks and a plain copy of the same bytes."""
    wb = Workbench(cfg, N, r, args.chunk, torch, su, want_full=False)
    plan, S = wb.plan, wb.S
    hp = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0}
    nbytes = 28 * S
    rows = []

    def region(fn):
        for t in range(1, 4):
            fn(t)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize(); a.record()
        for t in range(10, 10 + args.steps):
            fn(t)
        b.record(); torch.cuda.synchronize()
        return 1e3 * a.elapsed_time(b) / args.steps
    for block in (256, 128):
        for k in (0, 8, 6, 5, 4, 3):
            us = region(lambda t: su.shard_profile_adam_shape(plan, wb.w, wb.g, wb.m, wb.v, hp, t, block, k))
            rows.append({"threads": block, "workgroups_per_cu": k, "lds_bytes": 0 if k == 0 else 160 * 1024 // k - 1024,
                         "us": round(us, 1), "GBps": round(nbytes / us / 1e3, 1)})
            print("shape:", rows[-1], file=sys.stderr, flush=True)
    us_lib = region(lambda t: su.shard_update_adam(plan, r, wb.w, wb.g, wb.m, wb.v, hp, t))
    half = nbytes // 2 // 16 * 16
    ca = torch.empty(half, dtype=torch.uint8, device="cuda").zero_(); cb = torch.empty(half, dtype=torch.uint8, device="cuda")
    us_copy = region(lambda t: su.shard_profile_plain_copy(plan, cb, ca))
    print(json.dumps({"config": cfg.name, "N": N, "stage": "adam_shape_probe", "S": S, "launches": args.steps,
                      "bytes": nbytes, "shapes": rows,
                      "library_choice": {"us": round(us_lib, 1), "GBps": round(nbytes / us_lib / 1e3, 1)},
                      "plain_copy_same_bytes": {"us": round(us_copy, 1), "GBps": round(2 * half / us_copy / 1e3, 1)}}))
    wb.free()


def _adafactor_row(cfg, N, torch, su, warmup=10, iters=50):
    """Adafactor on the row plan of the same variables (matrices by rows, vectors as n x 1): 24 B/slot
    (g and w read by the reductions, g by the clipping sum, g and w read and w written by the update)."""
    shapes = [(s[0], s[1]) if len(s) == 2 else (s[0], 1) for s in cfg.shapes]
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, 8))
    _, _, total_rows, total_cols = su.shard_plan_rowcol_layout(plan)
    S = plan.S
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    w = _device_normal(S, cfg.weight_std, gen, torch)
    g = _device_normal(S, cfg.grad_std, gen, torch)
    R = torch.zeros(max(total_rows, 1), dtype=torch.float32, device="cuda")
    C = torch.zeros(max(total_cols, 1), dtype=torch.float32, device="cuda")
    hp = {"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2}
    tm = _time_stage(torch, su, plan, lambda t: su.shard_update_adafactor(plan, 0, w, g, R, C, hp, t),
                     ("rowcol_p1", "rowcol_p2", "adafactor_state", "adafactor_usq", "item_total", "adafactor_apply"),
                     warmup, iters)
    us = tm["region_us"]
    real = sum(plan.real_count(0))
    nbytes = 24 * S
    row = {"config": cfg.name, "N": N, "stage": "adafactor (row plan)", "S": S, "us": us, "total_us": us,
           "median_us": tm["median_us"], "kernel_us": tm["kernel_us"],
           "params_per_s": real / (us * 1e-6), "GBps": round(nbytes / (us * 1e-6) / 1e9, 1),
           "frac_hbm_peak": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "cache_resident": nbytes < 256e6}
    plan.free()
    return row


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one replica's shard on ONE GPU; --gpus %d is not supported "
              "(the cross-replica collectives are outside this library)" % args.gpus, file=sys.stderr)
        raise SystemExit(2)
    import torch
    if torch.cuda.device_count() < 1:           # counting devices does not initialise the GPU
        print("bench.py needs a GPU", file=sys.stderr)
        raise SystemExit(2)
    cpu = None
    if not args.no_cpu_baseline and not args.stage:
        # the oracle legs first: the all-cores one forks workers, which must happen before the GPU is touched
        from workloads import CONFIGS as _CFGS
        cfg0 = [c for c in _CFGS if c.name == args.config][0]
        cpu = (cpu_baseline(cfg0, args.replicas, args.replica_id),
               cpu_baseline_all_cores(cfg0, args.replicas, args.replica_id, min(16, os.cpu_count() or 1)))
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        raise SystemExit(2)
    import paper_2004_13336_amd as su
    from workloads import CONFIGS
    su.lib()
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    if args.stage:
        one_stage(args, torch, su, CONFIGS)
        return
    out = headline(args, torch, su, CONFIGS)
    if args.table:
        table(args, torch, su, CONFIGS, args.table)
    out["cpu_baseline"] = cpu[0] if cpu else None
    out["cpu_baseline_all_cores"] = cpu[1] if cpu else None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
