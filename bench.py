#!/usr/bin/env python3
"""Benchmark of the ReDrafter verification step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
rd_dedup -> rd_tree_attn (one layer's attention core) -> rd_accept, back to back on one
stream with all inputs resident in HBM.  The headline workload is the Vicuna-7B-shaped
configuration (B=1, context 1024, H=32, D=128, bf16 KV, W=8, L=5, vocab 32000).

To keep the infinity cache from serving the KV stream, step i works on copy i mod R of R
independent input copies whose K/V total exceeds 512 MiB, and a buffer larger than every cache is
overwritten before each timed region.  The timed region consists of HIP-graph replays only,
whatever --steps is: the library only enqueues kernels, so a caller can capture them; the steps
W .. W+K-1 of the rotation are cut into graphs of at most R consecutive steps, captured before the
clock starts, and replayed so that EXACTLY K steps run between the two events (--no-graph times
eager launches instead and says so in config.launch).

Beside the headline figures the JSON line carries a `configs` block with the attention launch time
(median and 10th / 90th percentile over graph replays), algorithmic bytes, fraction of the 8 TB/s
HBM peak, the plain streaming-read floor of the same bytes, the step time and the CPU oracle's rate
for each of the five synthetic configurations.

Prints one JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "rd_tree_attn_hbm_traffic.md")
LAYERS_BY_HEADS = {32: 32, 40: 40, 52: 60}      # decoder layers of the 7B / 13B / 33B models the shapes come from
FLUSH_BYTES = 1 << 30                           # larger than the 256 MB infinity cache plus every L2


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6400)
    ap.add_argument("--warmup", type=int, default=640)
    ap.add_argument("--config", type=int, default=2, help="headline workload 1..5 (default 2: Vicuna-7B-shaped layer)")
    ap.add_argument("--copies", type=int, default=0, help="rotating input copies (0 = enough for > 512 MiB of K/V)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-draft", action="store_true", help="skip the separate rd_draft timing")
    ap.add_argument("--no-floor", action="store_true", help="skip the plain streaming-read floor measurement")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration block (configs 1..5)")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline kernels only: no warm-cache figure, no rd_commit / rd_accept_sample / live-context "
                         "timings (so that a kernel trace or counter run holds the step's launches only)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="CPU time budget of the oracle baseline")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also run plain device copies of 64 MiB (reference dispatches for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def read_traffic_table():
    """HBM bytes per rd_tree_attn launch by configuration, from the committed counter summary
    (rows `| config | FETCH_SIZE | WRITE_SIZE | fetch scale | write scale | bytes |`)."""
    out = {}
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 6 and cells[0].isdigit():
                    out[int(cells[0])] = int(float(cells[5]))
    except OSError:
        pass
    return out


class Workload:
    """R independent synthetic batches of one configuration on the device, with the closures that
    enqueue the library's calls on them."""

    def __init__(self, cfg, R, rd, synth, torch, ctx_override=None):
        self.cfg, self.R, self.rd, self.torch = cfg, R, rd, torch
        dev = torch.device("cuda:0")
        self.esz = 4 if cfg.dtype == "f32" else 2
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        self.dt_code = rd.RD_F32 if cfg.dtype == "f32" else rd.RD_BF16
        self.scale = float(1.0 / np.sqrt(cfg.D))
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg.seed)
        self.copies = []
        for r in range(R):
            seed = cfg.seed + 7919 * r
            beams = torch.from_numpy(synth.make_beams(cfg.B, cfg.W, cfg.L, cfg.V, seed, cfg.share)).to(dev)
            ctx_np = synth.make_ctx_len(cfg.B, cfg.ctx_lo, cfg.ctx_hi, seed)
            if ctx_override is not None:
                ctx_np = np.full_like(ctx_np, ctx_override)
            c = dict(beams=beams, ctx_len=torch.from_numpy(ctx_np).to(dev), ctx_np=ctx_np)
            for name, n in (("q", cfg.N), ("k_new", cfg.N), ("v_new", cfg.N), ("k_cache", cfg.Cmax), ("v_cache", cfg.Cmax)):
                c[name] = torch.randn((cfg.B, cfg.H, n, cfg.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
            c["dedup"] = rd.rd_dedup(beams, c["ctx_len"])
            torch.cuda.synchronize()
            d = c["dedup"]
            c["n_packed_np"] = d["n_packed"].cpu().numpy()
            logits = synth.make_logits(cfg.B, cfg.N, cfg.V, seed, d["packed_tokens"].cpu().numpy(),
                                       d["parent"].cpu().numpy(), c["n_packed_np"], cfg.p_plant)
            c["logits"] = torch.from_numpy(logits).to(dev)
            c["attn_out"] = torch.empty_like(c["q"])
            c["accept"] = None
            self.copies.append(c)
        self.ws_attn = rd.new_workspace(rd.rd_tree_attn_workspace(cfg.B, cfg.H, cfg.N, cfg.D, cfg.Cmax, self.dt_code), "cuda")
        self.ws_acc = rd.new_workspace(rd.rd_accept_workspace(cfg.B, cfg.W, cfg.L, cfg.V), "cuda")
        # algorithmic bytes of one rd_tree_attn launch: every visible K/V element once, packed q/k/v/out once, mask bits
        words = (cfg.N + 63) // 64
        ab, pt = [], []
        for c in self.copies:
            P = c["n_packed_np"].astype(np.int64)
            C = c["ctx_np"].astype(np.int64)
            ab.append(self.esz * cfg.H * cfg.D * int((2 * C + 4 * P).sum()) + int(P.sum()) * words * 8)
            pt.append(int(P.sum()))
        self.attn_bytes = float(np.mean(ab))
        self.packed = float(np.mean(pt))
        for c in self.copies:                 # eager pass: allocates outputs, sets kernel attributes
            self.step(c)
        torch.cuda.synchronize()

    def attn(self, c, ctx_bound=None):
        d = c["dedup"]
        self.rd.rd_tree_attn(c["q"], c["k_cache"], c["v_cache"], c["ctx_len"], c["k_new"], c["v_new"],
                             d["n_packed"], d["tree_mask_bits"], self.scale, out=c["attn_out"], workspace=self.ws_attn,
                             ctx_bound=ctx_bound)

    def dedup(self, c):
        self.rd.rd_dedup(c["beams"], c["ctx_len"], out=c["dedup"])

    def accept(self, c):
        d = c["dedup"]
        c["accept"] = self.rd.rd_accept(c["logits"], c["beams"], d["unpack_index"], d["n_packed"],
                                        out=c["accept"], workspace=self.ws_acc)

    def step(self, c):
        self.dedup(c)
        self.attn(c)
        self.accept(c)

    def describe(self):
        cfg = self.cfg
        return "%s: B=%d ctx=%s H=%d D=%d %s KV, W=%d L=%d V=%d" % (
            cfg.name, cfg.B, cfg.ctx_lo if cfg.ctx_lo == cfg.ctx_hi else "U{%d..%d}" % (cfg.ctx_lo, cfg.ctx_hi),
            cfg.H, cfg.D, cfg.dtype, cfg.W, cfg.L, cfg.V)


class Rotation:
    """Enqueues `fn` on consecutive copies of a workload: as replays of HIP graphs that each hold at
    most R consecutive calls (captured on first use, i.e. outside any timed region when `plan` is
    called beforehand), or eagerly."""

    def __init__(self, wl, fn, stream, use_graph):
        self.wl, self.fn, self.stream, self.use_graph = wl, fn, stream, use_graph
        self.graphs = {}

    def _graph(self, start, count):
        torch = self.wl.torch
        key = (start, count)
        if key not in self.graphs:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.stream):
                for j in range(count):
                    self.fn(self.wl.copies[(start + j) % self.wl.R])
            self.graphs[key] = g
        return self.graphs[key]

    def plan(self, first, n):
        """Calls number first .. first+n-1 of the rotation as a list of things to run."""
        R = self.wl.R
        segs, pos, left = [], first % R, n
        while left > 0:
            cnt = min(left, R)
            segs.append((pos, cnt, self._graph(pos, cnt) if self.use_graph else None))
            pos = (pos + cnt) % R
            left -= cnt
        return segs

    def run(self, segs):
        for pos, cnt, g in segs:
            if g is not None:
                g.replay()
            else:
                for j in range(cnt):
                    self.fn(self.wl.copies[(pos + j) % self.wl.R])

    def timed(self, warmup, steps, flush):
        """(microseconds per call over exactly `steps` calls, wall ms) after `warmup` untimed calls."""
        torch = self.wl.torch
        with torch.cuda.stream(self.stream):
            w = self.plan(0, warmup)
            t = self.plan(warmup, steps)
            torch.cuda.synchronize()
            if flush is not None:
                flush.add_(1)
            self.run(w)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record(self.stream)
            self.run(t)
            e1.record(self.stream)
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) * 1e3 / steps, wall_ms

    def spread(self, target_ms=20.0, est_us=None):
        """Per-call time with every graph replay timed on its own: median and 10th / 90th percentile of
        the per-call mean of a replay.  A replay holds at least six calls and whole rotations."""
        torch = self.wl.torch
        R = self.wl.R
        rot = max(1, -(-6 // R))
        with torch.cuda.stream(self.stream):
            segs = self.plan(0, R) * rot
            self.run(segs)
            if est_us is None:
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(self.stream)
                self.run(segs)
                b.record(self.stream)
                torch.cuda.synchronize()
                est_us = a.elapsed_time(b) * 1e3 / (R * rot)
            reps = int(min(200, max(10, target_ms * 1e3 / max(est_us * R * rot, 1.0))))
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
            evs[0].record(self.stream)
            for i in range(reps):
                self.run(segs)
                evs[i + 1].record(self.stream)
            torch.cuda.synchronize()
        per = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 / (R * rot) for i in range(reps)])
        return {"p10": round(float(np.percentile(per, 10)), 3), "median": round(float(np.median(per)), 3),
                "p90": round(float(np.percentile(per, 90)), 3), "replays": reps, "launches_per_replay": R * rot,
                "launch": "hip_graph_replay" if self.use_graph else "eager"}


def stream_read_floor(wl, stream, use_graph):
    """The machine's floor for the dominant kernel: a plain streaming read of the same number of bytes,
    launched back to back over rotating buffers, best of a few workgroup counts."""
    torch, rd, R = wl.torch, wl.rd, wl.R
    nbytes = max(int(wl.attn_bytes) // 16 * 16, 16)
    slab = torch.empty((R, nbytes), dtype=torch.uint8, device="cuda").fill_(1)
    best = None
    for wgs in (256, 512, 1024, 2048):
        def fn(c, wgs=wgs):
            rd.rd_debug_stream_read(slab[c["slab"]], wgs)
        for r, c in enumerate(wl.copies):
            c["slab"] = r
        sp = Rotation(wl, fn, stream, use_graph).spread(target_ms=6.0)
        if best is None or sp["median"] < best[0]:
            best = (sp["median"], wgs)
    del slab
    return {"us_per_launch": round(best[0], 3), "workgroups": best[1], "bytes": nbytes,
            "GB/s": round(nbytes / best[0] / 1e3, 1), "launch": "hip_graph_replay" if use_graph else "eager"}


def cpu_baseline(cfg, synth, budget_s, max_seqs=None):
    """The CPU oracle as it stands, timed on this host on whole steps.  With max_seqs the sample is the
    first max_seqs sequences' worth of the batch (same generator, batch size reduced) and the rate is
    scaled by the fraction of the batch it covers."""
    import oracle                               # baseline leg only; the timed GPU path never touches it
    nb = cfg.B if max_seqs is None else min(cfg.B, max_seqs)
    cpu_cfg = cfg if nb == cfg.B else dataclasses.replace(cfg, B=nb)
    t = synth.make_attn_inputs(cpu_cfg, seed=cfg.seed, poison=False)
    scale = float(1.0 / np.sqrt(cpu_cfg.D))
    d = oracle.dedup(t["beams"], t["ctx_len"])
    logits = synth.make_logits(cpu_cfg.B, cpu_cfg.N, cpu_cfg.V, cfg.seed, d["packed_tokens"], d["parent"],
                               d["n_packed"], cpu_cfg.p_plant)
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.verify_step(t["beams"], t["ctx_len"], t["q"], t["k_cache"], t["v_cache"], t["k_new"], t["v_new"],
                           logits, cpu_cfg.dtype, scale)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or (reps >= 3 and el >= 0.5 * budget_s):
            break
    rate = reps / el * nb / cfg.B
    what = "%d whole steps of the same workload (%s), %.1f s" % (reps, cfg.name, el)
    if nb != cfg.B:
        what = "%d steps over %d of the %d sequences (%s), %.1f s, rate scaled by %d/%d" % (
            reps, nb, cfg.B, cfg.name, el, nb, cfg.B)
    return {"value": round(rate, 4), "unit": "steps/s", "cores": oracle.num_threads(), "kind": "oracle", "sample": what}


def copies_for(cfg, want):
    esz = 4 if cfg.dtype == "f32" else 2
    kv_bytes = 2 * cfg.B * cfg.H * cfg.Cmax * cfg.D * esz
    return want if want > 0 else min(33, max(2, -(-(512 << 20) // kv_bytes) + 1))


def config_entry(wl, stream, use_graph, flush, traffic, want_floor, cpu_s, synth):
    """One row of the `configs` block."""
    cfg = wl.cfg
    attn = Rotation(wl, wl.attn, stream, use_graph)
    with wl.torch.cuda.stream(stream):
        flush.add_(1)
    sp = attn.spread()
    step_us, _ = Rotation(wl, wl.step, stream, use_graph).timed(wl.R, max(2 * wl.R, 12), flush)
    gbs = wl.attn_bytes / sp["median"] / 1e3
    e = {"workload": wl.describe(), "rotating_copies": wl.R,
         "rd_tree_attn_us": sp, "algorithmic_bytes_per_launch": round(wl.attn_bytes, 1),
         "GB/s": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(cfg.idx),
         "step_us": round(step_us, 3), "steps_per_sec": round(1e6 / step_us, 1),
         "packed_tokens_per_step": round(wl.packed, 2),
         "rd_dedup_us": Rotation(wl, wl.dedup, stream, use_graph).spread(target_ms=3.0)["median"],
         "rd_accept_us": Rotation(wl, wl.accept, stream, use_graph).spread(target_ms=3.0)["median"]}
    if want_floor:
        fl = stream_read_floor(wl, stream, use_graph)
        e["stream_read_floor_us"] = fl["us_per_launch"]
        e["stream_read_floor_GB/s"] = fl["GB/s"]
    if cpu_s > 0:
        o = cpu_baseline(cfg, synth, cpu_s, max_seqs=2)
        e["oracle_steps_per_sec"] = o["value"]
        e["oracle_sample"] = o["sample"]
    return e


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the verification step shards over sequences and "
              "heads without communication; no multi-GPU path exists). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2403_09919_amd import binding as rd
    from paper_2403_09919_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    use_graph = not args.no_graph
    launch = "hip_graph_replay" if use_graph else "eager"
    traffic = read_traffic_table()
    stream = torch.cuda.Stream()          # default priority; capture needs a non-default stream
    flush = torch.zeros(FLUSH_BYTES, dtype=torch.uint8, device="cuda")

    wl = Workload(cfg, copies_for(cfg, args.copies), rd, synth, torch)
    R = wl.R

    if args.pmc_calib:                    # known traffic: each copy reads 64 MiB and writes 64 MiB
        src = torch.empty(32 << 20, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- timed region 1: whole steps (exactly --steps of them, graph replays only) ------------------
    steps_rot = Rotation(wl, wl.step, stream, use_graph)
    step_us, wall_ms = steps_rot.timed(args.warmup, args.steps, flush)
    ms_per_step = step_us / 1e3
    steps_per_s = 1e6 / step_us

    # ---- timed region 2: the dominant kernel alone (rd_tree_attn), events on its own stream ----------
    # At least ten rotations of launches, so that a short --steps (the step region above times exactly
    # --steps steps, however few) does not leave this figure to the first cold launches after the flush.
    attn_rot = Rotation(wl, wl.attn, stream, use_graph)
    attn_launches = max(args.steps, 10 * R)
    attn_us, _ = attn_rot.timed(max(args.warmup, R), attn_launches, flush)
    achieved = wl.attn_bytes / (attn_us * 1e-6) / 1e9
    attn_spread = attn_rot.spread(est_us=attn_us)

    # the other kernels of the step one by one
    kernels_us = {"rd_dedup": Rotation(wl, wl.dedup, stream, use_graph).spread(target_ms=5.0)["median"],
                  "rd_tree_attn": round(attn_us, 3),
                  "rd_accept": Rotation(wl, wl.accept, stream, use_graph).spread(target_ms=5.0)["median"]}
    valid_rows = float(np.mean([c["n_packed_np"].sum() for c in wl.copies]))
    kernels_gbs = {"rd_accept": round(valid_rows * cfg.V * 4 / kernels_us["rd_accept"] / 1e3, 1)}

    attn_warm_us = None
    if not args.no_extras:
        extras(wl, stream, use_graph, kernels_us, kernels_gbs, valid_rows, torch)
        # the same launch on one copy over and over (K/V then sit in the caches: reported beside the rotating
        # figure, never instead of it)
        one = Workload.__new__(Workload)
        one.__dict__.update(wl.__dict__)
        one.copies, one.R = [wl.copies[0]] * R, R
        attn_warm_us = Rotation(one, wl.attn, stream, use_graph).spread(target_ms=8.0)["median"]

    live_ctx = None if (args.no_extras or cfg.dtype == "f32") else live_context_point(cfg, rd, synth, torch, stream, use_graph)
    floor = None if args.no_floor else stream_read_floor(wl, stream, use_graph)
    draft = None if args.no_draft else time_draft(rd, cfg, stream, max(4, min(40, args.steps // 10)), torch)

    result = {
        "metric": "verify_steps_per_sec",
        "value": round(steps_per_s, 2),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": wl.describe(),
            "rotating_copies": R,
            "launch": launch,
            "graph_segments": [[p, c] for p, c, _ in steps_rot.plan(args.warmup, args.steps)][-2:],
            "step": "rd_dedup + rd_tree_attn + rd_accept",
        },
        "packed_tokens_per_sec": round(wl.packed * steps_per_s, 1),
        "packed_tokens_per_step": round(wl.packed, 2),
        "wall_ms_timed_region": round(wall_ms, 3),
        "kernels_us": kernels_us,
        "rd_tree_attn_us_spread": attn_spread,
        "rd_tree_attn_us_warm_cache": attn_warm_us,
        "rd_tree_attn_live_context": live_ctx,
        # not measured: one decoder layer's attention core times the layer count of the LLaMA-family model of this
        # shape (32 / 40 / 60 layers for 32 / 40 / 52 heads), plus the per-step calls; no projections, no MLP
        "derived_attention_us_per_model_step": None if cfg.H not in LAYERS_BY_HEADS else round(
            LAYERS_BY_HEADS[cfg.H] * attn_us + kernels_us["rd_dedup"] + kernels_us["rd_accept"], 1),
        "kernels_algorithmic_gbs": kernels_gbs,
        "rd_draft": draft,
        "roofline": {
            "kernel": "rd_tree_attn",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic.get(args.config),
            "algorithmic_bytes_per_launch": round(wl.attn_bytes, 1),
            "us_per_launch": round(attn_us, 3),
            "launches_timed": attn_launches,
            "launch": launch,
            "stream_read_floor": floor,
        },
    }

    if not args.no_configs:
        block = {}
        for idx in sorted(synth.CONFIGS):
            if idx == args.config:
                e = {"workload": wl.describe(), "rotating_copies": R, "rd_tree_attn_us": attn_spread,
                     "algorithmic_bytes_per_launch": round(wl.attn_bytes, 1),
                     "GB/s": round(wl.attn_bytes / attn_spread["median"] / 1e3, 1),
                     "frac": round(wl.attn_bytes / attn_spread["median"] / 1e3 / HBM_PEAK_GBS, 4),
                     "traffic": traffic.get(idx), "step_us": round(step_us, 3), "steps_per_sec": round(steps_per_s, 1),
                     "packed_tokens_per_step": round(wl.packed, 2),
                     "rd_dedup_us": kernels_us["rd_dedup"], "rd_accept_us": kernels_us["rd_accept"]}
                if floor:
                    e["stream_read_floor_us"], e["stream_read_floor_GB/s"] = floor["us_per_launch"], floor["GB/s"]
                block[str(idx)] = e
                continue
            c2 = synth.CONFIGS[idx]
            w2 = Workload(c2, copies_for(c2, 0), rd, synth, torch)
            block[str(idx)] = config_entry(w2, stream, use_graph, flush, traffic, not args.no_floor,
                                           0.0 if args.no_cpu_baseline else min(3.0, args.cpu_seconds / 2), synth)
            del w2
            torch.cuda.empty_cache()
        result["configs"] = block

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth, args.cpu_seconds)
        if "configs" in result:
            result["configs"][str(args.config)]["oracle_steps_per_sec"] = result["cpu_baseline"]["value"]
            result["configs"][str(args.config)]["oracle_sample"] = result["cpu_baseline"]["sample"]
    print(json.dumps(result), flush=True)


def live_context_point(cfg, rd, synth, torch, stream, use_graph, capacity=4096, live=600):
    """The headline shape with a cache allocated for `capacity` keys that holds `live` of them: rd_tree_attn plans
    from the capacity (all it knows), rd_tree_attn_bounded from the bound the caller passes."""
    c2 = dataclasses.replace(cfg, ctx_lo=capacity, ctx_hi=capacity)
    esz = 2
    per_launch = 2 * c2.B * c2.H * live * c2.D * esz
    R = min(64, max(2, -(-(512 << 20) // per_launch) + 1))           # > 512 MiB of K/V actually read per rotation
    wl = Workload(c2, R, rd, synth, torch, ctx_override=live)
    a = Rotation(wl, wl.attn, stream, use_graph).spread(target_ms=10.0)
    b = Rotation(wl, lambda c: wl.attn(c, ctx_bound=live), stream, use_graph).spread(target_ms=10.0)
    return {"workload": "%s with Cmax=%d, ctx_len=%d" % (cfg.name, capacity, live), "rotating_copies": R,
            "algorithmic_bytes_per_launch": round(wl.attn_bytes, 1),
            "rd_tree_attn_us": a["median"], "rd_tree_attn_bounded_us": b["median"],
            "frac_of_peak_bounded": round(wl.attn_bytes / b["median"] / 1e3 / HBM_PEAK_GBS, 4)}


def extras(wl, stream, use_graph, kernels_us, kernels_gbs, valid_rows, torch):
    """Kernels beside the step, one by one (reported beside the headline figures, not part of them)."""
    cfg, rd = wl.cfg, wl.rd
    # rd_commit (what follows the step, Sec. 3.4) appends the accepted rows behind position
    # ctx_len - L here, because the synthetic caches are allocated full.
    for c in wl.copies:
        c["ctx_commit"] = (c["ctx_len"] - cfg.L).clamp_(min=0)
        c["ctx_out"] = torch.empty_like(c["ctx_len"])
        c["n_comm"] = torch.empty_like(c["ctx_len"])
    ws_samp = rd.new_workspace(rd.rd_accept_sample_workspace(cfg.B, cfg.W, cfg.L, cfg.V), "cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed + 2)
    for c in wl.copies:                                  # sampling-mode acceptance: draft logits near the LLM's, uniform draws
        c["draft_logits"] = c["logits"] + torch.randn(c["logits"].shape, generator=gen, device="cuda")
        c["u_accept"] = torch.rand((cfg.B, cfg.N), generator=gen, device="cuda")
        c["u_next"] = torch.rand((cfg.B,), generator=gen, device="cuda")
        c["sample"] = rd.rd_accept_sample(c["logits"], c["draft_logits"], c["beams"], c["dedup"]["unpack_index"],
                                          c["dedup"]["n_packed"], c["u_accept"], c["u_next"], 1.0, workspace=ws_samp)

    def k_sample(c):
        rd.rd_accept_sample(c["logits"], c["draft_logits"], c["beams"], c["dedup"]["unpack_index"], c["dedup"]["n_packed"],
                            c["u_accept"], c["u_next"], 1.0, out=c["sample"], workspace=ws_samp)

    def k_commit(c):
        rd.rd_commit(c["k_new"], c["v_new"], c["accept"]["accepted_idx"], c["accept"]["best_len"], c["ctx_commit"],
                     c["k_cache"], c["v_cache"], ctx_len_out=c["ctx_out"], n_committed=c["n_comm"])

    # rotary embedding (LLaMA-family LLMs): as a launch of its own in front of the attention, and inside it
    max_pos = cfg.Cmax + cfg.L + 1
    inv = 1.0 / (10000.0 ** (torch.arange(0, cfg.D // 2, device="cuda", dtype=torch.float64) / (cfg.D // 2)))
    ang = torch.arange(max_pos, device="cuda", dtype=torch.float64)[:, None] * inv[None, :]
    cos_t, sin_t = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    if cfg.dtype != "f32":
        for c in wl.copies:
            c["k_rot"] = torch.zeros_like(c["k_new"])

        def k_rope(c):
            rd.rd_rope(c["q"], c["k_new"], c["dedup"]["position_ids"], c["dedup"]["n_packed"], cos_t, sin_t)

        def k_rope_then_attn(c):
            k_rope(c)
            wl.attn(c)

        def k_attn_rope(c):
            d = c["dedup"]
            rd.rd_tree_attn_rope(c["q"], c["k_cache"], c["v_cache"], c["ctx_len"], c["k_new"], c["v_new"], d["n_packed"],
                                 d["tree_mask_bits"], d["position_ids"], cos_t, sin_t, wl.scale, out=c["attn_out"],
                                 k_new_rot=c["k_rot"], workspace=wl.ws_attn)

        kernels_us["rd_rope"] = Rotation(wl, k_rope, stream, use_graph).spread(target_ms=4.0)["median"]
        kernels_us["rd_rope_then_rd_tree_attn"] = Rotation(wl, k_rope_then_attn, stream, use_graph).spread(target_ms=8.0)["median"]
        kernels_us["rd_tree_attn_rope"] = Rotation(wl, k_attn_rope, stream, use_graph).spread(target_ms=8.0)["median"]
    kernels_us["rd_commit"] = Rotation(wl, k_commit, stream, use_graph).spread(target_ms=4.0)["median"]
    kernels_us["rd_accept_sample"] = Rotation(wl, k_sample, stream, use_graph).spread(target_ms=5.0)["median"]
    # rd_accept_sample reads the valid logit rows and the draft rows of slots that are not at the last position
    leaf_rows = float(np.mean([sum(len(set(u[:, -1].tolist())) for u in c["dedup"]["unpack_index"].cpu().numpy())
                               for c in wl.copies]))
    kernels_gbs["rd_accept_sample"] = round((2 * valid_rows - leaf_rows) * cfg.V * 4 / kernels_us["rd_accept_sample"] / 1e3, 1)


def time_draft(rd, cfg, stream, n, torch):
    """rd_draft (Sec. 3.1, 3.2), the stage that feeds the verification step, timed on its own at the
    drafter dimensions that go with the workload: hidden size H*D, the workload's vocabulary, two MLP
    layers, its batch, beam width and length.  Reported beside the headline figures, not part of them.
    The weights (seeded normals, bf16, packed once into the library's operand-tiled layout as at model
    load) rotate over two copies so that no launch finds them in cache;
    the roofline figure is the weight bytes one call streams over its duration."""
    Dm, V, K, B, W, L = cfg.H * cfg.D, cfg.V, 2, cfg.B, cfg.W, cfg.L
    if B * W > 512 or W > 128:
        return None                                 # beyond rd_draft's present row limit
    G = 2 * Dm
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed + 1)

    def rn(*shape, s=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * s).to(torch.bfloat16)

    sets = [dict(emb=rn(V, Dm), rnn_u=rn(Dm, Dm, s=Dm ** -0.5), rnn_w=rn(Dm, Dm, s=Dm ** -0.5),
                 rnn_b=torch.randn(Dm, device="cuda", generator=gen) * 0.1,
                 mlp_w=rn(K, G, G, s=G ** -0.5), mlp_b=torch.randn(K, G, device="cuda", generator=gen) * 0.1,
                 head_w=rn(V, G, s=4 * G ** -0.5)) for _ in range(2)]
    sets = [rd.rd_draft_pack(p) for p in sets]      # the one-time layout change a model load would do
    h = rn(B, Dm)
    last = torch.randint(0, V, (B,), device="cuda", dtype=torch.int32, generator=gen)
    ws = torch.empty(rd.rd_draft_workspace(B, W, L, Dm, V), dtype=torch.uint8, device="cuda")
    with torch.cuda.stream(stream):                 # eager launches: replaying the call from a HIP graph was slower
        out = rd.rd_draft(sets[0], h, last, W, L, workspace=ws)     # (885 against 835 us at config 2)
        rd.rd_draft(sets[1], h, last, W, L, out=out, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(n):
            rd.rd_draft(sets[i % 2], h, last, W, L, out=out, workspace=ws)
        e1.record(stream)
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / n
    wbytes = (L - 1) * (K * G * G + V * G) * 2 + max(L - 2, 0) * 2 * Dm * Dm * 2
    gbs = wbytes / us / 1e3
    return {"us_per_call": round(us, 1), "config": "Dm=%d V=%d K=%d B=%d W=%d L=%d" % (Dm, V, K, B, W, L),
            "weights": "bf16, operand-tiled by rd_draft_pack_weights", "launch": "eager",
            "weight_bytes_streamed": wbytes, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}


if __name__ == "__main__":
    main()
