#!/usr/bin/env python3
"""Benchmark of the ReDrafter verification step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
rd_dedup -> rd_tree_attn (one layer's attention core) -> rd_accept, back to back on one
stream with all inputs resident in HBM.  The default workload is the Vicuna-7B-shaped
configuration (B=1, context 1024, H=32, D=128, bf16 KV, W=8, L=5, vocab 32000).

To keep the infinity cache from serving the KV stream, the step rotates over R
independent copies of the inputs whose K/V total exceeds 512 MiB.  The R steps are
captured once into a HIP graph (the library only enqueues kernels, so a caller can do
that) and the graph is replayed, which removes the Python/ctypes launch cost from the
timed region; --no-graph times eager launches instead.

Prints one JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per rd_tree_attn launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, each scaled
# by what the same counter reads for a 64 MiB copy); see profiles/bench_vicuna7b_layer_rocprofv3.md.
# Keyed by workload; None where no counter run has been made.
MEASURED_TRAFFIC_BYTES = {2: 21900746}
LAYERS_BY_HEADS = {32: 32, 40: 40, 52: 60}      # decoder layers of the 7B / 13B / 33B models the shapes come from


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6400)
    ap.add_argument("--warmup", type=int, default=640)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (default 2: Vicuna-7B-shaped layer)")
    ap.add_argument("--copies", type=int, default=0, help="rotating input copies (0 = enough for > 512 MiB of K/V)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-draft", action="store_true", help="skip the separate rd_draft timing")
    ap.add_argument("--no-floor", action="store_true", help="skip the plain streaming-read floor measurement")
    ap.add_argument("--no-warm-cache", action="store_true",
                    help="skip the warm-cache attention figure (so that a kernel trace holds rotating launches only)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle baseline")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also run plain device copies of 64 MiB (reference dispatches for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def build_copies(cfg, R, rd, synth, torch):
    """R independent synthetic batches on the device, plus their dedup results (from the HIP path)."""
    dev = torch.device("cuda:0")
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    copies = []
    for r in range(R):
        seed = cfg.seed + 7919 * r
        beams = torch.from_numpy(synth.make_beams(cfg.B, cfg.W, cfg.L, cfg.V, seed, cfg.share)).to(dev)
        ctx_np = synth.make_ctx_len(cfg.B, cfg.ctx_lo, cfg.ctx_hi, seed)
        ctx = torch.from_numpy(ctx_np).to(dev)
        c = dict(beams=beams, ctx_len=ctx, ctx_np=ctx_np)
        for name, n in (("q", cfg.N), ("k_new", cfg.N), ("v_new", cfg.N), ("k_cache", cfg.Cmax), ("v_cache", cfg.Cmax)):
            c[name] = torch.randn((cfg.B, cfg.H, n, cfg.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
        c["dedup"] = rd.rd_dedup(beams, ctx)
        torch.cuda.synchronize()
        d = c["dedup"]
        c["n_packed_np"] = d["n_packed"].cpu().numpy()
        logits = synth.make_logits(cfg.B, cfg.N, cfg.V, seed, d["packed_tokens"].cpu().numpy(),
                                   d["parent"].cpu().numpy(), c["n_packed_np"], cfg.p_plant)
        c["logits"] = torch.from_numpy(logits).to(dev)
        c["attn_out"] = torch.empty_like(c["q"])
        c["accept"] = None
        copies.append(c)
    return copies


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
    esz = 4 if cfg.dtype == "f32" else 2
    kv_bytes = 2 * cfg.B * cfg.H * cfg.Cmax * cfg.D * esz
    R = args.copies if args.copies > 0 else max(2, -(-(512 << 20) // kv_bytes) + 1)
    scale = float(1.0 / np.sqrt(cfg.D))
    dt_code = rd.RD_F32 if cfg.dtype == "f32" else rd.RD_BF16

    copies = build_copies(cfg, R, rd, synth, torch)
    ws_attn = rd.new_workspace(rd.rd_tree_attn_workspace(cfg.B, cfg.H, cfg.N, cfg.D, cfg.Cmax, dt_code), "cuda")
    ws_acc = rd.new_workspace(rd.rd_accept_workspace(cfg.B, cfg.W, cfg.L, cfg.V), "cuda")

    def attn(c):
        d = c["dedup"]
        rd.rd_tree_attn(c["q"], c["k_cache"], c["v_cache"], c["ctx_len"], c["k_new"], c["v_new"],
                        d["n_packed"], d["tree_mask_bits"], scale, out=c["attn_out"], workspace=ws_attn)

    def step(c):
        d = rd.rd_dedup(c["beams"], c["ctx_len"], out=c["dedup"])
        attn(c)
        c["accept"] = rd.rd_accept(c["logits"], c["beams"], d["unpack_index"], d["n_packed"],
                                   out=c["accept"], workspace=ws_acc)

    # algorithmic bytes of one rd_tree_attn launch: every visible K/V element once, packed q/k/v/out once, mask bits
    words = (cfg.N + 63) // 64
    attn_bytes = []
    packed_total = []
    for c in copies:
        P = c["n_packed_np"].astype(np.int64)
        C = c["ctx_np"].astype(np.int64)
        attn_bytes.append(esz * cfg.H * cfg.D * int((2 * C + 4 * P).sum()) + int(P.sum()) * words * 8)
        packed_total.append(int(P.sum()))
    attn_bytes_mean = float(np.mean(attn_bytes))
    packed_mean = float(np.mean(packed_total))

    for c in copies:                      # eager pass: allocates outputs, sets kernel attributes
        step(c)
    torch.cuda.synchronize()

    if args.pmc_calib:                    # known traffic: each copy reads 64 MiB and writes 64 MiB
        src = torch.empty(32 << 20, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()

    use_graph = not args.no_graph
    stream = torch.cuda.Stream()          # default priority; capture needs a non-default stream
    if use_graph:
        with torch.cuda.stream(stream):
            g_step = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_step, stream=stream):
                for c in copies:
                    step(c)
            g_attn = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_attn, stream=stream):
                for c in copies:
                    attn(c)
        torch.cuda.synchronize()

    def run_steps(n):
        """n steps on `stream` (graph replays of R steps each, remainder eagerly rotated)."""
        with torch.cuda.stream(stream):
            if use_graph:
                for _ in range(n // R):
                    g_step.replay()
                for i in range(n % R):
                    step(copies[i])
            else:
                for i in range(n):
                    step(copies[i % R])

    def run_attn(n):
        with torch.cuda.stream(stream):
            if use_graph:
                for _ in range(n // R):
                    g_attn.replay()
                for i in range(n % R):
                    attn(copies[i])
            else:
                for i in range(n):
                    attn(copies[i % R])

    # ---- timed region 1: whole steps -------------------------------------------------------------
    run_steps(args.warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        e0.record(stream)
    run_steps(args.steps)
    with torch.cuda.stream(stream):
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    step_ms = e0.elapsed_time(e1) / args.steps
    ms_per_step = max(step_ms, 0.0)
    steps_per_s = 1e3 / ms_per_step

    # ---- timed region 2: the dominant kernel alone (rd_tree_attn), events on its own stream --------
    run_attn(args.warmup)
    torch.cuda.synchronize()
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        a0.record(stream)
    run_attn(args.steps)
    with torch.cuda.stream(stream):
        a1.record(stream)
    torch.cuda.synchronize()
    attn_us = a0.elapsed_time(a1) * 1e3 / args.steps
    achieved = attn_bytes_mean / (attn_us * 1e-6) / 1e9

    # spread of the attention launch: every replay of the R-launch graph timed on its own (median, 10th and
    # 90th percentile of the per-launch mean), and the same launch on one copy over and over (K/V then sit in
    # the caches: reported beside the rotating figure, never instead of it)
    attn_spread = attn_warm_us = None
    if use_graph:
        reps = max(10, min(200, args.steps // R))
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        with torch.cuda.stream(stream):
            evs[0].record(stream)
            for i in range(reps):
                g_attn.replay()
                evs[i + 1].record(stream)
        torch.cuda.synchronize()
        per = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 / R for i in range(reps)])
        attn_spread = {"p10": round(float(np.percentile(per, 10)), 3), "median": round(float(np.median(per)), 3),
                       "p90": round(float(np.percentile(per, 90)), 3), "replays": reps, "launches_per_replay": R}
    if use_graph and not args.no_warm_cache:
        with torch.cuda.stream(stream):
            g_warm = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_warm, stream=stream):
                for _ in range(R):
                    attn(copies[0])
            g_warm.replay()
            w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            w0.record(stream)
            for _ in range(reps):
                g_warm.replay()
            w1.record(stream)
        torch.cuda.synchronize()
        attn_warm_us = round(w0.elapsed_time(w1) * 1e3 / (reps * R), 3)

    # ---- the other kernels one by one (reported beside the headline figures, not part of them) ------
    # rd_commit (what follows the step, Sec. 3.4) appends the accepted rows behind position
    # ctx_len - L here, because the synthetic caches are allocated full.
    for c in copies:
        c["ctx_commit"] = (c["ctx_len"] - cfg.L).clamp_(min=0)
        c["ctx_out"] = torch.empty_like(c["ctx_len"])
        c["n_comm"] = torch.empty_like(c["ctx_len"])

    def k_dedup(c):
        rd.rd_dedup(c["beams"], c["ctx_len"], out=c["dedup"])

    def k_accept(c):
        rd.rd_accept(c["logits"], c["beams"], c["dedup"]["unpack_index"], c["dedup"]["n_packed"],
                     out=c["accept"], workspace=ws_acc)

    dev = "cuda"
    ws_samp = rd.new_workspace(rd.rd_accept_sample_workspace(cfg.B, cfg.W, cfg.L, cfg.V), dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed + 2)
    for c in copies:                                  # sampling-mode acceptance: draft logits near the LLM's, uniform draws
        c["draft_logits"] = c["logits"] + torch.randn(c["logits"].shape, generator=gen, device=dev)
        c["u_accept"] = torch.rand((cfg.B, cfg.N), generator=gen, device=dev)
        c["u_next"] = torch.rand((cfg.B,), generator=gen, device=dev)
        c["sample"] = rd.rd_accept_sample(c["logits"], c["draft_logits"], c["beams"], c["dedup"]["unpack_index"],
                                          c["dedup"]["n_packed"], c["u_accept"], c["u_next"], 1.0, workspace=ws_samp)

    def k_sample(c):
        rd.rd_accept_sample(c["logits"], c["draft_logits"], c["beams"], c["dedup"]["unpack_index"], c["dedup"]["n_packed"],
                            c["u_accept"], c["u_next"], 1.0, out=c["sample"], workspace=ws_samp)

    def k_commit(c):
        rd.rd_commit(c["k_new"], c["v_new"], c["accept"]["accepted_idx"], c["accept"]["best_len"], c["ctx_commit"],
                     c["k_cache"], c["v_cache"], ctx_len_out=c["ctx_out"], n_committed=c["n_comm"])

    def time_kernel(fn):
        n = max(R, args.steps // 4)
        with torch.cuda.stream(stream):
            for c in copies:
                fn(c)
            g = None
            if use_graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for c in copies:
                        fn(c)
            k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            k0.record(stream)
            for i in range(n // R):
                if g is not None:
                    g.replay()
                else:
                    for c in copies:
                        fn(c)
            k1.record(stream)
        torch.cuda.synchronize()
        return round(k0.elapsed_time(k1) * 1e3 / (n // R * R), 3)

    kernels_us = {"rd_dedup": time_kernel(k_dedup), "rd_tree_attn": round(attn_us, 3),
                  "rd_accept": time_kernel(k_accept), "rd_commit": time_kernel(k_commit),
                  "rd_accept_sample": time_kernel(k_sample)}

    # algorithmic bytes of the other streaming kernels (means over the copies): rd_accept reads the valid logit
    # rows; rd_accept_sample reads them and the draft rows of slots that are not at the last position
    valid_rows = float(np.mean([c["n_packed_np"].sum() for c in copies]))
    leaf_rows = float(np.mean([sum(len(set(u[:, -1].tolist())) for u in c["dedup"]["unpack_index"].cpu().numpy())
                               for c in copies]))
    kernels_gbs = {
        "rd_accept": round(valid_rows * cfg.V * 4 / kernels_us["rd_accept"] / 1e3, 1),
        "rd_accept_sample": round((2 * valid_rows - leaf_rows) * cfg.V * 4 / kernels_us["rd_accept_sample"] / 1e3, 1),
    }

    # ---- the machine's floor for the dominant kernel: a plain streaming read of the same number of bytes,
    # launched back to back over rotating buffers, best of a few workgroup counts
    floor = None
    if not args.no_floor:
        nbytes = int(attn_bytes_mean) // 16 * 16
        slab = torch.empty((R, nbytes), dtype=torch.uint8, device="cuda").fill_(1)
        best = None
        for wgs in (256, 512, 1024, 2048):
            with torch.cuda.stream(stream):
                for r in range(R):
                    rd.rd_debug_stream_read(slab[r], wgs)
                gf = None
                if use_graph:                           # like the attention launches: R of them per replay
                    gf = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gf, stream=stream):
                        for r in range(R):
                            rd.rd_debug_stream_read(slab[r], wgs)
                    gf.replay()
                f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps = max(1, 660 // R)
                f0.record(stream)
                for _ in range(reps):
                    if gf is not None:
                        gf.replay()
                    else:
                        for r in range(R):
                            rd.rd_debug_stream_read(slab[r], wgs)
                f1.record(stream)
            torch.cuda.synchronize()
            us = f0.elapsed_time(f1) * 1e3 / (reps * R)
            if best is None or us < best[0]:
                best = (us, wgs)
        del slab
        floor = {"us_per_launch": round(best[0], 3), "workgroups": best[1], "bytes": nbytes,
                 "GB/s": round(nbytes / best[0] / 1e3, 1), "launch": "hip_graph_replay" if use_graph else "eager"}

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
            "workload": "%s: B=%d ctx=%s H=%d D=%d %s KV, W=%d L=%d V=%d" % (
                cfg.name, cfg.B, cfg.ctx_lo if cfg.ctx_lo == cfg.ctx_hi else "U{%d..%d}" % (cfg.ctx_lo, cfg.ctx_hi),
                cfg.H, cfg.D, cfg.dtype, cfg.W, cfg.L, cfg.V),
            "rotating_copies": R,
            "launch": "hip_graph_replay" if use_graph else "eager",
            "step": "rd_dedup + rd_tree_attn + rd_accept",
        },
        "packed_tokens_per_sec": round(packed_mean * steps_per_s, 1),
        "packed_tokens_per_step": round(packed_mean, 2),
        "wall_ms_timed_region": round(wall_ms, 3),
        "kernels_us": kernels_us,
        "rd_tree_attn_us_spread": attn_spread,
        "rd_tree_attn_us_warm_cache": attn_warm_us,
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
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.config),
            "algorithmic_bytes_per_launch": round(attn_bytes_mean, 1),
            "us_per_launch": round(attn_us, 3),
            "stream_read_floor": floor,
        },
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth, args.cpu_seconds)
    print(json.dumps(result), flush=True)


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
            "weights": "bf16, operand-tiled by rd_draft_pack_weights",
            "weight_bytes_streamed": wbytes, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}


def cpu_baseline(cfg, synth, budget_s):
    """The CPU oracle as it stands, timed on this host on whole steps of the same workload."""
    import oracle                               # baseline leg only; the timed GPU path never touches it
    cpu_cfg = cfg
    t = synth.make_attn_inputs(cpu_cfg, poison=False)
    scale = float(1.0 / np.sqrt(cpu_cfg.D))
    d = oracle.dedup(t["beams"], t["ctx_len"])
    logits = synth.make_logits(cpu_cfg.B, cpu_cfg.N, cpu_cfg.V, cpu_cfg.seed, d["packed_tokens"], d["parent"],
                               d["n_packed"], cpu_cfg.p_plant)
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.verify_step(t["beams"], t["ctx_len"], t["q"], t["k_cache"], t["v_cache"], t["k_new"], t["v_new"],
                           logits, cpu_cfg.dtype, scale)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or (reps >= 3 and el >= 0.5 * budget_s):
            break
    return {"value": round(reps / el, 4), "unit": "steps/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d whole steps of the same workload (%s), %.1f s" % (reps, cpu_cfg.name, el)}


if __name__ == "__main__":
    main()
