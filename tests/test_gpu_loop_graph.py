"""The whole sampling-mode loop on the device -- rd_draft -> rd_dedup -> rd_tree_attn ->
rd_accept_sample -> rd_commit -- chained without a host read-back, eagerly and as a captured HIP graph.
Every call only enqueues kernels (no allocation, no memset, no synchronisation), so the chain can be
captured; replays, with eager work and synchronisations in between, must reproduce the eager run bit
for bit, and the eager run is checked link by link against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host
from paper_2403_09919_amd import synth
from test_oracle_draft import make_params

pytestmark = pytest.mark.gpu


def test_sampling_loop_eager_and_graph():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding as rd
    announce("draft -> dedup -> attention -> accept_sample -> commit, eager and 3 graph replays")
    Dm, V, K, B, W, L, H, D, Cmax, t = 64, 900, 1, 3, 6, 4, 2, 64, 256, 1.0
    N = W * L
    p = make_params(V, Dm, K, seed=5, scale=4.0)
    rng = np.random.default_rng(5)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    ctx = np.array([100, 17, 200], np.int32)
    q, k_new, v_new = synth.make_qkv_new(B, H, N, D, "bf16", 5)
    k_cache, v_cache = synth.make_kv_cache(B, H, Cmax, D, "bf16", 5, ctx, False)
    logits = rng.standard_normal((B, N, V)).astype(np.float32)
    u_acc, u_next = synth.make_uniforms((B, N), 6), synth.make_uniforms((B,), 7)

    pd = {k: dev(v) for k, v in p.items()}
    g = dict(h=dev(h), last=dev(last), ctx=dev(ctx), q=dev(q), k_new=dev(k_new), v_new=dev(v_new),
             k_cache=dev(k_cache), v_cache=dev(v_cache), logits=dev(logits), u_acc=dev(u_acc), u_next=dev(u_next))
    ws_d = torch.empty(rd.rd_draft_workspace(B, W, L, Dm, V), dtype=torch.uint8, device="cuda")
    ws_a = rd.new_workspace(rd.rd_tree_attn_workspace(B, H, N, D, Cmax, rd.RD_BF16), "cuda")
    ws_s = rd.new_workspace(rd.rd_accept_sample_workspace(B, W, L, V), "cuda")
    st = {}

    def step():
        st["dr"] = rd.rd_draft(pd, g["h"], g["last"], W, L, out=st.get("dr"), workspace=ws_d, steps=True)
        st["d"] = rd.rd_dedup(st["dr"]["beams"], g["ctx"], out=st.get("d"))
        d = st["d"]
        st["o"] = rd.rd_tree_attn(g["q"], g["k_cache"], g["v_cache"], g["ctx"], g["k_new"], g["v_new"], d["n_packed"],
                                  d["tree_mask_bits"], 0.125, out=st.get("o"), workspace=ws_a)
        st["a"] = rd.rd_accept_sample(g["logits"], st["dr"]["step_logits"], st["dr"]["beams"], d["unpack_index"], d["n_packed"],
                                      g["u_acc"], g["u_next"], t, out=st.get("a"), workspace=ws_s, step_row=st["dr"]["step_row"])
        c = st.get("c") or {}
        st["c"] = rd.rd_commit(g["k_new"], g["v_new"], st["a"]["accepted_idx"], st["a"]["best_len"], g["ctx"], g["k_cache"],
                               g["v_cache"], ctx_len_out=c.get("ctx_len"), n_committed=c.get("n_committed"))

    def snapshot():
        torch.cuda.synchronize()
        s = {}
        for name in ("dr", "d", "a", "c"):
            s.update({name + "_" + k: host(v) for k, v in st[name].items() if v is not None})
        s["o"], s["k_cache"], s["v_cache"] = host(st["o"]), host(g["k_cache"]), host(g["v_cache"])
        dead = np.ones(B * W, bool)                              # rows of the first position that rd_draft does not write
        dead[::W] = False
        s["dr_step_logits"][0, dead] = 0
        return s

    step()
    eager = snapshot()

    # the eager run against the oracle, link by link (each link on the device's own inputs)
    beams = eager["dr_beams"]
    dref = oracle.dedup(beams, ctx)
    for k in ("packed_tokens", "n_packed", "unpack_index", "parent", "position_ids"):
        assert np.array_equal(eager["d_" + k], dref[k]), k
    aref = oracle.tree_attn(q, k_cache, v_cache, ctx, k_new, v_new, dref["n_packed"], dref["tree_mask"], "bf16", 0.125)
    assert np.abs(synth.to_f64(eager["o"], "bf16") - synth.to_f64(aref, "bf16")).max() <= 2e-2
    sref = oracle.accept_sample(logits, eager["dr_step_logits"], beams, dref["unpack_index"], u_acc, u_next, t,
                                diagnostics=True, step_row=eager["dr_step_row"])
    margin = np.abs(u_acc[np.arange(B)[:, None, None], dref["unpack_index"]].astype(np.float64) - sref["accept_ratio"])
    safe = ~((sref["accept_ratio"] >= 0) & (sref["accept_ratio"] < 1) & (margin <= 1e-4)).any(axis=(1, 2))
    assert safe.sum() >= B - 1
    for k in ("n_accept", "best_beam", "best_len", "accepted_idx"):
        assert np.array_equal(eager["a_" + k][safe], sref[k][safe]), k
    cref = oracle.commit(k_new, v_new, eager["a_accepted_idx"], eager["a_best_len"], ctx, k_cache, v_cache, "bf16")
    assert np.array_equal(eager["k_cache"], cref["k_cache"]) and np.array_equal(eager["v_cache"], cref["v_cache"])
    assert np.array_equal(eager["c_ctx_len"], cref["ctx_len"])

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step()
    for rep in range(3):
        for name in ("dr", "d", "a", "c"):                            # eager work between the replays
            for v in st[name].values():
                if v is not None:
                    v.zero_()
        st["o"].zero_()
        g["k_cache"].copy_(dev(k_cache))
        g["v_cache"].copy_(dev(v_cache))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for k in eager:
            assert np.array_equal(got[k], eager[k]), (rep, k)


def test_greedy_loop_at_the_widest_beams():
    """The token-matching loop at the widest beams of the paper's sweep (Sec. 4.3: 70 candidates of 5
    tokens, 350 packed slots): rd_draft -> rd_dedup -> rd_tree_attn -> rd_accept -> rd_commit on the
    device, every link checked against the oracle on the device's own inputs."""
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding as rd
    announce("draft -> dedup -> attention -> accept -> commit at W=70, L=5")
    Dm, V, K, B, W, L, H, D, Cmax = 64, 2000, 1, 2, 70, 5, 2, 128, 512
    N = W * L
    p = make_params(V, Dm, K, seed=70, scale=4.0)
    rng = np.random.default_rng(70)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    ctx = np.array([300, 41], np.int32)
    q, k_new, v_new = synth.make_qkv_new(B, H, N, D, "bf16", 70)
    k_cache, v_cache = synth.make_kv_cache(B, H, Cmax, D, "bf16", 70, ctx, False)

    dr = rd.rd_draft({k: dev(v) for k, v in p.items()}, dev(h), dev(last), W, L)
    d = rd.rd_dedup(dr["beams"], dev(ctx))
    torch.cuda.synchronize()
    beams = host(dr["beams"])
    assert (beams[:, :, 0] == last[:, None]).all()
    assert all(len({tuple(x) for x in beams[b].tolist()}) == W for b in range(B))
    dref = oracle.dedup(beams, ctx)
    for k in ("packed_tokens", "n_packed", "unpack_index", "parent", "position_ids"):
        assert np.array_equal(host(d[k]), dref[k]), k
    assert (dref["n_packed"] < N).all()                           # the candidates share their first token at least

    # logits that follow one candidate for a while: the planted path of synth.make_logits
    logits = synth.make_logits(B, N, V, 70, dref["packed_tokens"], dref["parent"], dref["n_packed"], 0.7)
    kd, vd = dev(k_cache), dev(v_cache)
    o = rd.rd_tree_attn(dev(q), kd, vd, dev(ctx), dev(k_new), dev(v_new), d["n_packed"], d["tree_mask_bits"], 0.0884)
    a = rd.rd_accept(dev(logits), dr["beams"], d["unpack_index"], d["n_packed"])
    c = rd.rd_commit(dev(k_new), dev(v_new), a["accepted_idx"], a["best_len"], dev(ctx), kd, vd)
    torch.cuda.synchronize()
    aref = oracle.tree_attn(q, k_cache, v_cache, ctx, k_new, v_new, dref["n_packed"], dref["tree_mask"], "bf16", 0.0884)
    assert np.abs(synth.to_f64(host(o), "bf16") - synth.to_f64(aref, "bf16")).max() <= 2e-2
    acc = oracle.accept(beams, dref["unpack_index"], oracle.argmax(logits, dref["n_packed"]))
    for k in ("n_accept", "best_beam", "best_len", "next_token", "accepted_idx"):
        assert np.array_equal(host(a[k]), acc[k]), k
    cref = oracle.commit(k_new, v_new, acc["accepted_idx"], acc["best_len"], ctx, k_cache, v_cache, "bf16")
    assert np.array_equal(host(kd), cref["k_cache"]) and np.array_equal(host(vd), cref["v_cache"])
    assert np.array_equal(host(c["ctx_len"]), cref["ctx_len"])
