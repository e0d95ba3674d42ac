"""GPU parity, integer steps: rd_dedup and rd_accept against the CPU oracle, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host, mask_bits_u64
from paper_2403_09919_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rd():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding
    return binding


def check_dedup(rd, beams, ctx_len):
    B, W, L = beams.shape
    ref = oracle.dedup(beams, ctx_len)
    got = rd.rd_dedup(dev(beams), None if ctx_len is None else dev(np.asarray(ctx_len, np.int32)))
    torch.cuda.synchronize()
    for k in ("prefix_tree", "packed_tokens", "n_packed", "unpack_index", "parent", "position_ids", "tree_mask"):
        assert np.array_equal(host(got[k]), ref[k]), k
    assert np.array_equal(mask_bits_u64(got["tree_mask_bits"]), ref["tree_mask_bits"])
    return ref, got


def test_dedup_worked_example(rd):
    announce("dedup worked example")
    beam = np.array([[[91, 92, 93, 95], [91, 92, 94, 96], [91, 92, 93, 97]]], np.int32)
    ref, got = check_dedup(rd, beam, np.array([10], np.int32))
    assert host(got["prefix_tree"])[0].tolist() == [[0, 0, 0, 0], [0, 0, 1, 1], [0, 0, 0, 2]]


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_dedup_configs(rd, idx):
    cfg = synth.CONFIGS[idx]
    announce("dedup config %d" % idx)
    beams = synth.make_beams(cfg.B, cfg.W, cfg.L, cfg.V, cfg.seed, cfg.share)
    ctx = synth.make_ctx_len(cfg.B, cfg.ctx_lo, cfg.ctx_hi, cfg.seed)
    check_dedup(rd, beams, ctx)


@pytest.mark.parametrize("W,L", [(1, 1), (1, 7), (1, 128), (2, 64), (3, 5), (7, 9), (16, 8), (25, 5),
                                 (32, 4), (33, 3), (63, 2), (64, 1), (64, 2), (42, 3), (12, 10),
                                 (70, 5), (128, 3), (1, 384), (127, 3), (65, 5), (96, 4), (2, 192)])
def test_dedup_shapes(rd, W, L):
    for seed, V, share in ((1, 3, "uniform"), (2, 1000, "high"), (3, 2, "high"), (4, 50, "uniform")):
        announce("dedup W=%d L=%d seed=%d V=%d" % (W, L, seed, V))
        beams = synth.make_beams(5, W, L, V, seed, share)
        ctx = np.array([0, 5, 1000, 77, 1 << 20], np.int32)
        check_dedup(rd, beams, ctx if seed % 2 else None)


def test_dedup_degenerate(rd):
    announce("dedup all identical / all distinct / optional outputs")
    W, L = 16, 5
    same = np.tile(np.array([9, 8, 7, 6, 5], np.int32), (2, W, 1))
    ref, _ = check_dedup(rd, same, None)
    assert (ref["n_packed"] == L).all()
    distinct = np.arange(2 * W * L, dtype=np.int32).reshape(2, W, L)
    ref, _ = check_dedup(rd, distinct, None)
    assert (ref["n_packed"] == W * L).all()
    neg = -np.abs(synth.make_beams(2, W, L, 4, 5)) - 1          # negative token ids are still just values
    check_dedup(rd, neg.astype(np.int32), None)
    got = rd.rd_dedup(dev(distinct), None, want_prefix_tree=False, want_mask=False)
    torch.cuda.synchronize()
    assert got["prefix_tree"] is None and got["tree_mask"] is None
    assert np.array_equal(host(got["unpack_index"]), ref["unpack_index"])


def run_accept(rd, logits, beams, d, root, workspace=None):
    got = rd.rd_accept(dev(logits), dev(beams), dev(d["unpack_index"]), dev(d["n_packed"]),
                       None if root is None else dev(np.asarray(root, np.int32)), workspace=workspace)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in got.items()}


def check_accept(rd, logits, beams, root, workspace=None):
    d = oracle.dedup(beams)
    am = oracle.argmax(logits, d["n_packed"])
    ref = oracle.accept(beams, d["unpack_index"], am, root)
    got = run_accept(rd, logits, beams, d, root, workspace)
    assert np.array_equal(got["argmax"], am)
    for k in ("n_accept", "best_beam", "best_len", "next_token", "accepted_idx"):
        assert np.array_equal(got[k], ref[k]), k
    return ref


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_accept_configs(rd, idx):
    cfg = synth.CONFIGS[idx]
    announce("accept config %d" % idx)
    beams = synth.make_beams(cfg.B, cfg.W, cfg.L, cfg.V, cfg.seed, cfg.share)
    d = oracle.dedup(beams)
    logits = synth.make_logits(cfg.B, cfg.N, cfg.V, cfg.seed, d["packed_tokens"], d["parent"],
                               d["n_packed"], cfg.p_plant)
    for root in (None, beams[:, 0, 0].copy()):
        ref = check_accept(rd, logits, beams, root)
    assert ref["best_len"].min() >= 0


@pytest.mark.parametrize("V", [1, 3, 4, 257, 1000, 2048, 2049, 4099, 32000, 32001, 151936])
def test_accept_vocab_sizes_and_ties(rd, V):
    announce("accept V=%d" % V)
    B, W, L = 3, 6, 4
    beams = synth.make_beams(B, W, L, min(V, 5), 7)
    d = oracle.dedup(beams)
    rng = np.random.default_rng(V)
    logits = rng.standard_normal((B, W * L, V)).astype(np.float32)
    logits[0, 0, :] = 1.5                                  # constant row
    logits[0, 1, :] = -np.inf                              # all -inf
    if V > 3:
        logits[1, 0, [V - 1, V // 2, 1]] = 30.0            # repeated maximum across chunks
        logits[1, 1, V - 1] = 31.0
        logits[2, 2, 0] = 31.0
    # quantised rows: many exact ties everywhere
    logits[2, 1, :] = np.round(logits[2, 1, :])
    check_accept(rd, logits, beams, None)
    check_accept(rd, logits, beams, np.array([beams[0, 0, 0], -5, beams[2, 1, 0]], np.int32))


def test_accept_signed_zeros_across_chunks(rd):
    """-0.0 and +0.0 are equal to the comparison that defines the arg max, so the smallest index
    among them wins even when the -0.0 sits in an earlier chunk of the row than the +0.0."""
    announce("accept signed zeros across chunks")
    B, W, L, V = 2, 4, 3, 32000
    beams = synth.make_beams(B, W, L, 5, 11)
    rng = np.random.default_rng(11)
    logits = -np.abs(rng.standard_normal((B, W * L, V)).astype(np.float32)) - 0.5     # everything below zero
    logits[0, 0, 100] = -0.0;  logits[0, 0, 20000] = 0.0        # -0.0 first, +0.0 in a later chunk -> 100
    logits[0, 1, 100] = 0.0;   logits[0, 1, 20000] = -0.0       # the other way round -> 100
    logits[1, 0, 31999] = -0.0; logits[1, 0, 5000] = -0.0; logits[1, 0, 9000] = 0.0    # -> 5000
    logits[1, 1, 3] = -0.0                                      # a lone -0.0 is the maximum -> 3
    check_accept(rd, logits, beams, None)                       # GPU == oracle, bit for bit
    am = oracle.argmax(logits, oracle.dedup(beams)["n_packed"])
    assert am[0, 0] == 100 and am[0, 1] == 100 and am[1, 0] == 5000 and am[1, 1] == 3


def test_accept_shapes_and_workspace_reuse(rd):
    announce("accept shapes + one workspace reused by successive calls of the same shape")
    up = lambda x: (x + 255) // 256 * 256
    for (B, W, L, V, seed) in [(1, 1, 1, 10, 0), (2, 1, 9, 300, 1), (4, 64, 2, 5000, 2), (16, 16, 5, 640, 3),
                               (3, 25, 5, 1200, 4), (2, 2, 64, 100, 5), (2, 70, 5, 900, 6), (1, 128, 3, 64, 7),
                               (2, 1, 384, 50, 8), (1, 65, 5, 32000, 9)]:
        ws = rd.new_workspace(rd.rd_accept_workspace(B, W, L, V), "cuda")
        for rep in range(3):
            beams = synth.make_beams(B, W, L, 4, seed + 10 * rep, "high")
            d = oracle.dedup(beams)
            logits = synth.make_logits(B, W * L, V, seed + rep, d["packed_tokens"], d["parent"], d["n_packed"], 0.8, 6.0)
            check_accept(rd, logits, beams, None, ws)
            check_accept(rd, logits, beams, beams[:, 0, 0].copy(), ws)
            assert int(ws.sum()) == 0                      # counters and row keys are left at zero


def test_accept_full_and_none(rd):
    announce("accept closed cases")
    W, L, V = 6, 5, 64
    beams = synth.make_beams(1, W, L, 40, 4)
    d = oracle.dedup(beams)
    ui = d["unpack_index"][0]
    N = W * L
    for w in range(W):
        logits = np.full((1, N, V), -1.0, np.float32)
        logits[0, :, 63] = 0.0
        for j in range(L - 1):
            logits[0, ui[w, j], beams[0, w, j + 1]] = 1.0
        ref = check_accept(rd, logits, beams, None)
        assert ref["best_len"][0] == L and ref["next_token"][0] == 63
    logits = np.full((1, N, V), -1.0, np.float32)
    logits[0, :, 63] = 0.0
    ref = check_accept(rd, logits, beams, np.array([63], np.int32))
    assert ref["best_len"][0] == 0 and ref["next_token"][0] == 63
