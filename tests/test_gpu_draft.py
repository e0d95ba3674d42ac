"""GPU parity for rd_draft against the CPU oracle.

Floating point decides integers here (which tokens survive), and the two sides sum in different
orders (fp32 on the GPU, fp64 in the oracle), so two candidates whose scores are closer than that
arithmetic resolves may swap.  What is unique is compared exactly: wherever the oracle's own
candidates are separated by more than the tolerance, beams must be identical.  The rest is checked for
validity: the oracle scores the GPU's candidates by teacher forcing; they must carry the scores the
GPU reports, be sorted, be distinct, and be as good as the oracle's own beam within the tolerance."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host
from paper_2403_09919_amd import synth
from draft_tolerance import DRAFT_SHAPES, TOL, TOL_7B, inputs_13b, inputs_7b, inputs_small
from test_oracle_draft import make_h, make_params

pytestmark = pytest.mark.gpu

# Log-probability units.  The two sides round every layer input to bf16, so a 1e-7 difference between
# fp32 and fp64 sums that straddles a rounding boundary moves that input by one bf16 ulp (2^-7 for
# values in [1, 2)); through an output-layer weight of these tests (sigma = 4/sqrt(2 Dm) = 0.35 at
# Dm = 64) one such flip shifts a logit by ~3e-3.  Flips are rare (a few per call) but with dozens of
# candidates some path meets one.  The bounds are not chosen here: tests/draft_tolerance.py derives them
# from the deviation a plain fp32 evaluation of the same models shows against the oracle, measured on
# the CPU over these very shapes (TOL) and over the 7B / 13B-sized inputs below (TOL_7B).


@pytest.fixture(scope="module")
def rd():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding
    return binding


def dev_params(p):
    return {k: dev(v) for k, v in p.items()}


def check(rd, p, h, last, W, L, what):
    got = rd.rd_draft(dev_params(p), dev(h), dev(last), W, L)
    torch.cuda.synchronize()
    return validate(p, h, last, W, L, got, what)


def validate(p, h, last, W, L, got, what):
    """Checks one rd_draft result (device tensors, already complete) against the oracle."""
    ref = oracle.draft(p, h, last, W, L)
    gb, gl = host(got["beams"]), host(got["beam_logp"])
    B = h.shape[0]
    V = p["emb"].shape[0]
    assert (gb[:, :, 0] == last[:, None]).all() and (gb >= 0).all() and (gb < V).all(), what
    if L == 1:
        assert (gl == 0).all()
        return 1.0
    tf = oracle.draft_path_logp(p, h, gb)                         # the oracle's score of the GPU's candidates
    assert np.abs(tf - gl).max() <= TOL, (what, np.abs(tf - gl).max())
    assert (np.diff(gl, axis=1) <= 1e-6).all(), what               # best first
    exact = 0
    for b in range(B):
        assert len({tuple(x) for x in gb[b].tolist()}) == W, what  # distinct
        # as good as the oracle's beam, candidate by candidate
        assert (tf[b] >= ref["beam_logp"][b].astype(np.float64) - TOL).all(), (what, b)
        if np.array_equal(gb[b], ref["beams"][b]):
            exact += 1
        else:
            # a swap is only legitimate between candidates the oracle itself holds closer than TOL
            rl = ref["beam_logp"][b].astype(np.float64)
            differs = [w for w in range(W) if not np.array_equal(gb[b, w], ref["beams"][b, w])]
            for w in differs:
                near = np.abs(rl - rl[w]) <= 2 * TOL
                assert near.sum() >= 2 or w == W - 1, (what, b, w, rl)
    return exact / B


@pytest.mark.parametrize("Dm,V,K,B,W,L", DRAFT_SHAPES)
def test_draft_matches_oracle(rd, Dm, V, K, B, W, L):
    announce(f"draft Dm={Dm} V={V} K={K} B={B} W={W} L={L}")
    p, h, last = inputs_small(Dm, V, K, B, W, L)
    frac = check(rd, p, h, last, W, L, "draft")
    assert frac >= 0.5                                   # random models: swaps are the exception


def test_draft_workspace_reused_by_different_inputs_back_to_back(rd):
    """Four different inputs through ONE workspace back to back with no synchronisation in between, at
    a shape whose layers split K over several workgroups per column group (partial tiles and arrival
    counters in the workspace); a partial or counter left by the previous call would show."""
    Dm, V, K, B, W, L = 512, 1200, 1, 5, 8, 4
    announce(f"draft stale-workspace check Dm={Dm} V={V} K={K} B={B} W={W} L={L}")
    p = make_params(V, Dm, K, seed=Dm + V, scale=4.0)
    pd = dev_params(p)
    ws = torch.empty(rd.rd_draft_workspace(B, W, L, Dm, V), dtype=torch.uint8, device="cuda")
    ins, outs = [], []
    for i in range(4):
        rng = np.random.default_rng(900 + i)
        h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
        last = rng.integers(0, V, B).astype(np.int32)
        ins.append((h, last, dev(h), dev(last)))
    torch.cuda.synchronize()
    for h, last, hd, ld in ins:
        outs.append(rd.rd_draft(pd, hd, ld, W, L, workspace=ws))
    torch.cuda.synchronize()
    for i, ((h, last, hd, ld), got) in enumerate(zip(ins, outs)):
        validate(p, h, last, W, L, got, "draft reuse #%d" % i)


def test_draft_uniform_model_tie_rule(rd):
    announce("draft uniform model")
    V, Dm, K, L, W = 70, 64, 1, 4, 3
    p = make_params(V, Dm, K, 5)
    p["head_w"][:] = 0
    h = synth.f32_to_bf16_bits(np.ones((1, Dm), np.float32))
    got = rd.rd_draft(dev_params(p), dev(h), dev(np.array([2], np.int32)), W, L)
    torch.cuda.synchronize()
    assert host(got["beams"])[0].tolist() == [[2, 0, 0, 0], [2, 0, 0, 1], [2, 0, 0, 2]]
    assert np.allclose(host(got["beam_logp"]), -(L - 1) * np.log(V), atol=1e-4)


def test_draft_feeds_the_verification_step(rd):
    """draft -> dedup on the device: the candidates are a valid input of rd_dedup (shared first token,
    distinct candidates, so the packed count is between L and W*(L-1)+1)."""
    announce("draft -> dedup")
    V, Dm, K, B, W, L = 2000, 128, 2, 2, 8, 5
    p = make_params(V, Dm, K, seed=77, scale=4.0)
    rng = np.random.default_rng(7)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    got = rd.rd_draft(dev_params(p), dev(h), dev(last), W, L)
    d = rd.rd_dedup(got["beams"])
    torch.cuda.synchronize()
    ref = oracle.dedup(host(got["beams"]))
    assert np.array_equal(host(d["n_packed"]), ref["n_packed"])
    assert ((ref["n_packed"] >= L) & (ref["n_packed"] <= W * (L - 1) + 1)).all()




def test_draft_vicuna7b_dimensions(rd):
    """Drafter dimensions of a 7B LLM (hidden 4096, vocabulary 32000, two MLP layers), the shape the
    benchmark times.  The oracle scores the GPU's candidates by teacher forcing (a few seconds) and
    runs its own beam search for the comparison.

    Tolerance: every linear layer's input is rounded to bf16, so an fp32-vs-fp64 difference of 1e-6
    in a hidden value that sits next to a rounding boundary moves that input by a whole bf16 ulp
    (2^-7 for values in [1, 2)).  With 8192 inputs a layer sees a few tens of such flips; each moves a
    logit by ulp * |head weight| ~ 3e-4 here, so a logit carries ~1e-3 per layer, and a score sums three
    layers over four steps.  tests/draft_tolerance.py measures what a plain numpy fp32 evaluation of the
    same model shows against the fp64 oracle on these very inputs; the bound is a multiple of that."""
    announce("draft Dm=4096 V=32000 K=2 B=1 W=8 L=5")
    Dm, V, K, B, W, L = 4096, 32000, 2, 1, 8, 5
    p, h, last = inputs_7b()
    pd = dev_params(p)
    got = rd.rd_draft(pd, dev(h), dev(last), W, L)
    packed = rd.rd_draft(rd.rd_draft_pack(pd), dev(h), dev(last), W, L)       # the layout bench.py times
    torch.cuda.synchronize()
    gb, gl = host(got["beams"]), host(got["beam_logp"])
    assert np.array_equal(host(packed["beams"]), gb) and np.array_equal(host(packed["beam_logp"]), gl)
    assert (gb[:, :, 0] == last[:, None]).all() and (gb >= 0).all() and (gb < V).all()
    assert (np.diff(gl, axis=1) <= 1e-6).all()
    assert len({tuple(x) for x in gb[0].tolist()}) == W
    tf = oracle.draft_path_logp(p, h, gb)
    assert np.abs(tf - gl).max() <= TOL_7B, np.abs(tf - gl).max()
    ref = oracle.draft(p, h, last, W, L)
    rl = ref["beam_logp"][0].astype(np.float64)
    assert (tf[0] >= rl - TOL_7B).all()
    # candidates the oracle separates from all others by more than the tolerance must be present
    got_set = {tuple(x) for x in gb[0].tolist()}
    for w in range(W - 1):
        if np.abs(np.delete(rl, w) - rl[w]).min() > 2 * TOL_7B and rl[w] - rl[W - 1] > 2 * TOL_7B:
            assert tuple(ref["beams"][0, w].tolist()) in got_set, w


def test_draft_vicuna13b_dimensions_many_rows(rd):
    """Drafter dimensions of a 13B LLM (hidden 5120, vocabulary 32000, two MLP layers) with B = 4 sequences
    of W = 16 candidates: 64 rows from the second position on, the shape at which the MLP and RNN layers
    split K over workgroups and the output layer uses 128-column workgroups, in the packed weight layout
    (what the benchmark times at this workload).  Two drafted positions keep the oracle to seconds.
    Tolerance as for the 7B-sized test."""
    announce("draft Dm=5120 V=32000 K=2 B=4 W=16 L=3")
    Dm, V, K, B, W, L = 5120, 32000, 2, 4, 16, 3
    p, h, last = inputs_13b()
    pd = dev_params(p)
    got = rd.rd_draft(pd, dev(h), dev(last), W, L)
    packed = rd.rd_draft(rd.rd_draft_pack(pd), dev(h), dev(last), W, L)
    torch.cuda.synchronize()
    gb, gl = host(got["beams"]), host(got["beam_logp"])
    assert np.array_equal(host(packed["beams"]), gb) and np.array_equal(host(packed["beam_logp"]), gl)
    assert (gb[:, :, 0] == last[:, None]).all() and (gb >= 0).all() and (gb < V).all()
    assert (np.diff(gl, axis=1) <= 1e-6).all()
    tf = oracle.draft_path_logp(p, h, gb)
    assert np.abs(tf - gl).max() <= TOL_7B, np.abs(tf - gl).max()
    ref = oracle.draft(p, h, last, W, L)
    for b in range(B):
        assert len({tuple(x) for x in gb[b].tolist()}) == W
        rl = ref["beam_logp"][b].astype(np.float64)
        assert (tf[b] >= rl - TOL_7B).all(), b
        got_set = {tuple(x) for x in gb[b].tolist()}
        for w in range(W - 1):
            if np.abs(np.delete(rl, w) - rl[w]).min() > 2 * TOL_7B and rl[w] - rl[W - 1] > 2 * TOL_7B:
                assert tuple(ref["beams"][b, w].tolist()) in got_set, (b, w)


@pytest.mark.parametrize("Dm,V,K,B,W,L", [(64, 500, 2, 2, 4, 5), (128, 4000, 1, 3, 8, 4), (64, 9000, 1, 3, 8, 3),
                                          (64, 300, 1, 2, 1, 4), (64, 200, 1, 2, 4, 1), (64, 3000, 1, 2, 70, 3)])
def test_draft_records_the_search(rd, Dm, V, K, B, W, L):
    """step_logits / step_row: the row recorded behind every candidate token must hold the draft
    distribution given that candidate's prefix (the oracle's record, where the beams agree), rows of
    candidates with a common prefix coincide, and the recorded distributions reproduce the scores."""
    announce(f"draft record Dm={Dm} V={V} K={K} B={B} W={W} L={L}")
    p = make_params(V, Dm, K, seed=Dm + V + 1, scale=4.0)
    rng = np.random.default_rng(V + W + 1)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    ref = oracle.draft(p, h, last, W, L, steps=True)
    got = rd.rd_draft(dev_params(p), dev(h), dev(last), W, L, steps=True)
    plain = rd.rd_draft(dev_params(p), dev(h), dev(last), W, L)
    torch.cuda.synchronize()
    gb, gl, sr = host(got["beams"]), host(got["beam_logp"]), host(got["step_row"])
    assert np.array_equal(gb, host(plain["beams"])) and np.array_equal(gl, host(plain["beam_logp"]))
    if L == 1:
        assert sr.shape == (B, W, 0)
        return
    sl = host(got["step_logits"]).astype(np.float64)
    M = B * W
    agree = 0
    for b in range(B):
        seen = {}
        for w in range(W):
            total = 0.0
            for j in range(L - 1):
                row = int(sr[b, w, j])
                assert b * W <= row < (b + 1) * W and (j > 0 or row == b * W)
                assert seen.setdefault((j, tuple(gb[b, w, : j + 1].tolist())), row) == row
                z = sl[j, row]
                lp = z - (z.max() + np.log(np.exp(z - z.max()).sum()))
                total += lp[gb[b, w, j + 1]]
            assert abs(total - gl[b, w]) <= 1e-4 * max(1.0, abs(total))       # the record reproduces the score
        if np.array_equal(gb[b], ref["beams"][b]):
            agree += 1
            assert np.array_equal(sr[b], ref["step_row"][b])
            for w in range(W):
                for j in range(L - 1):
                    z = sl[j, sr[b, w, j]]
                    lp = z - (z.max() + np.log(np.exp(z - z.max()).sum()))
                    # all V entries of a row, not just the few best: the maximum over thousands of entries of
                    # the same bf16 re-rounding effect that TOL bounds for a handful of path scores
                    assert np.abs(lp - ref["step_logp"][j, ref["step_row"][b, w, j]]).max() <= 3 * TOL
    assert agree >= (B + 1) // 2


@pytest.mark.parametrize("Dm,V,K,B,W,L", [(64, 500, 2, 2, 4, 5), (128, 4000, 1, 3, 8, 4), (64, 17000, 1, 5, 8, 3),
                                          (256, 1000, 2, 1, 16, 4), (64, 300, 0, 20, 8, 3)])
def test_draft_float16_model(rd, Dm, V, K, B, W, L):
    """The float16 storage type: same checks as for bf16 (fp16 carries three more significand bits, so a
    re-rounding flip is eight times smaller and the tolerance is kept)."""
    announce(f"draft fp16 Dm={Dm} V={V} K={K} B={B} W={W} L={L}")
    p = make_params(V, Dm, K, seed=Dm + V + 3, scale=4.0, dtype="f16")
    h = make_h(B, Dm, V + W + 3, "f16")
    last = np.random.default_rng(V + W + 3).integers(0, V, B).astype(np.int32)
    ref = oracle.draft(p, h, last, W, L, dtype="f16")
    got = rd.rd_draft(dev_params(p), dev(h), dev(last), W, L)
    torch.cuda.synchronize()
    gb, gl = host(got["beams"]), host(got["beam_logp"])
    assert (gb[:, :, 0] == last[:, None]).all() and (gb >= 0).all() and (gb < V).all()
    tf = oracle.draft_path_logp(p, h, gb, dtype="f16")
    assert np.abs(tf - gl).max() <= TOL
    assert (np.diff(gl, axis=1) <= 1e-6).all()
    exact = 0
    for b in range(B):
        assert len({tuple(x) for x in gb[b].tolist()}) == W
        assert (tf[b] >= ref["beam_logp"][b].astype(np.float64) - TOL).all()
        exact += int(np.array_equal(gb[b], ref["beams"][b]))
    assert exact >= (B + 1) // 2
    # not the bf16 model by accident: the same numbers stored as bf16 give other scores
    pb = make_params(V, Dm, K, seed=Dm + V + 3, scale=4.0)
    gbf = rd.rd_draft(dev_params(pb), dev(make_h(B, Dm, V + W + 3)), dev(last), W, L)
    torch.cuda.synchronize()
    assert not np.array_equal(host(gbf["beam_logp"]), gl)


def numpy_pack(w):
    """The operand-tiled layout written out with numpy: [N,K] -> tiles (n/16, k/32) of 64 lanes x 8
    elements, lane = ((k%32)/8)*16 + n%16, rows past N zero."""
    N, K = w.shape
    N16 = (N + 15) // 16 * 16
    wp = np.zeros((N16, K), w.dtype)
    wp[:N] = w
    t = wp.reshape(N16 // 16, 16, K // 32, 4, 8)              # nt, r16, ks, g, j
    return np.ascontiguousarray(t.transpose(0, 2, 3, 1, 4)).reshape(-1)


@pytest.mark.parametrize("N,K", [(16, 32), (100, 64), (1037, 128), (3, 256), (512, 8192)])
def test_pack_weights_layout(rd, N, K):
    announce(f"pack weights N={N} K={K}")
    w = np.random.default_rng(N + K).integers(0, 65536, (N, K)).astype(np.uint16)
    src = dev(w)                                               # bf16 bit patterns; the copy is bit for bit
    n = rd.raw().rd_draft_packed_elems(N, K)
    dst = torch.full((n,), -1.0, dtype=torch.bfloat16, device="cuda")
    code = rd.raw().rd_draft_pack_weights(src.data_ptr(), N, K, dst.data_ptr(), None)
    torch.cuda.synchronize()
    assert code == 0
    assert np.array_equal(host(dst), numpy_pack(w))


@pytest.mark.parametrize("Dm,V,K,B,W,L,dtype", [(64, 500, 2, 2, 4, 5, "bf16"), (128, 1037, 1, 3, 8, 4, "bf16"),
                                                (64, 17000, 1, 5, 8, 3, "bf16"), (64, 31000, 1, 3, 8, 3, "f16"),
                                                (64, 700, 1, 20, 8, 4, "bf16"), (256, 1000, 0, 1, 64, 3, "f16"),
                                                # K split over workgroups (more than 32 rows, hidden size a multiple of 256)
                                                (512, 1200, 1, 5, 8, 3, "bf16"), (256, 900, 1, 9, 8, 3, "f16"),
                                                # the many-row output layer (columns split over the waves)
                                                (256, 16400, 1, 10, 8, 3, "bf16"), (128, 17000, 1, 9, 8, 3, "f16"),
                                                (128, 17000, 1, 2, 8, 3, "bf16"), (256, 16500, 1, 3, 8, 3, "f16")])
def test_packed_weights_give_identical_results(rd, Dm, V, K, B, W, L, dtype):
    """The operand-tiled layout changes where the weights lie, not the arithmetic: beams, scores and the
    recorded logits must be bit-identical to the row-major run (which is checked against the oracle)."""
    announce(f"draft packed Dm={Dm} V={V} K={K} B={B} W={W} L={L} {dtype}")
    p = make_params(V, Dm, K, seed=Dm + V + 5, scale=4.0, dtype=dtype)
    h = make_h(B, Dm, V + 5, dtype)
    last = np.random.default_rng(V + 5).integers(0, V, B).astype(np.int32)
    pd = dev_params(p)
    a = rd.rd_draft(pd, dev(h), dev(last), W, L, steps=True)
    b = rd.rd_draft(rd.rd_draft_pack(pd), dev(h), dev(last), W, L, steps=True)
    torch.cuda.synchronize()
    for k in ("beams", "beam_logp", "step_row"):
        assert np.array_equal(host(a[k]), host(b[k])), k
    sa, sb = host(a["step_logits"]), host(b["step_logits"])
    live = np.ones(B * W, bool)
    assert np.array_equal(sa[1:], sb[1:]) and np.array_equal(sa[0, ::W], sb[0, ::W])


def test_many_random_small_models(rd):
    """Thirty seeded draws of model and beam sizes (both storage types, both weight layouts): a sweep for
    shape-dependent mistakes; every result is checked like the fixed cases."""
    rng = np.random.default_rng(77)
    for case in range(30):
        Dm = int(rng.choice([64, 128, 192]))
        V = int(rng.choice([40, 333, 1000, 4100, 8200, 16500]))
        K = int(rng.integers(0, 3))
        W = int(rng.choice([1, 2, 3, 5, 8, 13, 16, 33, 64]))
        W = min(W, V)
        B = int(rng.integers(1, max(2, min(8, 512 // W))))
        L = int(rng.integers(2, 6))
        dtype = "f16" if case % 3 == 0 else "bf16"
        announce(f"draft random case {case}: Dm={Dm} V={V} K={K} B={B} W={W} L={L} {dtype}")
        p = make_params(V, Dm, K, seed=500 + case, scale=4.0, dtype=dtype)
        h = make_h(B, Dm, 600 + case, dtype)
        last = rng.integers(0, V, B).astype(np.int32)
        ref = oracle.draft(p, h, last, W, L, dtype=dtype)
        pd = dev_params(p)
        if case % 2:
            pd = rd.rd_draft_pack(pd)
        got = rd.rd_draft(pd, dev(h), dev(last), W, L)
        torch.cuda.synchronize()
        gb, gl = host(got["beams"]), host(got["beam_logp"])
        assert (gb[:, :, 0] == last[:, None]).all() and (gb >= 0).all() and (gb < V).all(), case
        tf = oracle.draft_path_logp(p, h, gb, dtype=dtype)
        assert np.abs(tf - gl).max() <= TOL, (case, np.abs(tf - gl).max())
        assert (np.diff(gl, axis=1) <= 1e-6).all(), case
        for b in range(B):
            assert len({tuple(x) for x in gb[b].tolist()}) == W, (case, b)
            assert (tf[b] >= ref["beam_logp"][b].astype(np.float64) - TOL).all(), (case, b)


def test_split_layers_repeat_and_graph_replay(rd):
    """The layers that split K over workgroups keep arrival counters in the workspace: back-to-back calls
    on one workspace, and replays of a captured call with eager work in between, must all give the bits
    of the first call (which test_draft_matches_oracle checks against the oracle for this shape)."""
    announce("draft split layers: repeated calls and graph replays, Dm=512 B=5 W=8 L=4")
    Dm, V, K, B, W, L = 512, 1200, 2, 5, 8, 4
    p = make_params(V, Dm, K, seed=Dm + V + 9, scale=4.0)
    h = make_h(B, Dm, V + 9, "bf16")
    last = np.random.default_rng(V + 9).integers(0, V, B).astype(np.int32)
    pd = rd.rd_draft_pack(dev_params(p))
    hd, ld = dev(h), dev(last)
    ws = torch.zeros(rd.rd_draft_workspace(B, W, L, Dm, V), dtype=torch.uint8, device="cuda")
    out = rd.rd_draft(pd, hd, ld, W, L, workspace=ws, steps=True)
    torch.cuda.synchronize()
    first = {k: host(v).copy() for k, v in out.items()}
    ref = oracle.draft(p, h, last, W, L)
    tf = oracle.draft_path_logp(p, h, first["beams"])
    assert np.abs(tf - first["beam_logp"]).max() <= TOL
    assert (tf >= ref["beam_logp"].astype(np.float64) - TOL).all()

    def same(tag):
        torch.cuda.synchronize()
        for k in ("beams", "beam_logp", "step_row"):
            assert np.array_equal(host(out[k]), first[k]), (tag, k)
        assert np.array_equal(host(out["step_logits"])[1:], first["step_logits"][1:]), tag

    for rep in range(3):                                         # eager, same workspace
        rd.rd_draft(pd, hd, ld, W, L, out=out, workspace=ws, steps=True)
        same(("eager", rep))
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            rd.rd_draft(pd, hd, ld, W, L, out=out, workspace=ws, steps=True)
    for rep in range(3):
        for v in out.values():
            v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        same(("replay", rep))
