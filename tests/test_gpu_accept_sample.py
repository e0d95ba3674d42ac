"""GPU parity for rd_accept_sample against the CPU oracle.

Floating point decides integers here (u < p/q, and where u falls in a cumulative distribution), the
device in fp32 and the oracle in fp64.  What is unique is compared exactly: a sequence all of whose
examined tokens keep |u - ratio| above the tolerance must reproduce the oracle's integers, and the
drawn token must be one whose interval of the oracle's cumulative distribution contains u within
the tolerance (and carry positive weight).  Sequences with a decision inside the tolerance are
skipped and must be rare."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host
from paper_2403_09919_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4        # distance of a uniform number from a threshold below which fp32 and fp64 may disagree


@pytest.fixture(scope="module")
def rd():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding
    return binding


def make_case(B, W, L, V, seed, share="uniform", noise=1.0, p_plant=0.7, poison=True):
    beams = synth.make_beams(B, W, L, V, seed, share)
    d = oracle.dedup(beams, np.full(B, 16, np.int32))
    N = W * L
    logits = synth.make_logits(B, N, V, seed, d["packed_tokens"], d["parent"], d["n_packed"], p_plant, bump=4.0)
    draft = synth.make_draft_logits(logits, seed, noise)
    if poison:                                               # rows the contract says are never read
        for b in range(B):
            P = int(d["n_packed"][b])
            logits[b, P:] = np.nan
            draft[b, P:] = np.nan
            draft[b, d["unpack_index"][b, :, L - 1]] = np.nan
    return dict(beams=beams, d=d, logits=logits, draft=draft,
                u_accept=synth.make_uniforms((B, N), seed + 1), u_next=synth.make_uniforms((B,), seed + 2))


def run_gpu(rd, c, temperature, root=None):
    d = c["d"]
    got = rd.rd_accept_sample(dev(c["logits"]), dev(c["draft"]), dev(c["beams"]), dev(d["unpack_index"]),
                              dev(d["n_packed"]), dev(c["u_accept"]), dev(c["u_next"]), temperature,
                              root_token=None if root is None else dev(root))
    torch.cuda.synchronize()
    return {k: host(v) for k, v in got.items()}


def check(rd, c, temperature, root=None, what=""):
    d = c["d"]
    B, W, L = c["beams"].shape
    ref = oracle.accept_sample(c["logits"], c["draft"], c["beams"], d["unpack_index"], c["u_accept"], c["u_next"],
                               temperature, root, diagnostics=True)
    got = run_gpu(rd, c, temperature, root)
    compared = exact_tok = 0
    for b in range(B):
        ratio = ref["accept_ratio"][b]
        slots = d["unpack_index"][b]
        examined = ratio >= 0
        margin = np.abs(c["u_accept"][b][slots].astype(np.float64) - ratio)
        if (examined & (margin <= TOL) & (ratio < 1.0)).any():
            continue                                         # a decision too close to call
        compared += 1
        for k in ("n_accept", "best_beam", "best_len", "accepted_idx"):
            assert np.array_equal(got[k][b], ref[k][b]), (what, b, k)
        v = int(got["next_token"][b])
        if ref["best_len"][b] == 0:
            assert v == root[b], (what, b)
            exact_tok += 1
            continue
        wts = ref["next_weights"][b]
        cdf = np.cumsum(wts)
        assert 0 <= v < wts.shape[0] and wts[v] > 0, (what, b, v)
        lo, hi, u = (cdf[v - 1] if v else 0.0), cdf[v], float(c["u_next"][b])
        assert lo - TOL <= u < hi + TOL, (what, b, v, lo, u, hi)
        exact_tok += int(v == ref["next_token"][b])
    assert compared >= 0.8 * B, (what, compared, B)
    assert exact_tok >= 0.9 * compared, (what, exact_tok, compared)
    return ref, got


@pytest.mark.parametrize("B,W,L,V,t", [(1, 4, 4, 1000, 1.0), (3, 8, 5, 4096, 0.7), (2, 8, 5, 1037, 1.3),
                                       (5, 3, 6, 130, 1.0), (4, 16, 5, 9001, 0.9), (2, 1, 5, 5000, 1.0),
                                       (6, 5, 1, 777, 1.0), (2, 70, 5, 3000, 1.1), (1, 128, 3, 2048, 0.8),
                                       (40, 6, 4, 517, 1.0), (2, 4, 3, 40004, 1.0), (1, 3, 3, 70001, 0.8)])
def test_accept_sample_shapes(rd, B, W, L, V, t):
    announce(f"accept_sample B={B} W={W} L={L} V={V} t={t}")
    c = make_case(B, W, L, V, seed=B + W + V, share="high" if W > 8 else "uniform")
    check(rd, c, t, what="shapes")
    root = c["beams"][:, 0, 0].copy()
    root[::2] += 1                                           # every other sequence: first token refuted
    check(rd, c, t, root, what="shapes+root")


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_accept_sample_configs(rd, idx):
    cfg = synth.CONFIGS[idx]
    announce("accept_sample config %d" % idx)
    c = make_case(cfg.B, cfg.W, cfg.L, cfg.V, cfg.seed, cfg.share, p_plant=cfg.p_plant)
    ref, got = check(rd, c, 1.0, what="config")
    assert ref["best_len"].max() > 1                          # the workload does accept drafted tokens


def test_low_temperature_equals_token_matching(rd):
    """Temperature -> 0: the sampling mode must reproduce rd_accept (the device's own greedy path)."""
    announce("accept_sample low temperature")
    B, W, L, V = 6, 8, 5, 2000
    c = make_case(B, W, L, V, seed=21, poison=False)
    d = c["d"]
    greedy = rd.rd_accept(dev(c["logits"]), dev(c["beams"]), dev(d["unpack_index"]), dev(d["n_packed"]))
    got = run_gpu(rd, c, 1e-4)
    for k in ("n_accept", "best_beam", "best_len", "next_token", "accepted_idx"):
        assert np.array_equal(got[k], host(greedy[k])), k


def test_identical_models_accept_everything(rd):
    announce("accept_sample identical models")
    B, W, L, V, t = 4, 6, 4, 3000, 0.5
    c = make_case(B, W, L, V, seed=31, poison=False)
    c["logits"] = (c["draft"] * np.float32(t)).astype(np.float32)
    c["u_accept"][:] = 0.99
    ref, got = check(rd, c, t, what="identical")
    assert (got["best_len"] == L).all() and (got["best_beam"] == 0).all() and (got["n_accept"] == L).all()


def test_extreme_uniform_numbers_and_repeat_calls(rd):
    """u_next at both ends of [0,1); the same workspace used twice gives the same answer."""
    announce("accept_sample extremes")
    B, W, L, V = 8, 4, 4, 6000
    c = make_case(B, W, L, V, seed=41)
    c["u_next"][:4] = 0.0
    c["u_next"][4:] = np.float32(1.0 - 2.0 ** -24)
    ref, got = check(rd, c, 1.0, what="extremes")
    d = c["d"]
    ws = torch.zeros(rd.rd_accept_sample_workspace(B, W, L, V), dtype=torch.uint8, device="cuda")
    args = (dev(c["logits"]), dev(c["draft"]), dev(c["beams"]), dev(d["unpack_index"]), dev(d["n_packed"]),
            dev(c["u_accept"]), dev(c["u_next"]), 1.0)
    a = {k: host(v) for k, v in rd.rd_accept_sample(*args, workspace=ws).items()}
    b = {k: host(v) for k, v in rd.rd_accept_sample(*args, workspace=ws).items()}
    for k in a:
        assert np.array_equal(a[k], b[k]) and np.array_equal(a[k], got[k]), k
    torch.cuda.synchronize()
    assert int(ws[:256].view(torch.int32).abs().sum()) == 0        # the arrival counters are left at zero


def test_sampled_tokens_follow_the_llm_distribution(rd):
    """The published guarantee, on the device: one drafted token drawn from q, then accept or resample
    -> the emitted token is distributed as p."""
    announce("accept_sample distribution")
    rng = np.random.default_rng(7)
    V, B, t = 12, 60000, 0.9
    zp = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zq = (zp + rng.standard_normal(V)).astype(np.float32)
    p = np.exp(zp.astype(np.float64) / t); p /= p.sum()
    q = np.exp(zq.astype(np.float64)); q /= q.sum()
    x = rng.choice(V, size=B, p=q).astype(np.int32)
    beams = np.zeros((B, 1, 2), np.int32)
    beams[:, 0, 1] = x
    ui = np.tile(np.array([[0, 1]], np.int32), (B, 1, 1))
    got = rd.rd_accept_sample(dev(np.broadcast_to(zp, (B, 2, V)).copy()), dev(np.broadcast_to(zq, (B, 2, V)).copy()),
                              dev(beams), dev(ui), dev(np.full(B, 2, np.int32)),
                              dev(rng.random((B, 2), dtype=np.float32)), dev(rng.random(B, dtype=np.float32)), t)
    torch.cuda.synchronize()
    acc = host(got["best_len"]) == 2
    emitted = np.where(acc, x, host(got["next_token"]))
    freq = np.bincount(emitted, minlength=V) / B
    assert np.abs(freq - p).max() < 4.5 * np.sqrt(0.25 / B)
    assert abs(acc.mean() - np.minimum(p, q).sum()) < 4.5 * np.sqrt(0.25 / B)


def test_step_layout_against_the_oracle(rd):
    """Draft logits in the layout the beam search records (one matrix per position + the row behind
    every candidate token), synthetic rows that respect shared prefixes."""
    announce("accept_sample step layout")
    rng = np.random.default_rng(52)
    B, W, L, V, t = 5, 6, 5, 1500, 1.0
    rows = B * W
    c = make_case(B, W, L, V, seed=52, share="high", poison=False)
    beams, d = c["beams"], c["d"]
    step_row = np.zeros((B, W, L - 1), np.int32)
    for b in range(B):
        for j in range(L - 1):
            ids = {}
            for w in range(W):
                step_row[b, w, j] = ids.setdefault(tuple(beams[b, w, : j + 1].tolist()), b * W + (len(ids) * 5 + j) % W)
    step_logits = np.full((L - 1, rows, V), np.nan, np.float32)       # rows nobody names stay poisoned
    for b in range(B):
        for w in range(W):
            for j in range(L - 1):
                step_logits[j, step_row[b, w, j]] = c["draft"][b, d["unpack_index"][b, w, j]]
    ref = oracle.accept_sample(c["logits"], step_logits, beams, d["unpack_index"], c["u_accept"], c["u_next"], t,
                               step_row=step_row)
    packed = oracle.accept_sample(c["logits"], c["draft"], beams, d["unpack_index"], c["u_accept"], c["u_next"], t)
    got_step = rd.rd_accept_sample(dev(c["logits"]), dev(step_logits), dev(beams), dev(d["unpack_index"]), dev(d["n_packed"]),
                                   dev(c["u_accept"]), dev(c["u_next"]), t, step_row=dev(step_row))
    got_packed = run_gpu(rd, c, t)
    torch.cuda.synchronize()
    for k in packed:
        assert np.array_equal(ref[k], packed[k]), k                  # same data, two layouts
        assert np.array_equal(host(got_step[k]), got_packed[k]), k   # and the device agrees with itself bit for bit
    check(rd, c, t, what="step layout (packed twin)")                # ... and with the oracle


def test_draft_then_accept_sample(rd):
    """rd_draft -> rd_dedup -> rd_accept_sample with the draft's own record, no copy in between; the
    oracle runs on the same record (the device's logits are its input data)."""
    announce("draft -> dedup -> accept_sample")
    from test_oracle_draft import make_params
    Dm, V, K, B, W, L, t = 64, 1200, 1, 4, 6, 5, 1.0
    p = make_params(V, Dm, K, seed=77, scale=4.0)
    rng = np.random.default_rng(77)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    dr = rd.rd_draft({k: dev(v) for k, v in p.items()}, dev(h), dev(last), W, L, steps=True)
    dd = rd.rd_dedup(dr["beams"], dev(np.full(B, 9, np.int32)))
    torch.cuda.synchronize()
    beams, ui, npk = host(dr["beams"]), host(dd["unpack_index"]), host(dd["n_packed"])
    step_logits, step_row = host(dr["step_logits"]), host(dr["step_row"])
    N = W * L
    # the LLM agrees with its drafter up to noise: logits of slot s = draft logits of s + N(0,1) (leaves: noise only)
    logits = rng.standard_normal((B, N, V)).astype(np.float32)
    for b in range(B):
        for w in range(W):
            for j in range(L - 1):
                s = ui[b, w, j]
                logits[b, s] = step_logits[j, step_row[b, w, j]] + rng.standard_normal(V).astype(np.float32) * 0.7
    u_acc, u_next = synth.make_uniforms((B, N), 78), synth.make_uniforms((B,), 79)
    ref = oracle.accept_sample(logits, step_logits, beams, ui, u_acc, u_next, t, diagnostics=True, step_row=step_row)
    got = rd.rd_accept_sample(dev(logits), dr["step_logits"], dr["beams"], dd["unpack_index"], dd["n_packed"],
                              dev(u_acc), dev(u_next), t, step_row=dr["step_row"])
    torch.cuda.synchronize()
    compared = 0
    for b in range(B):
        ratio = ref["accept_ratio"][b]
        margin = np.abs(u_acc[b][ui[b]].astype(np.float64) - ratio)
        if ((ratio >= 0) & (margin <= TOL) & (ratio < 1.0)).any():
            continue
        compared += 1
        for k in ("n_accept", "best_beam", "best_len", "accepted_idx"):
            assert np.array_equal(host(got[k])[b], ref[k][b]), (b, k)
        v = int(host(got["next_token"])[b])
        cdf = np.cumsum(ref["next_weights"][b])
        assert ref["next_weights"][b][v] > 0 and (cdf[v - 1] if v else 0.0) - TOL <= float(u_next[b]) < cdf[v] + TOL
    assert compared >= B - 1 and ref["best_len"].max() > 1


@pytest.mark.parametrize("B,W,L,V", [(3, 4, 3, 1), (2, 5, 4, 3), (4, 6, 1, 50), (2, 128, 3, 300), (1, 1, 384, 64),
                                     (2, 2, 2, 5)])
def test_accept_sample_degenerate_shapes(rd, B, W, L, V):
    """One-token vocabularies, vocabularies below the vector width, no drafted tokens (L = 1), the widest
    beam and the longest candidate the library takes."""
    announce(f"accept_sample degenerate B={B} W={W} L={L} V={V}")
    c = make_case(B, W, L, V, seed=3 * B + W + L + V, share="high")
    check(rd, c, 1.0, what="degenerate")


def test_masked_vocabulary_entries(rd):
    """-inf logits (a masked vocabulary) carry no probability: never drawn, and a candidate token the LLM
    masks is rejected whatever the uniform number."""
    announce("accept_sample with -inf logits")
    B, W, L, V = 4, 6, 4, 1000
    c = make_case(B, W, L, V, seed=91, poison=False)
    rng = np.random.default_rng(91)
    masked = rng.random((B, 1, V)) < 0.5
    c["logits"] = np.where(masked, -np.inf, c["logits"]).astype(np.float32)
    c["u_accept"][:] = 1e-3                                  # small: nearly everything with p > 0 is accepted
    ref, got = check(rd, c, 1.0, what="masked")
    assert (got["n_accept"] < L).any() and (got["n_accept"] > 1).any()
    for b in range(B):
        assert not masked[b, 0, got["next_token"][b]]
        for w in range(W):
            assert not masked[b, 0, c["beams"][b, w, 1:got["n_accept"][b, w]]].any()


def test_many_random_small_shapes(rd):
    """Forty seeded shape draws (beam width, length, vocabulary, batch, temperature, with and without a
    root token, both draft layouts' common path): a sweep for shape-dependent mistakes."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        W = int(rng.integers(1, 20))
        L = int(rng.integers(1, 8))
        V = int(rng.choice([2, 3, 5, 17, 64, 257, 1000, 4099, 9000]))
        B = int(rng.integers(1, 7))
        t = float(rng.choice([0.5, 1.0, 1.7]))
        announce(f"accept_sample random case {case}: B={B} W={W} L={L} V={V} t={t}")
        c = make_case(B, W, L, V, seed=1000 + case, share="high" if case % 2 else "uniform", noise=float(rng.choice([0.3, 1.0, 2.0])))
        root = None
        if case % 3 == 0:
            root = c["beams"][:, 0, 0].copy()
            root[::2] += 1
        d = c["d"]
        ref = oracle.accept_sample(c["logits"], c["draft"], c["beams"], d["unpack_index"], c["u_accept"], c["u_next"], t, root,
                                   diagnostics=True)
        got = run_gpu(rd, c, t, root)
        for b in range(B):
            ratio = ref["accept_ratio"][b]
            margin = np.abs(c["u_accept"][b][d["unpack_index"][b]].astype(np.float64) - ratio)
            if ((ratio >= 0) & (ratio < 1.0) & (margin <= TOL)).any():
                continue
            for k in ("n_accept", "best_beam", "best_len", "accepted_idx"):
                assert np.array_equal(got[k][b], ref[k][b]), (case, b, k)
            v = int(got["next_token"][b])
            if ref["best_len"][b] == 0:
                assert v == root[b], (case, b)
                continue
            wts = ref["next_weights"][b]
            cdf = np.cumsum(wts)
            assert 0 <= v < V and wts[v] > 0, (case, b, v)
            assert (cdf[v - 1] if v else 0.0) - TOL <= float(c["u_next"][b]) < cdf[v] + TOL, (case, b, v)
