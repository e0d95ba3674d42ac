"""Pins for the oracle's draft model and beam search (Sec. 3.1, 3.2): an independent forward pass
written with numpy matrix products and scipy's log_softmax; width 1 = greedy decoding with it; a
beam as wide as the whole search space = exhaustive enumeration sorted by path probability; the
closed form of a uniform model, which also fixes the tie rule; teacher-forced path scores."""
import itertools

import numpy as np
import pytest
from scipy.special import log_softmax

import oracle
from paper_2403_09919_amd import synth


def make_params(V, Dm, K, seed, scale=1.0, dtype="bf16"):
    """Seeded draft-model weights in their 16-bit storage type: bf16 bit patterns or numpy float16."""
    rng = np.random.default_rng(seed)
    G = 2 * Dm

    def w16(shape, s):
        x = rng.standard_normal(shape, dtype=np.float32)
        x *= np.float32(s)
        return x.astype(np.float16) if dtype == "f16" else synth.f32_to_bf16_bits(x)

    return dict(
        emb=w16((V, Dm), 1.0),
        rnn_u=w16((Dm, Dm), Dm ** -0.5),
        rnn_w=w16((Dm, Dm), Dm ** -0.5),
        rnn_b=(0.1 * rng.standard_normal(Dm)).astype(np.float32),
        mlp_w=w16((K, G, G), G ** -0.5),
        mlp_b=(0.1 * rng.standard_normal((K, G))).astype(np.float32),
        head_w=w16((V, G), scale * G ** -0.5),
    )


def make_h(B, Dm, seed, dtype="bf16"):
    x = np.random.default_rng(seed).standard_normal((B, Dm)).astype(np.float32)
    return x.astype(np.float16) if dtype == "f16" else synth.f32_to_bf16_bits(x)


def f64(v):
    """Exact upcast of 16-bit storage (bf16 bit patterns or numpy float16) to float64."""
    if v.dtype == np.float16:
        return v.astype(np.float64)
    return synth.bf16_bits_to_f32(v).astype(np.float64)


def rb(x, dtype="bf16"):
    """Round float64 values to the 16-bit storage type (through float32, exact for these magnitudes' purposes)."""
    x32 = np.asarray(x, np.float64).astype(np.float32)
    if dtype == "f16":
        return x32.astype(np.float16).astype(np.float64)
    return f64(synth.f32_to_bf16_bits(x32))


def silu(x):
    return x / (1.0 + np.exp(-x))


class NumpyDrafter:
    """The draft model with library matrix products; operands of every product rounded to bf16."""

    def __init__(self, p, h_bits, dtype="bf16"):
        self.p = {k: (f64(v) if v.dtype in (np.uint16, np.float16) else v.astype(np.float64)) for k, v in p.items()}
        self.h = f64(h_bits)
        self.dtype = dtype

    def start(self, token):
        return self.p["emb"][token]

    def logp(self, s):
        x = np.concatenate([s, self.h])
        for k in range(self.p["mlp_w"].shape[0]):
            x = x + silu(self.p["mlp_w"][k] @ rb(x, self.dtype) + self.p["mlp_b"][k])
        return log_softmax(self.p["head_w"] @ rb(x, self.dtype))

    def step(self, s, token):
        return silu(self.p["rnn_u"] @ rb(s, self.dtype) + self.p["rnn_w"] @ self.p["emb"][token] + self.p["rnn_b"])

    def path_logp(self, path):
        s, total = self.start(path[0]), 0.0
        for t in range(1, len(path)):
            total += self.logp(s)[path[t]]
            s = self.step(s, path[t])
        return total


def _close(a, b, tol=1e-4):
    # the float32 -> bf16 operand rounding of this file goes through float32 first; a value that sits
    # within float32 rounding of a bf16 tie may round the other way than the oracle's direct rounding
    return abs(a - b) <= tol * max(1.0, abs(a), abs(b))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_width_one_is_greedy_decoding(seed):
    V, Dm, K, L = 50, 16, 2, 6
    p = make_params(V, Dm, K, seed, scale=3.0)
    h = synth.f32_to_bf16_bits(np.random.default_rng(seed + 10).standard_normal((2, Dm)).astype(np.float32))
    last = np.array([3, 41], np.int32)
    r = oracle.draft(p, h, last, W=1, L=L)
    for b in range(2):
        m = NumpyDrafter(p, h[b])
        s, path, total = m.start(last[b]), [int(last[b])], 0.0
        for t in range(1, L):
            lp = m.logp(s)
            v = int(np.argmax(lp))
            total += lp[v]
            path.append(v)
            s = m.step(s, v)
        assert r["beams"][b, 0].tolist() == path
        assert _close(float(r["beam_logp"][b, 0]), total)


@pytest.mark.parametrize("seed", [0, 1])
def test_beam_as_wide_as_the_search_space_is_exhaustive_search(seed):
    """A beam as wide as the vocabulary prunes nothing at the first step, so the result must be the
    best V of ALL V^(L-1) two-token continuations, found here by scoring every one of them."""
    V, Dm, K, L = 4, 8, 1, 3
    p = make_params(V, Dm, K, seed, scale=2.0)
    h = synth.f32_to_bf16_bits(np.random.default_rng(seed + 20).standard_normal((1, Dm)).astype(np.float32))
    last = np.array([1], np.int32)
    r = oracle.draft(p, h, last, W=V, L=L)
    m = NumpyDrafter(p, h[0])
    scored = []
    for tail in itertools.product(range(V), repeat=L - 1):
        scored.append((m.path_logp([1] + list(tail)), list(tail)))
    scored.sort(key=lambda x: -x[0])
    want = scored[:V]
    got = [(float(r["beam_logp"][0, w]), r["beams"][0, w, 1:].tolist()) for w in range(V)]
    assert [g[1] for g in got] == [w[1] for w in want]
    for g, w in zip(got, want):
        assert _close(g[0], w[0])


def test_uniform_model_closed_form_and_tie_rule():
    """Zero output weights: every token has probability 1/V at every step, so all candidates tie and
    the rule (smaller beam, then smaller token) decides: step 1 keeps tokens 0..W-1; afterwards the W
    best are beam 0 extended by tokens 0..W-1."""
    V, Dm, K, L, W = 7, 8, 1, 4, 3
    p = make_params(V, Dm, K, 5)
    p["head_w"][:] = 0
    h = synth.f32_to_bf16_bits(np.ones((1, Dm), np.float32))
    r = oracle.draft(p, h, np.array([2], np.int32), W=W, L=L)
    assert np.allclose(r["beam_logp"], -(L - 1) * np.log(V), atol=1e-6)
    assert r["beams"][0].tolist() == [[2, 0, 0, 0], [2, 0, 0, 1], [2, 0, 0, 2]]


@pytest.mark.parametrize("seed", [3, 4])
def test_invariants_and_teacher_forced_scores(seed):
    V, Dm, K, L, W, B = 200, 32, 2, 5, 6, 3
    p = make_params(V, Dm, K, seed, scale=4.0)
    rng = np.random.default_rng(seed)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    last = rng.integers(0, V, B).astype(np.int32)
    r = oracle.draft(p, h, last, W=W, L=L)
    beams, lp = r["beams"], r["beam_logp"]
    assert (beams[:, :, 0] == last[:, None]).all() and (beams >= 0).all() and (beams < V).all()
    assert (np.diff(lp, axis=1) <= 1e-6).all() and (lp < 0).all()          # best first
    for b in range(B):
        assert len({tuple(x) for x in beams[b].tolist()}) == W              # all candidates distinct
        m = NumpyDrafter(p, h[b])
        for w in range(W):
            assert _close(float(lp[b, w]), m.path_logp(beams[b, w].tolist()))
    tf = oracle.draft_path_logp(p, h, beams)
    assert np.allclose(tf, lp, rtol=1e-6, atol=1e-5)
    # a wider beam never has a worse best candidate, and contains the greedy path's score or better
    r1 = oracle.draft(p, h, last, W=1, L=L)
    assert (lp[:, 0] >= r1["beam_logp"][:, 0] - 1e-6).all()


def test_zero_mlp_is_the_identity_block():
    """With zero MLP weights and biases x + f(0) = x: the log-probabilities are log_softmax(O [s, h])."""
    V, Dm, L = 30, 8, 2
    p = make_params(V, Dm, 2, 9, scale=3.0)
    p["mlp_w"][:] = 0
    p["mlp_b"][:] = 0
    h = synth.f32_to_bf16_bits(np.random.default_rng(1).standard_normal((1, Dm)).astype(np.float32))
    r = oracle.draft(p, h, np.array([4], np.int32), W=V, L=L)
    g = np.concatenate([f64(p["emb"])[4], f64(h)[0]])                       # already bf16 values
    lp = log_softmax(f64(p["head_w"]) @ g)
    order = np.argsort(-lp, kind="stable")
    assert r["beams"][0, :, 1].tolist() == order.tolist()
    assert np.allclose(r["beam_logp"][0], lp[order], atol=1e-5)


@pytest.mark.parametrize("seed", [0, 3])
def test_step_rows_hold_the_distribution_behind_every_candidate_token(seed):
    """step_row/step_logp: for every final candidate and position, the recorded row must be the draft
    model's log-probabilities given that candidate's prefix (recomputed here with the numpy model), and
    candidates that share a prefix must point at the same row."""
    V, Dm, K, L, W, B = 40, 16, 1, 5, 6, 2
    p = make_params(V, Dm, K, seed, scale=3.0)
    h = synth.f32_to_bf16_bits(np.random.default_rng(seed + 30).standard_normal((B, Dm)).astype(np.float32))
    last = np.array([5, 17], np.int32)
    r = oracle.draft(p, h, last, W, L, steps=True)
    plain = oracle.draft(p, h, last, W, L)
    assert np.array_equal(r["beams"], plain["beams"]) and np.array_equal(r["beam_logp"], plain["beam_logp"])
    assert r["step_logp"].shape == (L - 1, B * W, V) and r["step_row"].shape == (B, W, L - 1)
    for b in range(B):
        m = NumpyDrafter(p, h[b])
        seen = {}
        for w in range(W):
            path = r["beams"][b, w].tolist()
            s, total = m.start(path[0]), 0.0
            for j in range(L - 1):
                row = int(r["step_row"][b, w, j])
                assert b * W <= row < (b + 1) * W
                want = m.logp(s)
                got = r["step_logp"][j, row].astype(np.float64)
                assert np.abs(got - want).max() < 1e-4
                assert seen.setdefault((j, tuple(path[: j + 1])), row) == row
                total += got[path[j + 1]]
                s = m.step(s, path[j + 1])
            assert _close(total, float(r["beam_logp"][b, w]))
        assert (r["step_row"][b, :, 0] == b * W).all()            # one live state at the first position


@pytest.mark.parametrize("seed", [0, 1])
def test_float16_model_greedy_and_teacher_forcing(seed):
    """The float16 storage type (App. A.2 runs its drafting in float16): width 1 = greedy decoding of
    the numpy model whose products read float16 operands, and candidates of a wider beam carry their
    teacher-forced scores."""
    V, Dm, K, L = 60, 16, 2, 5
    p = make_params(V, Dm, K, seed + 40, scale=3.0, dtype="f16")
    h = make_h(2, Dm, seed + 50, "f16")
    last = np.array([7, 33], np.int32)
    r = oracle.draft(p, h, last, W=1, L=L, dtype="f16")
    wide = oracle.draft(p, h, last, W=4, L=L, dtype="f16")
    tf = oracle.draft_path_logp(p, h, wide["beams"], dtype="f16")
    for b in range(2):
        m = NumpyDrafter(p, h[b], "f16")
        s, path, total = m.start(last[b]), [int(last[b])], 0.0
        for t in range(1, L):
            lp = m.logp(s)
            v = int(np.argmax(lp))
            total += lp[v]
            path.append(v)
            s = m.step(s, v)
        assert r["beams"][b, 0].tolist() == path
        assert _close(float(r["beam_logp"][b, 0]), total)
        for w in range(4):
            assert _close(m.path_logp(wide["beams"][b, w].tolist()), float(wide["beam_logp"][b, w]))
            assert _close(float(tf[b, w]), float(wide["beam_logp"][b, w]))
    bf = oracle.draft(make_params(V, Dm, K, seed + 40, scale=3.0), make_h(2, Dm, seed + 50), last, W=4, L=L)
    assert not np.array_equal(bf["beam_logp"], wide["beam_logp"])      # the storage type does matter
