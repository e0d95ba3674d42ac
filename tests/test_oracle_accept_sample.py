"""Pins for the oracle's rejection-sampling acceptance (Sec. 3.4's sampling mode; speculative sampling
as published by Leviathan et al. / Chen et al., 2023).  None of them reuses the oracle's arithmetic:
the published guarantee (the emitted token is distributed exactly as the LLM's own distribution, and
the acceptance rate is sum_v min(p, q)), the zero-temperature limit (= token matching), identical
models (everything accepted), library softmax / cumsum / searchsorted, and a literal walk over a
prefix trie."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
from bruteforce import trie_dedup
from paper_2403_09919_amd import synth


def _one_candidate(x):
    """beams/unpack_index of B sequences with one candidate [0, x_b]."""
    B = len(x)
    beams = np.zeros((B, 1, 2), np.int32)
    beams[:, 0, 1] = x
    ui = np.tile(np.array([[0, 1]], np.int32), (B, 1, 1))
    return beams, ui


@pytest.mark.parametrize("seed,temperature", [(0, 1.0), (1, 0.7), (2, 1.6)])
def test_emitted_token_follows_the_llm_distribution(seed, temperature):
    """One drafted token sampled from q, then accept / resample: the first emitted token must have
    the LLM's distribution p exactly, and P(accept) = sum_v min(p_v, q_v)."""
    rng = np.random.default_rng(seed)
    V, B = 6, 300_000
    zp = rng.standard_normal(V).astype(np.float32) * 1.5
    zq = (zp + rng.standard_normal(V)).astype(np.float32)
    p, q = softmax(zp.astype(np.float64) / temperature), softmax(zq.astype(np.float64))
    x = rng.choice(V, size=B, p=q).astype(np.int32)
    beams, ui = _one_candidate(x)
    logits = np.broadcast_to(zp, (B, 2, V)).copy()
    draft = np.broadcast_to(zq, (B, 2, V)).copy()
    r = oracle.accept_sample(logits, draft, beams, ui, rng.random((B, 2), dtype=np.float32),
                             rng.random(B, dtype=np.float32), temperature)
    accepted = r["best_len"] == 2
    emitted = np.where(accepted, x, r["next_token"])
    freq = np.bincount(emitted, minlength=V) / B
    assert np.abs(freq - p).max() < 4.5 * np.sqrt(0.25 / B)
    assert abs(accepted.mean() - np.minimum(p, q).sum()) < 4.5 * np.sqrt(0.25 / B)
    # after a fully accepted candidate the next token comes from the LLM's distribution at the last slot
    freq2 = np.bincount(r["next_token"][accepted], minlength=V) / accepted.sum()
    assert np.abs(freq2 - p).max() < 4.5 * np.sqrt(0.25 / accepted.sum())


def test_residual_distribution_and_inverse_cdf():
    """A forced rejection: the next token is drawn from max(0, p - q) normalised, by inverting the
    cumulative sum (library cumsum + searchsorted here)."""
    rng = np.random.default_rng(5)
    V, B, t = 9, 64, 0.8
    zp = rng.standard_normal((B, 2, V)).astype(np.float32)
    zq = rng.standard_normal((B, 2, V)).astype(np.float32)
    p, q = softmax(zp[:, 0].astype(np.float64) / t, axis=1), softmax(zq[:, 0].astype(np.float64), axis=1)
    x = np.argmin(p / q, axis=1).astype(np.int32)            # a token with p < q: rejected for u close to 1
    beams, ui = _one_candidate(x)
    u_acc = np.full((B, 2), 0.999999, np.float32)
    u_next = rng.random(B, dtype=np.float32)
    u_next[:3] = [0.0, 0.99999994, 0.5]
    r = oracle.accept_sample(zp, zq, beams, ui, u_acc, u_next, t, diagnostics=True)
    assert (r["best_len"] == 1).all() and (r["n_accept"] == 1).all()
    res = np.maximum(p - q, 0.0)
    res /= res.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(r["next_weights"], res, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["accept_ratio"][:, 0, 1], np.minimum(1.0, p[np.arange(B), x] / q[np.arange(B), x]), rtol=1e-12)
    for b in range(B):
        cdf = np.cumsum(res[b])
        want = int(np.searchsorted(cdf, np.float64(u_next[b]) * cdf[-1], side="right"))
        assert r["next_token"][b] == want and res[b, want] > 0
        assert r["next_token"][b] != x[b]                     # the rejected token has no residual mass


def test_zero_temperature_limit_is_token_matching():
    """As the temperature goes to zero p becomes one-hot on the arg max: a token is accepted iff it is
    the LLM's arg max, whatever the draft model says, and the next token is the arg max."""
    B, W, L, V = 6, 5, 4, 40
    beams = synth.make_beams(B, W, L, V, 3, "high")
    d = oracle.dedup(beams, np.full(B, 10, np.int32))
    logits = synth.make_logits(B, W * L, V, 3, d["packed_tokens"], d["parent"], d["n_packed"], 0.8)
    draft = synth.make_draft_logits(logits, 3, 2.0)
    am = oracle.argmax(logits, d["n_packed"])
    for root in (None, beams[:, 0, 0].copy()):
        if root is not None:
            root[1] += 1                                     # one sequence whose first token is refuted
        want = oracle.accept(beams, d["unpack_index"], am, root)
        got = oracle.accept_sample(logits, draft, beams, d["unpack_index"], synth.make_uniforms((B, W * L), 4),
                                   synth.make_uniforms((B,), 5), 1e-3, root)
        for k in want:
            assert np.array_equal(want[k], got[k]), k


def test_identical_models_accept_everything():
    """q == p: every ratio is 1, the whole first candidate is accepted for any uniform numbers below
    1, and the next token is the inverse CDF of p at the candidate's last slot."""
    B, W, L, V, t = 4, 3, 4, 17, 0.5
    beams = synth.make_beams(B, W, L, V, 8, "uniform")
    d = oracle.dedup(beams, np.full(B, 10, np.int32))
    rng = np.random.default_rng(8)
    draft = rng.standard_normal((B, W * L, V)).astype(np.float32)
    logits = (draft * np.float32(t)).astype(np.float32)       # logits / t == draft up to one rounding
    u_next = rng.random(B, dtype=np.float32)
    r = oracle.accept_sample(logits, draft, beams, d["unpack_index"], np.full((B, W * L), 0.999, np.float32), u_next, t)
    assert (r["n_accept"] == L).all() and (r["best_beam"] == 0).all() and (r["best_len"] == L).all()
    assert np.array_equal(r["accepted_idx"], d["unpack_index"][:, 0, :])
    for b in range(B):
        s = d["unpack_index"][b, 0, L - 1]
        cdf = np.cumsum(softmax(logits[b, s].astype(np.float64) / t))
        assert r["next_token"][b] == int(np.searchsorted(cdf, np.float64(u_next[b]) * cdf[-1], side="right"))


def _walk_trie(beam, logits, draft, u_acc, temperature):
    """Literal version on a prefix trie: node ids in creation order are the packed slots; the uniform
    number of a node decides its token once, for every candidate passing through it."""
    _, n_nodes, node_id, parent, token, _ = trie_dedup(beam)
    decided = {}
    for nid in range(n_nodes):
        if parent[nid] < 0:
            continue
        p = softmax(logits[parent[nid]].astype(np.float64) / temperature)
        q = softmax(draft[parent[nid]].astype(np.float64))
        decided[nid] = (np.float64(u_acc[nid]) < min(1.0, p[token[nid]] / q[token[nid]]), p[token[nid]] / q[token[nid]])
    lens = []
    for i in range(len(beam)):
        n = 1
        while n < len(beam[i]) and decided[node_id[i][n]][0]:
            n += 1
        lens.append(n)
    return lens, node_id, decided


@pytest.mark.parametrize("seed", range(6))
def test_tree_walk_on_a_literal_trie(seed):
    rng = np.random.default_rng(100 + seed)
    W, L, V, t = 6, 5, 4, 1.3                                 # tiny alphabet: heavy prefix sharing
    beam = rng.integers(0, V, (W, L)).astype(np.int32)
    beam[:, 0] = 2
    d = oracle.dedup(beam[None], np.array([7], np.int32))
    N = W * L
    logits = rng.standard_normal((1, N, V)).astype(np.float32)
    draft = (logits + 0.5 * rng.standard_normal((1, N, V))).astype(np.float32)
    u_acc = rng.random((1, N), dtype=np.float32)
    u_next = rng.random(1, dtype=np.float32)
    r = oracle.accept_sample(logits, draft, beam[None], d["unpack_index"], u_acc, u_next, t, diagnostics=True)
    lens, node_id, decided = _walk_trie(beam.tolist(), logits[0], draft[0], u_acc[0], t)
    assert all(abs(np.float64(u_acc[0, n]) - min(1.0, ratio)) > 1e-9 for n, (_, ratio) in decided.items())
    assert r["n_accept"][0].tolist() == lens
    best = int(np.argmax(lens))                               # first of the longest
    assert r["best_beam"][0] == best and r["best_len"][0] == lens[best]
    assert r["accepted_idx"][0, :lens[best]].tolist() == node_id[best][:lens[best]]
    assert (r["accepted_idx"][0, lens[best]:] == -1).all()
    s = node_id[best][lens[best] - 1]
    p = softmax(logits[0, s].astype(np.float64) / t)
    wts = p if lens[best] == L else np.maximum(p - softmax(draft[0, s].astype(np.float64)), 0.0)
    cdf = np.cumsum(wts)
    assert r["next_token"][0] == int(np.searchsorted(cdf, np.float64(u_next[0]) * cdf[-1], side="right"))


def test_refuted_first_token_returns_the_root_token():
    B, W, L, V = 2, 2, 3, 11
    beams = synth.make_beams(B, W, L, V, 1, "uniform")
    d = oracle.dedup(beams, np.full(B, 4, np.int32))
    z = np.zeros((B, W * L, V), np.float32)
    root = (beams[:, 0, 0] + 1).astype(np.int32)
    root[1] = beams[1, 0, 0]
    r = oracle.accept_sample(z, z, beams, d["unpack_index"], np.zeros((B, W * L), np.float32), np.zeros(B, np.float32), 1.0, root)
    assert r["best_len"][0] == 0 and r["next_token"][0] == root[0] and (r["accepted_idx"][0] == -1).all()
    assert r["best_len"][1] == L                               # uniform models: ratio 1, everything accepted


def test_last_position_draft_rows_are_never_read_and_foreign_tokens_are_rejected():
    B, W, L, V = 3, 4, 3, 13
    beams = synth.make_beams(B, W, L, V, 2, "uniform")
    d = oracle.dedup(beams, np.full(B, 4, np.int32))
    logits = np.random.default_rng(2).standard_normal((B, W * L, V)).astype(np.float32)
    draft = synth.make_draft_logits(logits, 2, 0.5)
    u_acc, u_next = synth.make_uniforms((B, W * L), 6), synth.make_uniforms((B,), 7)
    want = oracle.accept_sample(logits, draft, beams, d["unpack_index"], u_acc, u_next, 1.0)
    poisoned = draft.copy()
    for b in range(B):
        poisoned[b, d["unpack_index"][b, :, L - 1]] = np.nan       # the draft model has no distribution there
        poisoned[b, d["n_packed"][b]:] = np.nan                      # nor at padding slots
    got = oracle.accept_sample(logits, poisoned, beams, d["unpack_index"], u_acc, u_next, 1.0)
    for k in want:
        assert np.array_equal(want[k], got[k]), k
    bad = beams.copy()
    bad[0, :, 1] = V + 5                                             # not a token of the vocabulary
    bad[1, :, 1] = -1
    d2 = oracle.dedup(bad, np.full(B, 4, np.int32))
    r = oracle.accept_sample(logits, draft, bad, d2["unpack_index"], np.zeros((B, W * L), np.float32), u_next, 1.0)
    assert (r["n_accept"][:2] == 1).all()


def test_step_layout_equals_packed_layout():
    """Draft logits handed over as the beam search recorded them (one matrix per drafted position plus
    the row behind every candidate token) must give what the packed layout gives; the packed copy is
    gathered here with numpy."""
    rng = np.random.default_rng(12)
    B, W, L, V, t = 3, 5, 4, 9, 1.2
    rows = B * W
    beams = rng.integers(0, 3, (B, W, L)).astype(np.int32)          # tiny alphabet: shared prefixes
    beams[:, :, 0] = 1
    d = oracle.dedup(beams, np.full(B, 3, np.int32))
    # rows: candidates with the same prefix must name the same row (as a beam search guarantees)
    step_row = np.zeros((B, W, L - 1), np.int32)
    for b in range(B):
        for j in range(L - 1):
            ids = {}
            for w in range(W):
                key = tuple(beams[b, w, : j + 1].tolist())
                ids.setdefault(key, b * W + (len(ids) * 2 + j) % W)
                step_row[b, w, j] = ids[key]
            assert len(set(ids.values())) == len(ids)
    step_logits = rng.standard_normal((L - 1, rows, V)).astype(np.float32)
    packed = np.full((B, W * L, V), np.nan, np.float32)
    for b in range(B):
        for w in range(W):
            for j in range(L - 1):
                packed[b, d["unpack_index"][b, w, j]] = step_logits[j, step_row[b, w, j]]
    logits = rng.standard_normal((B, W * L, V)).astype(np.float32)
    u_acc, u_next = synth.make_uniforms((B, W * L), 3), synth.make_uniforms((B,), 4)
    want = oracle.accept_sample(logits, packed, beams, d["unpack_index"], u_acc, u_next, t, diagnostics=True)
    got = oracle.accept_sample(logits, step_logits, beams, d["unpack_index"], u_acc, u_next, t, diagnostics=True,
                               step_row=step_row)
    for k in want:
        assert np.array_equal(want[k], got[k]), k
    assert (want["best_len"] < L).any() and (want["best_len"] > 1).any()


def test_two_generated_tokens_follow_the_llm_joint_distribution():
    """Multi-token guarantee of speculative sampling: with the drafted tokens drawn autoregressively from
    q, the tokens a decoding loop emits are distributed as the LLM's own autoregressive process.  A toy
    first-order LM (logits = a table row of the previous token) drafts two tokens per step; the joint
    distribution of the first two generated tokens must be p(a | x0) p(b | a)."""
    rng = np.random.default_rng(21)
    V, B, t, x0 = 4, 400_000, 0.8, 2
    Tp = (rng.standard_normal((V, V)) * 1.2).astype(np.float32)
    Tq = (Tp + rng.standard_normal((V, V)) * 0.9).astype(np.float32)
    P = softmax(Tp.astype(np.float64) / t, axis=1)
    Q = softmax(Tq.astype(np.float64), axis=1)

    def draw(prob_rows):                                         # one sample per row of probabilities
        c = np.cumsum(prob_rows, axis=1)
        return (rng.random((len(prob_rows), 1)) * c[:, -1:] >= c).sum(axis=1).clip(0, V - 1).astype(np.int32)

    def step(prev):
        """One decoding step for every sequence: returns (number of tokens emitted, [n,3] tokens)."""
        x1 = draw(Q[prev])
        x2 = draw(Q[x1])
        beams = np.stack([prev, x1, x2], axis=1)[:, None, :].astype(np.int32)
        ui = np.tile(np.array([[0, 1, 2]], np.int32), (len(prev), 1, 1))
        logits = np.stack([Tp[prev], Tp[x1], Tp[x2]], axis=1)
        draft = np.stack([Tq[prev], Tq[x1], np.full((len(prev), V), np.nan, np.float32)], axis=1)
        r = oracle.accept_sample(logits, draft, beams, ui, rng.random((len(prev), 3), dtype=np.float32),
                                 rng.random(len(prev), dtype=np.float32), t)
        bl = r["best_len"]
        out = np.stack([np.where(bl >= 2, x1, r["next_token"]),
                        np.where(bl >= 3, x2, r["next_token"]), r["next_token"]], axis=1)
        return bl, out                                           # bl tokens emitted: out[:, :bl]

    prev = np.full(B, x0, np.int32)
    n1, e = step(prev)
    a = e[:, 0]
    b = e[:, 1].copy()
    short = n1 == 1                                              # only one token came out: run another step from it
    _, e2 = step(a[short])
    b[short] = e2[:, 0]
    joint = np.zeros((V, V))
    np.add.at(joint, (a, b), 1.0)
    joint /= B
    want = P[x0][:, None] * P
    assert np.abs(joint - want).max() < 4.5 * np.sqrt(0.25 / B)
    assert 0.15 < short.mean() < 0.85                            # both outcomes of the first test are exercised
