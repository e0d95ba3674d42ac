"""Pins for the oracle's commit of accepted tokens (Sec. 3.4): the same update written with
numpy's index arithmetic, what must stay untouched, agreement with attention (the committed
cache is exactly the context plus the accepted path), and the guarantee of Sec. 3.4 over many
steps: dedup -> tree attention -> accept -> commit in a loop reproduces plain greedy decoding of
a toy attention LM token for token."""
import numpy as np
import pytest

import oracle
from bruteforce import ToyAttentionLM
from paper_2403_09919_amd import synth


def _random_case(rng, B, H, N, D, Cmax, L, dtype):
    def t(shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    k_new, v_new = t((B, H, N, D)), t((B, H, N, D))
    kc, vc = t((B, H, Cmax, D)), t((B, H, Cmax, D))
    best_len = rng.integers(0, L + 1, B).astype(np.int32)
    acc = np.full((B, L), -1, np.int32)
    for b in range(B):
        acc[b, :best_len[b]] = rng.choice(N, best_len[b], replace=False)
    ctx = rng.integers(0, Cmax + 1, B).astype(np.int32)
    return k_new, v_new, acc, best_len, ctx, kc, vc


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_commit_equals_numpy_indexing_and_touches_nothing_else(dtype):
    rng = np.random.default_rng(11)
    B, H, N, D, Cmax, L = 5, 3, 12, 8, 20, 4
    k_new, v_new, acc, best_len, ctx, kc, vc = _random_case(rng, B, H, N, D, Cmax, L, dtype)
    ctx[0], best_len[0] = Cmax - 2, 4            # capacity: only two of four fit
    acc[0] = [3, 1, 7, 5]
    ctx[1], best_len[1] = Cmax, 3                # full cache: nothing fits
    acc[1, :3] = [0, 2, 4]
    best_len[2] = 0                              # nothing accepted
    acc[2] = -1
    hidden = rng.standard_normal((B, N, 6)).astype(np.float32)
    if dtype == "bf16":
        hidden = synth.f32_to_bf16_bits(hidden)
    r = oracle.commit(k_new, v_new, acc, best_len, ctx, kc, vc, dtype, hidden=hidden)
    ek, ev = kc.copy(), vc.copy()
    for b in range(B):
        n = int(min(best_len[b], Cmax - ctx[b]))
        assert r["n_committed"][b] == n and r["ctx_len"][b] == ctx[b] + n
        ek[b, :, ctx[b]:ctx[b] + n, :] = k_new[b][:, acc[b, :n], :]        # numpy fancy indexing
        ev[b, :, ctx[b]:ctx[b] + n, :] = v_new[b][:, acc[b, :n], :]
        if best_len[b] > 0:
            assert np.array_equal(r["hidden_last"][b], hidden[b, acc[b, best_len[b] - 1]])
        else:
            assert not r["hidden_last"][b].any()
    assert np.array_equal(r["k_cache"], ek) and np.array_equal(r["v_cache"], ev)
    assert r["n_committed"][0] == 2 and r["n_committed"][1] == 0 and r["n_committed"][2] == 0
    # inputs are not modified (the wrapper works on copies)
    assert not np.shares_memory(r["k_cache"], kc)


def test_committed_cache_is_context_plus_accepted_path():
    """The tree-attention output of the last accepted token (context + its ancestors + itself)
    equals plain softmax attention of the same query over the committed cache, computed here
    with numpy only.  A wrong slot, a wrong position or K/V rows that lost their pairing fail."""
    cfg = synth.CONFIGS[1]
    a = synth.make_attn_inputs(cfg, poison=False)
    ctx = a["ctx_len"]
    scale = 1.0 / np.sqrt(cfg.D)
    d = oracle.dedup(a["beams"], ctx)
    out = oracle.tree_attn(a["q"], a["k_cache"], a["v_cache"], ctx, a["k_new"], a["v_new"],
                           d["n_packed"], d["tree_mask"], "f32", scale)
    B, H, N, D = a["q"].shape
    Cmax = a["k_cache"].shape[2]
    # make room: the synthetic cache is full, so commit into a longer copy
    room = np.zeros((B, H, cfg.L, D), np.float32)
    kc = np.concatenate([a["k_cache"], room], axis=2)
    vc = np.concatenate([a["v_cache"], room], axis=2)
    for w in range(cfg.W):
        for bl in range(1, cfg.L + 1):
            acc = np.full((B, cfg.L), -1, np.int32)
            acc[0, :bl] = d["unpack_index"][0, w, :bl]
            r = oracle.commit(a["k_new"], a["v_new"], acc, np.array([bl], np.int32), ctx, kc, vc, "f32")
            C1 = int(r["ctx_len"][0])
            assert C1 == ctx[0] + bl
            last = acc[0, bl - 1]
            for h in range(H):
                q = a["q"][0, h, last].astype(np.float64)
                s = (r["k_cache"][0, h, :C1].astype(np.float64) @ q) * scale
                p = np.exp(s - s.max())
                ref = (p / p.sum()) @ r["v_cache"][0, h, :C1].astype(np.float64)
                assert np.allclose(out[0, h, last], ref, rtol=0, atol=2e-6), (w, bl, h)


def _spec_decode(lm, prompt, n_new, W, L, Cmax, seed, p_good=0.6):
    """Speculative greedy decoding of the toy LM with the oracle's step functions."""
    rng = np.random.default_rng(seed)
    truth = lm.greedy(prompt, n_new + 2 * L)                  # only used to build good candidates
    H, D = lm.H, lm.D
    kc = np.zeros((1, H, Cmax, D), np.float32)
    vc = np.zeros((1, H, Cmax, D), np.float32)
    seq = list(prompt)
    ctx = np.array([len(seq) - 1], np.int32)                  # all but the last token are context
    kc[0, :, :ctx[0]] = np.transpose(lm.Ek[seq[:-1]], (1, 0, 2))
    vc[0, :, :ctx[0]] = np.transpose(lm.Ev[seq[:-1]], (1, 0, 2))
    steps = 0
    while len(seq) < len(prompt) + n_new:
        root = seq[-1]                                        # the LLM's own (guaranteed) token
        beams = np.empty((1, W, L), np.int32)
        for w in range(W):
            beams[0, w, 0] = root
            cont = truth[len(seq):len(seq) + L - 1]
            good = rng.integers(0, L) if rng.random() < p_good else 0     # how many drafted tokens are right
            for j in range(1, L):
                beams[0, w, j] = cont[j - 1] if j <= good else rng.integers(0, lm.V)
        d = oracle.dedup(beams, ctx)
        P = int(d["n_packed"][0])
        tok = d["packed_tokens"][0]
        N = W * L
        q = np.zeros((1, H, N, D), np.float32)
        kn = np.zeros_like(q)
        vn = np.zeros_like(q)
        q[0, :, :P] = np.transpose(lm.Eq[tok[:P]], (1, 0, 2))
        kn[0, :, :P] = np.transpose(lm.Ek[tok[:P]], (1, 0, 2))
        vn[0, :, :P] = np.transpose(lm.Ev[tok[:P]], (1, 0, 2))
        out = oracle.tree_attn(q, kc, vc, ctx, kn, vn, d["n_packed"], d["tree_mask"], "f32", lm.scale)
        logits = lm.logits_from_attn(np.transpose(out[0], (1, 0, 2))).astype(np.float32)[None]   # [1,N,V]
        am = oracle.argmax(logits, d["n_packed"])
        acc = oracle.accept(beams, d["unpack_index"], am)
        bl, bw = int(acc["best_len"][0]), int(acc["best_beam"][0])
        assert bl >= 1                                        # position 0 is the guaranteed token
        r = oracle.commit(kn, vn, acc["accepted_idx"], acc["best_len"], ctx, kc, vc, "f32")
        kc, vc, ctx = r["k_cache"], r["v_cache"], r["ctx_len"]
        seq = seq[:-1] + [int(t) for t in beams[0, bw, :bl]] + [int(acc["next_token"][0])]
        steps += 1
    return seq, steps


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_speculative_loop_reproduces_greedy_decoding(seed):
    lm = ToyAttentionLM(V=40, H=2, D=16, seed=100 + seed)
    prompt = [3, 17, 5, 9]
    n_new = 30
    ref = lm.greedy(prompt, n_new + 8)
    got, steps = _spec_decode(lm, prompt, n_new, W=4, L=4, Cmax=80, seed=seed)
    assert got == ref[:len(got)]
    assert steps < n_new                                      # some drafts were accepted: more than one token per step
