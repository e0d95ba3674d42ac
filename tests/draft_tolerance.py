"""Where the tolerances of the rd_draft parity tests come from (R17 of the design notes).

Both sides of that comparison round every linear layer's input to the 16-bit storage type, and
accumulate in different precisions (fp32 on the GPU, fp64 in the oracle).  A difference of 1e-7
between the two sums that straddles a rounding boundary moves a layer input by a whole 16-bit ulp,
and a logit by that times an output-layer weight: that, not the accumulation error itself, is what
separates the two sides.  How large the effect is for a model size is MEASURED here, on the CPU: a
plain numpy fp32 evaluation of the model (same rounding points, fp32 sums) scores the oracle's own
candidates by teacher forcing, and the largest difference to the oracle's fp64 scores is the
deviation a correct fp32 implementation shows.  Another correct implementation that sums in another
order meets its rounding boundaries elsewhere and draws its own sample of the same effect, so the
tolerances are SAFETY = 2 x that deviation, rounded up to one significant digit; the deviations are stored in tests/golden/draft_fp32_deviation.txt
(written by tests/golden/make_draft_fp32_deviation.py, which calls only the oracle and numpy), and
tests/test_oracle_draft_tolerance.py recomputes them."""
import math
import os

import numpy as np

import oracle
from paper_2403_09919_amd import synth
from test_oracle_draft import make_params

SAFETY = 2.0
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "draft_fp32_deviation.txt")
# (Dm, V, K, B, W, L) of the small test models of tests/test_gpu_draft.py::test_draft_matches_oracle
DRAFT_SHAPES = [(64, 500, 2, 2, 4, 5), (128, 4000, 1, 3, 8, 5), (64, 300, 0, 1, 1, 4),
                                          (256, 1000, 2, 1, 16, 4), (64, 33, 1, 4, 32, 3), (64, 1037, 2, 5, 7, 6),
                                          (192, 2000, 3, 2, 8, 2), (64, 100, 1, 2, 4, 1),
                                          # many rows and a wide vocabulary: workgroups that own 32 and 64 columns
                                          (64, 9000, 1, 3, 8, 3), (64, 17000, 1, 5, 8, 3), (128, 16500, 2, 9, 8, 4),
                                          (64, 20000, 0, 4, 32, 3),
                                          # more rows than one linear-layer launch covers
                                          (64, 700, 1, 20, 8, 4), (64, 16400, 1, 9, 32, 3),
                                          # the widest beams (the paper's best GPU settings use 50 and more)
                                          (64, 3000, 1, 1, 64, 3), (64, 500, 1, 2, 48, 4), (128, 9000, 1, 2, 64, 3),
                                          (64, 70, 1, 1, 64, 3),
                                          # every token of the vocabulary is a candidate; the most rows; the shortest draft
                                          (64, 16, 1, 2, 16, 3), (64, 200, 0, 16, 32, 2), (64, 40, 1, 3, 5, 2),
                                          # output layers wide enough for workgroups of 128 columns
                                          (64, 31000, 1, 3, 8, 3), (64, 32768, 0, 5, 8, 2),
                                          # vocabularies of more than eight chunks of 4096 (one row per wave in the row pass)
                                          (64, 40000, 1, 2, 8, 3), (64, 70001, 0, 1, 4, 3), (64, 151936, 0, 2, 16, 2),
                                          (64, 262144, 0, 1, 2, 2),
                                          # layers whose K is split over 2, 4 and 8 workgroups per column group (hidden
                                          # sizes of 256, 512, 1024 at more than 32 rows), 16-row tiles x 4 and x 8, and
                                          # a second launch for the rows past 128 that does not split
                                          (256, 1000, 2, 5, 8, 4), (512, 1200, 1, 3, 16, 3), (1024, 900, 1, 5, 8, 3),
                                          (256, 1000, 1, 9, 8, 3), (256, 700, 1, 20, 8, 3), (512, 800, 1, 1, 64, 3),
                                          (1024, 600, 2, 10, 8, 3),
                                          # more than 64 candidates (two lists per lane in the beam step): the paper's widest
                                          # sweep (70), the limit (128), several sequences, a vocabulary of more than 8 chunks
                                          (64, 3000, 1, 1, 70, 3), (64, 2000, 1, 1, 128, 3), (128, 1500, 1, 3, 70, 4),
                                          (64, 500, 0, 4, 128, 2), (64, 40000, 0, 1, 70, 3), (64, 129, 1, 2, 128, 3),
                                          (256, 5000, 2, 1, 96, 5), (64, 4200, 1, 2, 65, 3),
                                          # 65 rows and more with a wide output layer: waves split the columns and the
                                          # activations pass through LDS in chunks of 256 (1, 2 and 3 chunks; a second
                                          # launch for the rows past 128)
                                          (128, 17000, 1, 9, 8, 3), (256, 16400, 1, 16, 8, 3), (384, 20000, 0, 10, 8, 3),
                                          (128, 16500, 2, 20, 8, 3),
                                          # the same kernel with 1, 2 and 4 row tiles (12, 16, 24 and 40 rows)
                                          (128, 16400, 1, 3, 4, 3), (128, 17000, 1, 2, 8, 3), (256, 16500, 1, 3, 8, 3),
                                          (128, 20000, 1, 5, 8, 3)]


def inputs_small(Dm, V, K, B, W, L):
    """Weights (output layer x 4), hidden states and last tokens of one small-model parity case."""
    p = make_params(V, Dm, K, seed=Dm + V, scale=4.0)
    rng = np.random.default_rng(V + W)
    h = synth.f32_to_bf16_bits(rng.standard_normal((B, Dm)).astype(np.float32))
    return p, h, rng.integers(0, V, B).astype(np.int32)


def inputs_7b():
    """The Vicuna-7B-sized drafter of the parity tests: hidden 4096, vocabulary 32000, two MLP layers, B = 1."""
    p = make_params(32000, 4096, 2, seed=4096, scale=4.0)
    rng = np.random.default_rng(11)
    h = synth.f32_to_bf16_bits(rng.standard_normal((1, 4096)).astype(np.float32))
    return p, h, rng.integers(0, 32000, 1).astype(np.int32)


def inputs_13b():
    """The Vicuna-13B-sized drafter of the parity tests: hidden 5120, B = 4."""
    p = make_params(32000, 5120, 2, seed=5120, scale=4.0)
    rng = np.random.default_rng(13)
    h = synth.f32_to_bf16_bits(rng.standard_normal((4, 5120)).astype(np.float32))
    return p, h, rng.integers(0, 32000, 4).astype(np.int32)


def _f32(v):
    return synth.bf16_bits_to_f32(v) if v.dtype == np.uint16 else v.astype(np.float32)


def _rb32(x):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.asarray(x, np.float32)))


def _silu(x):
    return x / (np.float32(1) + np.exp(-x))


def fp32_deviation(p, h, last, W, L):
    """max |fp32 teacher-forced score - oracle score| over the oracle's W candidates of every sequence."""
    B = h.shape[0]
    K = p["mlp_w"].shape[0]
    ref = oracle.draft(p, h, last, W, L)
    P = {k: _f32(v) for k, v in p.items()}
    worst = 0.0
    for b in range(B):
        hb = _f32(h)[b]

        def logp(s):
            x = np.concatenate([s, hb]).astype(np.float32)
            for k in range(K):
                x = x + _silu(P["mlp_w"][k] @ _rb32(x) + P["mlp_b"][k])
            z = (P["head_w"] @ _rb32(x)).astype(np.float32)
            m = z.max()
            return z - m - np.log(np.exp(z - m).sum(dtype=np.float32))

        for w in range(W):
            path = ref["beams"][b, w]
            s, tot = P["emb"][path[0]], 0.0
            for t in range(1, L):
                tot += float(logp(s)[path[t]])
                s = _silu(P["rnn_u"] @ _rb32(s) + P["rnn_w"] @ P["emb"][path[t]] + P["rnn_b"])
            worst = max(worst, abs(tot - float(ref["beam_logp"][b, w])))
    return worst


def small_deviation(shapes=None):
    return max(fp32_deviation(*inputs_small(*c), c[4], c[5]) for c in (DRAFT_SHAPES if shapes is None else shapes))


def stored():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def round_up(x):
    """x rounded up to one significant digit."""
    e = math.floor(math.log10(x))
    return math.ceil(x / 10 ** e - 1e-9) * 10 ** e


_S = stored()
TOL = round_up(SAFETY * _S["small"])                                  # small test models
TOL_7B = round_up(SAFETY * max(_S["vicuna7b"], _S["vicuna13b"]))      # hidden size 4096 / 5120, vocabulary 32000
