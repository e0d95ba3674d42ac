"""rd_accept_static, the entry point that allocates nothing (for callers under graph capture or in
loops that must not call hipMalloc): its outputs must equal rd_accept's bit for bit -- and the
oracle's -- on two calls in a row, the second with a smaller input, since both calls share the
library's static scratch array and the second finds what the first left there."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, dev, host
from paper_2403_09919_amd import synth

pytestmark = pytest.mark.gpu

KEYS = ("argmax", "n_accept", "best_beam", "best_len", "next_token", "accepted_idx")


def _case(B, W, L, V, seed, share="uniform"):
    beams = synth.make_beams(B, W, L, V, seed, share)
    d = oracle.dedup(beams)
    logits = synth.make_logits(B, W * L, V, seed, d["packed_tokens"], d["parent"], d["n_packed"], 0.7)
    return beams, d, logits


def _outputs(B, W, L):
    i32 = torch.int32
    return dict(argmax=torch.full((B, W * L), -9, dtype=i32, device="cuda"),
                n_accept=torch.full((B, W), -9, dtype=i32, device="cuda"),
                best_beam=torch.full((B,), -9, dtype=i32, device="cuda"),
                best_len=torch.full((B,), -9, dtype=i32, device="cuda"),
                next_token=torch.full((B,), -9, dtype=i32, device="cuda"),
                accepted_idx=torch.full((B, L), -9, dtype=i32, device="cuda"))


def test_static_scratch_entry_point_matches_rd_accept_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2403_09919_amd import binding as rd
    shapes = [(8, 16, 5, 32000, 41, "high"), (2, 8, 5, 4099, 42, "uniform")]     # the second call is smaller
    cases = []
    for (B, W, L, V, seed, share) in shapes:
        beams, d, logits = _case(B, W, L, V, seed, share)
        root = beams[:, 0, 0].copy()
        root[0] += 1                                            # one sequence whose first token is rejected
        cases.append(dict(shape=(B, W, L, V), beams=beams, d=d, logits=logits, root=root,
                          t=dict(logits=dev(logits), beams=dev(beams), ui=dev(d["unpack_index"]),
                                 n_packed=dev(d["n_packed"]), root=dev(root)),
                          out=_outputs(B, W, L)))
    torch.cuda.synchronize()
    for c in cases:                                             # back to back, nothing in between
        announce("rd_accept_static B=%d W=%d L=%d V=%d" % c["shape"])
        t = c["t"]
        rd.rd_accept_static(t["logits"], t["beams"], t["ui"], t["n_packed"], c["out"], root_token=t["root"])
    torch.cuda.synchronize()
    for c in cases:
        t = c["t"]
        want = rd.rd_accept(t["logits"], t["beams"], t["ui"], t["n_packed"], t["root"])
        torch.cuda.synchronize()
        am = oracle.argmax(c["logits"], c["d"]["n_packed"])
        ref = oracle.accept(c["beams"], c["d"]["unpack_index"], am, c["root"])
        ref["argmax"] = am
        for k in KEYS:
            assert np.array_equal(host(c["out"][k]), host(want[k])), (c["shape"], k)
            assert np.array_equal(host(c["out"][k]), ref[k]), (c["shape"], k, "oracle")
    # and once more without a root token, on the smaller shape, after the calls above
    c = cases[1]
    t = c["t"]
    out = _outputs(*c["shape"][:3])
    rd.rd_accept_static(t["logits"], t["beams"], t["ui"], t["n_packed"], out)
    want = rd.rd_accept(t["logits"], t["beams"], t["ui"], t["n_packed"])
    torch.cuda.synchronize()
    for k in KEYS:
        assert np.array_equal(host(out[k]), host(want[k])), k
