"""A caller may capture its very first call into a HIP graph.  Some kernels raise their dynamic LDS limit on
first use (attention, the beam step for more than 64 candidates, the many-row linear layers); that setup must
work while a capture is open.  The check needs a process in which nothing has run yet, so it runs once in a
child process (one GPU process besides this one)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

CHILD = r"""
import sys
import numpy as np, torch
root = sys.argv[1]
sys.path.insert(0, root); sys.path.insert(0, root + "/tests")
from paper_2403_09919_amd import binding as rd
from test_oracle_draft import make_params, make_h
from gpu_util import dev, host
Dm, V, K, B, W, L = 256, 16500, 1, 2, 70, 3        # 70 candidates (dynamic LDS in the beam step), 140 rows
p = make_params(V, Dm, K, seed=1, scale=4.0)
pd = rd.rd_draft_pack({k: dev(v) for k, v in p.items()})
h = dev(make_h(B, Dm, 3, "bf16")); last = dev(np.array([5, 7], np.int32))
ws = torch.zeros(rd.rd_draft_workspace(B, W, L, Dm, V), dtype=torch.uint8, device="cuda")
out = {"beams": torch.zeros((B, W, L), dtype=torch.int32, device="cuda"),
       "beam_logp": torch.zeros((B, W), dtype=torch.float32, device="cuda")}
stream = torch.cuda.Stream(); g = torch.cuda.CUDAGraph()
with torch.cuda.stream(stream):
    with torch.cuda.graph(g, stream=stream):
        rd.rd_draft(pd, h, last, W, L, out=out, workspace=ws)
        d = rd.rd_dedup(out["beams"])
g.replay(); torch.cuda.synchronize()
beams, n_packed = host(out["beams"]).copy(), host(d["n_packed"]).copy()
eager = rd.rd_draft(pd, h, last, W, L, workspace=ws)
de = rd.rd_dedup(eager["beams"])
torch.cuda.synchronize()
assert np.array_equal(beams, host(eager["beams"])) and np.array_equal(n_packed, host(de["n_packed"]))
assert (beams[:, :, 0] == np.array([5, 7])[:, None]).all()
print("CAPTURE-FIRST-OK")
"""


def test_first_call_inside_a_capture():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    print("first-ever rd_draft call inside a stream capture (child process)", flush=True)
    r = subprocess.run([sys.executable, "-c", CHILD, root], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "CAPTURE-FIRST-OK" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
