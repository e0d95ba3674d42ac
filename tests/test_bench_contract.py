"""bench.py's command-line contract that can be checked without a GPU: a run on more than one GPU is
refused with a message (this build is single-GPU), and the script never imports the oracle at
module level (the oracle is test infrastructure; only the CPU-baseline leg may load it)."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, cwd=ROOT, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""                       # no JSON line for a run that did not happen


def test_product_code_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2403_09919_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            src = open(os.path.join(pkg, name)).read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", src, flags=re.M), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    top_level = [l for l in bench.splitlines() if re.match(r"(import|from)\s+oracle\b", l)]
    assert top_level == []                              # only inside cpu_baseline()
    assert re.search(r"def cpu_baseline\(.*?\n(.*\n)*?\s+import oracle", bench)
