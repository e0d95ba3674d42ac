"""Writes tests/golden/draft_fp32_deviation.txt: the largest difference between a plain numpy fp32
evaluation of the draft model and the fp64 oracle on teacher-forced candidate scores (see
tests/draft_tolerance.py).  Calls only the oracle and numpy; run from the repository root:
    python tests/golden/make_draft_fp32_deviation.py"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

if __name__ == "__main__":
    path = os.path.join(HERE, "draft_fp32_deviation.txt")
    if not os.path.exists(path):                       # draft_tolerance reads the file when imported
        open(path, "w").write("small 1\nvicuna7b 1\nvicuna13b 1\n")
    import draft_tolerance as dt
    small = dt.small_deviation()
    big = dt.fp32_deviation(*dt.inputs_7b(), 8, 5)
    big13 = dt.fp32_deviation(*dt.inputs_13b(), 16, 3)
    with open(path, "w") as f:
        f.write("# max |numpy fp32 score - oracle fp64 score| over the oracle's candidates (log-probability units)\n")
        f.write("# written by tests/golden/make_draft_fp32_deviation.py\n")
        f.write("small %.6e\n" % small)
        f.write("vicuna7b %.6e\n" % big)
        f.write("vicuna13b %.6e\n" % big13)
    print(open(path).read())
