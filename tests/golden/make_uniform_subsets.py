"""Writes tests/golden/uniform_subsets.txt: token subsets of the Doc-Uniform baseline for a few
(seed, query, document, T, m).  Calls only the CPU oracle.  The generator is this build's own
definition (the paper fixes only "uniformly, without replacement": appendix "Compared Methods",
Doc-Uniform algorithm box), so the file freezes that definition; it is not a value the paper
prints.  Run from the repository root:  python tests/golden/make_uniform_subsets.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

cases = [(0, 0, 0, 32, 4), (0, 0, 1, 32, 4), (0, 1, 0, 32, 4), (1, 0, 0, 32, 4), (99, 127, 499999, 32, 8),
         (1234567, 3, 17, 24, 5), (7, 2, 1000, 64, 64), (7, 2, 1000, 64, 1), (7, 2, 1000, 7, 3),
         (2**63 + 5, 65534, 2**31 - 2, 32, 16)]
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "uniform_subsets.txt")
with open(out, "w") as f:
    f.write("# Doc-Uniform token subsets (appendix \"Compared Methods\"): Floyd sampling on a SplitMix64\n"
            "# stream per (query, document); written by make_uniform_subsets.py from the CPU oracle.\n"
            "# seed query document T m mask(hex, bit t = token t revealed)\n")
    for seed, q, i, T, m in cases:
        f.write(f"{seed} {q} {i} {T} {m} {oracle.uniform_subset(seed, q, i, T, m):x}\n")
print(open(out).read())
