"""Writes the stored expected values under tests/golden/ (calls the CPU oracle only).

    python tests/golden/make_golden.py

chain_fig6_style.json: a five-memory importance-propagation chain in the spirit of
the paper's Fig. 6 (query -> "locked door" -> "key" -> "table").  The figure's own
numbers are not in the paper's text; the scores here are this repository's, and the
expected sets are also derived by hand in tests/test_oracle_pins.py.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import keep_oracle as ko  # noqa: E402


def main():
    S = np.zeros((6, 5), dtype=np.float32)
    S[5] = [0.05, 0.10, 0.15, 0.12, 0.58]
    S[4] = [0.02, 0.03, 0.90, 0.05, 0.00]
    S[2] = [0.95, 0.05, 0.00, 0.00, 0.00]
    S[3] = [0.30, 0.30, 0.40, 0.00, 0.00]
    S[1] = [1.00, 0.00, 0.00, 0.00, 0.00]
    cases = []
    for ratio in (0.2, 0.4, 0.6, 0.8):
        for hops in (1, 2, 3, 8):
            got, runs = ko.select_multihop(S, list(range(5)), [1] * 5, ratio, hops)
            cases.append({"ratio": ratio, "hops": hops, "expect": got, "runs": runs})
    out = {"source": "Fig. 6 (structure only; numbers are this repository's own)",
           "scores": [[float(v) for v in row] for row in S], "cases": cases}
    with open(os.path.join(HERE, "chain_fig6_style.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
