#!/usr/bin/env python3
"""Writes tests/golden/tiny_lp_optima.json: small seeded (p, q, n) cases with the optimum of the relaxed
OTLP as an explicit linear program (Eq. "relaxed-lp"), the optimum of the OTLP itself (Eq. "opt-lp"),
and min psi over all subsets (Thm 3.1).  Calls nothing but oracle/brute.py; neither the checker's
prefix argument nor the HIP path has a hand in these values.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import brute  # noqa: E402


def main():
    rng = np.random.default_rng(20251115)
    cases = []
    for V, n, alpha in ((3, 2, 0.5), (4, 2, 0.5), (4, 3, 0.3), (5, 2, 1.0), (5, 3, 0.5), (6, 2, 0.3), (3, 4, 0.7), (6, 3, 0.2)):
        for _ in range(3):
            p = rng.dirichlet(np.full(V, alpha)).astype(np.float32)
            q = rng.dirichlet(np.full(V, alpha)).astype(np.float32)
            p = (p / p.sum(dtype=np.float32)).astype(np.float32)
            q = (q / q.sum(dtype=np.float32)).astype(np.float32)
            p64 = p.astype(np.float64) / float(np.sum(p, dtype=np.float64))
            q64 = q.astype(np.float64) / float(np.sum(q, dtype=np.float64))
            psi_min, subset = brute.psi_min_all_subsets(p64, q64, n)
            case = {"V": V, "n": n, "p": [float(x) for x in p], "q": [float(x) for x in q],
                    "relaxed_lp": brute.relaxed_otlp_value(p64, q64, n), "psi_min": psi_min,
                    "smallest_minimiser": [int(i) for i in subset]}
            if V ** (n + 1) <= 1500:
                case["otlp"] = brute.otlp_value(p64, q64, n)
            cases.append(case)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_lp_optima.json")
    with open(out, "w") as f:
        json.dump({"source": "oracle/brute.py: explicit LPs of Eq. (relaxed-lp) and Eq. (opt-lp), subset enumeration of Thm 3.1",
                   "cases": cases}, f, indent=1)
    print(out, len(cases))


if __name__ == "__main__":
    main()
