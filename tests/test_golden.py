"""Stored optima of explicit linear programs on tiny cases (tests/golden/tiny_lp_optima.json, written by
tests/golden/make_golden.py from oracle/brute.py alone): the checker's alpha* and H* against them on the
CPU, the HIP path's accept_prob and |H*| against them on the GPU."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_lp_optima.json")


def _cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


def test_fixture_is_self_consistent():
    """Thm 3.1: the LP optimum equals 1 + min psi; the relaxed and the equality-constrained LP agree."""
    cases = _cases()
    assert len(cases) >= 20
    for c in cases:
        assert abs(c["relaxed_lp"] - (1.0 + c["psi_min"])) < 1e-9
        if "otlp" in c:
            assert abs(c["otlp"] - c["relaxed_lp"]) < 1e-9


def test_checker_matches_the_stored_optima():
    from oracle import gr_oracle as G
    for c in _cases():
        p = np.array(c["p"], dtype=np.float32); q = np.array(c["q"], dtype=np.float32)
        sol = G.solve_row(p, q, c["n"], 0, tol=1e-9)
        assert abs(sol.alpha_star - c["relaxed_lp"]) < 1e-9, c
        assert sorted(int(t) for t in sol.order[:sol.h]) == c["smallest_minimiser"], c
        assert sol.status == 0


@pytest.mark.gpu
def test_hip_path_matches_the_stored_optima():
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    cases = _cases()
    for V in sorted({c["V"] for c in cases}):
        for n in sorted({c["n"] for c in cases if c["V"] == V}):
            grp = [c for c in cases if c["V"] == V and c["n"] == n]
            p = torch.tensor([c["p"] for c in grp], dtype=torch.float32, device=dev)
            q = torch.tensor([c["q"] for c in grp], dtype=torch.float32, device=dev)
            h = gr.gr_create(len(grp), V)
            try:
                acc, st = gr.gr_solve(h, p, q, n, 0, 1e-9)
                exp = gr.gr_policy_export(h, len(grp), dev)
                torch.cuda.synchronize()
                acc = acc.cpu().numpy(); order = exp["order"].cpu().numpy(); hs = exp["h_size"].cpu().numpy()
                assert np.all(st.cpu().numpy() == 0)
                for b, c in enumerate(grp):
                    assert abs(float(acc[b]) - c["relaxed_lp"]) < 1e-5, (c, acc[b])
                    assert sorted(int(t) for t in order[b, :hs[b]]) == c["smallest_minimiser"], c
            finally:
                gr.gr_destroy(h)
