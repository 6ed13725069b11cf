"""How many evaluator calls the solve spends per row on the paper-shaped batches (gr_solve_stats).  The counts are
deterministic for given inputs; the bounds leave room for a different rounding.  They guard the solver's treatment
of tokens whose target nearly exhausts the probability that they are drawn (Thm 6.5 / 6.4 programs whose plain
fixed-point step crawls): before that treatment the slowest rows of these batches took 35, 26 and 15 evaluations."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("make, tol, most, mean_most", [(W.small, 1e-4, 20, 9.5), (W.llm_shaped, 1e-4, 28, 9.0), (W.large_vocab, 1e-4, 14, 7.2)])
def test_evaluations_per_row_stay_bounded(make, tol, most, mean_most):
    import torch
    from paper_2511_15898_amd import binding as gr
    wl = make()
    dev = torch.device("cuda:0")
    p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n)
    try:
        _, st = gr.gr_solve(h, p, q, wl.n, wl.k, tol)
        ev = gr.gr_solve_stats(h, wl.B, dev)["evaluations"].cpu().numpy()
        torch.cuda.synchronize()
    finally:
        gr.gr_destroy(h)
    assert int(st.abs().sum()) == 0
    assert ev.max() <= most and ev.mean() <= mean_most, (int(ev.max()), float(ev.mean()))
