"""GPU parity of the full-vocabulary path (no top-k, support above GR_MAX_SUPPORT): ratio order by the
HBM sort, alpha*, residuals, blocks, truncation sets and row status, the convex programs of rows whose
truncation sets fit, the dense slice and the sampled token, against the CPU checker.  Same tolerances
as the top-k parity tests."""
import dataclasses

import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W
from parity_util import check_alpha_all_rows, compare_rows, run_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [2, 4, 8, 16])
def test_stress_full_vocab_cells(n):
    """Config 5's 'top-k = full V' cells at V = 128256 (4 rows per cell: the checker needs seconds per
    row).  Most rows are degenerate (alpha* = 1 with H* empty or everything) or exceed the cap on |T|;
    alpha* is checked on every row, everything else on the rows where it is unique."""
    wl = W.stress(B=4, n=n, k=0, seed_sub=900 + n)
    out = run_gpu(wl, 1e-4, export_rows=range(wl.B))
    check_alpha_all_rows(wl, out)
    stats = compare_rows(wl, out, range(wl.B), 1e-4)
    assert stats["rows"] == wl.B
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)


@pytest.mark.parametrize("V,n,tol", [(5000, 4, 1e-4), (5000, 2, 1e-4), (3000, 8, 1e-3), (777, 16, 1e-3)])
def test_mid_size_vocab_without_top_k(V, n, tol):
    """LLM-shaped rows on a vocabulary that the checker handles quickly: every row is compared, and
    rows with alpha* < 1 whose truncation sets fit exercise both kinds of convex program."""
    wl = W.llm_shaped(B=24, V=V, n=n, k=0, seed_sub=40 + n)
    out = run_gpu(wl, tol, export_rows=range(wl.B))
    check_alpha_all_rows(wl, out)
    stats = compare_rows(wl, out, range(wl.B), tol)
    assert stats["rows"] == wl.B and stats["fragile"] < wl.B
    assert np.any(out["status"] == 0) and out["iterations"].max() > 0


def test_residual_draws_walk_the_dense_residuals():
    """Uniforms close to 1 force the draw past the drafts wherever the conditional acceptance is below
    1, so the sampled token comes from the residual spread over all V tokens."""
    wl = W.llm_shaped(B=24, V=5000, n=2, k=0, seed_sub=77)
    wl = dataclasses.replace(wl, uniforms=np.full(wl.B, 0.9990234375, dtype=np.float32))
    out = run_gpu(wl, 1e-4, export_rows=range(wl.B))
    compare_rows(wl, out, range(wl.B), 1e-4)
    assert np.any(out["accepted"] == 0)


def test_flat_rows_and_exact_zeros():
    """Dirichlet rows (flat: every program exceeds the cap, the fallback transport is used) and rows
    with exact zeros in q (tokens outside the support rank nowhere and keep p as residual)."""
    wl = W.tiny(B=12, V=300, n=2)
    out = run_gpu(wl, 1e-2, export_rows=range(wl.B))
    compare_rows(wl, out, range(wl.B), 1e-2)
    rng = np.random.default_rng(5)
    wl = W.llm_shaped(B=8, V=2000, n=3, k=0, seed_sub=3)
    q = wl.q.copy()
    q[:, rng.permutation(2000)[:700]] = 0.0
    q = (q / q.sum(1, keepdims=True, dtype=np.float32)).astype(np.float32)
    drafts = W.draw_drafts(q, 0, wl.n, rng)
    wl = dataclasses.replace(wl, q=np.ascontiguousarray(q), drafts=drafts)
    out = run_gpu(wl, 1e-4, export_rows=range(wl.B))
    assert np.all(out["support"] == (q > 0).sum(1))
    check_alpha_all_rows(wl, out)
    compare_rows(wl, out, range(wl.B), 1e-4)


def test_bad_rows_bad_drafts_and_determinism():
    import torch
    from paper_2511_15898_amd import binding as gr
    wl = W.llm_shaped(B=6, V=1500, n=4, k=0, seed_sub=9)
    p = wl.p.copy(); q = wl.q.copy()
    p[1, 7] = np.nan
    q[2] = q[2] * np.float32(0.5)                       # row sum 0.5
    q[3, 11] = 0.0
    drafts = wl.drafts.copy()
    drafts[3, 0] = 11                                   # a draft with q = 0
    drafts[4, 1] = 1500                                 # out of range
    wl2 = dataclasses.replace(wl, p=p, q=q, drafts=drafts)
    a = run_gpu(wl2, 1e-4, export_rows=[0, 5])
    b = run_gpu(wl2, 1e-4, export_rows=[0, 5])
    assert a["status"][1] == gr.GR_ROW_BAD and a["status"][2] == gr.GR_ROW_BAD
    assert np.isnan(a["accept_prob"][1]) and a["token"][1] == -1 and a["token"][2] == -1
    assert a["token"][4] == -1 and a["accepted"][4] == 0
    if a["status"][3] == gr.GR_ROW_OK:
        assert a["token"][3] == -1 and a["accepted"][3] == 0
    compare_rows(wl2, a, [0, 5], 1e-4)
    for key in ("accept_prob", "status", "token", "accepted", "pi"):
        assert np.array_equal(a[key], b[key], equal_nan=True), key
    for r in (0, 5):
        assert np.array_equal(a["rows"][r]["order"], b["rows"][r]["order"])
        assert np.array_equal(a["rows"][r]["weight"], b["rows"][r]["weight"])


def test_uniform_rows_at_full_size():
    """p = q uniform over 128256 tokens: all ratios tie (order = token id), alpha* = 1; with a top-k of
    1000 all q tie as well and the support is the 1000 lowest token ids."""
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    V = 128256
    h = gr.gr_create(2, V, max_k=0)
    try:
        p = torch.full((2, V), 1.0 / V, device=dev)
        acc, st = gr.gr_solve(h, p, p, 4, V, 1e-6)
        d = torch.tensor([[5, 9, 5, 100000], [0, 1, 2, 3]], dtype=torch.int32, device=dev)
        u = torch.tensor([0.3, 0.9], device=dev)
        tok, ok = gr.gr_verify(h, d, u)
        row = gr.gr_policy_export_row(h, 0, V, dev)
        torch.cuda.synchronize()
        assert np.allclose(acc.cpu().numpy(), 1.0, atol=1e-6)
        assert np.array_equal(row["order"].cpu().numpy(), np.arange(V))
        assert np.all(tok.cpu().numpy() >= 0) and np.all(tok.cpu().numpy() < V)
        acc, st = gr.gr_solve(h, p, p, 4, 1000, 1e-6)    # ties in q: the 1000 lowest token ids
        row = gr.gr_policy_export_row(h, 1, 1000, dev)
        torch.cuda.synchronize()
        assert np.array_equal(row["order"].cpu().numpy(), np.arange(1000))
    finally:
        gr.gr_destroy(h)


def test_stress_full_vocab_cell_at_full_batch():
    """One 'full V' cell at config 5's own size (1024 rows x 128256 tokens, n = 8): alpha* against
    the checker on sampled rows, statuses and tokens valid on every row."""
    import torch
    from oracle import gr_oracle as G
    from paper_2511_15898_amd import binding as gr
    wl = W.stress(B=1024, n=8, k=0, seed_sub=908)
    out = run_gpu(wl, 1e-4, want_slice=False)
    assert np.all((out["status"] == gr.GR_ROW_OK) | (out["status"] == gr.GR_ROW_TRUNC_CAP))
    assert np.all((out["token"] >= 0) & (out["token"] < wl.V))
    assert np.all(out["support"] == (wl.q > 0).sum(1))
    for b in (0, 511, 1023):
        order = G.ratio_order(wl.p[b], wl.q[b], G.topk_support(wl.q[b], 0))
        pt = float(np.sum(wl.p[b], dtype=np.float64))
        _, _, F = G.prefix_psi(wl.p[b][order].astype(np.float64) / pt, wl.q[b][order], wl.n)
        assert abs(out["accept_prob"][b] - (1.0 + F.min())) < 1e-5
        assert out["h_size"][b] == int(np.argmin(F)) or np.sort(F)[1] - np.sort(F)[0] < 1e-13
    # rows whose programs ran (status OK with evaluations): order, |H*|, residuals, blocks, slice and token of
    # four of them against the checker, which orders all 128256 tokens of each
    ran = np.flatnonzero((out["status"] == gr.GR_ROW_OK) & (out["iterations"] > 0))
    assert ran.size >= wl.B // 20, ran.size
    rows = [int(b) for b in ran[:: max(1, ran.size // 4)][:4]]
    again = run_gpu(wl, 1e-4, export_rows=rows)
    assert np.array_equal(again["status"], out["status"]) and np.array_equal(again["token"], out["token"])
    stats = compare_rows(wl, again, rows, 1e-4)
    assert stats["rows"] == 4 and stats["solved_rows"] + stats["fragile"] == 4 and stats["solved_rows"] >= 2, stats


@pytest.mark.parametrize("V,n,k,tol", [(5000, 4, 300, 1e-4), (3000, 2, 1000, 1e-4), (1200, 8, 257, 1e-3)])
def test_top_k_above_the_lds_capacity(V, n, k, tol):
    """A top-k between GR_MAX_SUPPORT and V: the k largest q (ties by token id) are selected by a sort
    in HBM, everything after that is the full-vocabulary path."""
    wl = W.llm_shaped(B=12, V=V, n=n, k=k, seed_sub=60 + n)
    out = run_gpu(wl, tol, export_rows=range(wl.B))
    assert np.all(out["support"] == k)
    check_alpha_all_rows(wl, out)
    stats = compare_rows(wl, out, range(wl.B), tol)
    assert stats["rows"] == wl.B


@pytest.mark.parametrize("V,n,k,tail_mass,tol", [(5000, 4, 0, 1e-6, 1e-4), (5000, 2, 0, 1e-3, 1e-4), (3000, 8, 0, 1e-4, 1e-3),
                                                 (5000, 4, 300, 1e-3, 1e-4), (777, 3, 0, 0.05, 1e-3),
                                                 (5000, 4, 64, 1e-3, 1e-4), (1024, 3, 200, 0.05, 1e-3), (200, 2, 0, 0.01, 1e-4)])
def test_nucleus_cut_of_the_draft(V, n, k, tail_mass, tol):
    """gr_config.tail_mass (Sec. 5.1 / App. A: top-p sampling of the draft restricts the domain): every row
    against the checker with the same cut -- support size, order, blocks, programs, slice, token -- and
    alpha* against the uncut run within n * tail_mass.  The last three cases have supports of at most
    GR_MAX_SUPPORT tokens and run on the LDS-resident path."""
    from oracle import gr_oracle as G
    wl = W.llm_shaped(B=24, V=V, n=n, k=k, seed_sub=60 + n)
    out = run_gpu(wl, tol, export_rows=range(wl.B), tail_mass=tail_mass)
    check_alpha_all_rows(wl, out, tail_mass=tail_mass)
    for b in range(wl.B):
        assert out["support"][b] == len(G.topk_support(wl.q[b], k, tail_mass)), b
    stats = compare_rows(wl, out, range(wl.B), tol, tail_mass=tail_mass)
    assert stats["rows"] + stats.get("skipped", 0) == wl.B and stats["rows"] >= wl.B // 2 and stats["fragile"] < wl.B
    uncut = run_gpu(wl, tol, want_slice=False)
    assert np.all(np.abs(out["accept_prob"] - uncut["accept_prob"]) <= n * tail_mass + 2e-6)
    assert np.any(out["support"] < uncut["support"])            # the cut dropped tokens


def test_nucleus_cut_on_the_stress_cell_at_full_batch():
    """Config 5, 'top-k = full V', n = 8, B = 1024 at V = 128256 with tail_mass = 1e-8 (alpha* within 8e-8 of the
    uncut value): the supports shrink to what the checker orders in milliseconds, so alpha* is checked on
    every 4th row, 24 rows are compared in full (near-identical rows among them), rows with programs must
    be there, and four rows are held against the uncut checker."""
    from oracle import gr_oracle as G
    tm = 1e-8
    wl = W.stress(B=1024, n=8, k=0, seed_sub=908)
    near = [int(x) for x in np.flatnonzero(wl.meta["near"])[:6]]
    rows = sorted(set(range(5, wl.B, 57)) | set(near))
    out = run_gpu(wl, 1e-4, want_slice=False, export_rows=rows, tail_mass=tm)
    check_alpha_all_rows(wl, out, rows=range(0, wl.B, 4), tail_mass=tm)
    stats = compare_rows(wl, out, rows, 1e-4, tail_mass=tm)
    assert stats["rows"] >= len(rows) - 1 and stats["solved_rows"] >= 4, stats
    solved = (out["status"] == 0) & (out["iterations"] > 0)
    assert solved.sum() >= wl.B // 20, int(solved.sum())
    assert np.median(out["support"]) < wl.V // 4 and out["support"].min() >= 1
    for b in rows[:4]:
        order = G.ratio_order(wl.p[b], wl.q[b], G.topk_support(wl.q[b], 0))
        pt = float(np.sum(wl.p[b], dtype=np.float64))
        _, _, F = G.prefix_psi(wl.p[b][order].astype(np.float64) / pt, wl.q[b][order], wl.n)
        assert abs(out["accept_prob"][b] - (1.0 + F.min())) <= wl.n * tm + 2e-6
