"""GPU parity of gr_solve_logits (rows given as target / draft logits and a temperature per row; App. A, first
paragraph) against the checker's solve_row_from_logits, through the C ABI: alpha*, support, ratio order, H*,
blocks, residuals, weights through the dense slice, and the sampled token, on configs 2-4 given as logits;
plus the rows that the probability path and the logits path must agree on."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W
from parity_util import ABS_TOL, EDGE_TOL

pytestmark = pytest.mark.gpu


def _drafts_from_logits(wl, rows, seed):
    """n i.i.d. draws per row from the top-k renormalised softmax of the draft logits (float64), and uniforms."""
    from oracle import gr_oracle as G
    rng = np.random.default_rng(seed)
    drafts = np.zeros((wl.B, wl.n), np.int32)
    for b in range(wl.B):
        dl = wl.meta["draft_logits"][b].astype(np.float64)
        top = np.argsort(-dl, kind="stable")[: (wl.k if 0 < wl.k < wl.V else wl.V)]
        if b in rows:
            q = G.softmax_from_logits(wl.meta["draft_logits"][b], float(np.float32(wl.meta.get("draft_temps", wl.meta["temps"])[b])))
            assert sorted(int(t) for t in top) == G.topk_support(q, wl.k, key=dl)
        w = np.exp((dl[top] - dl[top].max()) / float(np.float32(wl.meta.get("draft_temps", wl.meta["temps"])[b])))
        drafts[b] = top[np.minimum(np.searchsorted(np.cumsum(w), rng.random(wl.n) * w.sum(), side="right"), top.size - 1)]
    return drafts


def _run_logits(wl, tol, drafts, export_rows=None):
    """A support above GR_MAX_SUPPORT has no dense export: its rows listed in `export_rows` are fetched one by one."""
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    full = (wl.V if (wl.k <= 0 or wl.k >= wl.V) else wl.k) > gr.GR_MAX_SUPPORT
    tl = torch.from_numpy(wl.meta["target_logits"]).to(dev); dl = torch.from_numpy(wl.meta["draft_logits"]).to(dev)
    T = torch.from_numpy(wl.meta["temps"].astype(np.float32)).to(dev)
    Td = torch.from_numpy(wl.meta["draft_temps"].astype(np.float32)).to(dev) if "draft_temps" in wl.meta else None
    d = torch.from_numpy(drafts).to(dev); u = torch.from_numpy(wl.uniforms).to(dev)
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n)
    try:
        acc, st = gr.gr_solve_logits(h, tl, dl, T, wl.n, wl.k, tol, draft_temperature=Td)
        tok, ok = gr.gr_verify(h, d, u)
        out = {"accept_prob": acc, "status": st, "token": tok, "accepted": ok}
        out["pi"], out["accept_given"] = gr.gr_policy_slice(h, d, wl.V)
        rows = {}
        if full:
            for name in ("support", "h_size", "iterations"):
                out[name] = torch.empty(wl.B, dtype=torch.int32, device=dev)
            rc = gr.load_library().gr_policy_export(h, None, None, None, None, out["support"].data_ptr(), out["h_size"].data_ptr(),
                                                    out["iterations"].data_ptr(), torch.cuda.current_stream().cuda_stream)
            assert rc == 0, rc
            torch.cuda.synchronize()
            sup = out["support"].cpu().numpy()
            for b in (export_rows or []):
                rows[b] = {k: v.cpu().numpy() for k, v in gr.gr_policy_export_row(h, b, int(sup[b]), dev).items()}
        else:
            out.update(gr.gr_policy_export(h, wl.B, dev))
        torch.cuda.synchronize()
        out = {k: v.cpu().numpy() for k, v in out.items()}
        if full:
            out["rows"] = rows
    finally:
        gr.gr_destroy(h)
    return out


def _compare(wl, out, rows, tol, drafts):
    from oracle import gr_oracle as G
    stats = {"rows": 0, "fragile": 0, "edge": 0, "programs": 0, "max_dpi": 0.0}
    for b in rows:
        T = float(np.float32(wl.meta["temps"][b]))
        Td = float(np.float32(wl.meta["draft_temps"][b])) if "draft_temps" in wl.meta else None
        sol, p, q = G.solve_row_from_logits(wl.meta["target_logits"][b], wl.meta["draft_logits"][b], T, wl.n, wl.k, tol=tol, max_T=128,
                                            draft_temperature=Td)
        tok, accepted, pi, acc_given, edge = G.verify_row(sol, p, drafts[b], wl.uniforms[b])
        stats["rows"] += 1
        assert abs(out["accept_prob"][b] - sol.alpha_star) < ABS_TOL, (b, out["accept_prob"][b], sol.alpha_star)
        assert abs(float(out["pi"][b].astype(np.float64).sum()) - 1.0) < 1e-5 and np.all(out["pi"][b] >= 0)
        if sol.fragile:
            stats["fragile"] += 1
            continue
        kk = len(sol.order)
        assert out["status"][b] == sol.status and out["support"][b] == kk and out["h_size"][b] == sol.h, (b, out["h_size"][b], sol.h)
        g = out["rows"][b] if "rows" in out else {k: out[k][b, :kk] for k in ("order", "block", "rho")}
        assert np.array_equal(g["order"], sol.order), (b, "ratio order differs")
        assert np.array_equal(g["block"], sol.block_of), (b, "block split differs")
        assert np.abs(g["rho"] - sol.rho).max() < 1e-12, (b, "residuals differ")
        stats["programs"] += sum(1 for blk in sol.blocks if blk.iters > 0)
        dpi = float(np.abs(out["pi"][b] - pi).max()); stats["max_dpi"] = max(stats["max_dpi"], dpi)
        assert dpi < ABS_TOL, (b, dpi)
        assert abs(out["accept_given"][b] - acc_given) < ABS_TOL
        if edge < EDGE_TOL:
            stats["edge"] += 1
        else:
            assert out["token"][b] == tok and bool(out["accepted"][b]) == accepted, (b, out["token"][b], tok, edge)
    assert stats["edge"] <= max(2, stats["rows"] // 20), stats
    return stats


def test_small_given_as_logits_all_rows():
    wl = W.small(keep_logits=True)                                   # config 2
    rows = range(wl.B)
    drafts = _drafts_from_logits(wl, set(rows), 11)
    out = _run_logits(wl, 1e-6, drafts)
    st = _compare(wl, out, rows, 1e-6, drafts)
    assert np.all(out["status"] == 0) and st["fragile"] == 0 and st["programs"] >= 32, st


@pytest.mark.parametrize("temperature", [0.7, 1.0])
def test_llm_shaped_given_as_logits(temperature):
    wl = W.llm_shaped(temperature=temperature, seed_sub=int(temperature * 10), keep_logits=True)      # config 3
    rows = list(range(0, wl.B, 16))
    drafts = _drafts_from_logits(wl, set(rows), 12)
    out = _run_logits(wl, 1e-6, drafts)
    st = _compare(wl, out, rows, 1e-6, drafts)
    assert np.all(out["status"] == 0) and st["fragile"] <= st["rows"] // 4 and st["programs"] >= 8, st


def test_large_vocab_given_as_logits_and_the_probability_path_beside_it():
    """Config 4 at full size as logits; every row's alpha* is also held against the probability path fed with the
    float32 softmaxes of the same logits (the two see p and q that differ by float32 rounding: 1e-6 on alpha*)."""
    import torch
    from paper_2511_15898_amd import binding as gr
    wl = W.large_vocab(keep_logits=True)
    rows = list(range(3, wl.B, 24))
    drafts = _drafts_from_logits(wl, set(rows), 13)
    out = _run_logits(wl, 1e-4, drafts)
    st = _compare(wl, out, rows, 1e-4, drafts)
    assert np.all(out["status"] == 0) and st["programs"] >= 6, st
    dev = torch.device("cuda:0")
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n)
    try:
        acc, _ = gr.gr_solve(h, torch.from_numpy(wl.p).to(dev), torch.from_numpy(wl.q).to(dev), wl.n, wl.k, 1e-4)
        torch.cuda.synchronize()
    finally:
        gr.gr_destroy(h)
    assert np.abs(acc.cpu().numpy() - out["accept_prob"]).max() < 5e-6


def test_logits_entry_point_rows_and_errors():
    """Per-row temperatures, a shift of a row's logits (no effect), a bad temperature and a NaN logit (GR_ROW_BAD),
    and the call-level refusals."""
    import torch
    from paper_2511_15898_amd import binding as gr
    wl = W.llm_shaped(B=12, V=6000, n=4, k=48, temperature=(0.5, 1.5), seed_sub=91, keep_logits=True)
    drafts = _drafts_from_logits(wl, set(range(wl.B)), 14)
    out = _run_logits(wl, 1e-6, drafts)
    _compare(wl, out, range(wl.B), 1e-6, drafts)
    dev = torch.device("cuda:0")
    tl = torch.from_numpy(wl.meta["target_logits"]).to(dev); dl = torch.from_numpy(wl.meta["draft_logits"]).to(dev)
    T = torch.from_numpy(wl.meta["temps"].astype(np.float32)).to(dev)
    tl2 = tl.clone(); dl2 = dl.clone(); T2 = T.clone()
    tl2[1] += 8.0; dl2[1] -= 16.0                       # exact in float32 for these magnitudes? compare loosely
    T2[2] = 0.0; tl2[3, 17] = float("nan"); dl2[4, 5] = float("inf")
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n)
    try:
        acc, st = gr.gr_solve_logits(h, tl2, dl2, T2, wl.n, wl.k, 1e-6)
        torch.cuda.synchronize()
        st = st.cpu().numpy(); acc = acc.cpu().numpy()
        assert list(st[2:5]) == [gr.GR_ROW_BAD] * 3 and np.all(np.isnan(acc[2:5]))
        assert st[0] == 0 and abs(acc[0] - out["accept_prob"][0]) < 1e-7 and abs(acc[1] - out["accept_prob"][1]) < 1e-5
        with pytest.raises(gr.GrError) as e:
            gr.gr_solve_logits(h, tl, dl, T, wl.n, 300, 1e-6)
        assert e.value.code == gr.GR_EINVAL                 # this handle holds no workspace for a support of 300
        with pytest.raises(TypeError):
            gr.gr_solve_logits(h, tl, dl, T[:3], wl.n, wl.k, 1e-6)
    finally:
        gr.gr_destroy(h)


@pytest.mark.parametrize("V,n,k,tol", [(3000, 4, 0, 1e-4), (5000, 2, 300, 1e-4), (2000, 8, 1000, 1e-3), (777, 3, 0, 1e-3)])
def test_logits_with_supports_above_the_lds_capacity(V, n, k, tol):
    """Rows given as logits whose support exceeds GR_MAX_SUPPORT (no top-k, or a large one): the HBM-resident path
    sorts on the draft logit and on draft minus target logit; every row against the checker."""
    wl = W.llm_shaped(B=10, V=V, n=n, k=k, temperature=(0.5, 1.5), near_identical_frac=0.2, seed_sub=300 + n, keep_logits=True)
    drafts = _drafts_from_logits(wl, set(range(wl.B)), 15)
    out = _run_logits(wl, tol, drafts, export_rows=range(wl.B))
    st = _compare(wl, out, range(wl.B), tol, drafts)
    assert st["rows"] == wl.B and st["fragile"] < wl.B
    assert np.any(out["status"] == 0)


@pytest.mark.parametrize("V,n,k,tol", [(8000, 4, 64, 1e-6), (3000, 3, 0, 1e-4)])
def test_a_cooled_target_with_the_draft_left_at_its_own_temperature(V, n, k, tol):
    """The paper's temperature study cools the target (0.2 ... 0.8) and leaves the draft at 1: two temperatures per row.
    One case on the LDS-resident path, one on the HBM-resident path; every row against the checker."""
    import dataclasses
    wl = W.llm_shaped(B=12, V=V, n=n, k=k, temperature=1.0, seed_sub=410 + n, keep_logits=True)
    rng = np.random.default_rng(17)
    meta = dict(wl.meta); meta["temps"] = rng.choice([0.4, 0.6, 0.8], size=wl.B); meta["draft_temps"] = np.ones(wl.B)
    wl = dataclasses.replace(wl, meta=meta)
    drafts = _drafts_from_logits(wl, set(range(wl.B)), 16)
    out = _run_logits(wl, tol, drafts, export_rows=range(wl.B))
    st = _compare(wl, out, range(wl.B), tol, drafts)
    assert st["rows"] == wl.B and st["fragile"] < wl.B and np.any(out["status"] == 0)
