"""Shared helpers of the GPU parity tests: run the HIP path on a workload, run the CPU checker
on chosen rows, compare element by element."""
from __future__ import annotations

import numpy as np

ABS_TOL = 1e-5          # spec tolerance on alpha* and on every policy entry
EDGE_TOL = 1e-5         # a uniform this close to a CDF edge may fall either way


def run_gpu(wl, tol, max_iter=0, max_T=0, rel_tol=0.0, want_slice=True, drafts=None, export_rows=None):
    """Run the HIP path.  A policy over more than GR_MAX_SUPPORT tokens (no top-k on a large V, or a large top-k) has no
    dense export: its rows listed in `export_rows` are fetched one by one into out["rows"]."""
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    full = (wl.V if (wl.k <= 0 or wl.k >= wl.V) else wl.k) > gr.GR_MAX_SUPPORT
    p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
    d = torch.from_numpy(wl.drafts if drafts is None else drafts).to(dev)
    u = torch.from_numpy(wl.uniforms).to(dev)
    h = gr.gr_create(wl.B, wl.V, max_iter=max_iter, max_T=max_T, rel_tol=rel_tol)
    try:
        acc, st = gr.gr_solve(h, p, q, wl.n, wl.k, tol)
        tok, ok = gr.gr_verify(h, d, u)
        out = {"accept_prob": acc, "status": st, "token": tok, "accepted": ok}
        if want_slice:
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


def compare_rows(wl, out, rows, tol, max_iter=4000, max_T=0, drafts=None):
    """Element-by-element comparison with the CPU checker on `rows`.  Returns statistics."""
    from oracle import gr_oracle as G
    drafts = wl.drafts if drafts is None else drafts
    max_T = max_T or 128                      # the library's GR_MAX_T applies when no cap is given
    stats = {"rows": 0, "fragile": 0, "edge": 0, "max_dacc": 0.0, "max_dpi": 0.0}
    for b in rows:
        sol = G.solve_row(wl.p[b], wl.q[b], wl.n, wl.k, tol=tol, max_T=max_T, max_iter=max_iter)
        tok, accepted, pi, acc_given, edge = G.verify_row(sol, wl.p[b], drafts[b], wl.uniforms[b])
        stats["rows"] += 1
        assert abs(out["accept_prob"][b] - sol.alpha_star) < ABS_TOL, (b, out["accept_prob"][b], sol.alpha_star)
        if sol.fragile:                       # several optimal H*: compare what is unique only
            stats["fragile"] += 1
            if "pi" in out:
                assert abs(float(out["pi"][b].sum()) - 1.0) < 1e-4
            continue
        assert out["status"][b] == sol.status, (b, out["status"][b], sol.status)
        kk = len(sol.order)
        assert out["support"][b] == kk and out["h_size"][b] == sol.h, (b, out["support"][b], kk, out["h_size"][b], sol.h)
        g_order, g_block, g_rho = (out["rows"][b]["order"], out["rows"][b]["block"], out["rows"][b]["rho"]) if "rows" in out \
            else (out["order"][b, :kk], out["block"][b, :kk], out["rho"][b, :kk])
        assert np.array_equal(g_order, sol.order), (b, "ratio order differs")
        assert np.array_equal(g_block, sol.block_of), (b, "block split differs")
        assert np.abs(g_rho - sol.rho).max() < 1e-12, (b, "residuals differ")
        if "pi" in out:
            dpi = float(np.abs(out["pi"][b] - pi).max())
            stats["max_dpi"] = max(stats["max_dpi"], dpi)
            assert dpi < ABS_TOL, (b, dpi)
            assert abs(out["accept_given"][b] - acc_given) < ABS_TOL, (b, out["accept_given"][b], acc_given)
        stats["max_dacc"] = max(stats["max_dacc"], abs(float(out["accept_prob"][b]) - sol.alpha_star))
        if edge < EDGE_TOL:
            stats["edge"] += 1
        else:
            assert out["token"][b] == tok and bool(out["accepted"][b]) == accepted, \
                (b, out["token"][b], tok, out["accepted"][b], accepted, edge)
    return stats


def check_alpha_all_rows(wl, out):
    """alpha* needs no convex solve (Sec. 6, step 1): cheap enough to check on every row."""
    from oracle import gr_oracle as G
    for b in range(wl.B):
        sup = G.topk_support(wl.q[b], wl.k)
        order = G.ratio_order(wl.p[b], wl.q[b], sup)
        pt = float(np.sum(wl.p[b], dtype=np.float64))
        _, _, F = G.prefix_psi(wl.p[b][order].astype(np.float64) / pt, wl.q[b][order], wl.n)
        assert abs(out["accept_prob"][b] - (1.0 + F.min())) < ABS_TOL, (b, out["accept_prob"][b], 1.0 + F.min())
