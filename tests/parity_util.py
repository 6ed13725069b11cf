"""Shared helpers of the GPU parity tests: run the HIP path on a workload, run the CPU checker
on chosen rows, compare element by element."""
from __future__ import annotations

import numpy as np

ABS_TOL = 1e-5          # spec tolerance on alpha* and on every policy entry
EDGE_TOL = 1e-5         # a uniform this close to a CDF edge may fall either way


def run_gpu(wl, tol, max_iter=0, max_T=0, rel_tol=0.0, want_slice=True, drafts=None, export_rows=None, tail_mass=0.0):
    """Run the HIP path.  A policy over more than GR_MAX_SUPPORT tokens (no top-k on a large V, or a large top-k) has no
    dense export: its rows listed in `export_rows` are fetched one by one into out["rows"]."""
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    full = (wl.V if (wl.k <= 0 or wl.k >= wl.V) else wl.k) > gr.GR_MAX_SUPPORT
    p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
    d = torch.from_numpy(wl.drafts if drafts is None else drafts).to(dev)
    u = torch.from_numpy(wl.uniforms).to(dev)
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n, max_iter=max_iter, max_T=max_T, rel_tol=rel_tol, tail_mass=tail_mass)
    try:
        acc, st = gr.gr_solve(h, p, q, wl.n, wl.k, tol)
        tok, ok = gr.gr_verify(h, d, u)
        out = {"accept_prob": acc, "status": st, "token": tok, "accepted": ok}
        # the one-call form must give the same bits (and leaves the same policy in the handle for what follows)
        one = gr.gr_solve_verify(h, p, q, wl.n, wl.k, tol, d, u)
        assert torch.equal(one[0].view(torch.int32), acc.view(torch.int32)) and torch.equal(one[1], st), "gr_solve_verify: solve outputs differ"
        assert torch.equal(one[2], tok) and torch.equal(one[3], ok), "gr_solve_verify: token / accepted differ"
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


def _gpu_policy_as_solution(wl, out, b):
    """The GPU's exported policy of row b in the shape oracle.policy_slice reads (only the fields it uses)."""
    from oracle import gr_oracle as G
    kk, h = int(out["support"][b]), int(out["h_size"][b])
    if "rows" in out:
        r = out["rows"][b]
        order, block, weight, rho = r["order"], r["block"], r["weight"], r["rho"]
    else:
        order, block, weight, rho = out["order"][b, :kk], out["block"][b, :kk], out["weight"][b, :kk], out["rho"][b, :kk]
    z = np.zeros(0)
    return G.RowSolution(wl.V, wl.n, np.asarray(order, int), {int(t): i for i, t in enumerate(order)}, z, z, z, z, z, z, h,
                         float(out["accept_prob"][b]), np.asarray(rho, float), z, np.asarray(block, int), [],
                         np.asarray(weight, float), int(out["status"][b]))


def check_row_validity(wl, out, b, drafts, alpha_star, tol=0.0):
    """What must hold for ANY correct result of row b, whichever optimal H* was taken (Sec. 3.1: the slice
    is a distribution; Eq. (cases): its mass sits on the drafts and, for drafts inside H*, on tokens outside
    H*; App. A: accepted iff the token is a draft).  On rows small enough to enumerate every draft tuple
    the coupling is rebuilt from the GPU's exported policy: marginal = p and acceptance = alpha*, both to within the
    truncated solver's bound when tol > 0 (App. "Truncated Solver Details": at most 15 tol in total variation)."""
    from oracle import brute, gr_oracle as G
    dset = set(int(t) for t in drafts[b])
    if "pi" in out:
        pi = out["pi"][b].astype(np.float64)
        assert np.all(pi >= 0.0), (b, "negative policy entry")
        assert abs(float(pi.sum()) - 1.0) < 1e-5, (b, float(pi.sum()))
        acc = float(sum(pi[t] for t in dset))
        assert acc <= 1.0 + 1e-6 and abs(float(out["accept_given"][b]) - acc) < ABS_TOL, (b, acc, out["accept_given"][b])
        if int(out["status"][b]) == 0 and ("rows" not in out or b in out["rows"]):
            sol = _gpu_policy_as_solution(wl, out, b)
            inside = set(int(t) for t in sol.order[: sol.h])
            bad = [int(t) for t in np.flatnonzero(pi > 0) if int(t) in inside and int(t) not in dset]
            assert not bad, (b, "mass on tokens of H* that were not drafted", bad[:5])
        tok = int(out["token"][b])
        assert 0 <= tok < wl.V and pi[tok] > 0.0, (b, tok, "token outside the slice's support")
    assert bool(out["accepted"][b]) == (int(out["token"][b]) in dset), (b, out["token"][b], out["accepted"][b])
    if wl.V <= 10 and wl.V ** wl.n <= 4096 and int(out["status"][b]) == 0 and ("rows" not in out or b in out["rows"]):
        sol = _gpu_policy_as_solution(wl, out, b)
        sup = G.topk_support(wl.q[b], wl.k)
        qq = np.zeros(wl.V); qq[sup] = wl.q[b][sup].astype(np.float64); qq /= qq.sum()
        if all(int(t) in sol.pos_of for t in sup):
            marg, acc, norm = brute.coupling_marginals(lambda t: G.policy_slice(sol, wl.p[b], t), qq, wl.n)
            p64 = wl.p[b].astype(np.float64); p64 /= p64.sum()
            slack = ABS_TOL + 15.0 * tol
            assert norm < 1e-9 and np.abs(marg - p64).max() < slack, (b, "marginal of the GPU's coupling", np.abs(marg - p64).max())
            assert abs(acc - alpha_star) < slack, (b, acc, alpha_star)


def compare_rows(wl, out, rows, tol, max_iter=4000, max_T=0, drafts=None, max_edge_frac=0.05, tail_mass=0.0):
    """Element-by-element comparison with the CPU checker on `rows`.  Rows the checker flags as fragile
    (several optimal H* within rounding) are compared on alpha* and on everything that holds for any
    correct result (check_row_validity).  Returns statistics; at most max_edge_frac of the rows (and
    never more than two when fewer than 40 rows are compared) may have their uniform within EDGE_TOL
    of a CDF edge."""
    from oracle import gr_oracle as G
    drafts = wl.drafts if drafts is None else drafts
    max_T = max_T or 128                      # the library's GR_MAX_T applies when no cap is given
    stats = {"rows": 0, "fragile": 0, "edge": 0, "max_dacc": 0.0, "max_dpi": 0.0, "inner_programs": 0, "outer_programs": 0,
             "solved_rows": 0}
    for b in rows:
        sol = G.solve_row(wl.p[b], wl.q[b], wl.n, wl.k, tol=tol, max_T=max_T, max_iter=max_iter, tail_mass=tail_mass)
        if tail_mass > 0 and sol.status != G.STATUS_BAD_ROW and not all(int(t) in sol.pos_of for t in drafts[b]):
            stats["skipped"] = stats.get("skipped", 0) + 1      # a draft from the cut tail: not a draw of the cut draft
            continue
        tok, accepted, pi, acc_given, edge = G.verify_row(sol, wl.p[b], drafts[b], wl.uniforms[b])
        stats["rows"] += 1
        assert abs(out["accept_prob"][b] - sol.alpha_star) < ABS_TOL, (b, out["accept_prob"][b], sol.alpha_star)
        in_support = all(int(t) in sol.pos_of for t in drafts[b]) if sol.status != G.STATUS_BAD_ROW else False
        if sol.fragile:                       # several optimal H*: compare what is unique, check that the rest is valid
            stats["fragile"] += 1
            if in_support and out["status"][b] != 3:
                check_row_validity(wl, out, b, drafts, sol.alpha_star, tol)
            continue
        assert out["status"][b] == sol.status, (b, out["status"][b], sol.status)
        kk = len(sol.order)
        assert out["support"][b] == kk and out["h_size"][b] == sol.h, (b, out["support"][b], kk, out["h_size"][b], sol.h)
        g_order, g_block, g_rho = (out["rows"][b]["order"], out["rows"][b]["block"], out["rows"][b]["rho"]) if "rows" in out \
            else (out["order"][b, :kk], out["block"][b, :kk], out["rho"][b, :kk])
        assert np.array_equal(g_order, sol.order), (b, "ratio order differs")
        assert np.array_equal(g_block, sol.block_of), (b, "block split differs")
        assert np.abs(g_rho - sol.rho).max() < 1e-12, (b, "residuals differ")
        if sol.status == G.STATUS_OK:
            stats["solved_rows"] += 1
            stats["inner_programs"] += sum(1 for blk in sol.blocks if blk.slack and blk.iters > 0)
            stats["outer_programs"] += sum(1 for blk in sol.blocks if not blk.slack and len(blk.active) >= 2)
        if "pi" in out:
            dpi = float(np.abs(out["pi"][b] - pi).max())
            stats["max_dpi"] = max(stats["max_dpi"], dpi)
            assert dpi < ABS_TOL, (b, dpi)
            assert np.all(out["pi"][b] >= 0.0), (b, "negative policy entry")
            assert abs(out["accept_given"][b] - acc_given) < ABS_TOL, (b, out["accept_given"][b], acc_given)
        stats["max_dacc"] = max(stats["max_dacc"], abs(float(out["accept_prob"][b]) - sol.alpha_star))
        if edge < EDGE_TOL:
            stats["edge"] += 1
        else:
            assert out["token"][b] == tok and bool(out["accepted"][b]) == accepted, \
                (b, out["token"][b], tok, out["accepted"][b], accepted, edge)
    assert stats["edge"] <= max(2, int(max_edge_frac * stats["rows"])), stats
    return stats


def rows_with_outer_programs(wl, candidates, tol, want=2):
    """Rows among `candidates` whose outer system has a block of two or more tokens of T with positive
    target (found with the checker's steps 1-2 only, no convex solve): the outer program Phi_T runs there."""
    from oracle import gr_oracle as G
    found = []
    for b in candidates:
        sol = G.solve_row(wl.p[b], wl.q[b], wl.n, wl.k, tol=tol, max_T=1)      # the cap stops before any solve
        if sol.fragile:
            continue
        if any(blk.slack == 0 and len(blk.active) >= 2 for blk in sol.blocks):
            found.append(int(b))
            if len(found) >= want:
                break
    return found


def check_alpha_all_rows(wl, out, rows=None, tail_mass=0.0):
    """alpha* needs no convex solve (Sec. 6, step 1): cheap enough to check on every row."""
    from oracle import gr_oracle as G
    for b in (range(wl.B) if rows is None else rows):
        sup = G.topk_support(wl.q[b], wl.k, tail_mass)
        order = G.ratio_order(wl.p[b], wl.q[b], sup)
        pt = float(np.sum(wl.p[b], dtype=np.float64))
        _, _, F = G.prefix_psi(wl.p[b][order].astype(np.float64) / pt, wl.q[b][order], wl.n)
        assert abs(out["accept_prob"][b] - (1.0 + F.min())) < ABS_TOL, (b, out["accept_prob"][b], 1.0 + F.min())
