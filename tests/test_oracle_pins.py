"""Pins for the CPU checker: brute force, closed forms and invariants fixed by the paper.

None of these re-types a formula of oracle/gr_oracle.py: the expected values come from
explicit LPs (Eq. opt-lp, Eq. relaxed-lp), from enumeration of all subsets (Thm 3.1) or
all draft tuples (Eq. cases), from the outer-residual LP (Thm 6.1) and from the classic
single-draft rule (App. A) that n = 1 must reduce to."""
import itertools
import math

import numpy as np
import pytest

from oracle import brute
from oracle import gr_oracle as G
from paper_2511_15898_amd import workloads as W


def _norm64(x):
    x = np.asarray(x, np.float64)
    return x / x.sum()


def _random_rows(seed, count, V, alphas=(0.2, 0.5, 1.0, 3.0), mix=True):
    rng = np.random.default_rng(seed)
    for t in range(count):
        a = rng.choice(alphas)
        p = rng.dirichlet(np.full(V, a)).astype(np.float32)
        q = rng.dirichlet(np.full(V, a)).astype(np.float32)
        if mix and t % 3 == 0:
            q = (0.7 * p + 0.3 * q).astype(np.float32)
        p = np.maximum(p, np.float32(1e-20)); q = np.maximum(q, np.float32(1e-20))
        yield (p / p.sum()).astype(np.float32), (q / q.sum()).astype(np.float32)


# ------------------------------------------------------------------ alpha*, H*
def test_alpha_star_equals_lp_optimum_on_tiny():
    """Thm 3.1: alpha* = optimum of the OTLP = optimum of the relaxed OTLP, V=8, n=2."""
    wl = W.tiny(B=16)
    for b in range(wl.B):
        sol = G.solve_row(wl.p[b], wl.q[b], 2, 0, tol=0.0)
        pp, qq = _norm64(wl.p[b]), _norm64(wl.q[b])
        assert abs(sol.alpha_star - brute.relaxed_otlp_value(pp, qq, 2)) < 1e-7
        if b < 4:
            assert abs(sol.alpha_star - brute.otlp_value(pp, qq, 2)) < 1e-6


def test_alpha_star_and_hstar_equal_subset_enumeration():
    """Thm 3.1 over all 2^V subsets; Sec. 5.1: a prefix of the ratio order attains it."""
    for n in (2, 3, 5):
        wl = W.tiny(B=60, n=n, seed_sub=n)
        for b in range(wl.B):
            sol = G.solve_row(wl.p[b], wl.q[b], n, 0, tol=0.0)
            val, H = brute.psi_min_all_subsets(_norm64(wl.p[b]), _norm64(wl.q[b]), n)
            assert abs(sol.alpha_star - (1.0 + val)) < 1e-12
            if not sol.fragile:
                assert sorted(int(t) for t in sol.order[: sol.h]) == sorted(H)


def test_n1_reduces_to_single_draft_speculative_sampling():
    """n = 1: alpha* = sum_i min(p_i, q_i); a drafted token i is kept with probability
    min(1, p_i/q_i) and otherwise replaced by a draw from (p - q)_+ normalised (App. A)."""
    for p, q in _random_rows(7, 30, 9):
        sol = G.solve_row(p, q, 1, 0, tol=0.0)
        pp, qq = _norm64(p), _norm64(q)
        assert abs(sol.alpha_star - np.minimum(pp, qq).sum()) < 1e-12
        resid = np.maximum(pp - qq, 0.0)
        for i in range(9):
            pi, acc = G.policy_slice(sol, p, (i,))
            keep = min(1.0, pp[i] / qq[i])
            assert abs(acc - keep) < 1e-9
            expect = (1.0 - keep) * resid / resid.sum() if keep < 1.0 else np.zeros(9)
            expect[i] += keep
            assert np.abs(pi - expect).max() < 1e-9


def test_acceptance_nondecreasing_in_n_and_one_when_p_equals_q():
    wl = W.small(B=8)
    for b in range(wl.B):
        prev = -1.0
        for n in (1, 2, 3, 4, 8, 16):
            sol = G.solve_row(wl.p[b], wl.q[b], n, 32, tol=1e-2, max_T=1)  # alpha* needs no solve
            assert sol.alpha_star >= prev - 1e-15
            prev = sol.alpha_star
    for p, _ in _random_rows(3, 5, 12):
        sol = G.solve_row(p, p, 3, 0, tol=0.0)
        assert abs(sol.alpha_star - 1.0) < 1e-12


# ------------------------------------------------------------------ outer residuals
def test_outer_targets_satisfy_outer_residual_lp():
    """Thm 6.1 by brute force over every S outside H*, and sum of residuals = 1 - alpha*."""
    for n in (2, 3):
        for p, q in _random_rows(11 + n, 40, 7):
            sol = G.solve_row(p, q, n, 0, tol=0.0, max_T=1)
            pp, qq = _norm64(p), _norm64(q)
            H = [int(t) for t in sol.order[: sol.h]]
            p_out = {int(t): sol.target[m] for m, t in enumerate(sol.order) if m >= sol.h}
            assert brute.outer_residual_violation(pp, qq, n, H, p_out) < 1e-7
            assert abs(sol.rho.sum() - (1.0 - sol.alpha_star)) < 1e-12
            assert np.all(sol.rho >= 0) and np.all(sol.target >= -1e-15)


# ------------------------------------------------------------------ evaluators
@pytest.mark.parametrize("slack", [0, 1])
def test_three_evaluators_agree(slack):
    """Definition by tuple enumeration == the paper's inclusion-exclusion grouping (App.
    "Truncated Solver Details") == the generating-function quadrature."""
    rng = np.random.default_rng(5 + slack)
    for _ in range(25):
        n = int(rng.integers(1, 5)); m = int(rng.integers(1, 6))
        mass = rng.dirichlet(np.ones(m + 1)) * rng.uniform(0.3, 1.0)
        ctx, q = float(mass[0]) * float(rng.integers(0, 2)), mass[1:]
        w = np.exp(rng.normal(0, 3, size=m))
        Re, R0e = G.routed_enum(n, ctx, slack, q, w)
        Rg, R0g = G.routed_grouped(n, ctx, slack, q, w)
        Rq, R0q = G.routed_quadrature(n, ctx, slack, q, w)
        assert np.abs(Re - Rg).max() < 1e-12 and abs(R0e - R0g) < 1e-12
        assert np.abs(Rq / Re - 1).max() < 1e-10
        if slack:
            assert abs(R0q / R0e - 1) < 1e-10
        total = (ctx + q.sum()) ** n - (0.0 if slack else ctx ** n)   # columns are exactly normalised
        assert abs(Re.sum() + R0e - total) < 1e-12


def test_quadrature_has_converged_in_its_step():
    rng = np.random.default_rng(9)
    q = rng.dirichlet(np.ones(40) * 0.3) * 0.9; w = np.exp(rng.normal(2, 4, size=40))
    for slack in (0, 1):
        a, a0 = G.routed_quadrature(8, 0.05, slack, q, w)
        b, b0 = G.routed_quadrature(8, 0.05, slack, q, w, step=0.1)
        assert np.abs(a / b - 1).max() < 1e-11 and abs(a0 - b0) <= 1e-11 * max(b0, 1e-300)
        assert abs(a.sum() + a0 - ((0.05 + q.sum()) ** 8 - (0 if slack else 0.05 ** 8))) < 1e-11


def test_quadrature_matches_grouping_at_moderate_size():
    rng = np.random.default_rng(10)
    q = rng.dirichlet(np.ones(12)) * 0.8; w = np.exp(rng.normal(0, 2, size=12))
    for slack in (0, 1):
        Rg, R0g = G.routed_grouped(3, 0.1, slack, q, w)
        Rq, R0q = G.routed_quadrature(3, 0.1, slack, q, w)
        assert np.abs(Rq / Rg - 1).max() < 1e-10 and abs(R0q - R0g) < 1e-12


# ------------------------------------------------------------------ the coupling itself
def _check_coupling(p, q, n, k, tol, marg_tol, acc_tol):
    sol = G.solve_row(p, q, n, k, tol=tol)
    assert sol.status == G.STATUS_OK
    qq = np.zeros(len(q)); sup = G.topk_support(q, k); qq[sup] = _norm64(q[sup])
    marg, acc, norm = brute.coupling_marginals(lambda t: G.policy_slice(sol, p, t), qq, n)
    assert norm < 1e-12                                  # every slice is a distribution
    assert np.abs(marg - _norm64(p)).sum() < marg_tol    # output marginal equals p
    assert abs(acc - sol.alpha_star) < acc_tol           # and the acceptance is the optimum
    return sol


def test_marginal_equals_p_and_acceptance_is_optimal_tiny():
    wl = W.tiny(B=40)
    for b in range(wl.B):
        _check_coupling(wl.p[b], wl.q[b], 2, 0, 0.0, 1e-6, 1e-9)


def test_marginal_with_nontrivial_outer_blocks_and_n3():
    seen_block = 0
    for i, (p, q) in enumerate(_random_rows(1, 120, 7)):
        n = 2 + i % 2
        sol = _check_coupling(p, q, n, 0, 0.0, 1e-6, 1e-9)
        seen_block += any(b.slack == 0 and b.hi - b.lo >= 2 for b in sol.blocks)
    assert seen_block >= 10          # the block rule was exercised


def test_truncated_runs_respect_the_papers_bounds():
    """Lemma 6.6 / Sec. 6.3: at most 15*tol L1 from p and 10*tol from alpha*."""
    for tol in (1e-2, 1e-3):
        hit = 0
        for i, (p, q) in enumerate(_random_rows(21, 60, 8, alphas=(0.1, 0.2))):
            n = 2 + i % 2
            full = G.solve_row(p, q, n, 0, tol=0.0)
            sol = _check_coupling(p, q, n, 0, tol, 15 * tol, 10 * tol)
            hit += sum(len(b.active) for b in sol.blocks) < sum(len(b.active) for b in full.blocks)
        assert hit >= 5               # truncation really dropped variables


def test_topk_is_the_full_problem_with_the_restricted_draft():
    """App. "Top-k Sampling ...": solving on V_0 with p sliced is the relaxed OTLP over
    all of V with the top-k renormalised draft.  The LP is built over the full V."""
    for i, (p, q) in enumerate(_random_rows(31, 12, 7, mix=False)):
        k = 3 + i % 3
        qq = np.zeros(7); sup = G.topk_support(q, k); qq[sup] = _norm64(q[sup])
        assert len(sup) == k
        sol = _check_coupling(p, q, 2, k, 0.0, 1e-6, 1e-9)
        assert abs(sol.alpha_star - brute.relaxed_otlp_value(_norm64(p), qq, 2)) < 1e-7
        assert sorted(int(t) for t in sol.order) == [int(t) for t in sup]


# ------------------------------------------------------------------ sampling and statuses
def test_inverse_cdf_reproduces_the_slice():
    rng = np.random.default_rng(2)
    pi = rng.dirichlet(np.ones(12) * 0.4); pi[3] = 0.0; pi /= pi.sum()
    drafts = (7, 2, 7, 9)
    N = 20000
    hist = np.zeros(12); acc = 0
    for j in range(N):
        tok, ok, _ = G.sample_token(pi, drafts, (j + 0.5) / N)
        hist[tok] += 1; acc += ok
    assert np.abs(hist / N - pi).max() <= 1.0 / N + 1e-12
    assert abs(acc / N - pi[[7, 2, 9]].sum()) <= 2.0 / N


def test_status_codes_and_fallback():
    wl = W.small(B=2)
    sol = G.solve_row(wl.p[0], wl.q[0], 4, 32, tol=1e-6, max_T=4)
    assert sol.status == G.STATUS_TRUNC_CAP
    pi, acc = G.policy_slice(sol, wl.p[0], wl.drafts[0])
    assert np.abs(pi - _norm64(wl.p[0])).max() < 1e-15       # valid fallback transport: sample from p
    sol = G.solve_row(wl.p[0], wl.q[0], 4, 32, tol=1e-6, max_iter=2)
    assert sol.status == G.STATUS_ITER_CAP
    bad = wl.p[1].copy(); bad[5] = np.nan
    assert G.solve_row(bad, wl.q[1], 4, 32).status == G.STATUS_BAD_ROW
    assert G.solve_row(wl.p[1] * np.float32(0.5), wl.q[1], 4, 32).status == G.STATUS_BAD_ROW


def test_zero_probability_tokens():
    p = np.array([0.5, 0.0, 0.25, 0.25, 0.0, 0.0], np.float32)
    q = np.array([0.2, 0.3, 0.0, 0.4, 0.1, 0.0], np.float32)
    sol = _check_coupling(p, q, 2, 0, 0.0, 1e-9, 1e-9)
    assert [int(t) for t in sol.order[:2]] == [1, 4]          # p = 0, q > 0 rank first
    assert 2 not in sol.pos_of and 5 not in sol.pos_of        # q = 0 is never drafted


def test_acceptance_sweep_against_subset_enumeration_and_closed_forms():
    """acceptance_sweep over (k, n): every cell equals 1 + min over ALL subsets of psi for the
    top-k restricted draft (Thm 3.1 by enumeration); n = 1 is sum_i min(p_i, q'_i) (single-draft
    rule, App. A); rows are nondecreasing in n; k >= V is the problem without top-k."""
    ks, ns = [1, 2, 3, 5, 8], [1, 2, 3, 5]
    for p, q in _random_rows(77, 12, 8):
        got = G.acceptance_sweep(p, q, ks, ns)
        p64 = _norm64(p)
        for a, k in enumerate(ks):
            qk = np.zeros(8)
            keep = sorted(range(8), key=lambda i: (-float(q[i]), i))[:k]
            qk[keep] = np.asarray(q, np.float64)[keep]
            qk = qk / qk.sum()
            for b, n in enumerate(ns):
                value, _ = brute.psi_min_all_subsets(p64, qk, n)
                assert abs(got[a, b] - (1.0 + value)) < 1e-12, (k, n)
            assert abs(got[a, 0] - np.minimum(p64, qk).sum()) < 1e-12
            assert np.all(np.diff(got[a]) >= -1e-15)
        assert np.array_equal(got[-1], G.acceptance_sweep(p, q, [0], ns)[0])


# ------------------------------------------------------------------ the quadrature evaluator beyond four drafts
@pytest.mark.parametrize("n", [5, 8, 12, 16])
@pytest.mark.parametrize("slack", [0, 1])
def test_quadrature_matches_the_papers_grouping_for_many_drafts(n, slack):
    """Per-token routed masses of the generating-function quadrature against the paper's own evaluator
    (App. "Truncated Solver Details": one term per set of at most n distinct tokens with its
    inclusion-exclusion coefficient), at the draft counts of the large configurations.  The grouping is
    exponential in the number of tokens only, so small programs reach n = 16."""
    rng = np.random.default_rng(1000 * n + slack)
    for m in (2, 4, 6):
        for with_ctx in (0, 1):
            for _ in range(3):
                mass = rng.dirichlet(np.ones(m + 1)) * rng.uniform(0.4, 1.0)
                ctx, q = float(mass[0]) * with_ctx, mass[1:]
                w = np.exp(rng.normal(0, 2.5, size=m))
                Rg, R0g = G.routed_grouped(n, ctx, slack, q, w)
                Rq, R0q = G.routed_quadrature(n, ctx, slack, q, w)
                assert np.abs(Rq - Rg).max() <= 1e-10 * Rg.max() + 1e-15, (n, m, with_ctx)
                assert np.abs(Rq / Rg - 1).max() < 1e-8, (n, m, with_ctx)      # also token by token
                assert abs(R0q - R0g) <= 1e-10 * max(R0g, 1e-3)
                total = (ctx + q.sum()) ** n - (0.0 if slack else ctx ** n)   # every tuple's mass is handed out
                assert abs(Rq.sum() + R0q - total) < 1e-11


def test_whole_chain_on_the_quadrature_alone(monkeypatch):
    """solve -> slice -> marginal by tuple enumeration with the quadrature as the ONLY evaluator (the
    dispatch to tuple enumeration is switched off): the output marginal equals p within 1e-6 and the
    acceptance is the optimum (Thm 3.1, Eq. (cases)).  This is the evaluator that every program of the
    larger configurations runs on."""
    calls = {"n": 0}
    real = G.routed_quadrature

    def only_quadrature(n, ctx, slack, q, w):
        calls["n"] += 1
        return real(n, ctx, slack, q, w)

    monkeypatch.setattr(G, "routed", only_quadrature)
    # solve_scaling binds its default evaluator at definition time: pass the replacement explicitly
    real_scaling = G.solve_scaling
    monkeypatch.setattr(G, "solve_scaling", lambda *a, **kw: real_scaling(*a, **{**kw, "evaluator": only_quadrature}))
    blocks = 0
    for i, (p, q) in enumerate(_random_rows(41, 24, 7)):
        sol = _check_coupling(p, q, 2 + i % 2, 0, 0.0, 1e-6, 1e-9)
        blocks += any(b.slack == 0 and b.hi - b.lo >= 2 for b in sol.blocks)
    assert calls["n"] > 100 and blocks >= 2


def test_whole_chain_where_the_dispatch_itself_picks_the_quadrature():
    """The same chain at sizes where routed() leaves tuple enumeration by itself ((m + 1)^n > 4096 for
    a program of m tokens) and enumerating every draft tuple for the marginal is still feasible."""
    seen = 0
    real = G.routed_quadrature
    counter = {"n": 0}

    def counting(*a, **kw):
        counter["n"] += 1
        return real(*a, **kw)

    G.routed_quadrature = counting
    try:
        rows = list(_random_rows(52, 6, 18, alphas=(1.0, 3.0))) + list(_random_rows(53, 4, 12, alphas=(1.0, 3.0)))
        for i, (p, q) in enumerate(rows):
            n = 3 if len(p) == 18 else 4
            before = counter["n"]
            _check_coupling(p, q, n, 0, 0.0, 1e-6, 1e-8)
            seen += counter["n"] > before
    finally:
        G.routed_quadrature = real
    assert seen >= 3, seen


# ------------------------------------------------------------------ truncation: what stays fixed outside T
def _draw_probability_by_enumeration(q_sys, ctx, j, n):
    """Pr[token j is among n i.i.d. draws from {context, tokens of the system}], all tuples written out."""
    probs = [ctx] + [float(x) for x in q_sys]
    tot = 0.0
    for tup in itertools.product(range(len(probs)), repeat=n):
        if (j + 1) in tup:
            mass = 1.0
            for a in tup:
                mass *= probs[a]
            tot += mass
    return tot


def test_truncated_slices_are_distributions_and_tokens_outside_T_keep_their_start_weight():
    """tol > 0.  (i) Every slice pi(.|omega) still sums to 1: the column sums of Eq. (approx-c) are exact
    whatever the weights (App. "Approximation Guarantee").  (ii) Thm 6.4 / 6.5: the objectives do not
    depend on alpha_i outside T, and every choice satisfies their bounds; this build's choice is
    w_i = target_i / Pr[i drawn within its own system] (inner ones in the slack's gauge,
    Q(H*)^n / (1 - alpha*)), with the draw probability taken here from the enumeration of all tuples of
    the system.  (iii) The deviations of Thm 6.4 / 6.5 themselves, with the actual epsilon_T / gamma_T of
    the sets chosen: total L1 deviation of the outer (inner) equality constraints at most 4 epsilon_T
    (4 gamma_T) at a point whose own gradient is within the shortfall."""
    checked_out = checked_in = 0
    for tol in (1e-2, 3e-3):
        for i, (p, q) in enumerate(_random_rows(61, 50, 8, alphas=(0.1, 0.2))):
            n = 2 + i % 2
            sol = G.solve_row(p, q, n, 0, tol=tol)
            assert sol.status == G.STATUS_OK
            qq = _norm64(q)
            marg, acc, norm = brute.coupling_marginals(lambda t: G.policy_slice(sol, p, t), qq, n)
            assert norm < 1e-12
            kk, h = len(sol.order), sol.h
            q_s = sol.q_s
            for blk in sol.blocks:
                T = set(blk.active)
                ctx_true = float(q_s[: blk.lo].sum())
                sys_tokens = list(range(blk.lo, blk.hi))
                for m in sys_tokens:
                    if m in T or not sol.target[m] > 0:
                        continue
                    if blk.slack == 0 and blk.hi - blk.lo < 2:
                        continue
                    pr = _draw_probability_by_enumeration(q_s[blk.lo:blk.hi], ctx_true, m - blk.lo, n)
                    gauge = (float(q_s[:h].sum()) ** n) / (1.0 - sol.alpha_star) if blk.slack else 1.0
                    expect = gauge * sol.target[m] / pr
                    assert abs(sol.w[m] / expect - 1.0) < 1e-9, (tol, i, m)
                    checked_in += blk.slack; checked_out += 1 - blk.slack
            # (iii) deviations of the two systems against the actual tunable errors of the sets chosen
            pp = _norm64(p)
            # gamma_T / epsilon_T of the minimal sets: the tokens the walk by decreasing q takes
            order_in = sorted(range(h), key=lambda m: (-q_s[m], sol.order[m]))
            Qh = float(q_s[:h].sum()); accq = 0.0; gamma_T = Qh ** n
            for m in order_in:
                if Qh ** n - accq ** n <= float(np.float32(tol)):
                    break
                accq += q_s[m]
            gamma_T = Qh ** n - accq ** n
            order_out = sorted(range(h, kk), key=lambda m: (-q_s[m], sol.order[m]))
            accq = Qh
            for m in order_out:
                if 1.0 - accq ** n <= float(np.float32(tol)):
                    break
                accq += q_s[m]
            eps_T = 1.0 - accq ** n
            dev_in = sum(abs(marg[int(sol.order[m])] - pp[int(sol.order[m])]) for m in range(h))
            # the marginal of a token outside H* also receives the residual lift: its outer-system share is p_i
            dev_total = float(np.abs(marg - pp).sum())
            assert dev_in <= 4.0 * gamma_T + 1e-9, (tol, i, dev_in, gamma_T)
            assert dev_total <= 4.0 * eps_T + 3.0 * (4.0 * gamma_T) + 1e-9, (tol, i, dev_total, eps_T, gamma_T)
    assert checked_in >= 5 and checked_out >= 1, (checked_in, checked_out)


# ------------------------------------------------------------------ the flag for rows with several optimal H*
def test_fragile_flag_covers_every_row_whose_discrete_structure_moves_under_rounding_noise():
    """Sec. 5.1 leaves the choice among several minimising prefixes open (psi(empty) = psi(V) = 0 whenever
    alpha* = 1), and the block split rests on comparisons F(m) <= G(m+1).  A row is flagged `fragile` when
    such a decision sits within 1e-13 of a tie.  Pin: on rows that are NOT flagged, perturbing F by up to
    4e-14 per entry (rounding noise of another summation order) changes neither |H*| nor the block split;
    rows with an exact tie by construction (p = q) are flagged."""
    rng = np.random.default_rng(71)
    flagged = moved_flagged = 0
    rows = list(_random_rows(72, 150, 8)) + [(p, p.copy()) for p, _ in _random_rows(73, 10, 8)]
    # near-identical rows: draft = target with tiny noise, the case that produces near ties in practice
    for p, _ in _random_rows(74, 60, 10):
        q = (p * np.exp(rng.normal(0, 1e-7, size=p.shape))).astype(np.float32)
        rows.append((p, (q / q.sum()).astype(np.float32)))
    for idx, (p, q) in enumerate(rows):
        for n in (2, 3):
            sol = G.solve_row(p, q, n, 0, tol=0.0, max_T=1)
            base_blocks = G.split_blocks(sol.F, sol.G, sol.h)
            moved = False
            for _ in range(20):
                F2 = sol.F + rng.uniform(-4e-14, 4e-14, size=sol.F.shape)
                F2[0] = 0.0
                h2 = int(np.argmin(F2))
                G2, _ = G.outer_targets(F2, h2)
                if h2 != sol.h or G.split_blocks(F2, G2, h2) != base_blocks:
                    moved = True
            if sol.fragile:
                flagged += 1; moved_flagged += moved
            else:
                assert not moved, (idx, n, "an unflagged row changed its H* or its blocks under 4e-14 noise")
            if np.array_equal(p, q):
                assert sol.fragile and abs(sol.alpha_star - 1.0) < 1e-12
    assert flagged >= 10 and moved_flagged >= 5, (flagged, moved_flagged)


# ------------------------------------------------------------------ rows given as logits
def test_logits_front_end_against_closed_forms_and_invariances():
    """App. A: temperature only changes how p, q come from the logits.  Two tokens: p_1 = 1 / (1 + e^{(b - a)/T})
    (the logistic function) and alpha* = 1 + min(0, p_1 - q_1^n, p_2 - q_2^n), the minimum of psi over the four
    subsets written out (Thm 3.1).  Any V: a shift of the logits changes nothing, logits and temperature scaled
    together change nothing, equal logits give alpha* = 1, and the result equals that of the softmaxed rows."""
    rng = np.random.default_rng(81)
    for _ in range(40):
        a, b, c, d = rng.normal(0, 2, size=4)
        T = float(rng.uniform(0.3, 2.0)); n = int(rng.integers(1, 6))
        sol, p, q = G.solve_row_from_logits([a, b], [c, d], T, n, tol=0.0)
        p1 = 1.0 / (1.0 + math.exp((b - a) / T)); q1 = 1.0 / (1.0 + math.exp((d - c) / T))
        assert abs(p[0] - p1) < 1e-14 and abs(q[0] - q1) < 1e-14
        expect = 1.0 + min(0.0, p1 - q1 ** n, (1.0 - p1) - (1.0 - q1) ** n)
        assert abs(sol.alpha_star - expect) < 1e-12, (a, b, c, d, T, n)
    for _ in range(10):
        V = int(rng.integers(5, 40)); n = int(rng.integers(2, 5)); k = int(rng.integers(2, V))
        tl = 3.0 * rng.standard_normal(V); dl = 0.8 * tl + rng.standard_normal(V); T = float(rng.uniform(0.5, 1.5))
        base, p, q = G.solve_row_from_logits(tl, dl, T, n, k, tol=1e-9)
        shifted, _, _ = G.solve_row_from_logits(tl + 7.25, dl - 3.5, T, n, k, tol=1e-9)
        scaled, _, _ = G.solve_row_from_logits(2.0 * tl, 2.0 * dl, 2.0 * T, n, k, tol=1e-9)
        direct = G.solve_row(p, q, n, k, tol=1e-9)
        for other in (shifted, scaled, direct):
            assert abs(other.alpha_star - base.alpha_star) < 1e-12 and np.array_equal(other.order, base.order)
            assert np.abs(other.w - base.w).max() <= 1e-7 * max(1.0, np.abs(base.w).max())
        same, _, _ = G.solve_row_from_logits(tl, tl, T, n, 0, tol=0.0)
        assert abs(same.alpha_star - 1.0) < 1e-12
        assert sorted(int(t) for t in base.order) == sorted(int(t) for t in np.argsort(-dl, kind="stable")[:k])   # top-k of q = top-k of the draft logits


def test_orders_taken_on_the_logits_are_the_orders_of_the_softmaxed_rows():
    """Sec. 5.1 asks for decreasing q/p; behind two softmaxes at one temperature that is decreasing d - t.  The
    checker's order from logits is held against q/p = exp((d - t) / T) evaluated with 60 decimal digits (exact
    for this purpose), with ties -- equal logit differences, equal draft logits -- resolved to the lower id."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    rng = np.random.default_rng(53)
    for trial in range(8):
        V = int(rng.integers(12, 40)); T = float(rng.uniform(0.4, 1.6))
        tl = (3.0 * rng.standard_normal(V)).astype(np.float32); dl = (0.8 * tl + rng.standard_normal(V)).astype(np.float32)
        if trial % 2:                                   # planted ties: the same difference twice, the same draft logit twice
            tl[7] = tl[2] + np.float32(0.5); dl[7] = dl[2] + np.float32(0.5)
            if float(dl[7]) - float(tl[7]) != float(dl[2]) - float(tl[2]):
                dl[7] = dl[2]; tl[7] = tl[2]
            dl[9] = dl[4]
        sol, p, q = G.solve_row_from_logits(tl, dl, T, 3, 0, tol=0.0, max_T=1)
        ratio = [((Decimal(float(dl[i])) - Decimal(float(tl[i])) ) / Decimal(T)).exp() for i in range(V)]
        want = sorted(range(V), key=lambda i: (-ratio[i], i))
        assert [int(t) for t in sol.order] == want
        qd = [(Decimal(float(dl[i])) / Decimal(T)).exp() for i in range(V)]
        k = V // 2
        want_k = sorted(sorted(range(V), key=lambda i: (-qd[i], i))[:k])
        assert G.topk_support(q, k, key=dl.astype(np.float64)) == want_k
        # the draft at its own temperature: q/p = exp(d / Td - t / Tt)
        Td = float(rng.uniform(0.4, 1.6))
        sol2, p2, q2 = G.solve_row_from_logits(tl, dl, T, 3, 0, tol=0.0, max_T=1, draft_temperature=Td)
        ratio2 = [(Decimal(float(dl[i])) / Decimal(Td) - Decimal(float(tl[i])) / Decimal(T)).exp() for i in range(V)]
        assert [int(t) for t in sol2.order] == sorted(range(V), key=lambda i: (-ratio2[i], i))
        e = np.exp((dl.astype(np.float64) - float(dl.max())) / Td)
        assert np.abs(q2 - e / e.sum()).max() < 1e-15 and np.abs(p2 - p).max() == 0.0


# ------------------------------------------------------------------ nucleus cut of the draft
def test_nucleus_cut_is_the_smallest_prefix_by_mass_and_costs_at_most_n_tail_mass():
    """Sec. 5.1 / App. A: top-p sampling of the draft restricts the domain like top-k.  The cut support is
    checked against the definition in exact rational arithmetic (the fewest tokens by decreasing q, ties to
    the lower id, whose mass reaches 1 - tail_mass of the row); with tail_mass = 0 nothing changes; the
    cut draft is the relaxed OTLP of the renormalised nucleus (LP over the full V); and against the uncut
    draft alpha* moves by at most n * tail_mass (n draws avoid the dropped tokens with at least that
    probability); drafts are then drawn from the cut, renormalised draft, under which the marginal is p."""
    from fractions import Fraction
    checked = cut_rows = 0
    for i, (p, q) in enumerate(_random_rows(77, 40, 7, alphas=(0.05, 0.1, 0.3), mix=False)):
        n = 2 + i % 2
        assert G.topk_support(q, 0, 0.0) == G.topk_support(q, 0)
        for delta in (1e-3, 3e-2, 0.2):
            sup = G.topk_support(q, 0, delta)
            ranked = sorted((j for j in range(7) if q[j] > 0), key=lambda j: (-Fraction(float(q[j])), j))
            total = sum(Fraction(float(x)) for x in q)
            need = (1 - Fraction(delta)) * total
            run, want = Fraction(0), []
            for j in ranked:
                want.append(j); run += Fraction(float(q[j]))
                if run >= need:
                    break
            # float64 running sums against exact ones: only a mass within rounding of the threshold could differ
            margin = min(abs(sum(Fraction(float(q[j])) for j in ranked[:c]) - need) for c in range(1, len(ranked) + 1))
            if margin > Fraction(1, 10 ** 12):
                assert sup == sorted(want), (i, delta)
                checked += 1
            cut_rows += len(sup) < len(ranked)
            full = G.solve_row(p, q, n, 0, tol=0.0)
            sol = G.solve_row(p, q, n, 0, tol=0.0, tail_mass=delta)
            assert sol.status == G.STATUS_OK and sorted(int(t) for t in sol.order) == sup
            dropped = float(sum(Fraction(float(q[j])) for j in range(7) if j not in sup) / total)
            assert dropped <= delta + 1e-12
            assert abs(sol.alpha_star - full.alpha_star) <= n * dropped + 1e-9, (i, delta, sol.alpha_star, full.alpha_star)
            qq = np.zeros(7); qq[sup] = _norm64(q[sup])
            assert abs(sol.alpha_star - brute.relaxed_otlp_value(_norm64(p), qq, n)) < 1e-7
            marg, acc, norm = brute.coupling_marginals(lambda t: G.policy_slice(sol, p, t), qq, n)
            assert norm < 1e-12 and np.abs(marg - _norm64(p)).sum() < 1e-6 and abs(acc - sol.alpha_star) < 1e-9
    assert checked >= 100 and cut_rows >= 40          # the cut really dropped tokens


# ------------------------------------------------------------------ multi-step walk over a draft tree
def test_tree_walk_emits_tokens_distributed_as_the_target_model():
    """App. "Multi-Step Experiments": K i.i.d. draft paths, n = the paths through the current node.  On a
    vocabulary of three tokens every draft tree (3^(K L) of them) and every outcome is enumerated with the exact
    slices in place of the uniform draws: the first token must have the root's target distribution, and given
    that it was accepted the second must have the target distribution of its prefix -- which fails if the walk
    kept the wrong paths, counted drafts wrongly or conditioned on the wrong rows.  Then the sampler itself:
    with uniforms it must pick, level by level, what the inverse CDF of those slices picks."""
    from oracle import tree_walk as TW
    rng = np.random.default_rng(404)
    V, K, L = 3, 2, 2
    rows = {}

    def node(prefix):
        if prefix not in rows:
            r = np.random.default_rng([7, len(prefix)] + list(prefix))
            rows[prefix] = (_norm64(r.dirichlet(np.ones(V)) + 0.05).astype(np.float32), _norm64(r.dirichlet(np.ones(V)) + 0.05).astype(np.float32))
        return rows[prefix]

    first = np.zeros(V); second = {x: np.zeros(V) for x in range(V)}; reach = {x: 0.0 for x in range(V)}
    for toks in itertools.product(range(V), repeat=K * L):
        paths = [toks[a * L:(a + 1) * L] for a in range(K)]
        mass = 1.0
        for a in range(K):
            for l in range(L):
                q = node(tuple(paths[a][:l]))[1].astype(np.float64)
                mass *= q[paths[a][l]] / q.sum()
        p0, q0 = node(())
        sol0 = G.solve_row(p0, q0, K, 0, tol=0.0)
        pi0, _ = G.policy_slice(sol0, p0, [paths[a][0] for a in range(K)])
        first += mass * pi0
        for x in set(paths[a][0] for a in range(K)):            # accepted first tokens
            act = [a for a in range(K) if paths[a][0] == x]
            p1, q1 = node((x,))
            sol1 = G.solve_row(p1, q1, len(act), 0, tol=0.0)
            pi1, _ = G.policy_slice(sol1, p1, [paths[a][1] for a in act])
            second[x] += mass * pi0[x] * pi1; reach[x] += mass * pi0[x]
    assert np.abs(first - _norm64(node(())[0])).max() < 1e-9
    for x in range(V):
        assert reach[x] > 0 and np.abs(second[x] / reach[x] - _norm64(node((x,))[0])).max() < 1e-9, x
    for trial in range(200):
        paths = []
        for a in range(K):
            pre = []
            for l in range(L):
                q = node(tuple(pre))[1].astype(np.float64)
                pre.append(int(rng.choice(V, p=q / q.sum())))
            paths.append(pre)
        u = rng.random(L)
        p_nodes = [[node(tuple(paths[a][:l]))[0] for l in range(L)] for a in range(K)]
        q_nodes = [[node(tuple(paths[a][:l]))[1] for l in range(L)] for a in range(K)]
        out, nacc, fb, _ = TW.tree_walk(p_nodes, q_nodes, paths, u, 0, 0.0)
        act = list(range(K)); want = []; oks = 0
        for l in range(L):
            pr, qr = node(tuple(want))
            sol = G.solve_row(pr, qr, len(act), 0, tol=0.0)
            pi, _ = G.policy_slice(sol, pr, [paths[a][l] for a in act])
            tok, ok, _ = G.sample_token(pi, [paths[a][l] for a in act], float(u[l]))
            want.append(tok)
            if not ok:
                break
            oks += 1
            act = [a for a in act if paths[a][l] == tok]
        assert out == want and fb == 0 and nacc == oks


# ------------------------------------------------------------------ the convex programs against the paper's own minimiser
def test_solver_reaches_the_minimiser_that_l_bfgs_b_finds_on_the_objective_itself():
    """Thm 6.5 / Thm 6.4 define the weights as the minimiser of Theta_T / Phi_T.  The objective is written out here by
    tuple enumeration (sum over draft tuples of pdraft * log(slack + sum of e^alpha over the distinct block tokens
    drawn) minus target . alpha) and minimised with SciPy's L-BFGS-B, the paper's own choice, on numerical gradients:
    nothing of the checker's evaluators or of its iteration enters.  The checker's solve_scaling must land on the same
    point; so must a manufactured problem whose targets are the routed masses of known weights."""
    from scipy.optimize import minimize
    rng = np.random.default_rng(606)
    for trial in range(10):
        slack = trial % 2
        m = int(rng.integers(2, 6)); n = int(rng.integers(2, 4))
        q = rng.dirichlet(np.ones(m + 1))[:m] * rng.uniform(0.5, 0.95)
        ctx = float(rng.uniform(0.0, 1.0 - q.sum())) if trial % 3 else 0.0
        w_true = np.exp(rng.normal(0.0, 1.5, size=m))
        target, slack_target = G.routed_enum(n, ctx, slack, q, w_true)         # a problem with a known solution
        probs = [ctx] + [float(x) for x in q]
        tuples = []
        for tup in itertools.product(range(m + 1), repeat=n):
            mass = float(np.prod([probs[a] for a in tup]))
            members = sorted({a - 1 for a in tup if a > 0})
            if mass > 0.0 and (members or slack):
                tuples.append((mass, members))

        def objective(alpha):
            w = np.exp(alpha)
            return sum(mass * math.log(slack + sum(w[j] for j in members)) for mass, members in tuples) - float(target @ alpha)

        best = minimize(objective, np.zeros(m), method="L-BFGS-B", options={"ftol": 1e-15, "gtol": 1e-10, "maxiter": 2000})
        w_ref = np.exp(best.x)
        w, evals, err = G.solve_scaling(n, ctx, slack, q, target, slack_target, np.ones(m))
        assert err <= 1e-10
        if slack == 0:                                  # Phi_T is flat along a common factor: compare shares
            w_ref = w_ref / w_ref.sum(); w = w / w.sum(); want = w_true / w_true.sum()
        else:
            want = w_true
        assert np.abs(w / want - 1.0).max() < 1e-8, (trial, w, want)
        assert np.abs(w_ref / want - 1.0).max() < 2e-4, (trial, w_ref, want)      # the library minimiser, to its own accuracy


def test_a_target_that_nearly_exhausts_its_token_is_still_solved():
    """A row met by a randomised run: the last token of H* has a target of 92 % of its draw probability, so its
    weight is large (about 380) and a mixed fixed-point step can throw it so far out that the routed masses stop
    feeling it.  The minimiser is unique (Thm 6.5): the checker must find it, and the coupling it builds must have
    marginal p and the optimal acceptance (Sec. 3.1, Thm 3.1)."""
    p = np.array([0.00347583, 0.81121342, 0.09828163, 0.05606862, 0.0309605], np.float64)
    q = np.array([0.03470613, 0.89321866, 0.05135588, 0.02071933, 0.0], np.float64)
    p = (p / p.sum()).astype(np.float32); q = (q / q.sum()).astype(np.float32)
    sol = _check_coupling(p, q, 3, 0, 0.0, 1e-6, 1e-9)
    assert sol.h == 4 and sol.status == G.STATUS_OK
    w = {int(t): float(sol.w[m]) for m, t in enumerate(sol.order)}
    assert 300.0 < w[3] < 500.0 and 50.0 < w[2] < 80.0
