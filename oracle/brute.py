"""Brute-force definitions used to pin gr_oracle (test infrastructure only).

Everything here is exponential in V or n and only meant for V <= 10, n <= 3."""
from __future__ import annotations

import itertools

import numpy as np
from scipy.optimize import linprog


def psi(H, p, q, n):
    """psi(H) = sum_{i in H} p(i) - sum_{tuples in H^n} pdraft  (Thm 3.1), the tuple sum
    written out as a product of n marginal sums (App. C)."""
    H = list(H)
    return float(sum(p[i] for i in H)) - float(sum(q[i] for i in H)) ** n


def psi_min_all_subsets(p, q, n):
    """min over all 2^V subsets; returns (value, smallest minimising subset as a tuple)."""
    V = len(p)
    best, arg = 0.0, ()
    for r in range(V + 1):
        for H in itertools.combinations(range(V), r):
            v = psi(H, p, q, n)
            if v < best - 1e-15:
                best, arg = v, H
    return best, arg


def tuples_with_mass(q, n):
    V = len(q)
    for tup in itertools.product(range(V), repeat=n):
        mass = 1.0
        for a in tup:
            mass *= float(q[a])
        yield tup, mass


def relaxed_otlp_value(p, q, n):
    """Optimum of the relaxed OTLP (Eq. relaxed-lp) as an explicit LP: one variable per
    (token i, tuple) pair with i in the tuple, row sums <= p(i), column sums <= pdraft."""
    V = len(p)
    tuples = list(tuples_with_mass(q, n))
    cols = []
    for ti, (tup, _) in enumerate(tuples):
        for i in sorted(set(tup)):
            cols.append((i, ti))
    nv = len(cols)
    A = np.zeros((V + len(tuples), nv))
    b = np.concatenate([np.asarray(p, float), np.array([m for _, m in tuples])])
    for c, (i, ti) in enumerate(cols):
        A[i, c] = 1.0
        A[V + ti, c] = 1.0
    res = linprog(-np.ones(nv), A_ub=A, b_ub=b, bounds=(0, None), method="highs")
    assert res.status == 0, res.message
    return -float(res.fun)


def otlp_value(p, q, n):
    """Optimum of the OTLP itself (Eq. opt-lp), equality-constrained, V^(n+1) variables.
    One of the V + V^n equalities is redundant; the last one is dropped so that rounding
    in sum p vs. sum pdraft cannot make the solver report infeasibility."""
    V = len(p)
    tuples = list(tuples_with_mass(q, n))
    nt = len(tuples)
    nv = V * nt
    c = np.zeros(nv)
    A = np.zeros((V + nt, nv))
    b = np.concatenate([np.asarray(p, float) / float(np.sum(p)), np.array([m for _, m in tuples]) / sum(m for _, m in tuples)])
    for ti, (tup, _) in enumerate(tuples):
        for i in range(V):
            v = i * nt + ti
            A[i, v] = 1.0
            A[V + ti, v] = 1.0
            if i in tup:
                c[v] = -1.0
    res = linprog(c, A_eq=A[:-1], b_eq=b[:-1], bounds=(0, None), method="highs")
    assert res.status == 0, res.message
    return -float(res.fun)


def outer_residual_violation(p, q, n, H, p_out):
    """Largest violation of the outer-residual LP (Thm 6.1): 0 <= p_i <= p(i),
    sum_{i in S} p_i <= sum_{i in S} p(i) + psi(V \\ S) for every S outside H, equality
    at S = V \\ H.  p_out maps token -> p_i for tokens outside H."""
    V = len(p)
    rest = [i for i in range(V) if i not in set(H)]
    worst = 0.0
    for i in rest:
        worst = max(worst, -p_out[i], p_out[i] - float(p[i]))
    for r in range(1, len(rest) + 1):
        for S in itertools.combinations(rest, r):
            comp = [i for i in range(V) if i not in set(S)]
            rhs = float(sum(p[i] for i in S)) + psi(comp, p, q, n)
            lhs = float(sum(p_out[i] for i in S))
            worst = max(worst, lhs - rhs)
            if r == len(rest):
                worst = max(worst, abs(lhs - rhs))
    return worst


def coupling_marginals(slice_fn, q, n):
    """Sum over every draft tuple of pdraft(tuple) * pi(.|tuple): returns the induced
    marginal over tokens and the total acceptance probability (the OTLP objective)."""
    V = len(q)
    marg = np.zeros(V); acc = 0.0; worst_norm = 0.0
    for tup, mass in tuples_with_mass(q, n):
        if mass == 0.0:
            continue
        pi, a = slice_fn(tup)
        worst_norm = max(worst_norm, abs(float(pi.sum()) - 1.0))
        marg += mass * pi
        acc += mass * a
    return marg, acc, worst_norm
