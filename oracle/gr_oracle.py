"""CPU checker for the Global Resolution verifier.  TEST INFRASTRUCTURE ONLY.

Plain, slow, single-threaded float64 NumPy, written from the paper
("Global Resolution: Optimal Multi-Draft Speculative Sampling via Convex
Minimization", Thomas & Pal).  It shares no code with the HIP path and must never be
imported by it: only tests, the smoke check and the bench's cpu_baseline leg use it.

Steps (paper citations in each function):
  1. top-k support of q                      App. "Top-k Sampling for the Relaxed OTLP"
  2. order by decreasing q/p, prefix psi     Sec. 5.1, Eq. (subset selection)
  3. H*, alpha* = 1 + psi(H*)                Thm 3.1, Sec. 5.1
  4. outer targets p_i by polymatroid greedy Thm 6.2, Lemma 6.3 (cumulative minima)
  5. truncated convex programs               Thm 6.4 (outer), Thm 6.5 (inner), Alg. 1
  6. transport slice pi(.|omega)             Eq. (cases), Eq. (approx-c), Lemma 6.6
  7. single-step multi-draft sampling        App. A, multi-draft procedure
  8. rows given as logits and a temperature  App. A, first paragraph; Sec. 5.1 for the orders
  9. nucleus (top-p) cut of the draft        Sec. 5.1, App. A (option of step 1)
The multi-step walk over a tree of draft paths (App. "Multi-Step Experiments") is in tree_walk.py.

Where the paper leaves a choice open the reading taken is stated at the function.
Parity status: every function below is pinned by tests/test_oracle_pins.py against brute
force (all 2^V subsets, the relaxed OTLP as an explicit LP, tuple enumeration, SciPy's
L-BFGS-B on the enumerated objective, exact rational and 60-digit arithmetic for the cuts
and orders), the n=1 closed form and the marginal / monotonicity invariants -- except the
inverse-CDF entry order of `sample_token` and the "not converged" status of a one-draft
program whose target reaches its token's draw probability, which are conventions of this
build (parity unpinned by the paper; the sampled distribution is pinned).
"""
from __future__ import annotations

import functools
import itertools
import math
from dataclasses import dataclass, field

import numpy as np

STATUS_OK, STATUS_TRUNC_CAP, STATUS_ITER_CAP, STATUS_BAD_ROW = 0, 1, 2, 3


# --------------------------------------------------------------------------- steps 1-4
def topk_support(q, k, tail_mass=0.0, key=None):
    """Tokens V_0 that top-k draft sampling can emit (App. "Top-k Sampling ..."): the k
    largest q (ties: lower token id), or every token with q > 0 when k <= 0 or k >= V.
    With tail_mass > 0 the support is also cut to a nucleus (App. A, first paragraph: top-p
    sampling, like top-k, only changes how q is computed): tokens are taken by decreasing q
    (ties: lower token id) until their running sum -- float64, added one after the other in
    that order -- reaches (1 - tail_mass) times the float64 row sum of q.  The tokens left
    out carry at most tail_mass of the draw mass, so n draws avoid them with probability
    at least 1 - n tail_mass: as an approximation of the uncut draft this moves alpha* and
    the coupling by at most n tail_mass in total variation.
    key: values that rise and fall with q (the draft logits behind a softmax); when given, "by
    decreasing q" is decided on them, so that two logits whose q round to one value keep their order."""
    q = np.asarray(q)
    by = q if key is None else np.asarray(key)
    pos = [i for i in range(q.shape[0]) if q[i] > 0]
    cut_k = 0 < k < q.shape[0] and len(pos) > k
    if cut_k or tail_mass > 0:
        pos.sort(key=lambda i: (-float(by[i]), i))
    if cut_k:
        pos = pos[:k]
    if tail_mass > 0:
        need = (1.0 - float(tail_mass)) * float(np.sum(q, dtype=np.float64))
        run = np.cumsum(np.array([float(q[i]) for i in pos]))          # sequential float64 sums
        reached = np.flatnonzero(run >= need)
        if reached.size:
            pos = pos[: int(reached[0]) + 1]
    return sorted(pos)


def ratio_order(p, q, support, key=None):
    """Sec. 5.1: tokens in decreasing order of q(i)/p(i).  The comparison is done by
    cross-multiplication (exact in float64 for float32-valued inputs); p = 0 ranks
    first; ties go to the lower token id.  key: values that rise and fall with q(i)/p(i)
    (draft logit minus target logit behind two softmaxes at one temperature); when given the
    order is taken on them."""
    if key is not None:
        return sorted(support, key=lambda i: (-float(key[i]), i))

    def before(a, b):
        lhs = float(q[a]) * float(p[b]); rhs = float(q[b]) * float(p[a])
        if lhs != rhs:
            return -1 if lhs > rhs else 1
        return -1 if a < b else (1 if a > b else 0)
    return sorted(support, key=functools.cmp_to_key(before))


def int_pow(x, n):
    r = x
    for _ in range(n - 1):
        r = r * x
    return r


def prefix_psi(p_sorted, q_sorted, n):
    """F(m) = psi({u_1..u_m}) = P_m - Q_m^n for m = 0..k' (Eq. subset selection with
    i.i.d. drafts, App. C: the draft mass of H^n is (sum_{i in H} q(i))^n).  q is
    renormalised over the support, so Q_{k'} = 1.  Sums run sequentially in the order."""
    S = np.cumsum(np.asarray(q_sorted, np.float64))
    Q = S / S[-1]
    P = np.cumsum(np.asarray(p_sorted, np.float64))
    F = np.concatenate(([0.0], P - int_pow(Q, n)))
    return P, Q, F


def pow_diff(a, d, n):
    """a^n - (a-d)^n without cancellation: d * sum_i a^(n-1-i) (a-d)^i."""
    b = a - d
    s = 0.0
    for i in range(n):
        s = s + a ** (n - 1 - i) * b ** i
    return d * s


def acceptance_sweep(p, q, ks, ns):
    """Optimal acceptance alpha*(k, n) = 1 + min_H psi(H) (Thm 3.1) of one decode position for every
    top-k size in `ks` and every number of i.i.d. drafts in `ns`: the quantity of the paper's
    acceptance-versus-(k, n) study (Sec. 7, first experiment).  For each k: the support V_0 of the
    top-k draft (App. "Top-k Sampling ..."), the order by decreasing q/p and the best prefix
    (Sec. 5.1).  p is divided by its float64 row sum, as in solve_row.  Returns [len(ks), len(ns)]."""
    p = np.asarray(p); q = np.asarray(q)
    pt = float(np.sum(p, dtype=np.float64))
    out = np.zeros((len(ks), len(ns)))
    for a, k in enumerate(ks):
        order = ratio_order(p, q, topk_support(q, int(k)))
        ps = p[order].astype(np.float64) / pt
        qs = q[order]
        for b, n in enumerate(ns):
            _, _, F = prefix_psi(ps, qs, int(n))
            out[a, b] = 1.0 + float(F.min())
    return out


@dataclass
class Block:
    """One transport sub-system: tokens at sorted positions lo..hi-1 (0-based), the mass
    of everything ranked before it, and slack 1 (inner system) or 0 (outer block)."""
    lo: int
    hi: int
    slack: int
    active: list = field(default_factory=list)   # positions that are optimised (T cap block)
    iters: int = 0
    resid: float = 0.0


@dataclass
class RowSolution:
    V: int
    n: int
    order: np.ndarray          # token ids, decreasing q/p  (length k')
    pos_of: dict               # token id -> sorted position
    p_s: np.ndarray            # p at the order
    q_s: np.ndarray            # renormalised q at the order
    P: np.ndarray
    Q: np.ndarray
    F: np.ndarray              # length k'+1
    G: np.ndarray              # suffix minima of F, length k'+1
    h: int
    alpha_star: float
    rho: np.ndarray            # residual p(i) - p_i at the order (0 on H*)
    target: np.ndarray         # p(i) on H*, p_i outside
    block_of: np.ndarray       # 0 for H*, 1.. for outer blocks, in rank order
    blocks: list
    w: np.ndarray              # softmax weights e^{alpha_i} at the order
    status: int = STATUS_OK
    fragile: bool = False      # a discrete decision sat within rounding of a tie


def outer_targets(F, h):
    """Thm 6.2 with v_1..v_k taken in increasing q/p (Sec. 6.1, last paragraph): the sets
    H_i are prefixes of the order, min_{T >= H_i} psi is a suffix minimum of F (Lemma
    6.3), so p_{u_m} = p(u_m) - (G(m) - G(m-1)) with G(m) = min_{j >= m} F(j).
    Tokens beyond the support have q = 0: F only rises there, so G(k') = F(k')."""
    G = np.minimum.accumulate(F[::-1])[::-1].copy()
    rho = np.zeros(F.shape[0] - 1)
    for m in range(h + 1, F.shape[0]):
        rho[m - 1] = G[m] - G[m - 1]
    return G, rho


def split_blocks(F, G, h):
    """The outer system decomposes at every rank m >= h with F(m) = G(m): there the Hall
    condition of the outer system (App. F, Eq. hall-outer) for the suffix {u_{m+1},...}
    holds with equality, so tuples that touch the suffix give it all their mass.  A
    tuple outside (H*)^n is therefore served inside the block of its lowest-ratio token.
    (The paper proves only that points of small gradient exist, Lemma G.1; this is the
    limit its minimising sequences approach.)"""
    kk = F.shape[0] - 1
    records = [m for m in range(h, kk + 1) if m == kk or F[m] <= G[m + 1]]
    return [(records[i], records[i + 1]) for i in range(len(records) - 1)]


# ------------------------------------------------------------------- routed mass (gradient)
def routed_enum(n, ctx, slack, q, w):
    """Definition: sum over tuples of n i.i.d. draws from {context, block tokens} of
    pdraft(tuple) * w_j / (slack + sum of w over the distinct block tokens drawn).  This
    is the row sum of S in Eq. (defined-s-outer) / (defined-s-inner), i.e. the gradient
    of Phi_T / Theta_T plus the target (App. G, App. H).  Also returns the mass left to
    the slack term, sum pdraft(tuple) * slack / (slack + ...)  (zero when slack = 0)."""
    m = len(q)
    probs = [ctx] + [float(x) for x in q]
    R = np.zeros(m); R0 = 0.0
    for tup in itertools.product(range(m + 1), repeat=n):
        mass = 1.0
        for a in tup:
            mass *= probs[a]
        members = sorted({a - 1 for a in tup if a > 0})
        if mass == 0.0 or (not members and slack == 0):
            continue
        den = slack + sum(w[j] for j in members)
        R0 += mass * slack / den
        for j in members:
            R[j] += mass * w[j] / den
    return R, R0


def routed_grouped(n, ctx, slack, q, w):
    """The paper's evaluator (App. "Truncated Solver Details"): one term per set A of at
    most n distinct block tokens, with the inclusion-exclusion coefficient
    sum_{A' <= A} (-1)^{|A|-|A'|} (ctx + Q(A'))^n."""
    m = len(q)
    R = np.zeros(m); R0 = slack * ctx ** n
    for size in range(1, min(n, m) + 1):
        for A in itertools.combinations(range(m), size):
            coef = 0.0
            for r in range(size + 1):
                for Ap in itertools.combinations(A, r):
                    coef += (-1.0) ** (size - r) * (ctx + sum(q[j] for j in Ap)) ** n
            den = slack + sum(w[j] for j in A)
            R0 += coef * slack / den
            for j in A:
                R[j] += coef * w[j] / den
    return R, R0


def routed_quadrature(n, ctx, slack, q, w, step=0.2, rel=1e-17):
    """Polynomial-time evaluator (derived here, pinned against the two above).
    1/x = int_0^inf e^{-xt} dt turns 1/(slack + W(set)) into a product of per-token
    factors x_i = e^{-t w_i}; for n i.i.d. draws
        E[ prod_{i in set} x_i ] = n! [z^n] e^{z ctx} prod_i (1 + x_i (e^{z q_i} - 1)),
    and requiring token j replaces its factor by x_j (e^{z q_j} - 1).  The t-integral is
    the trapezoid rule in s = log t (spectrally accurate for this integrand)."""
    q = np.asarray(q, np.float64); w = np.asarray(w, np.float64)
    m = q.shape[0]
    t_lo = rel / (slack + w.sum())
    # slowest decay: e^{-(slack + w_j) t} for token terms, e^{-slack t} for the slack term
    # of tuples drawn from the context alone
    t_hi = 46.0 / (slack + (w.min() if (slack == 0 or ctx == 0.0) else 0.0))
    N = int(math.ceil((math.log(t_hi) - math.log(t_lo)) / step)) + 1
    s = math.log(t_lo) + step * np.arange(N)
    t = np.exp(s)
    quad_w = step * t * np.exp(-slack * t)
    invfact = np.array([1.0 / math.factorial(d) for d in range(n + 1)])
    d_idx = np.arange(n + 1)

    def times_factor(A, j):
        """A(z) * (1 + x_j (e^{z q_j} - 1)) truncated at degree n, all nodes at once."""
        x = np.exp(-t * w[j])[:, None]
        e = q[j] ** d_idx * invfact
        out = (1.0 - x) * A
        for d in range(n + 1):
            out[:, d:] += x * e[d] * A[:, : n + 1 - d]
        return out

    pre = np.empty((m + 1, N, n + 1)); suf = np.empty((m + 1, N, n + 1))
    pre[0] = (ctx ** d_idx * invfact)[None, :]
    for j in range(m):
        pre[j + 1] = times_factor(pre[j], j)
    suf[m] = 0.0; suf[m][:, 0] = 1.0
    for j in range(m - 1, -1, -1):
        suf[j] = times_factor(suf[j + 1], j)
    R = np.zeros(m)
    for j in range(m):
        both = np.zeros((N, n + 1))
        for a in range(n + 1):
            both[:, a:] += pre[j][:, a:a + 1] * suf[j + 1][:, : n + 1 - a]
        e = q[j] ** d_idx * invfact
        coef = np.zeros(N)
        for d in range(1, n + 1):
            coef += e[d] * both[:, n - d]
        x = np.exp(-t * w[j])
        R[j] = w[j] * math.factorial(n) * float(np.sum(quad_w * x * coef))
    R0 = slack * math.factorial(n) * float(np.sum(quad_w * pre[m][:, n])) if slack else 0.0
    return R, R0


def routed(n, ctx, slack, q, w):
    m = len(q)
    if (m + 1) ** n <= 4096:
        return routed_enum(n, ctx, slack, q, w)
    return routed_quadrature(n, ctx, slack, q, w)


# ------------------------------------------------------------------------ convex solve
def newton_polish(n, ctx, slack, q, target, slack_target, alpha, rtol, max_iter, evaluator):
    """Damped Newton on  routed(alpha) = target  with a finite-difference Jacobian (the Hessian
    of Theta_T / Phi_T).  Without slack the system is singular along the common shift, so the
    last weight is pinned.  Used when the fixed-point iteration is too slow (a token whose
    target nearly exhausts the tuples that contain it).  Returns (alpha, evaluations, defect)."""
    m = alpha.shape[0]
    free = m if slack else m - 1
    evals = 0

    def defect(a):
        R, R0 = evaluator(n, ctx, slack, q, np.exp(a))
        f = np.log(target / R) - (math.log(slack_target / R0) if slack else math.log(target.sum() / R.sum()))
        return R, float(np.max(np.abs(f)))

    R, err = defect(alpha); evals += 1
    while err > rtol and evals < max_iter:
        J = np.empty((m, free))
        for k in range(free):
            a2 = alpha.copy(); a2[k] += 1e-6
            J[:, k] = (evaluator(n, ctx, slack, q, np.exp(a2))[0] - R) / 1e-6
        evals += free
        scale = 1.0 if slack else R.sum() / target.sum()
        try:
            step = np.linalg.solve(J[:free, :], (target * scale - R)[:free])
        except np.linalg.LinAlgError:
            # a weight so large that its difference quotients vanish: minimum-norm step instead
            step = np.linalg.lstsq(J[:free, :], (target * scale - R)[:free], rcond=None)[0]
        step = step * min(1.0, 2.0 / max(1e-300, float(np.max(np.abs(step)))))
        lam = 1.0
        while True:
            a2 = alpha.copy(); a2[:free] += lam * step
            R2, err2 = defect(a2); evals += 1
            if err2 < err or lam < 1e-4:
                break
            lam *= 0.5
        alpha, R, err = a2, R2, err2
    return alpha, evals, err


def solve_scaling(n, ctx, slack, q, target, slack_target, w0, rtol=1e-11, max_iter=4000, evaluator=routed):
    """Minimise Theta_T (slack 1, Thm 6.5) or Phi_T (slack 0, Thm 6.4) over the log
    weights alpha = log w: the gradient is routed(w) - target, and the minimiser is the
    point where it vanishes.  The paper runs L-BFGS-B; any convergent method reaches the
    same point because the objective is strictly convex (modulo a common shift when
    slack = 0).  Here: the exact coordinate update alpha_j += log(target_j / routed_j)
    (alternating minimisation, monotone).  With slack, the slack term is treated as the
    extra vertex a_0 of Lemma H.1 (weight pinned to 1, target = the system's slack
    mass) and updated with the rest, then the pin is restored.  Anderson mixing of
    depth 8 accelerates; if a mixed step ever raises the defect a hundredfold the
    iteration returns to its best point and takes plain steps for a while; after 400
    evaluations a damped Newton iteration takes over from the best point.
    Returns (w, evaluations, max relative defect)."""
    q = np.asarray(q, np.float64); target = np.asarray(target, np.float64)
    if n == 1:
        # One draft: a tuple is a single token, so Theta_T separates: routed_i = q_i w_i / (1 + w_i)
        # and the stationary point is w_i = target_i / (q_i - target_i) (the single-draft rule);
        # without slack routed_i = q_i whatever the weights, and the start weights are kept.
        # The point is exact wherever every target lies below its token's draw probability (no defect
        # is measured: re-evaluating it would lose all digits when a weight is huge); a target at or
        # above it has no finite weight and the program counts as not converged.
        w = np.asarray(w0, np.float64).copy()
        if slack:
            gap = q - target
            if not np.all(gap > 0):
                return np.where(gap > 0, target / np.where(gap > 0, gap, 1.0), 1e300), 0, float("inf")
            w = target / gap
        return w, 0, 0.0
    alpha = np.log(np.asarray(w0, np.float64))
    hist_a, hist_f = [], []
    err = np.inf
    best_err, best_alpha, best_f, plain = np.inf, alpha, None, 0
    for it in range(1, min(max_iter, 400) + 1):
        if slack == 0:
            alpha = alpha - alpha.max()
        R, R0 = evaluator(n, ctx, slack, q, np.exp(alpha))
        f = np.log(target / R)
        if slack:
            f = f - math.log(slack_target / R0)
        err = float(np.max(np.abs(f)))
        if err <= rtol:
            return np.exp(alpha), it, err
        if not np.isfinite(err) or err > 100.0 * best_err:
            # the mixed step went astray: back to the best point, plain (monotone) steps for a while
            alpha, f, err = best_alpha.copy(), best_f.copy(), best_err
            hist_a, hist_f, plain = [], [], 20
        elif err < best_err:
            best_err, best_alpha, best_f = err, alpha.copy(), f.copy()
        hist_a.append(alpha.copy()); hist_f.append(f.copy())
        if len(hist_a) > 9:
            hist_a.pop(0); hist_f.pop(0)
        step = f
        if plain > 0:
            plain -= 1
        elif len(hist_a) > 1:
            dF = np.stack([hist_f[-1] - x for x in hist_f[:-1]], axis=1)
            dA = np.stack([hist_a[-1] - x for x in hist_a[:-1]], axis=1)
            gam, *_ = np.linalg.lstsq(dF, f, rcond=1e-10)
            cand = f - (dA + dF) @ gam
            if np.all(np.isfinite(cand)) and np.max(np.abs(cand)) <= 10.0 * max(1.0, err):
                step = cand
            else:
                hist_a, hist_f = hist_a[-1:], hist_f[-1:]
        alpha = alpha + step
    if max_iter > 400:
        alpha, evals, err = newton_polish(n, ctx, slack, q, target, slack_target, best_alpha.copy(), rtol,
                                          max_iter - 400, evaluator)
        if err > rtol:
            # Both iterations can strand on a weight that a mixed step threw far beyond its value (the routed mass
            # of such a token no longer feels its weight).  The stationary point is unique (Thm 6.5; Thm 6.4 up
            # to a common factor), so a library root finder started from the start weights must reach the same
            # point: SciPy's hybrid Powell method on the same equations.
            from scipy.optimize import root

            def equations(a):
                R, R0 = evaluator(n, ctx, slack, q, np.exp(a if slack else a - a.max()))
                common = math.log(slack_target / R0) if slack else math.log(target.sum() / R.sum())
                return np.log(target / R) - common

            sol = root(equations, np.log(np.asarray(w0, np.float64)), method="hybr", tol=1e-13)
            a = sol.x if slack else sol.x - sol.x.max()
            f = equations(a)
            evals += int(sol.nfev) + 1
            if np.all(np.isfinite(f)) and float(np.max(np.abs(f))) < err:
                alpha, err = a, float(np.max(np.abs(f)))
        return np.exp(alpha), 400 + evals, err
    return np.exp(alpha), max_iter, err


# ----------------------------------------------------------------------- the row solve
def solve_row(p, q, n, k=0, tol=1e-6, max_T=0, max_iter=4000, rtol=1e-11, tail_mass=0.0, ratio_key=None, q_key=None):
    """Alg. 1 lines 1-2 and both convex programs, for one decode position (tail_mass: the nucleus cut of
    topk_support).

    Readings where the paper is silent:
      * "minimal T" (Alg. 1): the fewest tokens, taken by decreasing q (ties lower id),
        for which gamma_T (inner) / epsilon_T (outer) is at most tol.
      * Alg. 1 prints "T subset of H*" for the outer branch; Thm 6.4 has T outside H*.
      * the outer program is solved block by block (see split_blocks).
      * a program keeps only tuples drawn from its context and its tokens of T.  Their
        mass M_T falls short of the sum of the targets by at most gamma_T / epsilon_T, so
        the targets (with the inner system's slack mass 1 - alpha*) are scaled by one
        common factor to sum to M_T: the truncated system is then balanced and its
        gradient can vanish; the unscaled L1 gradient norm at that point is the
        shortfall, within Alg. 1's 5*tol.
      * tokens outside T keep the start weight w0_i = target_i / Pr[i drawn within its
        own system], divided for the inner system by the same ratio of the slack term
        ((1 - alpha*) / Q(H*)^n); tokens with target 0 have weight 0 and act as context.
        The common factor of an outer block's weights is fixed by sum w = sum w0 over
        its tokens of T.
      * p is divided by its float64 row sum first (the coupling needs sum p = 1 exactly;
        float32 rows only reach it to rounding); q is renormalised over the support.
      * max_T > 0 caps the variables of one program (App. "Truncated Solver Details",
        hard limits on |T|); hitting it, or the iteration cap, sets a status and the
        caller falls back to sampling from p (App. "Multi-Step Experiments")."""
    p = np.asarray(p); q = np.asarray(q)
    V = p.shape[0]
    bad = (not np.all(np.isfinite(p))) or (not np.all(np.isfinite(q))) or np.any(p < 0) or np.any(q < 0) \
        or abs(float(np.sum(p, dtype=np.float64)) - 1.0) > 1e-3 or abs(float(np.sum(q, dtype=np.float64)) - 1.0) > 1e-3
    if bad:
        return RowSolution(V, n, np.zeros(0, int), {}, *(np.zeros(0),) * 4, np.zeros(1), np.zeros(1), 0, float("nan"),
                           np.zeros(0), np.zeros(0), np.zeros(0, int), [], np.zeros(0), STATUS_BAD_ROW)
    support = topk_support(q, k, tail_mass, q_key)
    order = ratio_order(p, q, support, ratio_key)
    kk = len(order)
    p_total = float(np.sum(p, dtype=np.float64))   # float32 rows sum to 1 only to rounding
    p_s = np.array([float(p[i]) / p_total for i in order])
    q_raw = np.array([float(q[i]) for i in order])
    P, Q, F = prefix_psi(p_s, q_raw, n)
    q_s = q_raw / np.cumsum(q_raw)[-1]
    h = int(np.argmin(F))                       # smallest minimising prefix
    alpha_star = 1.0 + F[h]
    G, rho = outer_targets(F, h)
    target = p_s - rho
    fragile = False
    srt = np.sort(F)
    if kk >= 1 and srt[1] - srt[0] < 1e-13:
        fragile = True
    blocks_rng = split_blocks(F, G, h)
    for m in range(h, kk):
        if abs(F[m] - G[m + 1]) < 1e-13 and F[m] != G[m + 1]:
            fragile = True
    block_of = np.zeros(kk, int)
    for b, (lo, hi) in enumerate(blocks_rng):
        block_of[lo:hi] = b + 1
    tau = float(np.float32(tol))
    Qh = Q[h - 1] if h > 0 else 0.0
    w = np.zeros(kk)
    status = STATUS_OK
    blocks = []

    def by_q(positions):
        if q_key is not None:
            return sorted(positions, key=lambda m: (-float(q_key[order[m]]), order[m]))
        return sorted(positions, key=lambda m: (-q_raw[m], order[m]))

    # ---- truncation sets (Alg. 1: minimal T with gamma_T <= tol, resp. epsilon_T <= tol)
    T_in, acc = [], 0.0
    for m in by_q(range(h)):
        if int_pow(Qh, n) - int_pow(acc, n) <= tau:
            break
        T_in.append(m); acc = acc + q_s[m]
    T_out, acc = [], Qh
    for m in by_q(range(h, kk)):
        if 1.0 - int_pow(acc, n) <= tau:
            break
        T_out.append(m); acc = acc + q_s[m]
    T_out = set(T_out)

    # ---- start weights for every token of the support
    for lo, hi, slack in ([(0, h, 1)] if h > 0 else []) + [(lo, hi, 0) for lo, hi in blocks_rng]:
        top = Q[hi - 1] if hi > 0 else 0.0
        gauge = int_pow(top, n) / (-F[h]) if slack else 1.0
        for m in range(lo, hi):
            w[m] = gauge * target[m] / pow_diff(top, q_s[m], n) if target[m] > 0 else 0.0

    # ---- inner program, Thm 6.5
    if h > 0:
        act = [m for m in T_in if target[m] > 0]
        ctx = sum(q_s[m] for m in T_in if not target[m] > 0)
        blk = Block(0, h, 1, act)
        if max_T and len(act) > max_T:
            status = STATUS_TRUNC_CAP
        elif act:
            mass = int_pow(ctx + float(np.sum(q_s[act])), n)
            scale = mass / (float(np.sum(target[act])) - F[h])
            wa, blk.iters, blk.resid = solve_scaling(n, ctx, 1, q_s[act], target[act] * scale, -F[h] * scale,
                                                     w[act], rtol, max_iter)
            if blk.resid > rtol and status == STATUS_OK:
                status = STATUS_ITER_CAP
            w[act] = wa
        blocks.append(blk)
    # ---- outer programs, Thm 6.4, one per block of more than one token
    for lo, hi in blocks_rng:
        act = [m for m in range(lo, hi) if m in T_out and target[m] > 0]
        blk = Block(lo, hi, 0, act)
        if hi - lo >= 2 and len(act) >= 2:
            if max_T and len(act) > max_T:
                status = STATUS_TRUNC_CAP
            else:
                ctx = Q[lo - 1] if lo > 0 else 0.0
                qa = float(np.sum(q_s[act]))
                mass = pow_diff(ctx + qa, qa, n)
                w0sum = float(np.sum(w[act]))
                wa, blk.iters, blk.resid = solve_scaling(n, ctx, 0, q_s[act], target[act] * (mass / float(np.sum(target[act]))),
                                                         0.0, w[act], rtol, max_iter)
                if blk.resid > rtol and status == STATUS_OK:
                    status = STATUS_ITER_CAP
                w[act] = wa * (w0sum / float(np.sum(wa)))
        blocks.append(blk)
    return RowSolution(V, n, np.array(order, int), {int(t): i for i, t in enumerate(order)}, p_s, q_s, P, Q, F, G, h,
                       alpha_star, rho, target, block_of, blocks, w, status, fragile)


# ----------------------------------------------------------------- rows given as logits
def softmax_from_logits(logits, temperature=1.0):
    """App. A (review of single-step speculative sampling, first paragraph): temperature sampling only changes
    how p and q are computed from the models' logits -- softmax(logits / T), here in float64."""
    z = np.asarray(logits, np.float64) / float(temperature)
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def solve_row_from_logits(target_logits, draft_logits, temperature, n, k=0, tol=1e-6, max_T=0, max_iter=4000, rtol=1e-11,
                          draft_temperature=None):
    """Alg. 1 for a decode position given by its target and draft logits and the sampling temperatures (one for both
    models, or the draft's own in draft_temperature: the paper's temperature study cools the target and leaves the
    draft at 1): p and q are the float64 softmaxes.  Every order the method needs is decided on the logits
    themselves: q/p is proportional to exp(d / Td - t / Tt), so decreasing q/p (Sec. 5.1) is decreasing d - t with one
    temperature (exact for float32 logits) and decreasing d / Td - t / Tt with two (two rounded float64 products, one
    subtraction); decreasing q is decreasing d (top-k support, truncation sets); ties go to the lower token id.
    Returns (RowSolution, p, q)."""
    td = temperature if draft_temperature is None else draft_temperature
    p = softmax_from_logits(target_logits, temperature)
    q = softmax_from_logits(draft_logits, td)
    d64 = np.asarray(draft_logits, np.float64); t64 = np.asarray(target_logits, np.float64)
    inv_tt = 1.0 / float(temperature); inv_td = 1.0 / float(td)
    ratio_key = d64 - t64 if inv_td == inv_tt else d64 * inv_td - t64 * inv_tt
    return solve_row(p, q, n, k, tol=tol, max_T=max_T, max_iter=max_iter, rtol=rtol, ratio_key=ratio_key, q_key=d64), p, q


# ----------------------------------------------------------------- slice and sampling
def policy_slice(sol: RowSolution, p, drafts):
    """pi(.|omega) over all V tokens and the conditional acceptance a(omega)
    (Eq. (cases) / Eq. (approx-c), normalised by pdraft(omega) as in Alg. 1 'return
    normalized C').  A row whose solve failed uses the valid transport pi(.|omega) = p."""
    p = np.asarray(p, np.float64)
    p = p / p.sum()
    V = sol.V
    pi = np.zeros(V)
    distinct = list(dict.fromkeys(int(t) for t in drafts))
    if sol.status != STATUS_OK:
        pi[:] = p
        return pi, float(sum(pi[t] for t in distinct))
    pos = [sol.pos_of[t] for t in distinct]
    mmax = max(pos)
    if mmax < sol.h:                              # omega in (H*)^n: inner system + residual lift
        den = 1.0 + sum(sol.w[m] for m in pos)
        for t, m in zip(distinct, pos):
            pi[t] = sol.w[m] / den
        res = np.array(p, np.float64)             # residual p(i) - p_i of every token outside H*
        for m, t in enumerate(sol.order):
            res[t] = sol.rho[m]
        if res.sum() > 0:
            pi += (1.0 / den) * res / res.sum()
        return pi, float(1.0 - 1.0 / den)
    b = sol.block_of[mmax]
    members = [(t, m) for t, m in zip(distinct, pos) if m >= sol.h and sol.block_of[m] == b]
    den = sum(sol.w[m] for _, m in members)
    for t, m in members:
        pi[t] = sol.w[m] / den if den > 0 else 1.0 / len(members)
    return pi, 1.0


def sample_token(pi, drafts, u):
    """App. A, multi-draft procedure step 3: x0 ~ pi(.|drafts) by inverse CDF with one
    uniform.  Entry order (a convention of this build): the distinct drafts in order of
    first appearance, then every other token by ascending id.  Accepted iff x0 is one of
    the drafts.  Returns (token, accepted, distance of u to the nearest CDF edge)."""
    distinct = list(dict.fromkeys(int(t) for t in drafts))
    dset = set(distinct)
    c = 0.0; edge = 1.0; chosen = None; last = None
    for t in distinct + [i for i in range(len(pi)) if i not in dset]:
        if pi[t] <= 0.0:
            continue
        c += float(pi[t]); last = t
        edge = min(edge, abs(c - u))
        if chosen is None and u < c:
            chosen = t
    if chosen is None:
        chosen = last
    return chosen, chosen in dset, edge


def verify_row(sol, p, drafts, u):
    pi, acc = policy_slice(sol, p, drafts)
    tok, accepted, edge = sample_token(pi, drafts, float(u))
    return tok, accepted, pi, acc, edge
