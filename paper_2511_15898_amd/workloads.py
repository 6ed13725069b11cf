"""Seeded synthetic inputs for the Global Resolution verifier.

This module only *draws inputs*: target rows ``p``, draft rows ``q`` (before
top-k), the ``n`` i.i.d. drafts per row and one uniform per row.  It holds none
of the verifier's arithmetic, so both the HIP path and the CPU checker may be
fed from it.  Rows stand in for LLM next-token distributions (the paper measures
on Llama-3 / Gemma-2 logits, Section "Experiments"; those models are not
available here, so heavy-tailed synthetic logits with a correlated draft are
used instead).

Every array is produced in float64, rounded to float32 and re-normalised in
float32, so that every consumer reads the same bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20251115


@dataclass
class Workload:
    name: str
    B: int
    V: int
    n: int
    k: int                      # top-k on q; 0 means no top-k
    p: np.ndarray               # [B, V] float32, rows sum to 1
    q: np.ndarray               # [B, V] float32, rows sum to 1 (before top-k)
    drafts: np.ndarray          # [B, n] int32, i.i.d. from the top-k renormalised q row
    uniforms: np.ndarray        # [B] float32 in [0, 1)
    meta: dict = field(default_factory=dict)


def _softmax32(logits: np.ndarray) -> np.ndarray:
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    x = (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)
    # second normalisation in float32 so that the stored row is what sums to ~1
    x = x / x.sum(axis=-1, keepdims=True, dtype=np.float32)
    return x.astype(np.float32)


def topk_support(q_row: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest positive entries (ties: lower index first), ascending."""
    pos = np.flatnonzero(q_row > 0)
    if 0 < k < q_row.shape[0] and pos.size > k:
        vals = q_row[pos]
        kth = np.partition(vals, pos.size - k)[pos.size - k]      # the k-th largest value
        above = pos[vals > kth]
        ties = pos[vals == kth]                                   # ascending index
        pos = np.concatenate([above, ties[: k - above.size]])
    return np.sort(pos)


def draw_drafts(q: np.ndarray, k: int, n: int, rng: np.random.Generator) -> np.ndarray:
    """n i.i.d. inverse-CDF samples per row from q restricted to its top-k support."""
    B = q.shape[0]
    out = np.empty((B, n), dtype=np.int32)
    for b in range(B):
        sup = topk_support(q[b], k)
        cdf = np.cumsum(q[b, sup].astype(np.float64))
        u = rng.random(n) * cdf[-1]
        j = np.minimum(np.searchsorted(cdf, u, side="right"), sup.size - 1)
        out[b] = sup[j]
    return out


def _finish(name, p, q, n, k, rng, meta=None) -> Workload:
    B, V = p.shape
    drafts = draw_drafts(q, k, n, rng)
    uniforms = rng.random(B).astype(np.float32)
    uniforms = np.minimum(uniforms, np.float32(1.0 - 2.0 ** -24))
    return Workload(name, B, V, n, k, np.ascontiguousarray(p), np.ascontiguousarray(q),
                    drafts, uniforms, meta or {})


def tiny(B: int = 1000, V: int = 8, n: int = 2, seed_sub: int = 0) -> Workload:
    """Config 1: Dirichlet(0.5) target and draft rows, no top-k."""
    rng = np.random.default_rng(BASE_SEED + 1000 * 1 + seed_sub)
    p = rng.dirichlet(np.full(V, 0.5), size=B).astype(np.float32)
    q = rng.dirichlet(np.full(V, 0.5), size=B).astype(np.float32)
    p = np.maximum(p, np.float32(1e-30)); q = np.maximum(q, np.float32(1e-30))
    p = (p / p.sum(1, keepdims=True, dtype=np.float32)).astype(np.float32)
    q = (q / q.sum(1, keepdims=True, dtype=np.float32)).astype(np.float32)
    return _finish("tiny", p, q, n, 0, rng)


def small(B: int = 64, V: int = 1024, n: int = 4, k: int = 32, seed_sub: int = 0, keep_logits: bool = False) -> Workload:
    """Config 2: target logits 3*N(0,1); draft logits = target + N(0, std 0.5).  keep_logits: the float32 logits
    (before the division by the temperature, here 1) go to meta["target_logits"] / meta["draft_logits"]."""
    rng = np.random.default_rng(BASE_SEED + 1000 * 2 + seed_sub)
    tl = 3.0 * rng.standard_normal((B, V))
    dl = tl + 0.5 * rng.standard_normal((B, V))
    meta = {"temps": np.ones(B)}
    if keep_logits:
        meta.update(target_logits=tl.astype(np.float32), draft_logits=dl.astype(np.float32))
    return _finish("small", _softmax32(tl), _softmax32(dl), n, k, rng, meta)


def llm_shaped(B: int = 256, V: int = 32000, n: int = 4, k: int = 64, temperature=1.0,
               corr: float = 0.8, near_identical_frac: float = 0.0, seed_sub: int = 0,
               cfg: int = 3, name: str = "llm", keep_logits: bool = False) -> Workload:
    """Configs 3-5: heavy-tailed target logits 4*Gumbel(0,1); draft logits =
    corr*target + N(0,1); both divided by the row's temperature.  ``temperature`` may
    be a scalar or a (lo, hi) pair (uniform per row).  A fraction of rows may carry a
    draft that is the target plus N(0, std 0.01) noise (acceptance close to 1).  keep_logits: the float32
    logits (before the division by the temperature) go to meta["target_logits"] / meta["draft_logits"]."""
    rng = np.random.default_rng(BASE_SEED + 1000 * cfg + seed_sub)
    p = np.empty((B, V), np.float32); q = np.empty((B, V), np.float32)
    tls = np.empty((B, V), np.float32) if keep_logits else None
    dls = np.empty((B, V), np.float32) if keep_logits else None
    if np.ndim(temperature) == 0:
        temps = np.full(B, float(temperature))
    else:
        lo, hi = temperature
        temps = rng.uniform(lo, hi, size=B)
    near = rng.random(B) < near_identical_frac
    for b in range(B):                       # row by row: bounded host memory
        tl = 4.0 * rng.gumbel(0.0, 1.0, size=V)
        if near[b]:
            dl = tl + 0.01 * rng.standard_normal(V)
        else:
            dl = corr * tl + rng.standard_normal(V)
        p[b] = _softmax32(tl / temps[b]); q[b] = _softmax32(dl / temps[b])
        if keep_logits:
            tls[b] = tl; dls[b] = dl
    meta = {"temps": temps, "near": near}
    if keep_logits:
        meta.update(target_logits=tls, draft_logits=dls)
    return _finish(name, p, q, n, k, rng, meta)


def large_vocab(B: int = 256, V: int = 128256, n: int = 8, k: int = 128, seed_sub: int = 0, keep_logits: bool = False) -> Workload:
    """Config 4: the roofline configuration."""
    return llm_shaped(B, V, n, k, temperature=1.0, corr=0.7, seed_sub=seed_sub, cfg=4, name="large", keep_logits=keep_logits)


def stress(B: int = 1024, V: int = 128256, n: int = 8, k: int = 128, seed_sub: int = 0) -> Workload:
    """Config 5 cell: per-row temperature in [0.5, 1.5], 10 % near-identical rows."""
    return llm_shaped(B, V, n, k, temperature=(0.5, 1.5), corr=0.7, near_identical_frac=0.10,
                      seed_sub=seed_sub, cfg=5, name="stress")


def draft_tree(S: int = 8, K: int = 3, L: int = 4, V: int = 4096, k: int = 32, corr: float = 0.8, seed_sub: int = 0):
    """A tree of K i.i.d. draft paths of length L per sequence (stands in for the paper's multi-step runs on
    Gemma-2 27B/2B, App. "Multi-Step Experiments"): the target logits of a node are 4*Gumbel(0,1) and its draft
    logits corr*target + N(0,1), both a seeded function of the sequence and of the node's prefix, so that paths
    with equal prefixes see equal rows; each path draws its next token from the top-k renormalised draft row
    with its own stream.  Returns (p [S,K,L,V], q [S,K,L,V], paths [S,K,L] int32, uniforms [S,L] float32)."""
    p = np.empty((S, K, L, V), np.float32); q = np.empty((S, K, L, V), np.float32)
    paths = np.empty((S, K, L), np.int32)
    for s in range(S):
        for a in range(K):
            prefix = []
            for l in range(L):
                node = np.random.default_rng([BASE_SEED, 7000 + seed_sub, s] + prefix)
                tl = 4.0 * node.gumbel(0.0, 1.0, size=V)
                dl = corr * tl + node.standard_normal(V)
                p[s, a, l] = _softmax32(tl); q[s, a, l] = _softmax32(dl)
                draw = np.random.default_rng([BASE_SEED, 8000 + seed_sub, s, a, l])
                tok = int(draw_drafts(q[s, a, l][None, :], k, 1, draw)[0, 0])
                paths[s, a, l] = tok
                prefix.append(tok)
    u = np.random.default_rng([BASE_SEED, 9000 + seed_sub]).random((S, L)).astype(np.float32)
    return p, q, paths, np.minimum(u, np.float32(1.0 - 2.0 ** -24))
