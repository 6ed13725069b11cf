"""Seeded random configurations (shape, n, top-k, tau, cap on |T|, exact zeros): every row of every case
goes through the HIP path and the CPU checker.  A bounded version of the randomised differential runs
that found the one-draft and the large hard-program cases of test_gpu_edges.py."""
import dataclasses

import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W
from parity_util import compare_rows, run_gpu

pytestmark = pytest.mark.gpu


def _case(rng):
    kind = int(rng.integers(0, 4))
    n = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16]))
    tol = float(rng.choice([1e-2, 1e-3, 1e-4, 1e-6, 1e-7, 0.0]))
    max_T = int(rng.choice([0, 0, 0, 8, 64]))
    B = int(rng.integers(1, 7))
    sub = int(rng.integers(1_000_000))
    if kind == 0:
        V = int(rng.integers(2, 40)); k = min(int(rng.choice([0, 0, 1, 2, V])), V)
        wl = W.tiny(B=B, V=V, n=min(n, 4) if V ** min(n, 4) < 1e6 else 2, seed_sub=sub)
        wl = dataclasses.replace(wl, k=k, drafts=W.draw_drafts(wl.q, k, wl.n, rng))
    elif kind == 1:
        V = int(rng.integers(40, 3000)); k = min(int(rng.choice([1, 3, 8, 32, 100, 256, 300, 1000, 0])), V)
        wl = W.llm_shaped(B=B, V=V, n=n, k=k, temperature=(0.4, 1.6), near_identical_frac=0.2, seed_sub=sub)
    elif kind == 2:
        V = int(rng.integers(300, 2500))
        wl = W.llm_shaped(B=B, V=V, n=n, k=0, temperature=(0.4, 1.6), seed_sub=sub)
    else:
        V = int(rng.integers(64, 2000)); k = min(int(rng.choice([4, 16, 64, 128])), V)
        wl = W.small(B=B, V=V, n=min(n, 8), k=k, seed_sub=sub)
    if rng.random() < 0.4:                               # exact zeros in q and in p
        q = wl.q.copy(); p = wl.p.copy()
        zq = rng.random(q.shape) < 0.2; zq[np.arange(wl.B), q.argmax(1)] = False; q[zq] = 0
        zp = rng.random(p.shape) < 0.1; zp[np.arange(wl.B), p.argmax(1)] = False; p[zp] = 0
        q = (q / q.sum(1, keepdims=True, dtype=np.float32)).astype(np.float32)
        p = (p / p.sum(1, keepdims=True, dtype=np.float32)).astype(np.float32)
        wl = dataclasses.replace(wl, p=np.ascontiguousarray(p), q=np.ascontiguousarray(q),
                                 drafts=W.draw_drafts(q, wl.k, wl.n, rng))
    return wl, tol, max_T


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_configurations(seed):
    rng = np.random.default_rng(seed)
    rows = 0
    for _ in range(40):
        wl, tol, max_T = _case(rng)
        full = (wl.V if (wl.k <= 0 or wl.k >= wl.V) else wl.k) > 256
        out = run_gpu(wl, tol, max_T=max_T, export_rows=range(wl.B) if full else None)
        try:
            stats = compare_rows(wl, out, range(wl.B), tol, max_T=max_T)
        except AssertionError as e:
            raise AssertionError(f"{wl.name} B={wl.B} V={wl.V} n={wl.n} k={wl.k} tol={tol} max_T={max_T}: {e}") from e
        rows += stats["rows"]
    assert rows >= 40
