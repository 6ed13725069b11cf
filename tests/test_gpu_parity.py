"""GPU parity: the HIP path, called through the C ABI, against the CPU checker on the same seeded
inputs.  Tolerances: alpha* and every policy entry within 1e-5 absolute; token ids and the
accepted flag bit-exact unless the uniform lies within 1e-5 of a CDF edge; discrete structure
(ratio order, |H*|, block split) identical and residuals within 1e-12 on rows where H* is unique."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W
from parity_util import check_alpha_all_rows, compare_rows, rows_with_outer_programs, run_gpu

pytestmark = pytest.mark.gpu


def test_tiny_all_rows():
    wl = W.tiny()                                  # config 1: B=1000, V=8, n=2, no top-k
    out = run_gpu(wl, 0.0)
    st = compare_rows(wl, out, range(wl.B), 0.0)
    assert st["rows"] == 1000 and st["fragile"] < 20 and st["edge"] < 10, st     # exempt rows stay under 3 %
    assert st["inner_programs"] > 100 and st["outer_programs"] >= 10, st
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-5)


def test_small_all_rows():
    wl = W.small()                                 # config 2: B=64, V=1024, n=4, top-k 32
    out = run_gpu(wl, 1e-6)
    st = compare_rows(wl, out, range(wl.B), 1e-6)
    assert np.all(out["status"] == 0)
    assert st["fragile"] == 0 and st["inner_programs"] >= 32, st


@pytest.mark.parametrize("temperature", [0.7, 1.0])
def test_llm_shaped(temperature):
    wl = W.llm_shaped(temperature=temperature, seed_sub=int(temperature * 10))   # config 3
    out = run_gpu(wl, 1e-6)
    check_alpha_all_rows(wl, out)
    with_outer = rows_with_outer_programs(wl, range(wl.B), 1e-6, want=2)      # rare here: the inner program dominates
    st = compare_rows(wl, out, sorted(set(range(0, wl.B, 16)) | set(with_outer)), 1e-6)
    assert np.all(out["status"] == 0)
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)
    assert st["fragile"] <= st["rows"] // 4 and st["inner_programs"] >= 8 and st["outer_programs"] >= 1, st


@pytest.mark.parametrize("tol", [1e-6, 1e-4])
def test_large_vocab_full_size(tol):
    """Config 4 at full size, in the launch configuration bench.py times; the checker is run on
    sampled rows, alpha* and the normalisation of the slice on every row."""
    wl = W.large_vocab()
    out = run_gpu(wl, tol)
    check_alpha_all_rows(wl, out)
    # no row of this batch has an outer block with two active tokens (outside H* its F only rises): the sampled rows
    # exercise the inner program; outer programs at n = 8 are covered by the stress cells and the random configurations
    st = compare_rows(wl, out, range(3, wl.B, 24), tol)
    assert st["fragile"] <= st["rows"] // 4 and st["inner_programs"] >= 6, st
    assert np.all(out["status"] == 0)
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)
    assert np.all((out["token"] >= 0) & (out["token"] < wl.V))


_STRESS = {}


def _stress_base():
    """The 1024 x 128256 rows of config 5 (the batch `bench.py --workload stress` times), drawn once."""
    if "wl" not in _STRESS:
        _STRESS["wl"] = W.stress()
    return _STRESS["wl"]


@pytest.mark.parametrize("n", [2, 4, 8, 16])
@pytest.mark.parametrize("k", [8, 32, 128])
def test_stress_cells_at_full_batch(n, k):
    """Every top-k cell of config 5 at its own size (1024 rows x 128256 tokens; the full-V cells are in
    test_gpu_full_vocab.py): alpha* on every 16th row; order, |H*|, blocks, residuals, status, token and
    accepted flag on 10 rows (two of them near-identical p ~ q) taken from the full-batch launch; the
    policy entries of the same rows from a second launch on those rows alone, which must reproduce the
    full batch's tokens."""
    import dataclasses
    base = _stress_base()
    rng = np.random.default_rng(5000 + 100 * n + k)
    wl = dataclasses.replace(base, n=n, k=k, drafts=W.draw_drafts(base.q, k, n, rng))
    out = run_gpu(wl, 1e-6, want_slice=False)
    assert np.all((out["status"] == 0) | (out["status"] == 2)) and np.mean(out["status"] == 0) > 0.98
    sub = W.Workload(wl.name, 64, wl.V, n, k, wl.p[::16], wl.q[::16], wl.drafts[::16], wl.uniforms[::16])
    check_alpha_all_rows(sub, {"accept_prob": out["accept_prob"][::16]})
    near = [int(x) for x in np.flatnonzero(wl.meta["near"])[:2]]
    rows = sorted(set([0, 129, 333, 512, 700, 801, 950, 1023]) | set(near))
    st = compare_rows(wl, out, rows, 1e-6)
    assert st["rows"] >= 10 and st["fragile"] <= 3 and st["solved_rows"] >= 6, st
    pick = W.Workload(wl.name, len(rows), wl.V, n, k, np.ascontiguousarray(wl.p[rows]), np.ascontiguousarray(wl.q[rows]),
                      np.ascontiguousarray(wl.drafts[rows]), np.ascontiguousarray(wl.uniforms[rows]))
    out2 = run_gpu(pick, 1e-6)
    assert np.array_equal(out2["token"], out["token"][rows]) and np.array_equal(out2["accept_prob"], out["accept_prob"][rows])
    compare_rows(pick, out2, range(len(rows)), 1e-6)
    assert np.all(np.abs(out2["pi"].sum(1) - 1.0) < 1e-5)
