"""GPU parity: the HIP path, called through the C ABI, against the CPU checker on the same seeded
inputs.  Tolerances: alpha* and every policy entry within 1e-5 absolute; token ids and the
accepted flag bit-exact unless the uniform lies within 1e-5 of a CDF edge; discrete structure
(ratio order, |H*|, block split) identical and residuals within 1e-12 on rows where H* is unique."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W
from parity_util import check_alpha_all_rows, compare_rows, run_gpu

pytestmark = pytest.mark.gpu


def test_tiny_all_rows():
    wl = W.tiny()                                  # config 1: B=1000, V=8, n=2, no top-k
    out = run_gpu(wl, 0.0)
    st = compare_rows(wl, out, range(wl.B), 0.0)
    assert st["rows"] == 1000 and st["fragile"] < 20, st
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-5)


def test_small_all_rows():
    wl = W.small()                                 # config 2: B=64, V=1024, n=4, top-k 32
    out = run_gpu(wl, 1e-6)
    compare_rows(wl, out, range(wl.B), 1e-6)
    assert np.all(out["status"] == 0)


@pytest.mark.parametrize("temperature", [0.7, 1.0])
def test_llm_shaped(temperature):
    wl = W.llm_shaped(temperature=temperature, seed_sub=int(temperature * 10))   # config 3
    out = run_gpu(wl, 1e-6)
    check_alpha_all_rows(wl, out)
    compare_rows(wl, out, range(0, wl.B, 16), 1e-6)
    assert np.all(out["status"] == 0)
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)


@pytest.mark.parametrize("tol", [1e-6, 1e-4])
def test_large_vocab_full_size(tol):
    """Config 4 at full size, in the launch configuration bench.py times; the checker is run on
    sampled rows, alpha* and the normalisation of the slice on every row."""
    wl = W.large_vocab()
    out = run_gpu(wl, tol)
    check_alpha_all_rows(wl, out)
    compare_rows(wl, out, range(3, wl.B, 24), tol)
    assert np.all(out["status"] == 0)
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)
    assert np.all((out["token"] >= 0) & (out["token"] < wl.V))


@pytest.mark.parametrize("n", [2, 4, 8, 16])
@pytest.mark.parametrize("k", [8, 32, 128])
def test_stress_cells(n, k):
    """Config 5 cells with a top-k (batch reduced to 96 rows per cell; the full-V cells are in
    test_gpu_full_vocab.py)."""
    wl = W.stress(B=96, n=n, k=k, seed_sub=100 * n + k)
    out = run_gpu(wl, 1e-6)
    check_alpha_all_rows(wl, out)
    near = np.flatnonzero(wl.meta["near"])[:2]
    rows = sorted(set([0, 17, 50]) | set(int(x) for x in near))
    compare_rows(wl, out, rows, 1e-6)
    assert np.all(np.abs(out["pi"].sum(1) - 1.0) < 1e-4)


def test_stress_cell_at_full_batch():
    """One config 5 cell at its own size (1024 rows x 128256 tokens, n = 8, top-k 128), the launch
    shape `bench.py --workload stress` times: alpha* on every 16th row, everything on sampled rows."""
    wl = W.stress()
    out = run_gpu(wl, 1e-4, want_slice=False)
    assert np.all(out["status"] == 0)
    sub = W.Workload(wl.name, 64, wl.V, wl.n, wl.k, wl.p[::16], wl.q[::16], wl.drafts[::16], wl.uniforms[::16])
    check_alpha_all_rows(sub, {"accept_prob": out["accept_prob"][::16]})
    near = np.flatnonzero(wl.meta["near"])[:2]
    compare_rows(wl, out, sorted(set([0, 333, 1023]) | set(int(x) for x in near)), 1e-4)
