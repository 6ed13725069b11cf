"""The allocation-free sweep entry point (gr_accept_sweep_noalloc) against gr_accept_sweep, through the C ABI:
two calls in a row on one GPU, the second on a smaller input, every cell compared bit for bit (both run the
same kernels; only the home of the selection scratch differs), plus the capacity error."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_noalloc_sweep_matches_the_handle_based_sweep_on_two_calls_in_a_row():
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    cases = [(W.llm_shaped(B=96, V=20000, n=4, k=64, seed_sub=501), [8, 32, 100, 256], [1, 2, 4, 8]),
             (W.llm_shaped(B=17, V=3001, n=4, k=64, seed_sub=502), [1, 16, 64], [1, 3, 16, 64])]       # second call: smaller, ragged V
    for wl, ks, ns in cases:
        p = torch.from_numpy(wl.p).to(dev); q = torch.from_numpy(wl.q).to(dev)
        acc = torch.full((wl.B, len(ks), len(ns)), -1.0, dtype=torch.float32, device=dev)
        st = torch.full((wl.B,), -1, dtype=torch.int32, device=dev)
        gr.gr_accept_sweep_noalloc(p, q, ks, ns, acc, st)
        h = gr.gr_create(wl.B, wl.V)
        try:
            ref_acc, ref_st = gr.gr_accept_sweep(h, p, q, ks, ns)
            torch.cuda.synchronize()
        finally:
            gr.gr_destroy(h)
        assert torch.equal(st, ref_st) and int(st.abs().sum()) == 0
        assert torch.equal(acc, ref_acc)
        a = acc.cpu().numpy()
        assert np.all((a > 0.0) & (a <= 1.0 + 1e-6)) and np.all(np.diff(a, axis=2) >= -1e-6)    # nondecreasing in n


def test_noalloc_sweep_rejects_more_rows_than_its_scratch_holds():
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    B = gr.GR_NOALLOC_MAX_B + 1
    p = torch.full((B, 64), 1.0 / 64, device=dev)
    acc = torch.empty((B, 1, 1), dtype=torch.float32, device=dev); st = torch.empty(B, dtype=torch.int32, device=dev)
    with pytest.raises(gr.GrError) as e:
        gr.gr_accept_sweep_noalloc(p, p, [8], [2], acc, st)
    assert e.value.code == gr.GR_ECAPACITY and "GR_NOALLOC_MAX_B" in str(e.value)
