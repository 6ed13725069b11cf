"""gr_solve_verify (solve and verification in one launch) against gr_solve followed by gr_verify, through the C ABI:
the same kernels' arithmetic on the same policy, so acceptance probability, status, token and accepted flag are
compared bit for bit.  The two-call path is the one the other GPU tests hold against the CPU checker.  Cases: every
configuration that fits the LDS-resident path, rows that fall back to sampling from p (cap on |T|, iteration cap),
bad rows, draws that leave the drafts (uniforms near 1 walk the residual tokens), a support above GR_MAX_SUPPORT
(which keeps the two steps inside the call), a ragged tiny vocabulary, nine to sixteen drafts, and rows given as
logits (gr_solve_logits_verify against gr_solve_logits + gr_verify)."""
import numpy as np
import pytest

from paper_2511_15898_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(wl, tol, uniforms=None, drafts=None, p=None, **cfg):
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    pt = torch.from_numpy(wl.p if p is None else p).to(dev); qt = torch.from_numpy(wl.q).to(dev)
    d = torch.from_numpy(wl.drafts if drafts is None else drafts).to(dev)
    u = torch.from_numpy(wl.uniforms if uniforms is None else uniforms).to(dev)
    h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n, **cfg)
    try:
        acc, st = gr.gr_solve(h, pt, qt, wl.n, wl.k, tol)
        tok, ok = gr.gr_verify(h, d, u)
        two = [x.clone() for x in (acc, st, tok, ok)]
        one = gr.gr_solve_verify(h, pt, qt, wl.n, wl.k, tol, d, u)
        one = [x.clone() for x in one]
        tok2, ok2 = gr.gr_verify(h, d, u)              # the handle keeps the policy as after gr_solve
        torch.cuda.synchronize()
    finally:
        gr.gr_destroy(h)
    names = ("accept_prob", "status", "token", "accepted")
    for name, a, b in zip(names, two, one):
        if name == "accept_prob":
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), name      # NaN of a bad row included
        else:
            assert torch.equal(a, b), name
    assert torch.equal(tok2, two[2]) and torch.equal(ok2, two[3])
    return {n_: x.cpu().numpy() for n_, x in zip(names, one)}


def test_small_and_llm_shaped_and_large():
    for wl, tol in ((W.small(), 1e-6), (W.llm_shaped(seed_sub=3), 1e-6), (W.large_vocab(), 1e-4)):
        out = _both(wl, tol)
        assert np.all(out["status"] == 0)
        assert np.all((out["token"] >= 0) & (out["token"] < wl.V))
        assert 0 < out["accepted"].sum() <= wl.B


def test_draws_that_leave_the_drafts_walk_the_other_tokens():
    wl = W.large_vocab(B=64, seed_sub=7)
    rng = np.random.default_rng(11)
    u = (1.0 - rng.random(wl.B) * 0.004).astype(np.float32)               # the top of the CDF: where residual tokens sit
    u = np.minimum(u, np.float32(0.99999994))
    out = _both(wl, 1e-4, uniforms=u)
    assert (out["accepted"] == 0).sum() >= 3              # most slices leave little beyond the drafts
    wl = W.llm_shaped(B=48, V=777, n=3, k=16, seed_sub=8)                 # ragged V, one short tile
    out = _both(wl, 1e-6, uniforms=np.full(wl.B, 0.999, np.float32))
    assert (out["accepted"] == 0).sum() >= 1


def test_rows_that_fall_back_to_p_and_bad_rows():
    wl = W.large_vocab(B=32, seed_sub=9)
    p = wl.p.copy()
    p[3, 17] = np.nan                                                     # a bad row: token -1, accepted 0
    p[5] *= 0.5                                                           # row sum off by more than 1e-3
    out = _both(wl, 1e-6, p=p, max_T=8)                                   # most rows exceed the cap on |T|
    assert out["status"][3] == 3 and out["status"][5] == 3 and out["token"][3] == -1 and out["accepted"][5] == 0
    assert (out["status"] == 1).sum() >= 8                                # GR_ROW_TRUNC_CAP
    out = _both(wl, 1e-6, max_iter=2)                                     # iteration cap
    assert (out["status"] == 2).sum() >= 8                                # GR_ROW_ITER_CAP
    bad = wl.drafts.copy(); bad[1, 0] = wl.V + 5; bad[2, 1] = -1          # a draft outside the vocabulary
    out = _both(wl, 1e-4, drafts=bad)
    assert out["token"][1] == -1 and out["token"][2] == -1


def test_large_support_keeps_two_steps_and_many_drafts():
    wl = W.llm_shaped(B=8, V=5000, n=4, k=600, seed_sub=12)               # support above GR_MAX_SUPPORT: HBM-resident path
    out = _both(wl, 1e-4)
    assert np.all(out["status"] != 3)
    wl = W.llm_shaped(B=24, V=4096, n=12, k=48, seed_sub=13)              # the kernel for nine to sixteen drafts
    out = _both(wl, 1e-5)
    assert np.all(out["status"] == 0)


def test_rows_given_as_logits():
    import torch
    from paper_2511_15898_amd import binding as gr
    dev = torch.device("cuda:0")
    for wl, tol, two_temps in ((W.small(keep_logits=True), 1e-6, False), (W.large_vocab(B=64, seed_sub=21, keep_logits=True), 1e-4, True),
                               (W.llm_shaped(B=6, V=3000, n=3, k=500, seed_sub=22, keep_logits=True), 1e-4, False)):   # the last: HBM-resident support
        tl = torch.from_numpy(wl.meta["target_logits"]).to(dev); dl = torch.from_numpy(wl.meta["draft_logits"]).to(dev)
        T = torch.from_numpy(wl.meta["temps"].astype(np.float32)).to(dev)
        Td = (T * 1.25) if two_temps else None
        d = torch.from_numpy(wl.drafts).to(dev)                 # drawn from the float32 q: a draft that the logits' top-k does not
        u = torch.from_numpy(wl.uniforms).to(dev)               # hold gives token -1 on both paths alike
        h = gr.gr_create(wl.B, wl.V, max_k=wl.k, max_n=wl.n)
        try:
            acc, st = gr.gr_solve_logits(h, tl, dl, T, wl.n, wl.k, tol, draft_temperature=Td)
            tok, ok = gr.gr_verify(h, d, u)
            two = [x.clone() for x in (acc, st, tok, ok)]
            one = [x.clone() for x in gr.gr_solve_logits_verify(h, tl, dl, T, wl.n, wl.k, tol, d, u, draft_temperature=Td)]
            torch.cuda.synchronize()
        finally:
            gr.gr_destroy(h)
        for name, a, b in zip(("accept_prob", "status", "token", "accepted"), two, one):
            assert torch.equal(a.view(torch.int32) if name == "accept_prob" else a, b.view(torch.int32) if name == "accept_prob" else b), name
        assert int((one[1] == 0).sum()) >= wl.B // 2 and int((one[2] >= 0).sum()) >= wl.B // 2
