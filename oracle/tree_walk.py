"""CPU checker for the multi-step walk over a tree of draft paths.  TEST INFRASTRUCTURE ONLY.

App. "Multi-Step Experiments": K i.i.d. paths of length L are drafted autoregressively from the draft
model; the verifier then advances from the root of the tree, at every node with n = the number of
drafted continuations of that node (the paths that still agree with the tokens emitted so far), until the
emitted token is not one of them; a row whose solve fails falls back to sampling from p (status != 0 in
solve_row does exactly that).  Plain loops over gr_oracle.solve_row / verify_row; shares no code with the
HIP path.

Reading taken where the paper is silent: n counts paths, not distinct tokens (two paths that drew the same
token are two i.i.d. drafts of the node, which is what the coupling of Eq. (cases) is built for); after a
level whose token was accepted the walk continues with the paths that drew it; the walk emits one token per
level visited, so a tree accepted down to its leaves yields L tokens (no bonus token: the leaf's target
distribution is not among the inputs).
Pinned in tests/test_oracle_pins.py by exact enumeration of every draft tree and every outcome on a tiny
vocabulary: the emitted tokens are distributed as autoregressive sampling from the target model."""
from __future__ import annotations

from . import gr_oracle as G


def tree_walk(p_nodes, q_nodes, paths, uniforms, k=0, tol=1e-6, max_T=0, temperature=None):
    """p_nodes[a][l], q_nodes[a][l]: the target / draft distributions after the first l tokens of path a (paths with
    the same first l tokens carry the same rows); paths[a][l]: the drafted tokens; uniforms[l]: one per level.
    temperature: when given, p_nodes / q_nodes hold the models' logits and every level goes through
    solve_row_from_logits at that temperature (App. A, first paragraph).
    Returns (tokens emitted, number of them that were accepted drafts, levels that used the fallback, the smallest
    distance of a uniform to a CDF edge over the levels visited)."""
    K, L = len(paths), len(paths[0])
    active = list(range(K))
    out, accepted_count, fallbacks, edge_min = [], 0, 0, 1.0
    for l in range(L):
        a0 = active[0]
        drafts = [int(paths[a][l]) for a in active]
        if temperature is None:
            sol, p_row = G.solve_row(p_nodes[a0][l], q_nodes[a0][l], len(active), k, tol=tol, max_T=max_T), p_nodes[a0][l]
        else:
            sol, p_row, _ = G.solve_row_from_logits(p_nodes[a0][l], q_nodes[a0][l], temperature, len(active), k, tol=tol, max_T=max_T)
        fallbacks += sol.status != G.STATUS_OK
        tok, accepted, _, _, edge = G.verify_row(sol, p_row, drafts, uniforms[l])
        edge_min = min(edge_min, edge)
        out.append(int(tok))
        if not accepted:
            break
        accepted_count += 1
        active = [a for a in active if int(paths[a][l]) == tok]
    return out, accepted_count, fallbacks, edge_min
