"""The five benchmark programs written as compositions of oracle operators.

TEST INFRASTRUCTURE (see the package docstring).  Each function takes a
``workloads.Workload`` and returns a dict of numpy results.  Nothing here adds
arithmetic of its own beyond the loss gradient the harness feeds in.
"""
from __future__ import annotations

import numpy as np

from . import (dense_to_triples, damp_apply2_fwd, damp_apply2_bwd, filter_plan, damp_filter_fwd, damp_filter_bwd,
               union_plan, damp_union_fwd, damp_union_bwd, reach_fwd, reach_bwd, dtkp_init, dtkp_apply2,
               dense_to_tuples, damp_applyk_fwd, damp_applyk_bwd, dtkp_applyk, dtkp_prob_bwd)


def _sum_tri(sa, sb):
    t = (np.asarray(sa, np.int32)[:, None] + np.asarray(sb, np.int32)[None, :]).astype(np.int32)
    return dense_to_triples(t)


def sum2_fwd(w):
    """Config 1: apply(D1, D2, x+y) under DAMP (Fig. 2 with two digits)."""
    syms, out = damp_apply2_fwd(dense_to_triples(w["table"]), 10, 10, w["pa"], w["pb"])
    return dict(syms=syms, out=out)


def nll_grad(p_final, target):
    """Upstream gradient of loss = -log p[target] per sample (harness side)."""
    g = np.zeros_like(p_final)
    rows = np.arange(p_final.shape[0])
    pt = np.maximum(p_final[rows, target], np.finfo(np.float32).tiny)
    g[rows, target] = (-1.0 / pt.astype(np.float64)).astype(np.float32)
    return g


def sum_chain_fwd_bwd(w, want_bwd=True):
    """Config 2: left fold of apply(D_res, D_i, x+y) (Fig. 2), then the reverse
    sweep of vector-Jacobian products from loss = -log p[target]."""
    p = w["p"]
    n = p.shape[0]
    sym = np.asarray(w["sym"], np.int32)
    accs, syms_list, tris = [p[0]], [sym], []
    for t in range(1, n):
        tri = _sum_tri(syms_list[-1], sym)
        s, o = damp_apply2_fwd(tri, syms_list[-1].size, sym.size, accs[-1], p[t])
        tris.append(tri); syms_list.append(s); accs.append(o)
    res = dict(syms=syms_list[-1], out=accs[-1], accs=accs)
    if not want_bwd:
        return res
    g = nll_grad(accs[-1], w["target"])
    res["g_out"] = g
    grads = [None] * n
    for t in range(n - 1, 0, -1):
        ga, gb = damp_apply2_bwd(tris[t - 1], syms_list[t - 1].size, sym.size, accs[t - 1], p[t], g)
        grads[t] = gb
        g = ga
    grads[0] = g
    res["grad_p"] = np.stack(grads)
    return res


def product_chain_fwd_bwd(w, want_bwd=True):
    """Product-N (appendix on combinatorial explosions): the fold of Fig. 2 with f(x, y) = x * y over interned
    product symbols; the workload carries the symbol tables of its stages.  target is a column of the last stage."""
    p = w["p"]
    n = p.shape[0]
    tables, stage_ids = w["tables"], w["stage_ids"]
    accs, tris = [p[0]], []
    for t in range(1, n):
        tri = dense_to_triples(tables[t - 1])
        s, o = damp_apply2_fwd(tri, tables[t - 1].shape[0], 10, accs[-1], p[t])
        assert np.array_equal(s, stage_ids[t])
        tris.append(tri); accs.append(o)
    res = dict(syms=stage_ids[n - 1], out=accs[-1], accs=accs)
    if not want_bwd:
        return res
    g = nll_grad(accs[-1], w["target"])
    res["g_out"] = g
    grads = [None] * n
    for t in range(n - 1, 0, -1):
        ga, gb = damp_apply2_bwd(tris[t - 1], tables[t - 1].shape[0], 10, accs[t - 1], p[t], g)
        grads[t] = gb
        g = ga
    grads[0] = g
    res["grad_p"] = np.stack(grads)
    return res


def hashed_pipeline_fwd_bwd(w):
    """Config 3: apply with a hashed table, filter by a keep-mask over the output
    ids, union with a second Distribution over all ids; then backward."""
    na, nb, n_out = w["na"], w["nb"], w["n_out"]
    tri = dense_to_triples(w["table"])
    s1, o1 = damp_apply2_fwd(tri, na, nb, w["pa"], w["pb"])
    pred = w["keep"][s1]                      # predicate evaluated on the symbols present
    s2, _ = filter_plan(s1, pred)
    o2 = damp_filter_fwd(pred, o1)
    all_ids = np.arange(n_out, dtype=np.int32)
    s3, ia, ib = union_plan(s2, all_ids)
    o3 = damp_union_fwd(ia, ib, o2, w["p2"])
    g3 = w["g"][:, :s3.size]
    g2, gp2 = damp_union_bwd(ia, ib, o2, w["p2"], g3)
    g1 = damp_filter_bwd(pred, g2)
    ga, gb = damp_apply2_bwd(tri, na, nb, w["pa"], w["pb"], g1)
    return dict(s1=s1, o1=o1, s2=s2, o2=o2, s3=s3, o3=o3, g2=g2, gp2=gp2, g1=g1, ga=ga, gb=gb)


def dtkp_sum_chain(w):
    """Config 4: the sum fold under DTKP-AM; digit slot n, value d is fact 10n+d."""
    p = w["p"]
    n, B = p.shape[0], p.shape[1]
    k = w["k"]
    sym = np.asarray(w["sym"], np.int32)
    fp, grp = w["fact_prob"], w["fact_group"]
    m, pp, pr = dtkp_init(np.arange(10, dtype=np.int32), fp, k)
    syms = sym
    stages = []
    for t in range(1, n):
        dm, _, _ = dtkp_init(10 * t + np.arange(10, dtype=np.int32), fp, k)
        tri = _sum_tri(syms, sym)
        syms2, m, pp, pr = dtkp_apply2(tri, syms.size, sym.size, k, grp, fp, m, dm)
        syms = syms2
        stages.append((syms, m, pp, pr))
    return dict(syms=syms, mask=m, pprob=pp, prob=pr, stages=stages)


def transitive_closure_fwd_bwd(w, join_triples):
    """The recursion of App. B, Fig. 9: new = apply_if(paths, edges, join); merged = union(paths, new); stop when the
    merge adds no symbol and return it.  Then the reverse sweep from the upstream gradient over the final paths.
    `join_triples(path_ids, edge_ids, n_nodes)` is the symbol-side table of one step (workloads)."""
    n, eids, p = w["n_nodes"], np.asarray(w["edge_ids"], np.int32), w["p"]
    paths, tags, tape = eids, p, []
    while True:
        tri = join_triples(paths, eids, n)
        nsyms, new = damp_apply2_fwd(tri, paths.size, eids.size, tags, p)
        msyms, ia, ib = union_plan(paths, nsyms)
        merged = damp_union_fwd(ia, ib, tags, new)
        tape.append((tri, paths.size, tags, new, ia, ib))
        grew = msyms.size != paths.size
        paths, tags = msyms, merged
        if not grew:
            break
    g = np.ascontiguousarray(w["g"][:, paths])
    ge = np.zeros(p.shape, np.float64)
    for tri, n_paths, t_in, new, ia, ib in reversed(tape):
        g_paths, g_new = damp_union_bwd(ia, ib, t_in, new, g)
        ga, gb = damp_apply2_bwd(tri, n_paths, eids.size, t_in, p, g_new)
        ge += gb
        g = (g_paths.astype(np.float64) + ga).astype(np.float32)
    ge += g                                  # the first paths are the edges themselves
    return dict(syms=paths, out=tags, rounds=len(tape), grad_p=ge.astype(np.float32))


def grid_reach_fwd_bwd(w):
    """Config 5: fixed-round single-source reachability and its backward."""
    side = w["side"]
    n = side * side
    hist = reach_fwd(n, w["edge_u"], w["edge_v"], w["src"], w["rounds"], w["p"])
    gp = reach_bwd(n, w["edge_u"], w["edge_v"], w["rounds"], w["p"], hist, w["g"])
    return dict(r=hist[-1], hist=hist, grad_p=gp)


def hwf_pipeline_damp(w):
    """Formula pipeline (appendix on the HWF model) under DAMP: Filter every position to its admissible classes,
    fold Apply over the positions with the formula-building function, evaluate with a unary Apply; then the
    reverse sweep from the upstream gradient over the formula values back to the 14 class probabilities."""
    p, L = w["p"], w["length"]
    xs = [damp_filter_fwd(w["keep"][pos], np.ascontiguousarray(p[:, pos, :])) for pos in range(L)]
    accs, tris = [xs[0]], []
    for pos in range(1, L):
        tab = w["tables"][pos - 1]
        tri = dense_to_triples(tab)
        _, o = damp_apply2_fwd(tri, tab.shape[0], tab.shape[1], accs[-1], xs[pos])
        tris.append(tri); accs.append(o)
    idx, to = dense_to_tuples(w["final_map"])
    syms, out = damp_applyk_fwd(idx, to, [accs[-1]])
    (g,) = damp_applyk_bwd(idx, to, [accs[-1]], w["g"])
    grad_p = np.zeros_like(p)
    for pos in range(L - 1, 0, -1):
        tab = w["tables"][pos - 1]
        g, gx = damp_apply2_bwd(tris[pos - 1], tab.shape[0], tab.shape[1], accs[pos - 1], xs[pos], g)
        grad_p[:, pos, :] = damp_filter_bwd(w["keep"][pos], gx)
    grad_p[:, 0, :] = damp_filter_bwd(w["keep"][0], g)
    return dict(syms=syms, out=out, accs=accs, grad_p=grad_p)


def hwf_pipeline_dtkp(w):
    """The same pipeline under DTKP-AM: the kept classes of all positions are the input facts (one exclusion group
    per position); tags are initialised after the Filter, so only admissible classes take fact numbers."""
    p, L, k = w["p"], w["length"], w["k"]
    xs = [damp_filter_fwd(w["keep"][pos], np.ascontiguousarray(p[:, pos, :])) for pos in range(L)]
    fp = np.ascontiguousarray(np.concatenate(xs, axis=1))
    off = np.concatenate([[0], np.cumsum([x.shape[1] for x in xs])]).astype(np.int32)
    grp = np.concatenate([np.full(x.shape[1], pos, np.int32) for pos, x in enumerate(xs)])
    m, _, _ = dtkp_init(np.arange(off[0], off[1]), fp, k)
    stages = []
    for pos in range(1, L):
        tab = w["tables"][pos - 1]
        dm, _, _ = dtkp_init(np.arange(off[pos], off[pos + 1]), fp, k)
        _, m, pp, pr = dtkp_apply2(dense_to_triples(tab), tab.shape[0], tab.shape[1], k, grp, fp, m, dm)
        stages.append((m, pp, pr))
    idx, to = dense_to_tuples(w["final_map"])
    syms, om, op, opr = dtkp_applyk(idx, to, k, grp, fp, [m])
    gfact = dtkp_prob_bwd(om, fp, w["g"])
    grad_p = np.zeros_like(p)
    for pos in range(L):
        grad_p[:, pos, :] = damp_filter_bwd(w["keep"][pos], np.ascontiguousarray(gfact[:, off[pos]:off[pos + 1]]))
    return dict(syms=syms, mask=om, pprob=op, prob=opr, stages=stages, fact_prob=fp, fact_group=grp, fact_offset=off,
                gfact=gfact, grad_p=grad_p)
