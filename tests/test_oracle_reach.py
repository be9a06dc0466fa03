"""Pins for the CPU oracle's grid-reachability program (no GPU)."""
import numpy as np

import oracle
import workloads as W


def dense_round_matrix(n, eu, ev, p):
    """A[v,u] = p(u,v) (symmetric) in float64 for one sample."""
    A = np.zeros((n, n))
    for e, (u, v) in enumerate(zip(eu, ev)):
        A[v, u] = p[e]
        A[u, v] = p[e]
    return A


def f64_reach(n, eu, ev, src, rounds, p):
    A = dense_round_matrix(n, eu, ev, p.astype(np.float64))
    r = np.zeros(n); r[src] = 1.0
    for _ in range(rounds):
        r = np.minimum(1.0, r + A @ r)
    return r


def test_edge_numbering():
    u, v = W.grid_edges(3)
    assert list(zip(u, v)) == [(0, 1), (1, 2), (3, 4), (4, 5), (6, 7), (7, 8),
                               (0, 3), (1, 4), (2, 5), (3, 6), (4, 7), (5, 8)]
    u, v = W.grid_edges(32)
    assert u.size == 2 * 32 * 31 == 1984


def test_small_probabilities_match_matrix_power():
    """No clamping when all p <= 0.01 (except the source, pinned at 1): r_t = min(1, (I+A)^t e_src)."""
    side, rounds, B = 4, 6, 3
    eu, ev = W.grid_edges(side)
    p = (W.uniform01(3, B * eu.size) * 0.01).astype(np.float32).reshape(B, -1)
    hist = oracle.reach_fwd(side * side, eu, ev, 0, rounds, p)
    for s in range(B):
        A = dense_round_matrix(side * side, eu, ev, p[s].astype(np.float64))
        M = np.linalg.matrix_power(np.eye(side * side) + A, rounds)
        ref = M[:, 0]
        got = hist[-1, s].astype(np.float64)
        assert got[0] == 1.0                      # the source saturates
        # away from the source the clamp at the source perturbs by O(p^2): compare with the clamped recurrence too
        np.testing.assert_allclose(got[1:], ref[1:], rtol=5e-4)
        np.testing.assert_allclose(got, f64_reach(side * side, eu, ev, 0, rounds, p[s]), rtol=1e-6, atol=1e-12)


def test_first_round_and_distance_and_monotone():
    w = W.config5(batch=4, side=8, rounds=16, seed=1)
    eu, ev = w["edge_u"], w["edge_v"]
    hist = oracle.reach_fwd(64, eu, ev, 0, 16, w["p"])
    assert np.all(hist[0, :, 0] == 1) and np.all(hist[0, :, 1:] == 0)
    # r_1 at the two neighbours of the source equals the edge probability
    np.testing.assert_array_equal(hist[1, :, 1], w["p"][:, 0])                 # edge (0,1) is horizontal edge 0
    np.testing.assert_array_equal(hist[1, :, 8], w["p"][:, 8 * 7])             # edge (0,8) is the first vertical
    for v in range(64):
        d = v // 8 + v % 8
        assert np.all(hist[:d, :, v] == 0) if d > 0 else True
        if d <= 16:
            assert np.all(hist[d, :, v] > 0)
    assert np.all(np.diff(hist, axis=0) >= 0)
    assert hist.min() >= 0 and hist.max() <= 1


def test_full_size_all_nodes_reached():
    w = W.config5(batch=2, seed=0)
    hist = oracle.reach_fwd(1024, w["edge_u"], w["edge_v"], 0, 64, w["p"])
    assert np.all(hist[-1] > 0)               # farthest node is 62 steps away
    assert np.all(hist[61, :, 1023] == 0) and np.all(hist[62, :, 1023] > 0)


def test_backward_matches_finite_differences_with_clamping():
    side, rounds, B = 3, 5, 3
    eu, ev = W.grid_edges(side)
    p = W.beta22(7, B * eu.size).reshape(B, -1)
    g = W.normal(8, B * 9).astype(np.float32).reshape(B, 9)
    hist = oracle.reach_fwd(9, eu, ev, 0, rounds, p)
    assert (hist[-1] == 1.0).sum() > B          # some nodes besides the source saturate
    gp = oracle.reach_bwd(9, eu, ev, rounds, p, hist, g)
    h = 1e-7
    for s in range(B):
        for e in range(eu.size):
            d = np.zeros(eu.size); d[e] = h
            p64 = p[s].astype(np.float64)
            fp = (g[s].astype(np.float64) * f64_reach(9, eu, ev, 0, rounds, p64 + d)).sum()
            fm = (g[s].astype(np.float64) * f64_reach(9, eu, ev, 0, rounds, p64 - d)).sum()
            fd = (fp - fm) / (2 * h)
            assert abs(fd - gp[s, e]) < 2e-5 + 1e-5 * abs(fd), (s, e, fd, gp[s, e])


def test_backward_small_p_matches_matrix_calculus():
    """Without clamping (source excluded) the result is linear in each single edge to first order:
    check against finite differences of the float64 recurrence on a 4x4 grid."""
    side, rounds, B = 4, 6, 2
    eu, ev = W.grid_edges(side)
    p = (W.uniform01(4, B * eu.size) * 0.05).astype(np.float32).reshape(B, -1)
    g = W.normal(5, B * 16).astype(np.float32).reshape(B, 16)
    hist = oracle.reach_fwd(16, eu, ev, 0, rounds, p)
    gp = oracle.reach_bwd(16, eu, ev, rounds, p, hist, g)
    h = 1e-6
    for s in range(B):
        for e in range(0, eu.size, 3):
            d = np.zeros(eu.size); d[e] = h
            p64 = p[s].astype(np.float64)
            fd = ((g[s] * f64_reach(16, eu, ev, 0, rounds, p64 + d)).sum()
                  - (g[s] * f64_reach(16, eu, ev, 0, rounds, p64 - d)).sum()) / (2 * h)
            assert abs(fd - gp[s, e]) < 1e-6 + 1e-5 * abs(fd)


def test_round_equals_apply_with_stay_symbol():
    """One round is Apply over (node, edge-or-stay) tuples with a single disjunction per node:
    union(paths, apply_if(paths, edges)) with the conjunction identity on the 'stay' symbol.
    Values, the float decision quantity and gradients of the two formulations agree."""
    side, B = 5, 4
    w = W.config5(batch=B, side=side, rounds=3, seed=3)
    n, E = side * side, w["edge_u"].size
    tri = (w["tri_i"], w["tri_j"], w["tri_o"])
    pe = np.concatenate([w["p"], np.ones((B, 1), np.float32)], axis=1)
    hist = oracle.reach_fwd(n, w["edge_u"], w["edge_v"], 0, 3, w["p"])
    r = hist[0]
    outs = []
    for t in range(3):
        syms, r, pre32, _ = oracle.damp_apply2_fwd(tri, n, E + 1, r, pe, want_pre=True)
        assert list(syms) == list(range(n))
        np.testing.assert_array_equal(r, hist[t + 1])
        outs.append(r)
    g = w["g"]
    gp = oracle.reach_bwd(n, w["edge_u"], w["edge_v"], 3, w["p"], hist, g)
    acc = np.zeros((B, E), np.float64)
    gr = g
    for t in range(2, -1, -1):
        gr, gb = oracle.damp_apply2_bwd(tri, n, E + 1, hist[t], pe, gr)
        acc += gb[:, :E]
    np.testing.assert_allclose(acc, gp, rtol=1e-5, atol=1e-7)


# ---------------------------------------------------------------- all-pairs transitive closure (App. B, Fig. 9)

def _closure_matrices(w):
    n, B = w["n_nodes"], w["p"].shape[0]
    E = np.zeros((B, n, n))
    E[:, w["edge_u"], w["edge_v"]] = w["p"].astype(np.float64)
    return E


def test_closure_symbols_are_the_boolean_closure_and_tags_a_matrix_recurrence():
    """Without clamping one step is P <- P + P.E on the matrices of path and edge tags, so after R steps
    P = E (I + E)^R; the symbols are the reachable pairs (Warshall)."""
    from oracle import programs as P
    w = W.closure_workload(batch=5, n_nodes=9, n_edges=12, scale=0.05, seed=3)
    res = P.transitive_closure_fwd_bwd(w, W.join_triples)
    n = w["n_nodes"]
    reach = np.zeros((n, n), bool)
    reach[w["edge_u"], w["edge_v"]] = True
    for k in range(n):
        reach |= reach[:, [k]] & reach[[k], :]
    np.testing.assert_array_equal(res["syms"], np.flatnonzero(reach.ravel()))
    E = _closure_matrices(w)
    want = E @ np.linalg.matrix_power(np.eye(n)[None] + E, res["rounds"])
    assert want.max() < 1.0
    got = np.zeros_like(want).reshape(5, -1)
    got[:, res["syms"]] = res["out"]
    np.testing.assert_allclose(got.reshape(want.shape), want, rtol=2e-6, atol=1e-12)
    # the last step adds no symbol, every earlier one does
    assert 2 <= res["rounds"] <= n


def test_closure_gradient_matches_finite_differences_of_the_matrix_recurrence():
    from oracle import programs as P
    w = W.closure_workload(batch=2, n_nodes=6, n_edges=8, scale=0.05, seed=4)
    res = P.transitive_closure_fwd_bwd(w, W.join_triples)
    n, R = w["n_nodes"], res["rounds"]
    g = np.zeros((2, n * n))
    g[:, res["syms"]] = w["g"][:, res["syms"]]

    def loss(s, pe):
        E = np.zeros((n, n)); E[w["edge_u"], w["edge_v"]] = pe
        return float((g[s].reshape(n, n) * (E @ np.linalg.matrix_power(np.eye(n) + E, R))).sum())

    for s in range(2):
        p0 = w["p"][s].astype(np.float64)
        for e in range(p0.size):
            hi, lo = p0.copy(), p0.copy()
            hi[e] += 1e-6; lo[e] -= 1e-6
            fd = (loss(s, hi) - loss(s, lo)) / 2e-6
            assert abs(res["grad_p"][s, e] - fd) <= 1e-6 + 2e-5 * abs(fd), (s, e, res["grad_p"][s, e], fd)


def test_closure_with_clamping_stays_in_range():
    from oracle import programs as P
    w = W.closure_workload(batch=4, n_nodes=8, n_edges=20, scale=1.0, seed=5)
    res = P.transitive_closure_fwd_bwd(w, W.join_triples)
    assert res["out"].min() >= 0.0 and res["out"].max() == 1.0       # dense graph: re-derivations pile up to the clamp
    assert np.isfinite(res["grad_p"]).all()


def test_clamp_boundary_passes_gradient_in_the_rounds():
    """Two nodes, one edge.  With p = 0.5 the second round's sum at node 1 is 0.5 + 1 * 0.5 = 1 exactly: the clamp passes
    gradient on its bound (App. A.2), so d r_2[1] / d p = r_1[0] + d r_1[1] / d p = 1 + 1 = 2.  With p = 0.75 the sum is
    1.3125, the clamp acts and the gradient is 0; with p = 0.25 nothing clamps and the gradient is again 2."""
    eu, ev = np.array([0], np.int32), np.array([1], np.int32)
    g = np.array([[0.0, 1.0]], np.float32)
    for p, want_r, want_g in ((0.5, 1.0, 2.0), (0.75, 1.0, 0.0), (0.25, 0.5, 2.0)):
        pe = np.array([[p]], np.float32)
        hist = oracle.reach_fwd(2, eu, ev, 0, 2, pe)
        assert hist[2, 0, 1] == np.float32(want_r) and hist[1, 0, 1] == np.float32(p)
        gp = oracle.reach_bwd(2, eu, ev, 2, pe, hist, g)
        assert gp[0, 0] == np.float32(want_g), (p, gp)
