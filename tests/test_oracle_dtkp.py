"""Pins for the CPU oracle's DTKP-AM operators (no GPU).

Independent checks: the f(D,D) example of App. A.1, the identities of the
0-hat / 1-hat tags (App. A.2), agreement with DAMP when k covers every proof,
a brute-force top-k over all digit tuples, the add-mult >= exact WMC bound
(App. A.1) by enumeration of all fact assignments, and structural invariants.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads as W
from oracle import programs as P

ABSENT = np.uint64(0xFFFFFFFFFFFFFFFF)


def rand_probs(seed, B, n):
    return W.softmax_rows(W.normal(seed, B * n).reshape(B, n))


def test_natural_init():
    fp = rand_probs(1, 3, 6)
    m, pp, pr = oracle.dtkp_init([4, 0, 5], fp, 3)
    assert m.shape == (3, 3, 3)
    np.testing.assert_array_equal(m[:, :, 0], np.tile(np.array([16, 1, 32], np.uint64), (3, 1)))
    assert np.all(m[:, :, 1:] == ABSENT) and np.all(pp[:, :, 1:] == 0)
    np.testing.assert_array_equal(pp[:, :, 0], fp[:, [4, 0, 5]])
    np.testing.assert_array_equal(pr, fp[:, [4, 0, 5]])


@pytest.mark.parametrize("n,k", [(3, 3), (2, 3), (3, 5)])
def test_f_of_D_D_example(n, k):
    """App. A.1: f(a,b) = T if a==b else F applied to the SAME Distribution D of mutually exclusive
    symbols.  Top-k set semantics: D(i) (x) D(i) = D(i), so Pr(T) = sum_i D(i) = 1 when |D| <= k;
    mixed pairs hold two values of one slot and are dropped, so F has no proof.  DAMP gives sum D(i)^2."""
    D = rand_probs(7, 5, n)
    m, pp, pr = oracle.dtkp_init(np.arange(n), D, k)
    table = np.where(np.eye(n, dtype=bool), 1, 0).astype(np.int32)      # T=1, F=0
    tri = oracle.dense_to_triples(table)
    syms, om, op, prob = oracle.dtkp_apply2(tri, n, n, k, np.zeros(n, np.int32), D, m, m)
    assert list(syms) == [0, 1]
    np.testing.assert_allclose(prob[:, 1], 1.0, atol=3e-7)
    assert np.all(prob[:, 0] == 0) and np.all(om[:, 0, :] == ABSENT)
    # every proof of T is a single fact
    for s in range(5):
        kept = [int(x) for x in om[s, 1] if x != ABSENT]
        assert sorted(kept) == [1 << i for i in range(n)]
    _, damp = oracle.damp_apply2_fwd(tri, n, n, D, D)
    np.testing.assert_allclose(damp[:, 1], (D.astype(np.float64) ** 2).sum(1), rtol=1e-6)


def test_without_exclusion_groups_mixed_pairs_survive():
    D = rand_probs(8, 2, 3)
    m, _, _ = oracle.dtkp_init(np.arange(3), D, 3)
    table = np.where(np.eye(3, dtype=bool), 1, 0).astype(np.int32)
    _, om, op, prob = oracle.dtkp_apply2(oracle.dense_to_triples(table), 3, 3, 3, None, D, m, m)
    # F now holds the 3 distinct two-fact proofs {i,j} (each reachable as (i,j) and (j,i): counted once)
    for s in range(2):
        assert sorted(int(x) for x in om[s, 0]) == [3, 5, 6]
        want = sorted((float(np.float32(D[s, i]) * np.float32(D[s, j])) for i, j in ((0, 1), (0, 2), (1, 2))),
                      reverse=True)
        np.testing.assert_array_equal(op[s, 0], np.array(want, np.float32))


def test_one_hat_and_zero_hat_identities():
    """App. A.2: 1-hat is one empty proof (probability 1), 0-hat has no proofs (probability 0);
    t (x) 1-hat = t and t (+) 0-hat = t."""
    k = 3
    fp = rand_probs(2, 4, 8)
    # a tag with several proofs: sum of two 2-symbol slots gives symbol 1 two proofs
    a0, _, _ = oracle.dtkp_init([0, 1], fp, k)
    a1, _, _ = oracle.dtkp_init([2, 3], fp, k)
    grp = np.array([0, 0, 1, 1, 2, 2, 3, 3], np.int32)
    syms, tm, tp, tpr = oracle.dtkp_apply2(oracle.dense_to_triples(W.sum_table([0, 1], [0, 1])), 2, 2, k, grp, fp, a0, a1)
    assert list(syms) == [0, 1, 2] and np.all(tm[:, 1, :2] != ABSENT) and np.all(tm[:, 1, 2] == ABSENT)
    one = np.full((4, 1, k), ABSENT, np.uint64)
    one[:, 0, 0] = 0
    ident = np.arange(3, dtype=np.int32).reshape(3, 1)          # f(s, unit) = s
    s2, om, op, opr = oracle.dtkp_apply2(oracle.dense_to_triples(ident), 3, 1, k, grp, fp, tm, one)
    np.testing.assert_array_equal(om, tm)
    np.testing.assert_array_equal(op, tp)
    np.testing.assert_array_equal(opr, tpr)
    # Pr(1-hat) = 1, Pr(0-hat) = 0 through the union's probability output
    zero_m = np.full((4, 3, k), ABSENT, np.uint64)
    zero_p = np.zeros((4, 3, k), np.float32)
    _, ia, ib = oracle.union_plan(syms, syms)
    um, up, upr = oracle.dtkp_union(ia, ib, tm, tp, zero_m, zero_p)
    np.testing.assert_array_equal(um, tm)
    np.testing.assert_array_equal(up, tp)
    np.testing.assert_array_equal(upr, tpr)
    zm, zp, zpr = oracle.dtkp_union(ia, ib, zero_m, zero_p, zero_m, zero_p)
    assert np.all(zpr == 0) and np.all(zm == ABSENT)
    one_p = np.zeros((4, 1, k), np.float32)
    one_p[:, 0, 0] = 1.0
    _, ja, jb = oracle.union_plan([0], [])
    _, _, opr1 = oracle.dtkp_union(ja, jb, one, one_p, np.zeros((4, 0, k), np.uint64), np.zeros((4, 0, k), np.float32))
    assert np.all(opr1 == 1.0)


def test_union_dedupes_and_orders():
    k = 3
    am = np.array([[[0b011, 0b100, ABSENT]]], np.uint64)
    ap = np.array([[[0.25, 0.5, 0.0]]], np.float32)
    bm = np.array([[[0b100, 0b1000, 0b1]]], np.uint64)
    bp = np.array([[[0.5, 0.25, 0.125]]], np.float32)
    _, ia, ib = oracle.union_plan([3], [3])
    om, op, pr = oracle.dtkp_union(ia, ib, am, ap, bm, bp)
    # 0b100 appears on both sides: one proof.  0.25 tie: smaller mask (0b011) first.
    assert [int(x) for x in om[0, 0]] == [0b100, 0b011, 0b1000]
    np.testing.assert_array_equal(op[0, 0], np.array([0.5, 0.25, 0.25], np.float32))
    assert pr[0, 0] == 1.0      # 0.5+0.25+0.25
    om1, op1, pr1 = oracle.dtkp_union(ia, ib, am[:, :, :1].copy(), ap[:, :, :1].copy(),
                                      bm[:, :, 1:2].copy(), bp[:, :, 1:2].copy())
    assert [int(x) for x in om1[0, 0]] == [0b011] and pr1[0, 0] == 0.25     # k=1, tie -> smaller mask
    # the tag probability is clamped at 1 (Sec. 3.2): 0.75 + 0.5 -> 1
    cm = np.array([[[0b01, ABSENT, ABSENT]]], np.uint64)
    cp = np.array([[[0.75, 0, 0]]], np.float32)
    dm = np.array([[[0b10, ABSENT, ABSENT]]], np.uint64)
    dp = np.array([[[0.5, 0, 0]]], np.float32)
    om2, op2, pr2 = oracle.dtkp_union(ia, ib, cm, cp, dm, dp)
    assert [int(x) for x in om2[0, 0]] == [0b01, 0b10, int(ABSENT)] and pr2[0, 0] == 1.0


def test_large_k_equals_damp():
    """With k >= the number of proofs of every symbol nothing is pruned, the proofs of a sum over distinct slots
    are pairwise exclusive, and the tag probability is the DAMP probability (up to rounding)."""
    n_dig, k, B = 3, 8, 6
    p = np.stack([rand_probs(40 + t, B, 3) for t in range(n_dig)])      # digits 0..2, at most 7 proofs per sum
    fp = np.ascontiguousarray(p.transpose(1, 0, 2).reshape(B, 9))
    grp = (np.arange(9) // 3).astype(np.int32)
    sym = np.arange(3, dtype=np.int32)
    m, _, _ = oracle.dtkp_init(np.arange(3), fp, k)
    syms, acc = sym, p[0]
    for t in range(1, n_dig):
        dm, _, _ = oracle.dtkp_init(3 * t + np.arange(3), fp, k)
        tri = oracle.dense_to_triples(W.sum_table(syms, sym))
        s2, m, pp, pr = oracle.dtkp_apply2(tri, syms.size, 3, k, grp, fp, m, dm)
        _, acc = oracle.damp_apply2_fwd(tri, syms.size, 3, acc, p[t])
        syms = s2
    np.testing.assert_allclose(pr, acc, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("n_dig,k", [(3, 3), (4, 3), (5, 3), (4, 1), (3, 5)])
def test_staged_topk_matches_brute_force_over_all_tuples(n_dig, k):
    B = 3
    w = W.config4(batch=B, n_digits=n_dig, k=k, seed=50 + n_dig)
    r = P.dtkp_sum_chain(w)
    p = w["p"]
    tuples = np.array(list(itertools.product(range(10), repeat=n_dig)))
    sums = tuples.sum(1)
    masks = np.zeros(len(tuples), np.uint64)
    for t in range(n_dig):
        masks |= np.uint64(1) << (np.uint64(10 * t) + tuples[:, t].astype(np.uint64))
    n_checked = 0
    for s in range(B):
        prob = np.ones(len(tuples), np.float32)
        for t in range(n_dig):                       # ascending fact index = ascending slot
            prob = (prob * p[t, s, tuples[:, t]]).astype(np.float32)
        for c in range(9 * n_dig + 1):
            sel = np.nonzero(sums == c)[0]
            order = sorted(sel, key=lambda q: (-float(prob[q]), int(masks[q])))
            top = order[:k]
            if len(order) > k and prob[order[k]] == prob[order[k - 1]]:
                continue                              # float tie at the cut: pruning order may differ
            want_m = [int(masks[q]) for q in top] + [int(ABSENT)] * (k - len(top))
            want_p = [prob[q] for q in top] + [np.float32(0)] * (k - len(top))
            assert [int(x) for x in r["mask"][s, c]] == want_m
            np.testing.assert_array_equal(r["pprob"][s, c], np.array(want_p, np.float32))
            tot = np.float32(0)
            for v in want_p:
                tot = np.float32(tot + v)
            assert r["prob"][s, c] == min(np.float32(1), tot)
            n_checked += 1
    assert n_checked >= 0.9 * B * (9 * n_dig + 1)


def test_config4_structural_invariants():
    w = W.config4(batch=16, seed=2)
    r = P.dtkp_sum_chain(w)
    assert list(r["syms"]) == list(range(46))
    for s in range(16):
        for c in range(46):
            ms = [int(x) for x in r["mask"][s, c]]
            ps = r["pprob"][s, c]
            valid = [m for m in ms if m != int(ABSENT)]
            assert len(set(valid)) == len(valid)
            assert ms[:len(valid)] == valid                      # absent slots come last
            assert all(ps[x] >= ps[x + 1] for x in range(len(ps) - 1))
            for m in valid:
                digits = []
                for t in range(5):
                    bits = (m >> (10 * t)) & 0x3FF
                    assert bin(bits).count("1") == 1              # one value per slot
                    digits.append(bits.bit_length() - 1)
                assert sum(digits) == c
    # sums 0 and 45 have exactly one proof; interior sums have 3
    assert np.all(r["mask"][:, 0, 1:] == ABSENT) and np.all(r["mask"][:, 45, 1:] == ABSENT)
    assert np.all(r["mask"][:, 20, :] != ABSENT)


def exact_wmc(masks, fact_prob):
    """P(at least one proof holds) for independent facts, by enumerating all fact assignments."""
    n = len(fact_prob)
    tot = 0.0
    for assign in range(1 << n):
        if any((assign & m) == m for m in masks):
            w = 1.0
            for j in range(n):
                w *= fact_prob[j] if (assign >> j) & 1 else 1.0 - fact_prob[j]
            tot += w
    return tot


def test_add_mult_upper_bounds_exact_wmc():
    """App. A.1: sum_i Pr(t_i) >= exact WMC of the same proofs (it double counts shared models)."""
    n, k, B = 10, 4, 6
    fp = W.uniform01(5, B * n).astype(np.float32).reshape(B, n)
    rng_bits = W.splitmix64(99, np.arange(B * 2 * k)).reshape(B, 2, k)
    am = (rng_bits[:, 0, :] % np.uint64(1 << n)).astype(np.uint64).reshape(B, 1, k)
    bm = (rng_bits[:, 1, :] % np.uint64(1 << n)).astype(np.uint64).reshape(B, 1, k)

    def probs(m):
        out = np.ones(m.shape, np.float32)
        for j in range(n):
            has = ((m >> np.uint64(j)) & np.uint64(1)).astype(bool)
            out = np.where(has, (out * fp[:, j].reshape(B, 1, 1)).astype(np.float32), out)
        return out
    _, ia, ib = oracle.union_plan([0], [0])
    om, op, pr = oracle.dtkp_union(ia, ib, am, probs(am), bm, probs(bm))
    for s in range(B):
        kept = [int(x) for x in om[s, 0] if x != ABSENT]
        assert len(kept) >= 1
        wmc = exact_wmc(kept, fp[s].astype(np.float64))
        am_sum = float(op[s, 0].astype(np.float64).sum())
        assert am_sum >= wmc - 1e-7
        assert pr[s, 0] >= min(1.0, wmc) - 1e-6


def test_filter_copies_tags():
    w = W.config4(batch=4, n_digits=2, seed=1)
    r = P.dtkp_sum_chain(w)
    pred = (np.arange(19) % 3 == 0).astype(np.uint8)
    om, op, pr = oracle.dtkp_filter(pred, r["mask"], r["pprob"], r["prob"])
    sel = pred.astype(bool)
    np.testing.assert_array_equal(om, r["mask"][:, sel])
    np.testing.assert_array_equal(op, r["pprob"][:, sel])
    np.testing.assert_array_equal(pr, r["prob"][:, sel])


# ---------------------------------------------------------------- gradient of the tag probabilities

def _masks(rows, k):
    """[[proof bit lists per symbol]] -> mask[1, n, k]"""
    m = np.full((1, len(rows), k), ABSENT, np.uint64)
    for i, proofs in enumerate(rows):
        for x, bits in enumerate(proofs):
            m[0, i, x] = np.uint64(sum(1 << b for b in bits))
    return m


def test_prob_gradient_by_hand():
    """Pr = p0*p1 + p2 for the first symbol, p3 for the second: d/dp = (p1, p0, 1 | 1), scaled by the upstream
    gradient; a symbol over 1 passes nothing, a symbol at exactly 1 passes (App. A.2)."""
    m = _masks([[[0, 1], [2]], [[3]]], 3)
    fp = np.array([[0.5, 0.25, 0.125, 0.75]], np.float32)
    g = np.array([[2.0, -3.0]], np.float32)
    np.testing.assert_array_equal(oracle.dtkp_prob_bwd(m, fp, g), [[0.5, 1.0, 2.0, -3.0]])
    over = np.array([[1.0, 0.75, 0.5, 0.75]], np.float32)           # 0.75 + 0.5 > 1
    np.testing.assert_array_equal(oracle.dtkp_prob_bwd(m, over, g), [[0.0, 0.0, 0.0, -3.0]])
    edge = np.array([[1.0, 0.5, 0.5, 1.0]], np.float32)             # exactly 1 on both symbols
    np.testing.assert_array_equal(oracle.dtkp_prob_bwd(m, edge, g), [[1.0, 2.0, 2.0, -3.0]])
    shared = _masks([[[0, 1], [0, 2]]], 2)                          # a fact in two proofs: p0*(p1 + p2)
    np.testing.assert_allclose(oracle.dtkp_prob_bwd(shared, fp[:, :3], np.array([[1.0]], np.float32)),
                               [[0.375, 0.5, 0.5]], rtol=1e-7)


def test_prob_gradient_matches_finite_differences_of_the_definition():
    """Central differences of sum_i prod_j p_j over the proof sets the forward pass kept (held fixed)."""
    w = W.config4(batch=4, n_digits=4, k=3, seed=5)
    ref = P.dtkp_sum_chain(w)
    mask, fp = ref["mask"], w["fact_prob"].astype(np.float64)
    B, n, k = mask.shape
    g = W.normal(9, B * n).astype(np.float32).reshape(B, n)

    def loss(s, q):
        tot = 0.0
        for i in range(n):
            pr = 0.0
            for x in range(k):
                mm = int(mask[s, i, x])
                if mm == int(ABSENT):
                    continue
                pr += np.prod([q[f] for f in range(q.size) if (mm >> f) & 1])
            assert pr < 1.0
            tot += float(g[s, i]) * pr
        return tot

    got = oracle.dtkp_prob_bwd(mask, w["fact_prob"], g)
    for s in range(B):
        for f in range(fp.shape[1]):
            hi, lo = fp[s].copy(), fp[s].copy()
            hi[f] += 1e-6; lo[f] -= 1e-6
            fd = (loss(s, hi) - loss(s, lo)) / 2e-6
            assert abs(got[s, f] - fd) <= 1e-6 + 1e-5 * abs(fd), (s, f, got[s, f], fd)


def test_prob_gradient_equals_damp_gradient_when_nothing_is_pruned():
    """With k >= the number of proofs of every symbol the tag probabilities are DAMP's (pinned above), and so are
    their gradients w.r.t. the digit probabilities: fact 3n+d is digit slot n taking value d."""
    n_dig, k, B = 3, 8, 5
    p = np.stack([rand_probs(60 + t, B, 3) for t in range(n_dig)])
    fp = np.ascontiguousarray(p.transpose(1, 0, 2).reshape(B, 9))
    grp = (np.arange(9) // 3).astype(np.int32)
    sym = np.arange(3, dtype=np.int32)
    m, _, _ = oracle.dtkp_init(np.arange(3), fp, k)
    syms, accs, tris = sym, [p[0]], []
    for t in range(1, n_dig):
        dm, _, _ = oracle.dtkp_init(3 * t + np.arange(3), fp, k)
        tri = oracle.dense_to_triples(W.sum_table(syms, sym))
        s2, m, _, _ = oracle.dtkp_apply2(tri, syms.size, 3, k, grp, fp, m, dm)
        accs.append(oracle.damp_apply2_fwd(tri, syms.size, 3, accs[-1], p[t])[1])
        tris.append((tri, syms.size))
        syms = s2
    g = W.normal(7, B * syms.size).astype(np.float32).reshape(B, syms.size)
    got = oracle.dtkp_prob_bwd(m, fp, g)
    want, gr = [None] * n_dig, g
    for t in range(n_dig - 1, 0, -1):
        gr, want[t] = oracle.damp_apply2_bwd(tris[t - 1][0], tris[t - 1][1], 3, accs[t - 1], p[t], gr)
    want[0] = gr
    want = np.stack(want).transpose(1, 0, 2).reshape(B, 9)
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=1e-7)
