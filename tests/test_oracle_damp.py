"""Pins for the CPU oracle's DAMP operators (no GPU).

Each test checks the oracle against something other than itself: values the
paper prints, closed forms (discrete convolution), brute-force enumeration of
all symbol tuples, invariants, and finite differences of an independent float64
evaluation written here with Python dicts.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads as W
from oracle import programs as P


# ---------------------------------------------------------------- independent helpers

def brute_apply(table, a, b):
    """Eq. 1-3 by dictionaries, float64, one sample: {symbol: sum of a[i]*b[j]} (unclamped)."""
    acc = {}
    for i in range(table.shape[0]):
        for j in range(table.shape[1]):
            s = int(table[i, j])
            if s < 0:
                continue
            acc[s] = acc.get(s, 0.0) + float(a[i]) * float(b[j])
    return acc


def rand_probs(seed, B, n):
    return W.softmax_rows(W.normal(seed, B * n).reshape(B, n))


# ---------------------------------------------------------------- paper examples

def test_paper_example_3_2(golden):
    d1 = np.array([golden["ex31_d1"]], np.float32)
    d2 = np.array([golden["ex31_d2"]], np.float32)
    syms, out = oracle.damp_apply2_fwd(oracle.dense_to_triples(W.sum_table(range(10), range(10))), 10, 10, d1, d2)
    assert syms.size == int(golden["ex32_n_symbols"][0])
    assert list(syms) == list(range(19))
    assert abs(out[0, 1] - golden["ex32_out1_exact"][0]) < 1e-6
    assert round(float(out[0, 1]), 2) == golden["ex32_out1_2dp"][0]
    assert round(float(out[0, 0]), 2) == golden["ex32_out0_2dp"][0]
    assert round(float(out[0, 18]), 2) == golden["ex32_out18_2dp"][0]


def test_paper_example_3_3_filter(golden):
    x = np.array([golden["ex33_in"]], np.float32)
    pred = (np.arange(10) % 2 == 0).astype(np.uint8)
    syms, idx = oracle.filter_plan(np.arange(10), pred)
    assert list(syms) == [int(v) for v in golden["ex33_syms"]]
    out = oracle.damp_filter_fwd(pred, x)
    assert out.shape == (1, 5)
    assert out[0, 0] == np.float32(golden["ex33_out0"][0])
    assert out[0, 1] == np.float32(golden["ex33_out2"][0])
    assert out[0, 4] == np.float32(golden["ex33_out8"][0])
    assert list(idx) == [0, 2, 4, 6, 8]


def test_paper_union_example(golden):
    sa = np.array(golden["union_a_syms"], np.int32)
    sb = np.array(golden["union_b_syms"], np.int32)
    a = np.array([golden["union_a_tags"]], np.float32)
    b = np.array([golden["union_b_tags"]], np.float32)
    syms, ia, ib = oracle.union_plan(sa, sb)
    assert list(syms) == [int(v) for v in golden["union_out_syms"]]
    out = oracle.damp_union_fwd(ia, ib, a, b)
    np.testing.assert_allclose(out[0], np.array(golden["union_out_tags"], np.float32), rtol=0, atol=1e-7)


def test_sumn_label_count(golden):
    mult, add = (int(v) for v in golden["sumn_labels_per_n"])
    for n in (2, 3, 5):
        w = W.config2(batch=3, n_digits=n, seed=n)
        r = P.sum_chain_fwd_bwd(w, want_bwd=False)
        assert r["syms"].size == mult * n + add
        assert list(r["syms"]) == list(range(mult * n + add))


# ---------------------------------------------------------------- closed forms / brute force

def test_sum2_is_discrete_convolution():
    w = W.config1(batch=64, seed=3)
    r = P.sum2_fwd(w)
    for s in range(64):
        ref = np.convolve(w["pa"][s].astype(np.float64), w["pb"][s].astype(np.float64))
        np.testing.assert_allclose(r["out"][s], ref, rtol=2e-7, atol=1e-9)


def test_convolution_is_order_sensitive():
    """Operands of different sizes: a transposed operand or swapped index would not fit/agree."""
    a, b = rand_probs(11, 5, 7), rand_probs(12, 5, 4)
    syms, out = oracle.damp_apply2_fwd(oracle.dense_to_triples(W.sum_table(range(7), range(4))), 7, 4, a, b)
    assert list(syms) == list(range(10))
    for s in range(5):
        np.testing.assert_allclose(out[s], np.convolve(a[s].astype(np.float64), b[s].astype(np.float64)), rtol=2e-7)


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_sum_chain_matches_enumeration_of_all_tuples(n):
    """All 10^N digit tuples (Sec. 2: 10^N states): P(sum=s) = sum over tuples of the product."""
    w = W.config2(batch=4, n_digits=n, seed=20 + n)
    r = P.sum_chain_fwd_bwd(w, want_bwd=False)
    p = w["p"].astype(np.float64)          # [n, B, 10]
    digits = np.array(list(itertools.product(range(10), repeat=n)))     # [10^n, n]
    sums = digits.sum(1)
    for s in range(4):
        prod = np.ones(len(digits))
        for t in range(n):
            prod *= p[t, s, digits[:, t]]
        ref = np.bincount(sums, weights=prod, minlength=9 * n + 1)
        np.testing.assert_allclose(r["out"][s], ref, rtol=1e-6, atol=1e-12)


def test_random_table_matches_dict_brute_force():
    na, nb = 6, 9
    tab = W.hashed_table(5, na, nb, 13)
    tab[2, 3] = -1          # an ApplyIf-rejected tuple
    tab[5, 8] = -1
    a, b = rand_probs(1, 8, na), rand_probs(2, 8, nb)
    syms, out, pre32, pre64 = oracle.damp_apply2_fwd(oracle.dense_to_triples(tab), na, nb, a, b, want_pre=True)
    for s in range(8):
        ref = brute_apply(tab, a[s], b[s])
        assert sorted(ref) == list(syms)
        np.testing.assert_allclose(pre64[s], [ref[k] for k in sorted(ref)], rtol=1e-14)
        np.testing.assert_allclose(out[s], [min(1.0, ref[k]) for k in sorted(ref)], rtol=1e-7)
        np.testing.assert_allclose(pre32[s], pre64[s], rtol=1e-6)


def test_mass_is_conserved_without_drops():
    w = W.config3(batch=32, seed=9)
    syms, out = oracle.damp_apply2_fwd(oracle.dense_to_triples(w["table"]), 64, 64, w["pa"], w["pb"])
    assert syms.size <= 256 and np.all(np.diff(syms) > 0)
    np.testing.assert_allclose(out.astype(np.float64).sum(1), 1.0, atol=2e-6)


def test_constant_function_gives_one_symbol_with_all_mass():
    a, b = rand_probs(3, 4, 5), rand_probs(4, 4, 6)
    syms, out = oracle.damp_apply2_fwd(oracle.dense_to_triples(np.full((5, 6), 42, np.int32)), 5, 6, a, b)
    assert list(syms) == [42]
    np.testing.assert_allclose(out[:, 0], 1.0, atol=3e-7)


def test_disjunction_clamps_at_one():
    """Table 1: t (+) t' = clamp(t + t').  Tags 0.7,0.6 against 1,1 all landing on one symbol -> 1."""
    a = np.array([[0.7, 0.6]], np.float32)
    b = np.array([[1.0]], np.float32)
    syms, out, pre32, pre64 = oracle.damp_apply2_fwd(oracle.dense_to_triples(np.zeros((2, 1), np.int32)), 2, 1, a, b,
                                                     want_pre=True)
    assert out[0, 0] == 1.0 and abs(pre64[0, 0] - 1.3) < 1e-6 and pre32[0, 0] > 1.0


def test_out_syms_sorted_unique():
    assert list(oracle.out_syms(np.array([5, -1, 3, 5, 0, 3], np.int32))) == [0, 3, 5]
    assert oracle.out_syms(np.array([-1, -1], np.int32)).size == 0


def test_rejects_unsorted_tuples():
    with pytest.raises(ValueError):
        oracle.damp_apply2_fwd((np.array([1, 0]), np.array([0, 0]), np.array([0, 0])), 2, 1,
                               np.ones((1, 2), np.float32), np.ones((1, 1), np.float32))


# ---------------------------------------------------------------- backward

def f64_loss(table, a, b, g):
    """sum_c g_c * min(1, pre_c) in float64 for one sample, by the dict brute force."""
    acc = brute_apply(table, a, b)
    return sum(float(g[n]) * min(1.0, acc[k]) for n, k in enumerate(sorted(acc)))


def test_apply_backward_matches_finite_differences():
    na, nb = 5, 7
    tab = W.hashed_table(77, na, nb, 9)
    tab[1, 1] = -1
    a, b = rand_probs(5, 3, na), rand_probs(6, 3, nb)
    S = oracle.out_syms(tab[tab >= 0]).size
    g = W.normal(8, 3 * S).astype(np.float32).reshape(3, S)
    ga, gb = oracle.damp_apply2_bwd(oracle.dense_to_triples(tab), na, nb, a, b, g)
    h = 1e-6
    for s in range(3):
        a64, b64 = a[s].astype(np.float64), b[s].astype(np.float64)
        for i in range(na):
            e = np.zeros(na); e[i] = h
            fd = (f64_loss(tab, a64 + e, b64, g[s]) - f64_loss(tab, a64 - e, b64, g[s])) / (2 * h)
            assert abs(fd - ga[s, i]) < 1e-6 + 1e-5 * abs(fd)
        for j in range(nb):
            e = np.zeros(nb); e[j] = h
            fd = (f64_loss(tab, a64, b64 + e, g[s]) - f64_loss(tab, a64, b64 - e, g[s])) / (2 * h)
            assert abs(fd - gb[s, j]) < 1e-6 + 1e-5 * abs(fd)


def test_apply_backward_euler_identity():
    """pre is bilinear: sum_i a_i ga_i = sum_c gh_c pre_c = sum_j b_j gb_j (no clamping here)."""
    w = W.config3(batch=16, seed=4)
    tri = oracle.dense_to_triples(w["table"])
    syms, out, pre32, pre64 = oracle.damp_apply2_fwd(tri, 64, 64, w["pa"], w["pb"], want_pre=True)
    g = w["g"][:, :syms.size]
    ga, gb = oracle.damp_apply2_bwd(tri, 64, 64, w["pa"], w["pb"], g)
    lhs_a = (w["pa"].astype(np.float64) * ga).sum(1)
    lhs_b = (w["pb"].astype(np.float64) * gb).sum(1)
    rhs = (g.astype(np.float64) * pre64).sum(1)
    np.testing.assert_allclose(lhs_a, rhs, rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(lhs_b, rhs, rtol=1e-5, atol=1e-7)


def test_clamp_gradient_convention():
    """App. A.2: gradient 1 inside the clamp and on its boundary, 0 beyond.  a+b = 0.875, 1.0, 1.125
    (exact in binary) through apply with a one-symbol function and through union."""
    for total, want in ((0.875, 1.0), (1.0, 1.0), (1.125, 0.0)):
        a = np.array([[0.5, total - 0.5]], np.float32)
        b = np.array([[1.0]], np.float32)
        g = np.array([[2.0]], np.float32)
        ga, gb = oracle.damp_apply2_bwd(oracle.dense_to_triples(np.zeros((2, 1), np.int32)), 2, 1, a, b, g)
        np.testing.assert_array_equal(ga[0], [2.0 * want, 2.0 * want])
        assert gb[0, 0] == np.float32(2.0 * want * total)
        ua, ub = np.array([[0.5]], np.float32), np.array([[total - 0.5]], np.float32)
        _, ia, ib = oracle.union_plan([7], [7])
        assert oracle.damp_union_fwd(ia, ib, ua, ub)[0, 0] == np.float32(min(1.0, total))
        gua, gub = oracle.damp_union_bwd(ia, ib, ua, ub, g)
        assert gua[0, 0] == 2.0 * want and gub[0, 0] == 2.0 * want


def test_chain_gradient_closed_forms():
    """loss = -log p[target].  d p[target] / d p_n[d] = (convolution of the other rows)[target - d]."""
    n = 4
    w = W.config2(batch=6, n_digits=n, seed=31)
    w.arrays["target"][0] = 0          # all-zero digits is the only way to sum to 0
    r = P.sum_chain_fwd_bwd(w)
    p = w["p"].astype(np.float64)
    for s in range(6):
        tgt = int(w["target"][s])
        ptgt = float(r["out"][s, tgt])
        for t in range(n):
            others = np.array([1.0])
            for u in range(n):
                if u != t:
                    others = np.convolve(others, p[u, s])
            for d in range(10):
                k = tgt - d
                dp = others[k] if 0 <= k < others.size else 0.0
                want = -dp / ptgt
                got = r["grad_p"][t, s, d]
                assert abs(got - want) <= 1e-6 * abs(want) + 1e-30
    # target 0: only digit 0 of each row gets gradient, equal to -1/p_n[0]
    for t in range(n):
        assert np.all(r["grad_p"][t, 0, 1:] == 0)
        np.testing.assert_allclose(r["grad_p"][t, 0, 0], -1.0 / p[t, 0, 0], rtol=1e-6)


# ---------------------------------------------------------------- filter / union

def test_filter_identity_and_transpose():
    x = rand_probs(9, 4, 11)
    ones = np.ones(11, np.uint8)
    np.testing.assert_array_equal(oracle.damp_filter_fwd(ones, x), x)
    pred = W.keep_mask(3, 11)
    out = oracle.damp_filter_fwd(pred, x)
    np.testing.assert_array_equal(out, x[:, pred.astype(bool)])
    g = W.normal(1, 4 * out.shape[1]).astype(np.float32).reshape(4, -1)
    gi = oracle.damp_filter_bwd(pred, g)
    assert np.all(gi[:, ~pred.astype(bool)] == 0)
    np.testing.assert_array_equal(gi[:, pred.astype(bool)], g)
    none = np.zeros(11, np.uint8)
    assert oracle.damp_filter_fwd(none, x).shape == (4, 0)


def test_union_with_empty_is_identity_and_one_sided_copy():
    x = rand_probs(10, 3, 5)
    syms, ia, ib = oracle.union_plan([1, 4, 6, 8, 9], [])
    assert list(syms) == [1, 4, 6, 8, 9] and np.all(ib == -1)
    np.testing.assert_array_equal(oracle.damp_union_fwd(ia, ib, x, np.zeros((3, 0), np.float32)), x)
    y = rand_probs(11, 3, 3)
    syms, ia, ib = oracle.union_plan([1, 4, 6, 8, 9], [0, 4, 9])
    assert list(syms) == [0, 1, 4, 6, 8, 9]
    out = oracle.damp_union_fwd(ia, ib, x, y)
    np.testing.assert_array_equal(out[:, 0], y[:, 0])
    np.testing.assert_array_equal(out[:, 1], x[:, 0])
    np.testing.assert_allclose(out[:, 2], np.minimum(1.0, x[:, 1].astype(np.float64) + y[:, 1]), rtol=1e-7)
    g = W.normal(2, 3 * 6).astype(np.float32).reshape(3, 6)
    ga, gb = oracle.damp_union_bwd(ia, ib, x, y, g)
    np.testing.assert_array_equal(ga[:, 0], g[:, 1])
    np.testing.assert_array_equal(gb[:, 0], g[:, 0])


def test_config3_pipeline_shapes_and_mass():
    w = W.config3(batch=8, seed=0)
    r = P.hashed_pipeline_fwd_bwd(w)
    keep = w["keep"].astype(bool)
    assert list(r["s2"]) == [int(s) for s in r["s1"] if keep[s]]
    assert list(r["s3"]) == list(range(256))
    # union output = p2 + (kept apply mass), nothing near the clamp
    tot = r["o3"].astype(np.float64).sum(1)
    np.testing.assert_allclose(tot, 1.0 + r["o2"].astype(np.float64).sum(1), rtol=1e-6)
    assert r["ga"].shape == (8, 64) and r["gb"].shape == (8, 64) and r["gp2"].shape == (8, 256)


# ---------------------------------------------------------------- Product-N fold

def test_product_chain_zero_probability_closed_form_and_enumeration():
    """Pr(product = 0) = 1 - prod_t (1 - p_t[0]); every other value by enumeration of all digit tuples."""
    B, n = 4, 4
    w = W.product_workload(batch=B, n_digits=n, seed=3)
    r = P.product_chain_fwd_bwd(w, want_bwd=False)
    p = w["p"].astype(np.float64)
    values = w["values"]
    assert values[0] == 0 and list(r["syms"]) == list(range(len(values)))
    np.testing.assert_allclose(r["out"][:, 0], 1.0 - np.prod(1.0 - p[:, :, 0], axis=0), rtol=1e-6)
    want = np.zeros((B, len(values)))
    col = {v: c for c, v in enumerate(values)}
    for tup in itertools.product(range(10), repeat=n):
        v = int(np.prod(tup))
        pr = np.ones(B)
        for t, d in enumerate(tup):
            pr = pr * p[t, :, d]
        want[:, col[v]] += pr
    np.testing.assert_allclose(r["out"], want, rtol=1e-6, atol=1e-10)
    np.testing.assert_allclose(r["out"].sum(1), 1.0, rtol=1e-6)


def test_product_stage_symbol_counts():
    """Distinct products of t digits: 10, 37, 101, 226 (counted here from scratch by enumeration)."""
    _, stage_ids, tables = W.product_stage_tables(4)
    for t, ids in enumerate(stage_ids):
        vals = {int(np.prod(tup)) for tup in itertools.product(range(10), repeat=t + 1)}
        assert ids.size == len(vals)
    assert [tb.shape for tb in tables] == [(10, 10), (37, 10), (101, 10)]


def test_product_chain_gradient_matches_finite_differences():
    B, n = 2, 3
    w = W.product_workload(batch=B, n_digits=n, seed=5)
    r = P.product_chain_fwd_bwd(w)
    p = w["p"].astype(np.float64)
    values = w["values"]
    tgt = w["target"]

    def loss(pp, s):
        tot = 0.0
        for tup in itertools.product(range(10), repeat=n):
            if int(np.prod(tup)) == values[tgt[s]]:
                tot += np.prod([pp[t, s, d] for t, d in enumerate(tup)])
        return -np.log(tot)

    h = 1e-6
    for s in range(B):
        for t in range(n):
            for d in (0, 3, 7):
                hi, lo = p.copy(), p.copy()
                hi[t, s, d] += h
                lo[t, s, d] -= h
                fd = (loss(hi, s) - loss(lo, s)) / (2 * h)
                assert abs(fd - r["grad_p"][t, s, d]) <= 2e-4 * max(1.0, abs(fd))
