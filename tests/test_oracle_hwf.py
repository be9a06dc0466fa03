"""Pins for the formula pipeline (no GPU): the symbol-side tables against Python's own expression evaluation, the
DAMP result against enumeration of every formula, its gradient against finite differences, the DTKP-AM result
against a brute-force top-k over all formulas."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W
from oracle import programs as P

ABSENT = np.uint64(0xFFFFFFFFFFFFFFFF)
ALPHABET = [str(d) for d in range(10)] + list(W.HWF_OPS)


def python_value(tokens):
    """The formula's value by Python's parser over exact rationals; None for a division by zero."""
    src = "".join("Fraction(%s)" % t if t.isdigit() else t for t in tokens)
    try:
        return eval(src, {"Fraction": Fraction})        # noqa: S307 (test-side arithmetic on generated digits/operators)
    except ZeroDivisionError:
        return None


def all_formulas(L):
    kinds = [range(10) if pos % 2 == 0 else range(10, 14) for pos in range(L)]
    return itertools.product(*kinds)


def walk(tables, final_map, classes):
    """Follow the tables from the first digit through every later class (position-local index) to the value index."""
    st = classes[0]
    for pos in range(1, len(classes)):
        st = tables[pos - 1][st, classes[pos] - (10 if pos % 2 else 0)]
    return final_map[st]


@pytest.mark.parametrize("L", [1, 3, 5])
def test_tables_agree_with_python_evaluation_on_every_formula(L):
    states, tables, values, final_map = W.hwf_symbol_tables(L)
    seen = set()
    for classes in all_formulas(L):
        v = python_value([ALPHABET[c] for c in classes])
        got = values[walk(tables, final_map, classes)]
        assert got == v, (classes, got, v)
        seen.add(v)
    assert seen == set(values)
    fr = [v for v in values if v is not None]
    assert fr == sorted(fr) and (None not in values or values[-1] is None)


def test_tables_agree_with_python_evaluation_on_sampled_long_formulas():
    L = 7
    states, tables, values, final_map = W.hwf_symbol_tables(L)
    draws = W.splitmix64(99, np.arange(3000 * L)).reshape(3000, L)
    for row in draws:
        classes = [int(r % 10) if pos % 2 == 0 else 10 + int(r % 4) for pos, r in enumerate(row)]
        assert values[walk(tables, final_map, classes)] == python_value([ALPHABET[c] for c in classes])
    for pos, tab in enumerate(tables):
        assert tab.shape == (len(states[pos]), 4 if pos % 2 == 0 else 10)
        assert sorted(set(tab.reshape(-1))) == list(range(len(states[pos + 1])))


def enumerate_values(w, L):
    """{value index: list of (formula classes, float64 probability per sample)} over every formula."""
    p = w["p"].astype(np.float64)
    values = w["values"]
    vidx = {v: i for i, v in enumerate(values)}
    table = {}
    for classes in all_formulas(L):
        pr = np.ones(p.shape[0])
        for pos, c in enumerate(classes):
            pr = pr * p[:, pos, c]
        table.setdefault(vidx[python_value([ALPHABET[c] for c in classes])], []).append((classes, pr))
    return table


@pytest.mark.parametrize("L", [3, 5])
def test_damp_pipeline_equals_enumeration(L):
    w = W.hwf_workload(batch=3, length=L, seed=L)
    r = P.hwf_pipeline_damp(w)
    table = enumerate_values(w, L)
    want = np.zeros((3, len(w["values"])))
    for v, items in table.items():
        for _, pr in items:
            want[:, v] += pr
    np.testing.assert_allclose(r["out"], np.minimum(want, 1.0), rtol=1e-6, atol=1e-10)
    assert list(r["syms"]) == list(range(len(w["values"])))
    # classes a position does not admit carry no gradient
    for pos in range(L):
        assert np.all(r["grad_p"][:, pos, w["keep"][pos] == 0] == 0)


def test_damp_pipeline_gradient_matches_finite_differences():
    L = 3
    w = W.hwf_workload(batch=2, length=L, seed=11)
    r = P.hwf_pipeline_damp(w)
    g = w["g"].astype(np.float64)

    def loss(p, s):
        tot = 0.0
        vidx = {v: i for i, v in enumerate(w["values"])}
        for classes in all_formulas(L):
            v = vidx[python_value([ALPHABET[c] for c in classes])]
            tot += g[s, v] * np.prod([p[s, pos, c] for pos, c in enumerate(classes)])
        return tot

    p = w["p"].astype(np.float64)
    h = 1e-6
    for s in range(2):
        for pos, c in [(0, 0), (0, 7), (1, 10), (1, 13), (2, 0), (2, 5)]:
            hi, lo = p.copy(), p.copy()
            hi[s, pos, c] += h
            lo[s, pos, c] -= h
            fd = (loss(hi, s) - loss(lo, s)) / (2 * h)
            assert abs(fd - r["grad_p"][s, pos, c]) <= 1e-5 * max(1.0, abs(fd))


@pytest.mark.parametrize("L,k", [(3, 3), (5, 3), (5, 1)])
def test_dtkp_pipeline_equals_brute_force_top_k(L, k):
    B = 2
    w = W.hwf_workload(batch=B, length=L, k=k, seed=20 + L)
    r = P.hwf_pipeline_dtkp(w)
    off = r["fact_offset"]
    assert off[-1] == 10 * ((L + 1) // 2) + 4 * (L // 2)
    p32 = w["p"]
    vidx = {v: i for i, v in enumerate(w["values"])}
    cands = {}
    for classes in all_formulas(L):
        mask, pr = 0, np.ones(B, np.float32)
        for pos, c in enumerate(classes):                    # ascending position = ascending fact number
            mask |= 1 << (int(off[pos]) + c - (10 if pos % 2 else 0))
            pr = (pr * p32[:, pos, c]).astype(np.float32)
        cands.setdefault(vidx[python_value([ALPHABET[c] for c in classes])], []).append((mask, pr))
    checked = 0
    for s in range(B):
        for v, items in cands.items():
            order = sorted(items, key=lambda it: (-float(it[1][s]), it[0]))
            if len(order) > k and order[k][1][s] == order[k - 1][1][s]:
                continue                                      # float tie at the cut
            top = order[:k]
            want_m = [it[0] for it in top] + [int(ABSENT)] * (k - len(top))
            assert [int(x) for x in r["mask"][s, v]] == want_m
            np.testing.assert_array_equal(r["pprob"][s, v][:len(top)], np.array([it[1][s] for it in top], np.float32))
            tot = np.float32(0)
            for it in top:
                tot = np.float32(tot + it[1][s])
            assert r["prob"][s, v] == min(np.float32(1), tot)
            checked += 1
    assert checked >= 0.95 * B * len(cands)
