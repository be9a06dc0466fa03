"""Pins for the CPU oracle's Apply over K Distributions, unary Apply and ApplyIf (no GPU).

Independent checks: the double convolution a sum of three digits is, dictionary
brute force over all symbol tuples for K = 1..4, segment sums for the unary case,
agreement with the separately pinned two-operand routines, finite differences of
a float64 evaluation written here, and for DTKP-AM enumeration of every proof and
composition through an injective pairing function.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads as W

ABSENT = np.uint64(0xFFFFFFFFFFFFFFFF)


def rand_probs(seed, B, n):
    return W.softmax_rows(W.normal(seed, B * n).reshape(B, n))


def rand_table(seed, shape, n_ids, drop_every=0):
    t = (W.splitmix64(seed, np.arange(int(np.prod(shape)))) % np.uint64(n_ids)).astype(np.int32).reshape(shape)
    if drop_every:
        t.reshape(-1)[::drop_every] = -1
    return t


def brute(table, rows):
    """Eq. 1-3 by a dictionary, float64, one sample: {symbol: sum of products} (unclamped)."""
    acc = {}
    for tup in itertools.product(*[range(n) for n in table.shape]):
        s = int(table[tup])
        if s < 0:
            continue
        v = 1.0
        for l, i in enumerate(tup):
            v *= float(rows[l][i])
        acc[s] = acc.get(s, 0.0) + v
    return acc


# ---------------------------------------------------------------- DAMP

def test_sum_of_three_digits_is_a_double_convolution():
    B = 5
    ins = [rand_probs(900 + l, B, 10) for l in range(3)]
    t = np.add.outer(np.add.outer(np.arange(10), np.arange(10)), np.arange(10)).astype(np.int32)
    idx, to = oracle.dense_to_tuples(t)
    syms, out = oracle.damp_applyk_fwd(idx, to, ins)
    assert list(syms) == list(range(28))
    for s in range(B):
        ref = np.convolve(np.convolve(ins[0][s].astype(np.float64), ins[1][s]), ins[2][s])
        np.testing.assert_allclose(out[s], np.minimum(ref, 1.0), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(out.sum(1), 1.0, rtol=1e-6)


@pytest.mark.parametrize("shape,scale", [((7,), 1.0), ((4, 5), 1.0), ((3, 4, 3), 1.0), ((2, 3, 2, 3), 1.0),
                                         ((3, 4, 3), 3.0), ((9,), 8.0)])
def test_dictionary_brute_force(shape, scale):
    B = 4
    K = len(shape)
    ins = [(rand_probs(910 + l, B, n) * scale).astype(np.float32) for l, n in enumerate(shape)]
    table = rand_table(77 + K, shape, 5, drop_every=4)
    idx, to = oracle.dense_to_tuples(table)
    syms, out, pre32, pre64 = oracle.damp_applyk_fwd(idx, to, ins, want_pre=True)
    clamped = 0
    for s in range(B):
        acc = brute(table, [x[s] for x in ins])
        assert sorted(acc) == list(syms)
        for c, sym in enumerate(syms):
            assert abs(pre64[s, c] - acc[sym]) <= 1e-12 * max(1.0, acc[sym])
            assert abs(out[s, c] - min(1.0, acc[sym])) <= 1e-6
            assert abs(pre32[s, c] - acc[sym]) <= 1e-5 * max(1.0, acc[sym])
            clamped += acc[sym] > 1.0
    if scale > 1.0:
        assert clamped > 0


def test_unary_apply_is_a_segment_sum():
    B, n = 6, 23
    x = rand_probs(920, B, n)
    f = (np.arange(n) % 4).astype(np.int32)
    f[5] = -1                                              # ApplyIf rejects symbol 5
    idx, to = oracle.dense_to_tuples(f)
    syms, out = oracle.damp_applyk_fwd(idx, to, [x])
    assert list(syms) == [0, 1, 2, 3]
    keep = f >= 0
    for s in range(B):
        ref = np.bincount(f[keep], weights=x[s, keep].astype(np.float64), minlength=4)
        np.testing.assert_allclose(out[s], np.minimum(ref, 1.0), rtol=1e-6)
    g = W.normal(921, B * 4).reshape(B, 4).astype(np.float32)
    (gx,) = oracle.damp_applyk_bwd(idx, to, [x], g)
    want = np.where(keep[None, :], g[:, np.maximum(f, 0)], 0.0)
    np.testing.assert_array_equal(gx, want.astype(np.float32))


def test_two_operands_agree_with_the_binary_routine():
    B = 7
    a, b = (rand_probs(930, B, 9) * 2.0).astype(np.float32), (rand_probs(931, B, 6) * 2.0).astype(np.float32)
    table = rand_table(5, (9, 6), 7, drop_every=5)
    tri = oracle.dense_to_triples(table)
    idx, to = oracle.dense_to_tuples(table)
    s2, o2, p32, p64 = oracle.damp_apply2_fwd(tri, 9, 6, a, b, want_pre=True)
    sk, ok, k32, k64 = oracle.damp_applyk_fwd(idx, to, [a, b], want_pre=True)
    np.testing.assert_array_equal(s2, sk)
    np.testing.assert_array_equal(o2, ok)
    np.testing.assert_array_equal(p32, k32)
    assert (p32 > 1).any() and (p32 < 1).any()
    g = W.normal(932, B * s2.size).reshape(B, -1).astype(np.float32)
    ga, gb = oracle.damp_apply2_bwd(tri, 9, 6, a, b, g)
    ka, kb = oracle.damp_applyk_bwd(idx, to, [a, b], g)
    np.testing.assert_array_equal(ga, ka)
    np.testing.assert_array_equal(gb, kb)


def test_apply_if_equals_leaving_the_tuples_out():
    B = 3
    ins = [rand_probs(940 + l, B, n) for l, n in enumerate((4, 3, 5))]
    table = rand_table(9, (4, 3, 5), 6)
    cond = (np.add.outer(np.add.outer(np.arange(4), np.arange(3)), np.arange(5)) % 3) != 0
    idx_all = np.argwhere(np.ones_like(table, bool)).astype(np.int32)
    to_all = np.where(cond, table, -1).astype(np.int32)[tuple(idx_all.T)]
    idx_kept, to_kept = oracle.dense_to_tuples(np.where(cond, table, -1))
    assert idx_kept.shape[0] < idx_all.shape[0]
    r1 = oracle.damp_applyk_fwd(idx_all, to_all, ins)
    r2 = oracle.damp_applyk_fwd(idx_kept, to_kept, ins)
    np.testing.assert_array_equal(r1[0], r2[0])
    np.testing.assert_array_equal(r1[1], r2[1])
    g = W.normal(941, B * r1[0].size).reshape(B, -1).astype(np.float32)
    for x, y in zip(oracle.damp_applyk_bwd(idx_all, to_all, ins, g), oracle.damp_applyk_bwd(idx_kept, to_kept, ins, g)):
        np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("shape", [(6,), (4, 3), (3, 4, 3), (2, 3, 2, 3)])
def test_gradient_matches_finite_differences(shape):
    K = len(shape)
    ins = [rand_probs(950 + l, 1, n) for l, n in enumerate(shape)]
    table = rand_table(31 + K, shape, 4, drop_every=7)
    idx, to = oracle.dense_to_tuples(table)
    syms, out, pre32, _ = oracle.damp_applyk_fwd(idx, to, ins, want_pre=True)
    assert (pre32 < 1).all()
    g = W.normal(951, syms.size).reshape(1, -1).astype(np.float32)
    grads = oracle.damp_applyk_bwd(idx, to, ins, g)

    def loss(rows):
        acc = brute(table, rows)
        return sum(float(g[0, c]) * acc[int(sym)] for c, sym in enumerate(syms))

    h = 1e-6
    for l in range(K):
        for i in range(shape[l]):
            hi = [x[0].astype(np.float64).copy() for x in ins]
            lo = [x[0].astype(np.float64).copy() for x in ins]
            hi[l][i] += h
            lo[l][i] -= h
            fd = (loss(hi) - loss(lo)) / (2 * h)
            assert abs(fd - grads[l][0, i]) <= 1e-5 * max(1.0, abs(fd))


def test_clamped_columns_pass_no_gradient():
    B = 5
    shape = (4, 3, 4)
    ins = [(rand_probs(960 + l, B, n) * 1.45).astype(np.float32) for l, n in enumerate(shape)]
    table = rand_table(12, shape, 3)
    idx, to = oracle.dense_to_tuples(table)
    syms, out, pre32, pre64 = oracle.damp_applyk_fwd(idx, to, ins, want_pre=True)
    assert (pre64 > 1.001).any() and (pre64 < 0.999).any() and (np.abs(pre64 - 1) > 1e-3).all()
    g = W.normal(961, B * syms.size).reshape(B, -1).astype(np.float32)
    got = oracle.damp_applyk_bwd(idx, to, ins, g)
    gated = np.where(pre64 <= 1.0, g, 0.0).astype(np.float32)
    for s in range(B):
        for l in range(3):
            for i in range(shape[l]):
                want = 0.0
                for tup in itertools.product(*[range(n) for n in shape]):
                    if tup[l] != i:
                        continue
                    c = int(np.searchsorted(syms, table[tup]))
                    others = 1.0
                    for m in range(3):
                        if m != l:
                            others *= float(ins[m][s, tup[m]])
                    want += float(gated[s, c]) * others
                assert abs(got[l][s, i] - want) <= 1e-5 * max(1.0, abs(want))


# ---------------------------------------------------------------- DTKP-AM

def digit_tags(seed, B, n_slots, n_val, k):
    """n_slots Distributions over n_val values each, one fact per (slot, value), naturally initialised."""
    fp = np.concatenate([rand_probs(seed + t, B, n_val) for t in range(n_slots)], axis=1)
    grp = np.repeat(np.arange(n_slots), n_val).astype(np.int32)
    tags = []
    for t in range(n_slots):
        m, _, _ = oracle.dtkp_init(np.arange(n_val) + n_val * t, fp, k)
        tags.append(m)
    return fp, grp, tags


def test_dtkp_two_operands_agree_with_the_binary_routine():
    B, k = 4, 3
    fp, grp, tags = digit_tags(970, B, 2, 5, k)
    table = rand_table(15, (5, 5), 4, drop_every=6)
    r2 = oracle.dtkp_apply2(oracle.dense_to_triples(table), 5, 5, k, grp, fp, tags[0], tags[1])
    idx, to = oracle.dense_to_tuples(table)
    rk = oracle.dtkp_applyk(idx, to, k, grp, fp, tags)
    for x, y in zip(r2, rk):
        np.testing.assert_array_equal(x, y)


def test_dtkp_unary_merges_the_proofs_of_symbols_with_one_image():
    B, k = 5, 3
    fp, grp, tags = digit_tags(975, B, 2, 4, k)
    sum_t = np.add.outer(np.arange(4), np.arange(4)).astype(np.int32)
    idx2, to2 = oracle.dense_to_tuples(sum_t)
    syms, m, pp, pr = oracle.dtkp_applyk(idx2, to2, k, grp, fp, tags)      # 7 symbols, up to 3 proofs each
    f = np.array([0, 1, 0, -1, 1, 0, 2], np.int32)
    idx1, to1 = oracle.dense_to_tuples(f)
    s1, m1, p1, pr1 = oracle.dtkp_applyk(idx1, to1, k, grp, fp, [m])
    assert list(s1) == [0, 1, 2]
    for s in range(B):
        for c, sym in enumerate(s1):
            proofs = {}
            for i in np.nonzero(f == sym)[0]:
                for x in range(k):
                    if m[s, i, x] != ABSENT:
                        proofs[int(m[s, i, x])] = pp[s, i, x]
            order = sorted(proofs, key=lambda q: (-float(proofs[q]), q))[:k]
            assert [int(v) for v in m1[s, c]] == order + [int(ABSENT)] * (k - len(order))
            tot = np.float32(0)
            for q in order:
                tot = np.float32(tot + proofs[q])
            assert pr1[s, c] == min(np.float32(1), tot)


def test_dtkp_three_operands_without_pruning_enumerate_every_proof():
    B, k, nv = 3, 8, 3
    fp, grp, tags = digit_tags(980, B, 3, nv, k)
    t = np.add.outer(np.add.outer(np.arange(nv), np.arange(nv)), np.arange(nv)).astype(np.int32)
    idx, to = oracle.dense_to_tuples(t)
    syms, m, pp, pr = oracle.dtkp_applyk(idx, to, k, grp, fp, tags)       # at most 7 tuples per sum: nothing pruned
    _, damp = oracle.damp_applyk_fwd(idx, to, [fp[:, nv * l:nv * (l + 1)] for l in range(3)])
    np.testing.assert_allclose(pr, damp, rtol=1e-6, atol=1e-9)
    for s in range(B):
        for c, sym in enumerate(syms):
            want = {}
            for tup in itertools.product(range(nv), repeat=3):
                if sum(tup) != sym:
                    continue
                mask = sum(1 << (nv * l + v) for l, v in enumerate(tup))
                p = np.float32(1)
                for l, v in enumerate(tup):
                    p = np.float32(p * fp[s, nv * l + v])
                want[mask] = p
            order = sorted(want, key=lambda q: (-float(want[q]), q))
            assert [int(v) for v in m[s, c][:len(order)]] == order
            assert (m[s, c][len(order):] == ABSENT).all()
            np.testing.assert_array_equal(pp[s, c][:len(order)], np.array([want[q] for q in order], np.float32))


def test_dtkp_three_operands_fold_left_through_an_injective_pairing():
    B, k = 4, 2
    fp, grp, tags = digit_tags(985, B, 4, 3, k)
    # operand 0: sums of slots 0 and 1 (up to 2 proofs per symbol); operands 1, 2: slots 2 and 3
    sum_t = np.add.outer(np.arange(3), np.arange(3)).astype(np.int32)
    _, a, _, _ = oracle.dtkp_apply2(oracle.dense_to_triples(sum_t), 3, 3, k, grp, fp, tags[0], tags[1])
    na = a.shape[1]
    f3 = rand_table(21, (na, 3, 3), 5, drop_every=5)
    idx, to = oracle.dense_to_tuples(f3)
    got = oracle.dtkp_applyk(idx, to, k, grp, fp, [a, tags[2], tags[3]])
    # the same function through pair symbols: (i, j) -> 3*i + j keeps every intermediate tag apart
    pair = (3 * np.arange(na)[:, None] + np.arange(3)[None, :]).astype(np.int32)
    ps, pm, _, _ = oracle.dtkp_apply2(oracle.dense_to_triples(pair), na, 3, k, grp, fp, a, tags[2])
    assert list(ps) == list(range(3 * na))
    want = oracle.dtkp_apply2(oracle.dense_to_triples(f3.reshape(3 * na, 3)), 3 * na, 3, k, grp, fp, pm, tags[3])
    for x, y in zip(got, want):
        np.testing.assert_array_equal(x, y)
