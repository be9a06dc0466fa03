"""Parity of the HIP library against the CPU oracle, element by element, through the C ABI (needs an MI355X).

Floating-point bar: |gpu - oracle| <= 1e-7 + 1e-5 * |oracle| (oracle accumulates in float64).
Integer / index / proof-mask bar: bit-exact.
Stress cases with unnormalised tags use a one-signed upstream gradient: a float32 sum of mixed-sign terms of order 1
cannot meet an absolute 1e-7 where it cancels to ~0, whatever the kernel.
"""
import numpy as np
import pytest

import oracle
import workloads as W
from oracle import programs as OP

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_03348_amd import programs
    return programs


@pytest.fixture(scope="module")
def dol():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_03348_amd import binding
    return binding


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def assert_close(got, want, what=""):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    err = np.abs(got - want)
    tol = 1e-7 + 1e-5 * np.abs(want)
    bad = err > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst excess %g at %s" % (
        what, int(bad.sum()), bad.size, float((err - tol).max()), np.unravel_index(np.argmax(err - tol), err.shape))


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


# ---------------------------------------------------------------- config 1

@pytest.mark.parametrize("batch", [64, 1, 257])
def test_config1_sum2(gp, batch):
    w = W.config1(batch=batch, seed=batch)
    ref = OP.sum2_fwd(w)
    prog = gp.Sum2Forward(w)
    prog.forward()
    out = prog.out
    np.testing.assert_array_equal(out.sym_ids, ref["syms"])
    assert_close(host(out.prob), ref["out"], "sum2")


# ---------------------------------------------------------------- config 2

@pytest.mark.parametrize("batch,n", [(4096, 15), (300, 15), (37, 4), (1, 2)])
def test_config2_sum_chain(gp, batch, n):
    w = W.config2(batch=batch, n_digits=n, seed=n)
    ref = OP.sum_chain_fwd_bwd(w)
    prog = gp.SumChain(w)
    prog.step()
    np.testing.assert_array_equal(prog.accs[-1].sym_ids, ref["syms"])
    for t in range(1, n):
        assert_close(host(prog.accs[t].prob), ref["accs"][t], "chain stage %d" % t)
    assert_close(host(prog.g_acc[-1]), ref["g_out"], "loss gradient")
    assert_close(host(prog.grad_p), ref["grad_p"], "chain grad")


@pytest.mark.parametrize("batch,n", [(4096, 15), (301, 15), (37, 4), (1, 2), (64, 32), (6401, 15), (8192, 6)])
def test_config2_fused_fold(gp, batch, n):
    """dol_fold_apply2: the same results as the chain of per-operator calls, and as the oracle.  The two largest batches
    take the form of the kernel that keeps the reverse sweep's operands in registers."""
    w = W.config2(batch=batch, n_digits=n, seed=n + 100)
    ref = OP.sum_chain_fwd_bwd(w)
    prog = gp.SumChainFused(w)
    prog.step()
    np.testing.assert_array_equal(prog.out.sym_ids, ref["syms"])
    assert_close(host(prog.out.prob), ref["out"], "fold forward")
    assert_close(host(prog.grad_p), ref["grad_p"], "fold grad")
    chain = gp.SumChain(w)
    chain.step()
    np.testing.assert_array_equal(host(prog.out.prob), host(chain.accs[-1].prob))    # same arithmetic, bit for bit


@pytest.mark.parametrize("batch,n,pad", [(1, 1, 0), (5, 3, 0), (1000, 19, 0), (4099, 136, 0), (333, 2050, 0), (70, 19, 5)])
def test_nll_grad(dol, batch, n, pad):
    """dol_nll_grad: -1 / max(p[target], FLT_MIN) at the target, zero elsewhere; rows that are not a multiple of 16 bytes,
    a last workgroup with fewer rows, a padded tensor (the element-wise kernel), a tag of zero."""
    p = W.uniform01(3, batch * n).astype(np.float32).reshape(batch, n)
    target = (np.arange(batch) * 7 % n).astype(np.int32)
    p[0, target[0]] = 0.0
    buf = torch.full((batch, n + pad), 9.0, device="cuda")
    buf[:, :n] = dev(p)
    grad = torch.full((batch, n + pad), 7.0, device="cuda")
    dol.nll_grad(dol.Dist(np.arange(n), buf[:, :n]), dev(target), grad[:, :n])
    want = np.zeros((batch, n), np.float32)
    want[np.arange(batch), target] = np.float32(-1.0) / np.maximum(p[np.arange(batch), target], np.float32(1.17549435e-38))
    got = host(grad)
    np.testing.assert_array_equal(got[:, :n] != 0, want != 0)
    assert_close(got[:, :n], want, "nll gradient")
    assert np.all(got[:, n:] == 7.0)


@pytest.mark.parametrize("widths", [[7, 3, 10, 16, 2], [5, 1, 9, 4, 13, 6, 11]])
@pytest.mark.parametrize("B", [77, 6203])
def test_fused_fold_with_clamping_and_explicit_gradient(dol, B, widths):
    """Unnormalised tags drive several stages over 1; the fold must gate exactly like the per-operator path.
    Also: explicit upstream gradient, padded leading dimensions, mixed operand widths, forward-only call.  The larger
    batch takes the kernel's other form (history in registers); the second list of widths covers second operands of
    1, 4, 6, 9, 11 and 13 symbols (how the lanes share out a short operand's gradient sums depends on that count)."""
    ins = [(W.uniform01(10 + t, B * n) * 0.9).astype(np.float32).reshape(B, n) for t, n in enumerate(widths)]
    syms = [np.arange(n, dtype=np.int32) for n in widths]
    tabs, tris, accs, cur = [], [], [ins[0]], syms[0]
    for t in range(1, len(widths)):
        tab = W.sum_table(cur, syms[t])
        tri = oracle.dense_to_triples(tab)
        cur, o = oracle.damp_apply2_fwd(tri, tab.shape[0], tab.shape[1], accs[-1], ins[t])
        tabs.append(tab); tris.append(tri); accs.append(o)
    assert (accs[-1] == 1.0).any() and (accs[2] == 1.0).any()
    g = np.abs(W.normal(5, B * cur.size)).astype(np.float32).reshape(B, -1)
    want, gr = [None] * len(widths), g
    for t in range(len(widths) - 1, 0, -1):
        gr, want[t] = oracle.damp_apply2_bwd(tris[t - 1], tabs[t - 1].shape[0], tabs[t - 1].shape[1], accs[t - 1], ins[t], gr)
    want[0] = gr
    pad = 3
    d_in = []
    for t, n in enumerate(widths):
        buf = torch.zeros((B, n + pad), device="cuda")
        buf[:, :n] = dev(ins[t])
        d_in.append(dol.Dist(syms[t], buf[:, :n]))
    ftabs = [dol.FnTable.create_dense(t) for t in tabs]
    out = dol.Dist.empty(cur, B)
    gbuf = torch.zeros((B, cur.size + 5), device="cuda")
    gbuf[:, :cur.size] = dev(g)
    gins = [torch.full((B, n + pad), 7.0, device="cuda") for n in widths]
    gins[2] = None                                   # a skipped gradient
    dol.fold_apply2(dol.Fold(d_in, ftabs, out=out, grad_out=gbuf[:, :cur.size], grad_inputs=gins))
    assert_close(host(out.prob), accs[-1], "fold forward (clamped)")
    np.testing.assert_array_equal(host(out.prob) == 1.0, accs[-1] == 1.0)
    for t, n in enumerate(widths):
        if gins[t] is None:
            continue
        assert_close(host(gins[t])[:, :n], want[t], "fold grad %d" % t)
        assert np.all(host(gins[t])[:, n:] == 7.0)
    out2 = dol.Dist.empty(cur, B)
    dol.fold_apply2(dol.Fold(d_in, ftabs, out=out2))                  # forward only
    np.testing.assert_array_equal(host(out2.prob), host(out.prob))
    hashed = dol.FnTable.create_dense(W.hashed_table(1, widths[0], widths[1], 9))
    with pytest.raises(dol.DolError) as ei:
        dol.fold_apply2(dol.Fold(d_in[:2], [hashed], out=dol.Dist.empty(hashed.out_syms, B)))
    assert ei.value.status == 5


# ---------------------------------------------------------------- config 3

@pytest.mark.parametrize("batch,na,nb,n_out", [(16384, 64, 64, 256), (1000, 64, 64, 256), (129, 17, 33, 40), (3, 5, 2, 300)])
def test_config3_hashed_pipeline(gp, batch, na, nb, n_out):
    w = W.config3(batch=batch, na=na, nb=nb, n_out=n_out, seed=7)
    ref = OP.hashed_pipeline_fwd_bwd(w)
    prog = gp.HashedPipeline(w)
    prog.step()
    np.testing.assert_array_equal(prog.o1.sym_ids, ref["s1"])
    np.testing.assert_array_equal(prog.o2.sym_ids, ref["s2"])
    np.testing.assert_array_equal(prog.o3.sym_ids, ref["s3"])
    assert_close(host(prog.o1.prob), ref["o1"], "apply")
    np.testing.assert_array_equal(host(prog.o2.prob), host(prog.o1.prob)[:, prog.pred.astype(bool)])
    assert_close(host(prog.o3.prob), ref["o3"], "union")
    assert_close(host(prog.g2), ref["g2"], "union bwd a")
    assert_close(host(prog.gp2), ref["gp2"], "union bwd b")
    assert_close(host(prog.g1), ref["g1"], "filter bwd")
    assert_close(host(prog.ga), ref["ga"], "apply bwd a")
    assert_close(host(prog.gb), ref["gb"], "apply bwd b")


@pytest.mark.parametrize("batch,na,nb,n_out", [(16384, 64, 64, 256), (1000, 64, 64, 256), (129, 17, 33, 40), (3, 5, 2, 300)])
def test_config3_fused_filter_union(gp, batch, na, nb, n_out):
    """dol_filter_union and its backward: the same results as filter then union, without the filtered tensor."""
    w = W.config3(batch=batch, na=na, nb=nb, n_out=n_out, seed=9)
    ref = OP.hashed_pipeline_fwd_bwd(w)
    prog = gp.HashedPipelineFused(w)
    prog.step()
    np.testing.assert_array_equal(prog.o3.sym_ids, ref["s3"])
    assert_close(host(prog.o3.prob), ref["o3"], "filter-union")
    assert_close(host(prog.gp2), ref["gp2"], "filter-union bwd b")
    assert_close(host(prog.g1), ref["g1"], "filter-union bwd a")
    assert_close(host(prog.ga), ref["ga"], "apply bwd a")
    assert_close(host(prog.gb), ref["gb"], "apply bwd b")
    per_op = gp.HashedPipeline(w)
    per_op.step()
    np.testing.assert_array_equal(host(prog.o3.prob), host(per_op.o3.prob))
    np.testing.assert_array_equal(host(prog.g1), host(per_op.g1))
    np.testing.assert_array_equal(host(prog.gp2), host(per_op.gp2))


@pytest.mark.parametrize("batch,na,nb,n_out,scale", [(16384, 64, 64, 256, 1.0), (16421, 64, 64, 256, 6.0), (12301, 64, 64, 256, 6.0), (1000, 64, 64, 256, 1.0), (333, 64, 64, 256, 12.0),
                                                      (65, 32, 16, 64, 9.0), (1, 16, 16, 8, 1.0), (200, 64, 64, 128, 30.0),
                                                      (130, 4, 64, 8, 3.0)])
def test_config3_apply_filter_union_in_one_launch(gp, dol, batch, na, nb, n_out, scale):
    """dol_apply2_filter_union and its reverse: the results of dol_apply2 + dol_filter_union + two dol_backward calls
    (bit for bit) and of the oracle.  scale > 1 multiplies the tags (capped at 1) so that sums of the Apply and of the
    union land on both sides of the clamp: those tiles re-derive every decision."""
    w = W.config3(batch=batch, na=na, nb=nb, n_out=n_out, seed=11)
    if scale != 1.0:
        for key in ("pa", "pb", "p2"):
            w.arrays[key] = np.minimum(w[key] * np.float32(scale), np.float32(1.0))
        w.arrays["g"] = np.abs(w["g"])         # one-signed upstream gradient: see the tolerance note in the module docstring
    ref = OP.hashed_pipeline_fwd_bwd(w)
    prog = gp.HashedPipelineMerged(w)
    prog.step()
    np.testing.assert_array_equal(prog.o3.sym_ids, ref["s3"])
    assert_close(host(prog.o3.prob), ref["o3"], "apply-filter-union")
    np.testing.assert_array_equal(host(prog.o3.prob) == 1.0, ref["o3"] == 1.0)
    assert_close(host(prog.gp2), ref["gp2"], "apply-filter-union grad c")
    assert_close(host(prog.ga), ref["ga"], "apply-filter-union grad a")
    assert_close(host(prog.gb), ref["gb"], "apply-filter-union grad b")
    # some clamp acted in a sample <=> the saved word says so
    both = np.isin(ref["s3"], ref["s2"])
    o2_in_3 = np.zeros_like(ref["o3"], dtype=np.float32)
    o2_in_3[:, both] = ref["o2"]
    pre32 = oracle.damp_apply2_fwd(oracle.dense_to_triples(w["table"]), na, nb, w["pa"], w["pb"], want_pre=True)[2]
    acted = (pre32 > 1.0).any(axis=1) | (((o2_in_3 + w["p2"].astype(np.float32)) > np.float32(1.0)) & both[None, :]).any(axis=1)
    np.testing.assert_array_equal(host(prog.saved) != 0, acted)
    per_op = gp.HashedPipelineFused(w)
    per_op.step()
    np.testing.assert_array_equal(host(prog.o3.prob), host(per_op.o3.prob))
    np.testing.assert_array_equal(host(prog.gp2), host(per_op.gp2))
    assert_close(host(prog.ga), host(per_op.ga).astype(np.float64), "one launch against three: grad a")
    assert_close(host(prog.gb), host(per_op.gb).astype(np.float64), "one launch against three: grad b")
    # without the saved words every tile re-derives its decisions: same results; accumulate adds
    m2 = dol.ApplyMerge(prog.a, prog.b, prog.table, prog.pred, prog.p2, prog.o3, None)
    ga, gb, gc = prog.ga.clone(), prog.gb.clone(), prog.gp2.clone()
    dol.apply2_filter_union_backward(m2, prog.g3, ga, gb, gc, accumulate=7)
    assert_close(host(ga), 2.0 * host(prog.ga).astype(np.float64), "accumulated grad a")
    assert_close(host(gb), 2.0 * host(prog.gb).astype(np.float64), "accumulated grad b")
    assert_close(host(gc), 2.0 * host(prog.gp2).astype(np.float64), "accumulated grad c")
    dol.apply2_filter_union_backward(m2, prog.g3, None, gb, None)
    np.testing.assert_array_equal(host(gb), host(prog.gb))


@pytest.mark.parametrize("batch,scale", [(16384, 1.0), (16421, 6.0), (12301, 6.0), (333, 12.0), (64, 1.0), (1, 1.0)])
def test_config3_forward_and_backward_in_one_launch(gp, dol, batch, scale):
    """dol_apply2_filter_union_forward_backward: the results of the two separate calls, bit for bit (clamp words included),
    with samples in which clamps act (scale > 1) and without."""
    w = W.config3(batch=batch, seed=21)
    if scale != 1.0:
        for key in ("pa", "pb", "p2"):
            w.arrays[key] = np.minimum(w[key] * np.float32(scale), np.float32(1.0))
    two = gp.HashedPipelineMerged(w)
    two.step()
    one = gp.HashedPipelineMerged(w, one_launch=True)
    assert len(one.launches) == 1
    for t in (one.o3.prob, one.ga, one.gb, one.gp2):
        t.fill_(-3.0)
    one.saved.fill_(-3)
    one.step()
    np.testing.assert_array_equal(host(one.o3.prob), host(two.o3.prob))
    np.testing.assert_array_equal(host(one.saved), host(two.saved))
    np.testing.assert_array_equal(host(one.ga), host(two.ga))
    np.testing.assert_array_equal(host(one.gb), host(two.gb))
    np.testing.assert_array_equal(host(one.gp2), host(two.gp2))
    if scale != 1.0:
        assert host(one.saved).any()
    ref = OP.hashed_pipeline_fwd_bwd(w)
    assert_close(host(one.o3.prob), ref["o3"], "one-launch forward")
    if scale == 1.0:                          # (mixed-sign gradients over unnormalised tags cannot meet the absolute bar)
        assert_close(host(one.ga), ref["ga"], "one-launch grad a")
        assert_close(host(one.gp2), ref["gp2"], "one-launch grad c")
    with pytest.raises(dol.DolError) as ei:   # the backward pass of this call needs the clamp words
        dol.apply2_filter_union_forward_backward(dol.ApplyMerge(one.a, one.b, one.table, one.pred, one.p2, one.o3, None), one.g3,
                                                 one.ga, one.gb, one.gp2)
    assert ei.value.status == 1


def test_apply_filter_union_rejects_what_it_cannot_take(dol):
    w = W.config3(batch=8, na=17, nb=33, n_out=40, seed=3)                     # symbol counts that are not multiples of 4
    f = dol.FnTable.create_dense(w["table"])
    a, b = dol.Dist(np.arange(17), dev(w["pa"])), dol.Dist(np.arange(33), dev(w["pb"]))
    c = dol.Dist(np.arange(40), dev(w["p2"]))
    pred = np.ones(f.n_out, np.uint8)
    out = dol.Dist.empty(dol.filter_union_plan(dol.Dist(f.out_syms, None, batch=8), pred, c), 8)
    with pytest.raises(dol.DolError) as ei:
        dol.apply2_filter_union(dol.ApplyMerge(a, b, f, pred, c, out))
    assert ei.value.status == 5


def test_filter_union_edge_cases(dol):
    """Everything dropped, nothing dropped, disjoint and empty second operand, padded rows, clamped sums, accumulate."""
    B = 37
    sd = np.array([1, 4, 6, 8, 9], np.int32)
    sc = np.array([0, 4, 9, 12], np.int32)
    a = (W.uniform01(1, B * 5) * 0.9).astype(np.float32).reshape(B, 5)
    c = (W.uniform01(2, B * 4) * 0.9).astype(np.float32).reshape(B, 4)
    g_all = np.abs(W.normal(3, B * 9)).astype(np.float32).reshape(B, 9)
    for pred in ([1, 1, 1, 1, 1], [0, 0, 0, 0, 0], [0, 1, 0, 1, 1], [1, 0, 1, 0, 0]):
        pred = np.array(pred, np.uint8)
        kept, fa = oracle.filter_plan(sd, pred)[0], np.ascontiguousarray(a[:, pred.astype(bool)])
        usyms, ia, ib = oracle.union_plan(kept, sc)
        want = oracle.damp_union_fwd(ia, ib, fa, c)
        ta = torch.zeros((B, 8), device="cuda"); ta[:, :5] = dev(a)            # padded rows
        da, dc = dol.Dist(sd, ta[:, :5]), dol.Dist(sc, dev(c))
        np.testing.assert_array_equal(dol.filter_union_plan(da, pred, dc), usyms)
        out = dol.Dist.empty(usyms, B)
        dol.filter_union(da, pred, dc, None, out)
        assert_close(host(out.prob), want, "filter-union %s" % pred)
        np.testing.assert_array_equal(host(out.prob) == 1.0, want == 1.0)
        g = g_all[:, :usyms.size]
        wfa, wc = oracle.damp_union_bwd(ia, ib, fa, c, g)
        wa = np.zeros((B, 5), np.float32); wa[:, pred.astype(bool)] = wfa
        ga, gc = torch.full((B, 8), 3.0, device="cuda"), torch.zeros((B, 4), device="cuda")
        rec = dol.OpRecord(dol.OP_FILTER_UNION, da, dc, out, pred_mask=pred)
        dol.backward(rec, dev(g), ga, gc)
        assert_close(host(ga)[:, :5], wa, "filter-union bwd a %s" % pred)
        assert np.all(host(ga)[:, 5:] == 3.0)
        assert_close(host(gc), wc, "filter-union bwd c %s" % pred)
        dol.backward(dol.OpRecord(dol.OP_FILTER_UNION, da, dc, out, pred_mask=pred, accumulate=2), dev(g), None, gc)
        assert_close(host(gc), 2.0 * wc.astype(np.float64), "filter-union bwd c accumulated")
    empty = dol.Dist(np.zeros(0, np.int32), torch.zeros((B, 0), device="cuda"))
    da = dol.Dist(sd, dev(a))
    out = dol.Dist.empty(dol.filter_union_plan(da, np.ones(5, np.uint8), empty), B)
    dol.filter_union(da, np.ones(5, np.uint8), empty, None, out)
    np.testing.assert_array_equal(host(out.prob), a)


# ---------------------------------------------------------------- config 4

@pytest.mark.parametrize("batch,n,k", [(1024, 5, 3), (130, 5, 1), (65, 4, 8), (7, 3, 5), (1, 2, 2)])
def test_config4_dtkp_sum(gp, dol, batch, n, k):
    w = W.config4(batch=batch, n_digits=n, k=k, seed=k)
    ref = OP.dtkp_sum_chain(w)
    prog = gp.DtkpSumChain(w)
    prog.step()
    for t in range(1, n):
        syms, m, pp, pr = ref["stages"][t - 1]
        d = prog.accs[t]
        np.testing.assert_array_equal(d.sym_ids, syms)
        np.testing.assert_array_equal(host(d.proof_mask).view(np.uint64), m, err_msg="masks stage %d" % t)
        np.testing.assert_array_equal(host(d.proof_prob), pp, err_msg="proof probs stage %d" % t)
        assert_close(host(d.prob), pr, "tag prob stage %d" % t)
    # gradient of -log Pr(target sum) w.r.t. the digit probabilities through the kept proofs
    last = prog.accs[-1]
    S = last.n_sym
    target = (W.splitmix64(77, np.arange(batch)) % np.uint64(S)).astype(np.int64)
    g = np.zeros((batch, S), np.float32)
    g[np.arange(batch), target] = -1.0 / np.maximum(ref["prob"][np.arange(batch), target], np.float32(1e-30))
    want = oracle.dtkp_prob_bwd(ref["mask"], w["fact_prob"], g)
    gpad = torch.zeros((batch, S + 3), device="cuda")             # a padded gradient tensor
    gpad[:, :S] = dev(g)
    gf = torch.empty((batch, 10 * n), device="cuda")
    dol.dtkp_backward(last, prog.prov, gpad, gf)
    assert_close(host(gf), want, "dtkp gradient of the digit probabilities")
    with pytest.raises(dol.DolError) as ei:                        # the per-operator backward does not take DTKP
        dol.backward(dol.OpRecord(dol.OP_APPLY2, prog.accs[0], prog.digits[1], prog.accs[1], f=prog.tables[0],
                                  prov=prog.prov), gpad, None, None)
    assert ei.value.status == 5


@pytest.mark.parametrize("batch,n,k", [(1024, 5, 3), (130, 5, 1), (65, 4, 8), (7, 3, 5), (1, 2, 2), (3, 6, 2)])
def test_config4_fused_dtkp_fold(gp, dol, batch, n, k):
    """dol_dtkp_fold_apply2: initialisation + all applies (+ the gradient of -log Pr(target)) in one launch."""
    w = W.config4(batch=batch, n_digits=n, k=k, seed=k + 10)
    ref = OP.dtkp_sum_chain(w)
    prog = gp.DtkpSumChainFused(w, with_gradient=True)
    prog.step()
    np.testing.assert_array_equal(prog.out.sym_ids, ref["syms"])
    np.testing.assert_array_equal(host(prog.out.proof_mask).view(np.uint64), ref["mask"])
    np.testing.assert_array_equal(host(prog.out.proof_prob), ref["pprob"])
    assert_close(host(prog.out.prob), ref["prob"], "fused dtkp tag prob")
    S = ref["syms"].size
    target = np.arange(batch) % S
    g = np.zeros((batch, S), np.float32)
    g[np.arange(batch), target] = -1.0 / np.maximum(ref["prob"][np.arange(batch), target], np.float32(1.17549435e-38))
    assert_close(host(prog.grad_fact), oracle.dtkp_prob_bwd(ref["mask"], w["fact_prob"], g), "fused dtkp gradient")
    per_op = gp.DtkpSumChain(w)
    per_op.step()
    np.testing.assert_array_equal(host(prog.out.proof_mask), host(per_op.accs[-1].proof_mask))
    np.testing.assert_array_equal(host(prog.out.proof_prob), host(per_op.accs[-1].proof_prob))
    np.testing.assert_array_equal(host(prog.out.prob), host(per_op.accs[-1].prob))
    # an explicit upstream gradient instead of a target; forward only
    gsym = W.normal(5, batch * S).astype(np.float32).reshape(batch, S)
    gf = torch.empty((batch, 10 * n), device="cuda")
    out2 = dol.Dist.empty(ref["syms"], batch, k=k)
    dol.dtkp_fold_apply2(dol.DtkpFold(prog.digits, prog.facts, prog.tables, out2, grad_out=dev(gsym), grad_fact_prob=gf), prog.prov)
    assert_close(host(gf), oracle.dtkp_prob_bwd(ref["mask"], w["fact_prob"], gsym), "fused dtkp gradient, explicit")
    out3 = dol.Dist.empty(ref["syms"], batch, k=k)
    dol.dtkp_fold_apply2(dol.DtkpFold(prog.digits, prog.facts, prog.tables, out3), prog.prov)
    np.testing.assert_array_equal(host(out3.proof_mask), host(prog.out.proof_mask))


@pytest.mark.parametrize("k", [1, 3, 8])
def test_fused_dtkp_fold_when_a_stage_brings_no_new_facts(dol, k):
    """The fused fold with inputs whose facts are not new to the fold: facts below the ones already in the proofs (the
    product over ascending facts is then redone, not continued), an input given twice (the same fact is idempotent, a
    rival of it excludes the proof), an input that shares its exclusion group with an earlier one under other facts,
    and one with new facts again.  Against the oracle's operator-by-operator composition, bit for bit."""
    batch, nv = 70, 4
    fact_sets = [8 + np.arange(nv), 4 + np.arange(nv), 8 + np.arange(nv), np.arange(nv), 12 + np.arange(nv), 16 + np.arange(nv)]
    n_facts = 20
    grp = (np.arange(n_facts) // nv).astype(np.int32)
    grp[16:20] = grp[0:4]                    # the last input's facts are rivals of the fourth input's
    fp = W.uniform01(77, batch * n_facts).astype(np.float32).reshape(batch, n_facts)
    fp[:, 5] = fp[:, 6]                      # equal probabilities: ties decided by the masks
    fp[3] = 0.0
    sym = np.arange(nv, dtype=np.int32)
    m, pp, pr = oracle.dtkp_init(fact_sets[0].astype(np.int32), fp, k)
    syms, tables = sym, []
    for t in range(1, len(fact_sets)):
        dm, _, _ = oracle.dtkp_init(fact_sets[t].astype(np.int32), fp, k)
        tab = W.sum_table(syms, sym)
        syms, m, pp, pr = oracle.dtkp_apply2(oracle.dense_to_triples(tab), syms.size, nv, k, grp, fp, m, dm)
        tables.append(dol.FnTable.create_dense(tab))
    prov = dol.Prov(dol.DTKP, k, dev(fp), grp)
    digits = [dol.Dist(sym, torch.empty((batch, nv), device="cuda")) for _ in fact_sets]
    out = dol.Dist.empty(syms, batch, k=k)
    g = W.normal(9, batch * syms.size).astype(np.float32).reshape(batch, -1)
    gf = torch.empty((batch, n_facts), device="cuda")
    dol.dtkp_fold_apply2(dol.DtkpFold(digits, [f.astype(np.int32) for f in fact_sets], tables, out, grad_out=dev(g), grad_fact_prob=gf), prov)
    np.testing.assert_array_equal(host(out.proof_mask).view(np.uint64), m)
    np.testing.assert_array_equal(host(out.proof_prob), pp)
    assert_close(host(out.prob), pr, "fold tag prob")
    assert_close(host(gf), oracle.dtkp_prob_bwd(m, fp, g), "fold gradient")


# ---------------------------------------------------------------- config 5

@pytest.mark.parametrize("batch,side,rounds", [(256, 32, 64), (33, 7, 20), (2, 3, 5)])
def test_config5_grid_reach(gp, batch, side, rounds):
    w = W.config5(batch=batch, side=side, rounds=rounds, seed=side)
    ref = OP.grid_reach_fwd_bwd(w)
    prog = gp.GridReach(w)
    prog.step()
    hist = host(prog.hist)
    assert_close(hist, ref["hist"], "reach history")
    # the clamp decisions: saturated entries agree exactly
    np.testing.assert_array_equal(hist == 1.0, ref["hist"] == 1.0)
    assert_close(host(prog.grad_p), ref["grad_p"], "reach grad")


@pytest.mark.parametrize("batch,side,rounds", [(256, 32, 64), (33, 7, 20), (2, 3, 5), (5, 4, 1), (3, 3, 0)])
def test_config5_fused_iteration(gp, dol, batch, side, rounds):
    """dol_iterate_apply2 / dol_iterate_backward: all rounds in one launch, same results as round-by-round calls."""
    w = W.config5(batch=batch, side=side, rounds=rounds, seed=side + 1)
    ref = OP.grid_reach_fwd_bwd(w)
    prog = gp.GridReachFused(w, ckpt_every=0)
    prog.step()
    hist = host(prog.hist)
    assert_close(hist, ref["hist"], "fused reach history")
    np.testing.assert_array_equal(hist == 1.0, ref["hist"] == 1.0)
    assert_close(host(prog.grad_p), ref["grad_p"], "fused reach grad")
    if rounds:
        per_round = gp.GridReach(w)
        per_round.step()
        np.testing.assert_array_equal(hist, host(per_round.hist))          # same arithmetic, bit for bit
    g0 = torch.empty((batch, side * side), device="cuda")
    dol.iterate_backward(prog.edges, prog.table, rounds, prog.hist, prog.g_out, g0, None)
    if rounds == 0:
        np.testing.assert_array_equal(host(g0), w["g"])
    with pytest.raises(dol.DolError) as ei:                                 # a table that is not square
        f = dol.FnTable.create_dense(W.sum_table(range(4), range(3)))
        dol.iterate_apply2(dol.Dist(np.arange(4), torch.ones((2, 4), device="cuda")),
                           dol.Dist(np.arange(3), torch.ones((2, 3), device="cuda")), f, 2,
                           torch.empty((3, 2, 4), device="cuda"))
    assert ei.value.status == 5


@pytest.mark.parametrize("batch,side,rounds,every", [(256, 32, 64, 8), (256, 32, 64, 16), (33, 7, 20, 6), (33, 7, 20, 1),
                                                      (2, 3, 5, 5), (2, 3, 5, 9), (5, 4, 1, 3), (3, 3, 0, 2), (7, 32, 64, 30), (9, 32, 64, 32)])
def test_config5_checkpointed_iteration(gp, dol, batch, side, rounds, every):
    """dol_iterate_apply2_ckpt / dol_iterate_backward_ckpt: only the last round and a checkpoint every `every` rounds
    leave the chip; the reverse sweep replays the rounds in between.  Same results as the oracle, and bit for bit
    those of the sweeps that keep the whole history."""
    w = W.config5(batch=batch, side=side, rounds=rounds, seed=side + 2)
    ref = OP.grid_reach_fwd_bwd(w)
    prog = gp.GridReachFused(w, ckpt_every=every)
    prog.step()
    out = host(prog.out.prob)
    assert_close(out, ref["hist"][-1], "checkpointed reach result")
    np.testing.assert_array_equal(out == 1.0, ref["hist"][-1] == 1.0)
    assert_close(host(prog.grad_p), ref["grad_p"], "checkpointed reach grad")
    n_ck = dol.iterate_ckpt_count(rounds, every)
    assert n_ck == max(0, -(-rounds // every) - 1)
    assert 1 <= dol.iterate_ckpt_every(prog.table, batch, rounds) <= max(rounds, 1)
    for x in range(n_ck):                                                   # the checkpoints are rounds of the history
        assert_close(host(prog.ckpt[x]), ref["hist"][(x + 1) * every], "checkpoint %d" % x)
    full = gp.GridReachFused(w, ckpt_every=0)
    full.step()
    np.testing.assert_array_equal(out, host(full.hist[rounds]))
    np.testing.assert_array_equal(host(prog.g_e), host(full.g_e))
    g0a, g0b = torch.empty((batch, side * side), device="cuda"), torch.empty((batch, side * side), device="cuda")
    dol.iterate_backward_ckpt(prog.r0, prog.edges, prog.table, rounds, every, prog.ckpt, prog.g_out, g0a, None)
    dol.iterate_backward(full.edges, full.table, rounds, full.hist, full.g_out, g0b, None)
    np.testing.assert_array_equal(host(g0a), host(g0b))
    with pytest.raises(dol.DolError) as ei:
        dol.iterate_apply2_ckpt(prog.r0, prog.edges, prog.table, rounds, 0, prog.out, prog.ckpt)
    assert ei.value.status == 1


@pytest.mark.parametrize("batch,side,rounds,every", [(256, 32, 64, 22), (256, 32, 64, 32), (33, 7, 20, 6), (5, 4, 1, 8), (40, 12, 30, 30), (3, 3, 7, 2),
                                                      (600, 7, 20, 6), (520, 32, 11, 8)])
def test_config5_iteration_in_one_launch(gp, dol, batch, side, rounds, every):
    """dol_iterate_apply2_backward: both sweeps in one launch (in two, issued by the one call, for batches above 512).  With an upstream gradient: bit for bit the results of
    the two separate calls.  With a target node per sample (loss = -log r[target]): against the oracle's sweeps fed
    the gradient of that loss at the oracle's own result."""
    w = W.config5(batch=batch, side=side, rounds=rounds, seed=side + 3)
    two = gp.GridReachFused(w, ckpt_every=every)
    two.step()
    one = gp.GridReachFused(w, ckpt_every=every, one_launch=True)
    assert len(one.launches) == (1 if batch <= 512 else 2)
    one.step()
    np.testing.assert_array_equal(host(one.out.prob), host(two.out.prob))
    np.testing.assert_array_equal(host(one.g_e), host(two.g_e))
    if one.ckpt is not None:
        np.testing.assert_array_equal(host(one.ckpt), host(two.ckpt))
    n = side * side
    g0a, g0b = torch.empty((batch, n), device="cuda"), torch.empty((batch, n), device="cuda")
    dol.iterate_apply2_backward(one.r0, one.edges, one.table, rounds, every, one.out, one.ckpt, None, one.g_out, g0a, None)
    dol.iterate_backward_ckpt(two.r0, two.edges, two.table, rounds, every, two.ckpt, two.g_out, g0b, None)
    np.testing.assert_array_equal(host(g0a), host(g0b))
    # a target node per sample
    ref = OP.grid_reach_fwd_bwd(w)
    near = np.array([r * side + c for r in range(side) for c in range(side) if r + c <= rounds], np.int32)   # reachable in time
    target = near[np.arange(batch) * 7 % near.size]
    r_t = ref["hist"][-1][np.arange(batch), target]
    assert (r_t > 0).all()
    g = np.zeros((batch, n), np.float32)
    g[np.arange(batch), target] = -1.0 / np.maximum(r_t, np.float32(1.17549435e-38))
    wd = {k: w[k] for k in ("side", "edge_u", "edge_v", "src", "rounds", "p")}
    wd["g"] = g
    want = OP.grid_reach_fwd_bwd(wd)["grad_p"]
    ge = torch.empty_like(one.g_e)
    dol.iterate_apply2_backward(one.r0, one.edges, one.table, rounds, every, one.out, one.ckpt, dev(target), None, None, ge)
    assert_close(host(one.out.prob), ref["hist"][-1], "one-launch reach result")
    assert_close(host(ge)[:, :w["p"].shape[1]], want, "one-launch reach grad from a target")
    for args in ((None, None), (dev(target), one.g_out)):
        with pytest.raises(dol.DolError) as ei:
            dol.iterate_apply2_backward(one.r0, one.edges, one.table, rounds, every, one.out, one.ckpt, args[0], args[1], None, ge)
        assert ei.value.status == 1


def test_iterated_apply_passes_gradient_on_the_clamp_bound(dol):
    """Two nodes, one edge, a "stay" symbol of tag 1: with p = 0.5 the second round's sum at node 1 is exactly 1 and the
    clamp passes gradient (App. A.2), d r_2[1] / d p = 2; with p = 0.75 the clamp acts (0); with 0.25 nothing clamps (2).
    The same case pins the oracle (tests/test_oracle_reach.py)."""
    tri = (np.array([0, 0, 1, 1], np.int32), np.array([0, 1, 0, 1], np.int32), np.array([1, 0, 0, 1], np.int32))
    f = dol.FnTable.create_sparse(2, 2, *tri)
    ps = np.array([0.5, 0.75, 0.25], np.float32)
    r0 = dol.Dist(np.arange(2), dev(np.tile(np.array([[1.0, 0.0]], np.float32), (3, 1))))
    e = dol.Dist(np.arange(2), dev(np.stack([ps, np.ones(3, np.float32)], axis=1)))
    g = dev(np.tile(np.array([[0.0, 1.0]], np.float32), (3, 1)))
    hist = torch.empty((3, 3, 2), device="cuda")
    dol.iterate_apply2(r0, e, f, 2, hist)
    np.testing.assert_array_equal(host(hist[2])[:, 1], np.array([1.0, 1.0, 0.5], np.float32))
    ge = torch.empty((3, 2), device="cuda")
    dol.iterate_backward(e, f, 2, hist, g, None, ge)
    np.testing.assert_array_equal(host(ge)[:, 0], np.array([2.0, 0.0, 2.0], np.float32))
    out, ge2 = dol.Dist.empty(np.arange(2), 3), torch.empty((3, 2), device="cuda")
    ck = torch.empty((1, 3, 2), device="cuda")
    dol.iterate_apply2_ckpt(r0, e, f, 2, 1, out, ck)
    dol.iterate_backward_ckpt(r0, e, f, 2, 1, ck, g, None, ge2)
    np.testing.assert_array_equal(host(ge2), host(ge))


@pytest.mark.parametrize("batch,n_nodes,n_edges,scale", [(64, 10, 16, 0.5), (130, 12, 30, 1.0), (3, 5, 4, 0.9), (70, 16, 40, 0.3)])
def test_transitive_closure_program(gp, batch, n_nodes, n_edges, scale):
    """The recursion of App. B, Fig. 9 over a random directed graph: symbol sets grow step by step, tags pile up
    towards the clamp, gradients of Distributions used twice are summed with the accumulate flags."""
    w = W.closure_workload(batch=batch, n_nodes=n_nodes, n_edges=n_edges, scale=scale, seed=n_nodes)
    w.arrays["g"] = np.abs(w["g"])         # one-signed upstream gradient: see the tolerance note in the module docstring
    ref = OP.transitive_closure_fwd_bwd(w, W.join_triples)
    prog = gp.TransitiveClosure(w, W.join_triples)
    prog.step()
    assert len(prog.rounds) == ref["rounds"]
    np.testing.assert_array_equal(prog.out.sym_ids, ref["syms"])
    assert_close(host(prog.out.prob), ref["out"], "closure tags")
    np.testing.assert_array_equal(host(prog.out.prob) == 1.0, ref["out"] == 1.0)
    assert_close(host(prog.grad_p), ref["grad_p"], "closure gradient of the edge probabilities")


@pytest.mark.parametrize("long_a,long_b", [((5, 9), (0, 1, 2)), ((5,), (0,)), ((), (0, 1, 2))])
def test_fused_iteration_with_long_rows(dol, long_a, long_b):
    """A square table in which some symbols of either operand meet more than 64 tuples: the fused sweeps sum the
    first two such rows with the whole workgroup and leave the others to single threads."""
    na, nb, B, rounds = 150, 80, 9, 5
    ti, tj, to = [], [], []
    for j in long_b:                                   # symbol j of e combines with every symbol of r
        for i in range(na):
            ti.append(i); tj.append(j); to.append((i * (2 * j + 1) + j) % na)
    for i in long_a:                                   # symbol i of r combines with every remaining symbol of e
        for j in range(3, nb):
            ti.append(i); tj.append(j); to.append((i + 3 * j) % na)
    for i in range(20, 140):                           # a few ordinary tuples
        ti.append(i); tj.append(3 + i % 70); to.append((i + 1) % na)
    order = np.lexsort((tj, ti))
    tri = tuple(np.asarray(x, np.int32)[order] for x in (ti, tj, to))
    assert np.unique(tri[2]).size == na
    r0 = (W.uniform01(1, B * na) * 0.3).astype(np.float32).reshape(B, na)
    r0[:, 7] = 1.0                                     # stays on the clamp in every round
    e = (W.uniform01(2, B * nb) * 0.02).astype(np.float32).reshape(B, nb)
    e[:, 0] = 1.0
    hist = [r0]
    for t in range(rounds):
        hist.append(oracle.damp_apply2_fwd(tri, na, nb, hist[-1], e)[1])
    g = np.abs(W.normal(3, B * na)).astype(np.float32).reshape(B, na)
    want_ge = np.zeros((B, nb), np.float64)
    gr = g
    for t in reversed(range(rounds)):
        gr, ge = oracle.damp_apply2_bwd(tri, na, nb, hist[t], e, gr)
        want_ge += ge
    f = dol.FnTable.create_sparse(na, nb, *tri)
    d0, de = dol.Dist(np.arange(na), dev(r0)), dol.Dist(np.arange(nb), dev(e))
    dh = torch.empty((rounds + 1, B, na), device="cuda")
    dol.iterate_apply2(d0, de, f, rounds, dh)
    got = host(dh)
    assert_close(got, np.stack(hist), "iterated apply")
    np.testing.assert_array_equal(got == 1.0, np.stack(hist) == 1.0)
    g0, ge = torch.empty((B, na), device="cuda"), torch.empty((B, nb), device="cuda")
    dol.iterate_backward(de, f, rounds, dh, dev(g), g0, ge)
    assert_close(host(g0), gr, "iterated apply: gradient of r0")
    assert_close(host(ge), want_ge, "iterated apply: gradient of e")
    # the shares of d loss / d e meet in a fixed order: a second run and the checkpointed sweeps give the same bits
    g0b, geb = torch.empty_like(g0), torch.empty_like(ge)
    dol.iterate_backward(de, f, rounds, dh, dev(g), g0b, geb)
    np.testing.assert_array_equal(host(ge), host(geb))
    np.testing.assert_array_equal(host(g0), host(g0b))
    for every in (2, 3, 7):
        out = dol.Dist.empty(np.arange(na), B)
        n_ck = dol.iterate_ckpt_count(rounds, every)
        ck = torch.empty((n_ck, B, na), device="cuda") if n_ck else None
        dol.iterate_apply2_ckpt(d0, de, f, rounds, every, out, ck)
        np.testing.assert_array_equal(host(out.prob), got[-1])
        g0c, gec = torch.empty_like(g0), torch.empty_like(ge)
        dol.iterate_backward_ckpt(d0, de, f, rounds, every, ck, dev(g), g0c, gec)
        np.testing.assert_array_equal(host(gec), host(ge))
        np.testing.assert_array_equal(host(g0c), host(g0))


@pytest.mark.parametrize("B,na", [(5, 300), (5, 700), (520, 700)])
def test_fused_iteration_with_six_tuples_per_symbol(dol, B, na):
    """Every column and every row of the table holds six tuples: the builds that keep six tuples in registers, without
    tail loops, in each launch shape (one symbol per thread; 1024 threads; two symbols per thread for the larger
    batch, whose combined call issues its two sweeps as two launches)."""
    nb, rounds, every = 40, 10, 4
    i = np.repeat(np.arange(na, dtype=np.int32), 6)
    d = np.tile(np.arange(6, dtype=np.int32), na)
    ti, tj, to = i, (i + 5 * d) % nb, (i + np.array([0, 1, 7, 31, 100, 211], np.int32)[d]) % na
    order = np.lexsort((tj, ti))
    tri = tuple(x[order].astype(np.int32) for x in (ti, tj, to))
    assert np.bincount(tri[2], minlength=na).max() == 6 and np.bincount(tri[0]).max() == 6
    r0 = (W.uniform01(1, B * na) * 0.5).astype(np.float32).reshape(B, na)
    r0[:, 3] = 1.0
    e = (W.uniform01(2, B * nb) * 0.45).astype(np.float32).reshape(B, nb)
    hist = [r0]
    for t in range(rounds):
        hist.append(oracle.damp_apply2_fwd(tri, na, nb, hist[-1], e)[1])
    assert (hist[-1] == 1.0).any() and (hist[-1] < 1.0).any()
    g = np.abs(W.normal(3, B * na)).astype(np.float32).reshape(B, na)
    want_ge, gr = np.zeros((B, nb), np.float64), g
    for t in reversed(range(rounds)):
        gr, ge = oracle.damp_apply2_bwd(tri, na, nb, hist[t], e, gr)
        want_ge += ge
    f = dol.FnTable.create_sparse(na, nb, *tri)
    d0, de = dol.Dist(np.arange(na), dev(r0)), dol.Dist(np.arange(nb), dev(e))
    n_ck = dol.iterate_ckpt_count(rounds, every)
    out, ck = dol.Dist.empty(np.arange(na), B), torch.empty((n_ck, B, na), device="cuda")
    g0, ge = torch.empty((B, na), device="cuda"), torch.empty((B, nb), device="cuda")
    dol.iterate_apply2_ckpt(d0, de, f, rounds, every, out, ck)
    dol.iterate_backward_ckpt(d0, de, f, rounds, every, ck, dev(g), g0, ge)
    assert_close(host(out.prob), hist[-1], "six tuples: result")
    np.testing.assert_array_equal(host(out.prob) == 1.0, hist[-1] == 1.0)
    assert_close(host(g0), gr, "six tuples: gradient of r0")
    assert_close(host(ge), want_ge, "six tuples: gradient of e")
    out2, ck2 = dol.Dist.empty(np.arange(na), B), torch.empty_like(ck)
    g0b, geb = torch.empty_like(g0), torch.empty_like(ge)
    dol.iterate_apply2_backward(d0, de, f, rounds, every, out2, ck2, None, dev(g), g0b, geb)
    for a, b in ((out2.prob, out.prob), (ck2, ck), (g0b, g0), (geb, ge)):
        np.testing.assert_array_equal(host(a), host(b))


def test_fused_iteration_with_more_than_1024_symbols(dol):
    """Four symbols of the first operand per thread (the widest build of the fused sweeps)."""
    na, nb, B, rounds = 1100, 40, 3, 4
    i = np.arange(na, dtype=np.int32)
    ti = np.concatenate([i, i]); tj = np.concatenate([np.zeros(na, np.int32), 1 + i % 39])
    to = np.concatenate([i, (i * 7 + 3) % na]).astype(np.int32)
    order = np.lexsort((tj, ti))
    tri = tuple(x[order].astype(np.int32) for x in (ti, tj, to))
    r0 = (W.uniform01(1, B * na) * 0.3).astype(np.float32).reshape(B, na)
    r0[:, 11] = 1.0
    e = (W.uniform01(2, B * nb) * 0.3).astype(np.float32).reshape(B, nb)
    e[:, 0] = 1.0
    hist = [r0]
    for t in range(rounds):
        hist.append(oracle.damp_apply2_fwd(tri, na, nb, hist[-1], e)[1])
    g = np.abs(W.normal(3, B * na)).astype(np.float32).reshape(B, na)
    want_ge, gr = np.zeros((B, nb), np.float64), g
    for t in reversed(range(rounds)):
        gr, ge = oracle.damp_apply2_bwd(tri, na, nb, hist[t], e, gr)
        want_ge += ge
    f = dol.FnTable.create_sparse(na, nb, *tri)
    d0, de = dol.Dist(np.arange(na), dev(r0)), dol.Dist(np.arange(nb), dev(e))
    dh = torch.empty((rounds + 1, B, na), device="cuda")
    dol.iterate_apply2(d0, de, f, rounds, dh)
    got = host(dh)
    assert_close(got, np.stack(hist), "iterated apply, 1100 symbols")
    np.testing.assert_array_equal(got == 1.0, np.stack(hist) == 1.0)
    g0, ge = torch.empty((B, na), device="cuda"), torch.empty((B, nb), device="cuda")
    dol.iterate_backward(de, f, rounds, dh, dev(g), g0, ge)
    assert_close(host(g0), gr, "iterated apply, 1100 symbols: gradient of r0")
    assert_close(host(ge), want_ge, "iterated apply, 1100 symbols: gradient of e")
    out = dol.Dist.empty(np.arange(na), B)
    ck = torch.empty((1, B, na), device="cuda")
    dol.iterate_apply2_ckpt(d0, de, f, rounds, 2, out, ck)
    np.testing.assert_array_equal(host(out.prob), got[-1])
    g0c, gec = torch.empty_like(g0), torch.empty_like(ge)
    dol.iterate_backward_ckpt(d0, de, f, rounds, 2, ck, dev(g), g0c, gec)
    np.testing.assert_array_equal(host(gec), host(ge))
    np.testing.assert_array_equal(host(g0c), host(g0))


def test_backward_of_tables_with_long_rows(dol):
    """A table whose rows hold hundreds of tuples (one symbol of b combines with every symbol of a)."""
    na, B = 300, 20
    i = np.arange(na, dtype=np.int32)
    tri = (np.concatenate([i, i]), np.concatenate([np.zeros(na, np.int32), np.ones(na, np.int32)]),
           np.concatenate([i % 7, 7 + i % 5]))
    order = np.lexsort((tri[1], tri[0]))
    tri = tuple(x[order].astype(np.int32) for x in tri)
    a = W.softmax_rows(W.normal(1, B * na).reshape(B, na))
    b = (W.uniform01(2, B * 2)).astype(np.float32).reshape(B, 2)
    syms, want = oracle.damp_apply2_fwd(tri, na, 2, a, b)
    f = dol.FnTable.create_sparse(na, 2, *tri)
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(2), dev(b))
    do = dol.Dist.empty(syms, B)
    dol.apply2(da, db, f, None, do)
    assert_close(host(do.prob), want, "long-row apply")
    g = np.abs(W.normal(3, B * syms.size)).astype(np.float32).reshape(B, -1)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f), dev(g), ga, gb)
    wa, wb = oracle.damp_apply2_bwd(tri, na, 2, a, b, g)
    assert_close(host(ga), wa, "long-row bwd a")
    assert_close(host(gb), wb, "long-row bwd b")


# ---------------------------------------------------------------- operators on their own: edge cases

def test_apply_with_rejected_tuples_and_padding(dol):
    na, nb, B = 9, 6, 70
    tab = W.hashed_table(3, na, nb, 11)
    tab[0, :] = -1                     # symbol 0 of a never admitted
    tab[4, 2] = -1
    a = W.softmax_rows(W.normal(1, B * na).reshape(B, na))
    b = W.softmax_rows(W.normal(2, B * nb).reshape(B, nb))
    tri = oracle.dense_to_triples(tab)
    syms, want = oracle.damp_apply2_fwd(tri, na, nb, a, b)
    f = dol.FnTable.create_dense(tab)
    np.testing.assert_array_equal(f.out_syms, syms)
    # padded leading dimensions on every tensor
    ta = torch.zeros((B, na + 3), device="cuda"); ta[:, :na] = dev(a)
    tb = torch.zeros((B, nb + 5), device="cuda"); tb[:, :nb] = dev(b)
    to = torch.full((B, f.n_out + 2), -7.0, device="cuda")
    da, db, do = dol.Dist(np.arange(na), ta[:, :na]), dol.Dist(np.arange(nb), tb[:, :nb]), dol.Dist(syms, to[:, :f.n_out])
    assert da.ld == na + 3 and do.ld == f.n_out + 2
    dol.apply2(da, db, f, None, do)
    assert_close(host(to)[:, :f.n_out], want, "apply padded")
    assert np.all(host(to)[:, f.n_out:] == -7.0)          # padding untouched
    g = W.normal(9, B * f.n_out).astype(np.float32).reshape(B, -1)
    tg = torch.zeros((B, f.n_out + 2), device="cuda"); tg[:, :f.n_out] = dev(g)
    ga = torch.full((B, na + 3), 5.0, device="cuda")
    gb = torch.full((B, nb + 5), 5.0, device="cuda")
    rec = dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f)
    dol.backward(rec, tg, ga, gb)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    assert_close(host(ga)[:, :na], wa, "bwd a padded")
    assert_close(host(gb)[:, :nb], wb, "bwd b padded")
    assert np.all(host(ga)[:, 0] == 0) and np.all(host(ga)[:, na:] == 5.0) and np.all(host(gb)[:, nb:] == 5.0)
    # accumulate flags add to what is there
    rec2 = dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f, accumulate=3)
    dol.backward(rec2, tg, ga, gb)
    assert_close(host(ga)[:, :na], 2 * wa.astype(np.float64), "bwd a accumulated")
    assert_close(host(gb)[:, :nb], 2 * wb.astype(np.float64), "bwd b accumulated")


def test_clamp_decisions_match_oracle(dol):
    """Tags large enough that many columns exceed 1: values clamp, gradients gate, decisions agree bit for bit."""
    na, nb, B = 12, 12, 200
    tab = W.hashed_table(5, na, nb, 6)
    a = (W.uniform01(1, B * na) * 0.4).astype(np.float32).reshape(B, na)
    b = (W.uniform01(2, B * nb) * 0.4).astype(np.float32).reshape(B, nb)
    # exact boundary cases: rows 0..2 make column sums of exactly 0.875, 1.0, 1.125
    for r, tot in enumerate((0.875, 1.0, 1.125)):
        a[r] = 0; b[r] = 0
        a[r, 0] = 1.0; b[r, 0] = tot
    tri = oracle.dense_to_triples(tab)
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    assert 0.2 < (pre32 > 1).mean() < 0.8
    f = dol.FnTable.create_dense(tab)
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    do = dol.Dist.empty(syms, B)
    dol.apply2(da, db, f, None, do)
    got = host(do.prob)
    assert_close(got, want, "clamped apply")
    np.testing.assert_array_equal(got == 1.0, pre32 >= 1.0)
    g = W.normal(3, B * syms.size).astype(np.float32).reshape(B, -1)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f), dev(g), ga, gb)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    assert_close(host(ga), wa, "gated bwd a")
    assert_close(host(gb), wb, "gated bwd b")


@pytest.mark.parametrize("na,nb,n_out,B,scale", [(12, 12, 8, 200, 0.4), (64, 64, 256, 130, 0.7), (128, 4, 16, 64, 0.25),
                                                  (16, 128, 100, 257, 0.2), (4, 4, 4, 4160, 1.0), (64, 64, 256, 64, 0.05)])
def test_hashed_tables_in_lds_with_clamping(dol, na, nb, n_out, B, scale):
    """Hashed tables whose sizes are multiples of four (whole tiles of 64 samples go through the LDS kernels, the
    remainder through the direct ones), some tuples rejected, tags scaled so that columns land on both sides of
    the clamp (the last case: all far below it); rows 0..2 hit 0.875 / 1.0 / 1.125 exactly."""
    tab = W.hashed_table(7, na, nb, n_out)
    tab[1, :] = -1
    tab[na - 1, nb // 2] = -1
    a = (W.uniform01(1, B * na) * scale).astype(np.float32).reshape(B, na)
    b = (W.uniform01(2, B * nb) * scale).astype(np.float32).reshape(B, nb)
    for r, tot in enumerate((0.875, 1.0, 1.125)):
        a[r] = 0; b[r] = 0
        a[r, 0] = 1.0; b[r, 0] = tot
    tri = oracle.dense_to_triples(tab)
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    f = dol.FnTable.create_dense(tab)
    if syms.size % 4 == 0:                 # operand rows that fit in registers: code written for the table; else LDS gathers
        kind = "table" if max(na, nb) <= 64 else "lds"
        assert f.kernel_fwd == "damp_%s_fwd_kernel" % kind and f.kernel_bwd == "damp_%s_bwd_kernel" % kind
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    do = dol.Dist.empty(syms, B)
    dol.apply2(da, db, f, None, do)
    got = host(do.prob)
    assert_close(got, want, "lds apply")
    np.testing.assert_array_equal(got == 1.0, pre32 >= 1.0)
    g = np.abs(W.normal(3, B * syms.size)).astype(np.float32).reshape(B, -1)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f), dev(g), ga, gb)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    assert_close(host(ga), wa, "lds bwd a")
    assert_close(host(gb), wb, "lds bwd b")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f, accumulate=3), dev(g), ga, gb)
    assert_close(host(ga), 2.0 * wa.astype(np.float64), "lds bwd a accumulated")
    assert_close(host(gb), 2.0 * wb.astype(np.float64), "lds bwd b accumulated")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f, accumulate=1), dev(g), ga, None)     # one side only
    assert_close(host(ga), 3.0 * wa.astype(np.float64), "lds bwd a alone")


@pytest.mark.parametrize("na,nb,B", [(127, 10, 300), (10, 10, 65), (1, 3, 70), (200, 16, 130), (5, 7, 64), (70, 1, 33),
                                      (9, 17, 40), (64, 4, 129), (300, 10, 50), (257, 2, 9), (256, 16, 5)])
def test_sum_tables_with_clamping(dol, na, nb, B):
    """Sum-shaped tables of every supported width, with unnormalised tags so that many columns exceed 1 and the
    backward pass has to re-derive the clamp decisions; rows 0..2 hit 0.875 / 1.0 / 1.125 exactly."""
    check_sum_table(dol, na, nb, B)


@pytest.mark.parametrize("na,nb,B", [(127, 10, 16384 + 37), (19, 10, 16384), (17, 16, 20001), (192, 16, 16385), (64, 4, 16401),
                                      (70, 1, 16390), (100, 8, 16384 + 63), (37, 3, 16387), (118, 10, 32768), (10, 10, 16389),
                                      (3, 16, 16400), (1, 1, 16385), (16, 2, 16384), (127, 10, 40005), (30, 10, 70001)])
def test_sum_tables_at_batches_that_fill_the_chip(dol, na, nb, B):
    """The same at batches where a lane owns a sample and a workgroup a tile of 64: whole tiles and a ragged last
    one, tiles that must re-derive the clamp decisions and (the second half of the batch) tiles that need not."""
    check_sum_table(dol, na, nb, B, calm_from=B // 2, kernel="rows")


def check_sum_table(dol, na, nb, B, calm_from=None, kernel=None):
    tab = W.sum_table(range(na), range(nb))
    x = min(1.0, 2.2 / np.sqrt(min(na, nb)))        # column sums of min(na, nb) terms scatter around 1
    a = (W.uniform01(na, B * na) * x).astype(np.float32).reshape(B, na)
    b = (W.uniform01(nb + 100, B * nb) * x).astype(np.float32).reshape(B, nb)
    for r, tot in enumerate((0.875, 1.0, 1.125)):
        a[r] = 0; b[r] = 0
        a[r, na - 1] = 1.0; b[r, 0] = tot
    a[3] *= 0.01                       # a sample far below the clamp takes the shortcut
    if calm_from is not None:
        a[calm_from:] *= 0.01
    tri = oracle.dense_to_triples(tab)
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    f = dol.FnTable.create_dense(tab)
    if kernel:
        assert f.kernel_at(False, B).startswith("damp_conv_fwd_%s_kernel" % (kernel if na > 16 else "small")), f.kernel_at(False, B)
        assert f.kernel_at(True, B).startswith("damp_conv_bwd_%s_kernel" % kernel), f.kernel_at(True, B)
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    do = dol.Dist.empty(syms, B)
    dol.apply2(da, db, f, None, do)
    got = host(do.prob)
    assert_close(got, want, "sum apply")
    np.testing.assert_array_equal(got == 1.0, pre32 >= 1.0)
    # one-signed upstream gradient: with tags of order 1 a float32 sum of mixed-sign terms cannot meet an
    # absolute 1e-7 where it cancels to ~0, whatever the kernel; the clamp decisions are what is under test here
    g = np.abs(W.normal(3, B * syms.size)).astype(np.float32).reshape(B, -1)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f), dev(g), ga, gb)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    assert_close(host(ga), wa, "sum bwd a")
    assert_close(host(gb), wb, "sum bwd b")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f, accumulate=3), dev(g), ga, gb)
    assert_close(host(ga), 2.0 * wa.astype(np.float64), "sum bwd a accumulated")
    assert_close(host(gb), 2.0 * wb.astype(np.float64), "sum bwd b accumulated")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f), dev(g), None, gb)      # one side only
    assert_close(host(gb), wb, "sum bwd b alone")


@pytest.mark.parametrize("B", [3, 70])
def test_tuple_list_backward_with_the_gradient_row_staged(dol, B):
    """A sparse table of 700 x 600 symbols onto 400 with a long row in either operand, tags large enough to put many
    results on the clamp: dol_backward through the kernel that works out the gated gradient row once per sample, with
    accumulation, one-sided calls and the decisions on the clamp compared with the oracle's."""
    na, nb, S = 700, 600, 400
    ti, tj, to = [], [], []
    for i in range(na):                                 # a few tuples per symbol of a
        for d in range(3):
            ti.append(i); tj.append((i * 7 + d * 131) % (nb - 1) + 1); to.append((i * 3 + d * 17) % S)
    for j in range(1, nb):                              # row 5 of a meets every symbol of b, symbol 0 of b every symbol of a
        ti.append(5); tj.append(j); to.append((j * 11) % S)
    for i in range(na):
        ti.append(i); tj.append(0); to.append((i * 13 + 1) % S)
    keys = sorted(set(zip(ti, tj)))
    first = {}
    for i, j, o in zip(ti, tj, to):
        first.setdefault((i, j), o)
    tri = tuple(np.asarray(x, np.int32) for x in ([k[0] for k in keys], [k[1] for k in keys], [first[k] for k in keys]))
    a = (W.uniform01(1, B * na) * 0.9).astype(np.float32).reshape(B, na)
    b = (W.uniform01(2, B * nb) * 0.5).astype(np.float32).reshape(B, nb)
    b[:, 0] = 1.0
    f = dol.FnTable.create_sparse(na, nb, *tri)
    assert f.kernel_bwd == "damp_apply2_bwd_staged_kernel", f.kernel_bwd
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    assert (pre32 > 1.0).mean() > 0.1 and (pre32 <= 1.0).mean() > 0.1
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    do = dol.Dist.empty(syms, B)
    dol.apply2(da, db, f, None, do)
    np.testing.assert_array_equal(host(do.prob) == 1.0, pre32 >= 1.0)
    g = np.abs(W.normal(3, B * syms.size)).astype(np.float32).reshape(B, -1)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    rec = dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f)
    dol.backward(rec, dev(g), ga, gb)
    assert_close(host(ga), wa, "staged bwd a")
    assert_close(host(gb), wb, "staged bwd b")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, do, f=f, accumulate=3), dev(g), ga, gb)
    assert_close(host(ga), 2.0 * wa.astype(np.float64), "staged bwd a accumulated")
    assert_close(host(gb), 2.0 * wb.astype(np.float64), "staged bwd b accumulated")
    ga2, gb2 = torch.empty_like(ga), torch.empty_like(gb)
    dol.backward(rec, dev(g), ga2, None)
    dol.backward(rec, dev(g), None, gb2)
    ga3, gb3 = torch.empty_like(ga), torch.empty_like(gb)
    dol.backward(rec, dev(g), ga3, gb3)
    np.testing.assert_array_equal(host(ga2), host(ga3))            # a fixed summation order: the same bits on every run
    np.testing.assert_array_equal(host(gb2), host(gb3))


def test_union_and_filter_edge_cases(dol):
    B = 50
    sa, sb = np.array([1, 4, 6, 8, 9], np.int32), np.array([0, 4, 9, 12], np.int32)
    a = (W.uniform01(4, B * 5) * 0.9).astype(np.float32).reshape(B, 5)
    b = (W.uniform01(5, B * 4) * 0.9).astype(np.float32).reshape(B, 4)
    a[0, 1], b[0, 1] = 0.5, 0.5          # a+b == 1 exactly: passes gradient
    a[1, 1], b[1, 1] = 0.75, 0.5         # clamps
    da, db = dol.Dist(sa, dev(a)), dol.Dist(sb, dev(b))
    syms = dol.union_plan(da, db)
    want_syms, ia, ib = oracle.union_plan(sa, sb)
    np.testing.assert_array_equal(syms, want_syms)
    do = dol.Dist.empty(syms, B)
    dol.union(da, db, None, do)
    assert_close(host(do.prob), oracle.damp_union_fwd(ia, ib, a, b), "union")
    g = W.normal(6, B * syms.size).astype(np.float32).reshape(B, -1)
    ga, gb = torch.empty_like(da.prob), torch.empty_like(db.prob)
    dol.backward(dol.OpRecord(dol.OP_UNION, da, db, do), dev(g), ga, gb)
    wa, wb = oracle.damp_union_bwd(ia, ib, a, b, g)
    np.testing.assert_array_equal(host(ga), wa)
    np.testing.assert_array_equal(host(gb), wb)
    # union with an empty Distribution is the identity
    de = dol.Dist(np.empty(0, np.int32), torch.empty((B, 0), device="cuda"))
    d2 = dol.Dist.empty(dol.union_plan(da, de), B)
    dol.union(da, de, None, d2)
    np.testing.assert_array_equal(host(d2.prob), a)
    # filter: all kept = identity, none kept = empty result, and the transpose
    d3 = dol.Dist.empty(sa, B)
    dol.filter(da, np.ones(5, np.uint8), None, d3)
    np.testing.assert_array_equal(host(d3.prob), a)
    assert dol.filter_plan(da, np.zeros(5, np.uint8)).size == 0
    d4 = dol.Dist(np.empty(0, np.int32), torch.empty((B, 0), device="cuda"))
    dol.filter(da, np.zeros(5, np.uint8), None, d4)
    pred = np.array([1, 0, 0, 1, 1], np.uint8)
    d5 = dol.Dist.empty(dol.filter_plan(da, pred), B)
    dol.filter(da, pred, None, d5)
    np.testing.assert_array_equal(host(d5.prob), oracle.damp_filter_fwd(pred, a))
    g5 = W.normal(7, B * 3).astype(np.float32).reshape(B, 3)
    gi = torch.full((B, 5), 9.0, device="cuda")
    dol.backward(dol.OpRecord(dol.OP_FILTER, da, None, d5, pred_mask=pred), dev(g5), gi, None)
    np.testing.assert_array_equal(host(gi), oracle.damp_filter_bwd(pred, g5))


def test_empty_batch_and_errors(dol):
    f = dol.FnTable.create_dense(W.sum_table(range(3), range(3)))
    e3 = dol.Dist(np.arange(3), torch.empty((0, 3), device="cuda"))
    e5 = dol.Dist(f.out_syms, torch.empty((0, 5), device="cuda"))
    dol.apply2(e3, e3, f, None, e5)                       # batch 0 is legal
    a = dol.Dist(np.arange(3), torch.ones((2, 3), device="cuda"))
    wrong = dol.Dist(np.arange(4), torch.ones((2, 4), device="cuda"))
    out = dol.Dist.empty(f.out_syms, 2)
    out.prob.fill_(-3.0)
    with pytest.raises(dol.DolError) as ei:
        dol.apply2(a, wrong, f, None, out)
    assert ei.value.status == 2 and "table" in str(ei.value)
    assert np.all(host(out.prob) == -3.0)                  # outputs untouched on error
    with pytest.raises(dol.DolError) as ei:
        dol.FnTable.create_sparse(2, 2, [0, 0], [1, 1], [5, 6])       # a function has one value per tuple
    assert ei.value.status == 1
    with pytest.raises(dol.DolError) as ei:
        dol.FnTable.create_sparse(2, 2, [0, 2], [1, 1], [5, 6])       # index outside the operand
    assert ei.value.status == 2
    none = dol.FnTable.create_dense(np.full((3, 3), -1, np.int32))     # nothing admitted: empty result, zero gradients
    assert none.n_out == 0
    o0 = dol.Dist(np.empty(0, np.int32), torch.empty((2, 0), device="cuda"))
    dol.apply2(a, a, none, None, o0)
    ga = torch.full((2, 3), 4.0, device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, a, a, o0, f=none), torch.empty((2, 0), device="cuda"), ga, None)
    assert np.all(host(ga) == 0)
    prov = dol.Prov(dol.DTKP, 3, torch.ones((2, 4), device="cuda"), None)
    with pytest.raises(dol.DolError) as ei:
        dol.backward(dol.OpRecord(dol.OP_APPLY2, a, a, out, f=f, prov=prov), out.prob, ga, None)
    assert ei.value.status == 5


def test_dtkp_general_conjunction_union_filter(dol):
    """k x k conjunction with overlapping fact sets, exclusion groups, then union and filter under DTKP."""
    B, k, n_facts = 40, 3, 12
    fp = W.uniform01(11, B * n_facts).astype(np.float32).reshape(B, n_facts)
    grp = np.array([0, 0, 0, 1, 1, 1, 2, 3, 4, 5, 6, 7], np.int32)
    d_fp = dev(fp)
    prov = dol.Prov(dol.DTKP, k, d_fp, grp)
    # two stages of apply so that the second sees multi-proof tags on both sides
    s0, s1 = np.arange(3, dtype=np.int32), np.arange(3, dtype=np.int32)
    tabs = [W.hashed_table(21, 3, 3, 4), W.hashed_table(22, 3, 3, 4)]
    facts = [[0, 1, 6], [3, 4, 7], [2, 8, 9], [5, 10, 11]]
    o_m = [oracle.dtkp_init(f, fp, k) for f in facts]
    g_d = []
    for f in facts:
        d = dol.Dist.empty(np.arange(3), B, k=k)
        dol.dtkp_init(d, f, prov)
        g_d.append(d)
    for x in range(4):
        np.testing.assert_array_equal(host(g_d[x].proof_mask).view(np.uint64), o_m[x][0])
        np.testing.assert_array_equal(host(g_d[x].proof_prob), o_m[x][1])
        np.testing.assert_array_equal(host(g_d[x].prob), o_m[x][2])
    mids_o, mids_g = [], []
    for x, tab in enumerate(tabs):
        tri = oracle.dense_to_triples(tab)
        so, om, op, opr = oracle.dtkp_apply2(tri, 3, 3, k, grp, fp, o_m[2 * x][0], o_m[2 * x + 1][0])
        f = dol.FnTable.create_dense(tab)
        out = dol.Dist.empty(f.out_syms, B, k=k)
        dol.apply2(g_d[2 * x], g_d[2 * x + 1], f, prov, out)
        np.testing.assert_array_equal(out.sym_ids, so)
        np.testing.assert_array_equal(host(out.proof_mask).view(np.uint64), om)
        np.testing.assert_array_equal(host(out.proof_prob), op)
        assert_close(host(out.prob), opr, "dtkp apply")
        mids_o.append((so, om, op, opr)); mids_g.append(out)
    # k x k conjunction of the two multi-proof results (facts of groups 0 and 1 overlap across sides)
    na, nb = mids_o[0][0].size, mids_o[1][0].size
    tab2 = W.hashed_table(23, na, nb, 5)
    tri2 = oracle.dense_to_triples(tab2)
    so, om, op, opr = oracle.dtkp_apply2(tri2, na, nb, k, grp, fp, mids_o[0][1], mids_o[1][1])
    f2 = dol.FnTable.create_dense(tab2)
    out2 = dol.Dist.empty(f2.out_syms, B, k=k)
    dol.apply2(mids_g[0], mids_g[1], f2, prov, out2)
    np.testing.assert_array_equal(host(out2.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(out2.proof_prob), op)
    assert_close(host(out2.prob), opr, "dtkp k x k apply")
    assert (om[:, :, 1] != oracle.ABSENT).any()
    # union of the two mid results (their symbol lists overlap)
    usyms, ia, ib = oracle.union_plan(mids_o[0][0], mids_o[1][0])
    um, up, upr = oracle.dtkp_union(ia, ib, mids_o[0][1], mids_o[0][2], mids_o[1][1], mids_o[1][2])
    uo = dol.Dist.empty(dol.union_plan(mids_g[0], mids_g[1]), B, k=k)
    np.testing.assert_array_equal(uo.sym_ids, usyms)
    dol.union(mids_g[0], mids_g[1], prov, uo)
    np.testing.assert_array_equal(host(uo.proof_mask).view(np.uint64), um)
    np.testing.assert_array_equal(host(uo.proof_prob), up)
    assert_close(host(uo.prob), upr, "dtkp union")
    # gradient of the k x k result's and the union's tag probabilities w.r.t. the facts (uniform fact probabilities
    # put several symbols over 1, so the clamp gate is exercised; proofs share facts across slots)
    for name, dist, masks, prob in (("k x k", out2, om, opr), ("union", uo, um, upr)):
        gsym = W.normal(31, B * masks.shape[1]).astype(np.float32).reshape(B, -1)
        want = oracle.dtkp_prob_bwd(masks, fp, gsym)
        gf = torch.full((B, n_facts), 7.0, device="cuda")
        dol.dtkp_backward(dist, prov, dev(gsym), gf)
        assert_close(host(gf), want, "dtkp gradient, " + name)
    assert (upr == 1.0).any() and (upr < 1.0).any()
    # filter
    pred = (np.arange(usyms.size) % 2 == 0).astype(np.uint8)
    fm, fpp, fpr = oracle.dtkp_filter(pred, um, up, upr)
    fo = dol.Dist.empty(dol.filter_plan(uo, pred), B, k=k)
    dol.filter(uo, pred, prov, fo)
    np.testing.assert_array_equal(host(fo.proof_mask).view(np.uint64), fm)
    np.testing.assert_array_equal(host(fo.proof_prob), fpp)
    np.testing.assert_array_equal(host(fo.prob), fpr)


@pytest.mark.parametrize("which", ["chain", "fold", "hashed", "hashed-fused", "dtkp-fold", "reach-fused", "reach-one-launch", "hashed-merged", "hashed-one-launch", "product",
                                   "formula-damp", "formula-dtkp"])
def test_hip_graph_replay_matches_eager(gp, which):
    """Every entry point issues only asynchronous launches once its symbol-side plans exist, so a whole step can be
    captured; replays (with eager work and synchronisations between them) equal the eager result."""
    if which == "chain":
        prog = gp.SumChain(W.config2(batch=512, n_digits=6, seed=5)); key = lambda: prog.grad_p
    elif which == "fold":
        prog = gp.SumChainFused(W.config2(batch=512, n_digits=6, seed=5)); key = lambda: prog.grad_p
    elif which == "hashed":
        prog = gp.HashedPipeline(W.config3(batch=320, seed=5)); key = lambda: prog.ga
    elif which == "hashed-fused":
        prog = gp.HashedPipelineFused(W.config3(batch=320, seed=5)); key = lambda: prog.ga
    elif which == "hashed-merged":
        prog = gp.HashedPipelineMerged(W.config3(batch=320, seed=5)); key = lambda: prog.ga
    elif which == "hashed-one-launch":
        prog = gp.HashedPipelineMerged(W.config3(batch=320, seed=5), one_launch=True); key = lambda: prog.ga
    elif which == "reach-one-launch":
        prog = gp.GridReachFused(W.config5(batch=16, side=8, rounds=12, seed=5), one_launch=True); key = lambda: prog.grad_p
    elif which == "dtkp-fold":
        prog = gp.DtkpSumChainFused(W.config4(batch=200, seed=5), with_gradient=True); key = lambda: prog.grad_fact
    elif which == "product":
        prog = gp.ProductChain(W.product_workload(batch=40, n_digits=7, seed=5)); key = lambda: prog.grad_p
    elif which == "formula-damp":
        prog = gp.HwfPipeline(W.hwf_workload(batch=24, length=5, seed=5), "damp"); key = lambda: prog.grad_p
    elif which == "formula-dtkp":
        prog = gp.HwfPipeline(W.hwf_workload(batch=24, length=5, seed=5), "dtkp"); key = lambda: prog.grad_p
    else:
        prog = gp.GridReachFused(W.config5(batch=16, side=8, rounds=12, seed=5)); key = lambda: prog.grad_p
    prog.step()
    eager = host(key()).copy()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        prog.step()
    torch.cuda.current_stream().wait_stream(s)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        prog.step()
    for _ in range(3):
        key().fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        np.testing.assert_array_equal(host(key()), eager)


# ---------------------------------------------------------------- large batches: sampled rows against the oracle

def _rows_of(w, idx, per_sample):
    """A sub-workload holding only the samples `idx` (samples are independent, so the oracle can run on them alone)."""
    arrays = {}
    for name, arr in w.arrays.items():
        axis = per_sample.get(name)
        arrays[name] = arr if axis is None else np.ascontiguousarray(np.take(arr, idx, axis=axis))
    params = dict(w.params, batch=len(idx))
    return W.Workload(w.name, params, arrays)


def _sample_rows(batch, n=48):
    picks = (W.splitmix64(batch, np.arange(n, dtype=np.uint64)) % np.uint64(batch)).astype(np.int64)
    return np.unique(np.concatenate([[0, 1, 63, 64, batch // 2, batch - 2, batch - 1], picks]))


@pytest.mark.parametrize("cfg,batch", [(2, 200003), (3, 70001), (4, 50021), (5, 1031)])
def test_large_batches_sampled_rows(gp, cfg, batch):
    """The launch shapes of the B-scaled bench variants (odd batches, many tiles per workgroup, grids of 10^5
    workgroups): rows sampled over the whole batch against the oracle run on those samples alone."""
    w = W.make_config(cfg, batch=batch, seed=11)
    idx = _sample_rows(batch)
    if cfg == 2:
        prog = gp.SumChainFused(w)
        prog.step()
        ref = OP.sum_chain_fwd_bwd(_rows_of(w, idx, dict(p=1, target=0)))
        assert_close(host(prog.out.prob)[idx], ref["out"], "fold forward, sampled rows")
        assert_close(host(prog.grad_p)[:, idx], ref["grad_p"], "fold gradient, sampled rows")
    elif cfg == 3:
        ref = OP.hashed_pipeline_fwd_bwd(_rows_of(w, idx, dict(pa=0, pb=0, p2=0, g=0)))
        for cls in (gp.HashedPipelineMerged, gp.HashedPipelineFused):     # the bench's two launches; Apply, then Filter + Union
            prog = cls(w)
            prog.step()
            assert_close(host(prog.o3.prob)[idx], ref["o3"], "hashed pipeline forward, sampled rows")
            assert_close(host(prog.ga)[idx], ref["ga"], "hashed pipeline grad a, sampled rows")
            assert_close(host(prog.gb)[idx], ref["gb"], "hashed pipeline grad b, sampled rows")
            assert_close(host(prog.gp2)[idx], ref["gp2"], "hashed pipeline grad p2, sampled rows")
            del prog
    elif cfg == 4:
        prog = gp.DtkpSumChainFused(w)
        prog.step()
        ref = OP.dtkp_sum_chain(_rows_of(w, idx, dict(p=1, fact_prob=0)))
        np.testing.assert_array_equal(host(prog.out.proof_mask).view(np.uint64)[idx], ref["mask"])
        np.testing.assert_array_equal(host(prog.out.proof_prob)[idx], ref["pprob"])
        assert_close(host(prog.out.prob)[idx], ref["prob"], "dtkp fold, sampled rows")
    else:
        ref = OP.grid_reach_fwd_bwd(_rows_of(w, idx, dict(p=0, g=0)))
        for one_launch in (True, False):                                   # the bench's single launch; the two sweeps apart
            prog = gp.GridReachFused(w, one_launch=one_launch)
            prog.step()
            assert_close(host(prog.out.prob)[idx], ref["r"], "reachability, sampled rows")
            assert_close(host(prog.grad_p)[idx], ref["grad_p"], "reachability gradient, sampled rows")
            del prog


# ---------------------------------------------------------------- Apply over K Distributions, unary Apply, ApplyIf

def _rand_table(seed, shape, n_ids, drop_every=0):
    t = (W.splitmix64(seed, np.arange(int(np.prod(shape)))) % np.uint64(n_ids)).astype(np.int32).reshape(shape)
    if drop_every:
        t.reshape(-1)[::drop_every] = -1
    return t


@pytest.mark.parametrize("shape,n_ids,scale,batch", [
    ((37,), 6, 1.0, 300), ((37,), 6, 9.0, 45),                      # unary, second one clamps
    ((10, 10), 19, 1.0, 129), ((10, 10, 10), 28, 1.0, 513),         # sums of two and three digits
    ((9, 5, 7), 40, 3.2, 200), ((4, 3, 5, 4), 23, 1.0, 77), ((3, 2, 3, 2, 3), 11, 2.0, 64),
    ((2, 3, 2, 2, 3, 2), 9, 1.0, 33), ((300, 4, 3), 500, 1.0, 1000), ((2100,), 2100, 1.0, 3)])
def test_apply_k_damp_forward_and_backward(dol, shape, n_ids, scale, batch):
    K = len(shape)
    if n_ids in (19, 28):      # digit sums
        table = np.zeros(shape, np.int32)
        for l in range(K):
            table = table + np.arange(10).reshape([-1 if m == l else 1 for m in range(K)])
        table = table.astype(np.int32)
    else:
        table = _rand_table(300 + K, shape, n_ids, drop_every=5)
    ins = [(W.softmax_rows(W.normal(310 + l, batch * n).reshape(batch, n)) * scale).astype(np.float32)
           for l, n in enumerate(shape)]
    idx, to = oracle.dense_to_tuples(table)
    syms, want, pre32, _ = oracle.damp_applyk_fwd(idx, to, ins, want_pre=True)
    f = dol.FnkTable.create_dense(table)
    np.testing.assert_array_equal(f.out_syms, syms)
    if K == 1:      # rows of fewer than 2 048 tags stay with the cached gathers
        want_names = ("damp_apply1_fwd_kernel", "damp_apply1_bwd_kernel") if shape[0] < 2048 else \
                     ("damp_apply1_fwd_staged_kernel", "damp_apply1_bwd_staged_kernel")
    else:
        want_names = ("damp_applyk_fwd_kernel<%d>" % K, "damp_applyk_bwd_kernel<%d>" % K)
    assert (f.kernel_fwd, f.kernel_bwd) == want_names
    lds = [n + (3 if l % 2 else 0) for l, n in enumerate(shape)]       # some operands with padded rows
    d_in = []
    for x, n, ld in zip(ins, shape, lds):
        buf = torch.zeros((batch, ld), device="cuda")
        buf[:, :n] = dev(x)
        d_in.append(dol.Dist(np.arange(n), buf[:, :n]))
    out = dol.Dist.empty(f.out_syms, batch)
    dol.apply_k(d_in, f, None, out)
    assert_close(host(out.prob), want, "apply_k forward")
    if scale > 1.0:
        assert (pre32 > 1).any() and (pre32 < 1).any()
    sign = np.float32(1.0) if scale > 1.0 else None
    g = W.normal(320, batch * syms.size).astype(np.float32).reshape(batch, -1)
    if sign is not None:
        g = np.abs(g)
    wants = oracle.damp_applyk_bwd(idx, to, ins, g)
    grads = [torch.full((batch, ld), 5.0, device="cuda") for ld in lds]
    skip = 1 if K >= 3 else None
    dol.apply_k_backward(d_in, f, out, dev(g), [None if l == skip else gr for l, gr in enumerate(grads)])
    for l, n in enumerate(shape):
        got = host(grads[l])
        if l == skip:
            assert np.all(got == 5.0)
            continue
        assert_close(got[:, :n], wants[l], "apply_k grad of operand %d" % l)
        assert np.all(got[:, n:] == 5.0)


@pytest.mark.parametrize("batch", [3, 300])
def test_wide_operand_rows_staged_in_lds(dol, batch):
    """Unary and binary Apply over operand rows of thousands of tags (the kernels that copy a sample's rows into LDS
    and gather there): a few workgroups per sample at batch 3, one at batch 300; padded rows whose starts fall off
    16-byte boundaries; columns of every length from 1 up, one of them long enough for the wavefront kernel; tags
    scaled so that columns clamp, with pre exactly 1 (gradient passes) and pre > 1 (blocked) in sample 0."""
    # ---- unary
    n_in, n_ids = 5001, 700
    table = _rand_table(6100, (n_in,), n_ids, drop_every=9)
    table[:200:2] = 5                                                  # 100 symbols on one column
    x = (W.softmax_rows(W.normal(6101, batch * n_in).reshape(batch, n_in)) * 700.0).astype(np.float32)
    x[0, :] = 0.125                                                    # columns of 8 symbols sum to exactly 1
    idx, to = oracle.dense_to_tuples(table)
    syms, want, pre32, _ = oracle.damp_applyk_fwd(idx, to, [x], want_pre=True)
    assert (pre32[0] == 1).any() and (pre32 > 1).any() and (pre32 < 1).any()
    f = dol.FnkTable.create_dense(table)
    assert (f.kernel_fwd, f.kernel_bwd) == ("damp_apply1_fwd_staged_kernel", "damp_apply1_bwd_staged_kernel")
    buf = torch.zeros((batch, n_in + 3), device="cuda")
    buf[:, :n_in] = dev(x)
    d_in = [dol.Dist(np.arange(n_in), buf[:, :n_in])]
    out = dol.Dist.empty(f.out_syms, batch)
    dol.apply_k(d_in, f, None, out)
    assert_close(host(out.prob), want, "wide unary forward")
    g = np.abs(W.normal(6102, batch * syms.size).astype(np.float32).reshape(batch, -1)) + np.float32(0.5)
    (wx,) = oracle.damp_applyk_bwd(idx, to, [x], g)
    gx = torch.full((batch, n_in + 3), 5.0, device="cuda")
    dol.apply_k_backward(d_in, f, out, dev(g), [gx])
    got = host(gx)
    np.testing.assert_array_equal(got[:, :n_in], wx)                   # each entry is a gradient entry or 0
    assert np.all(got[:, n_in:] == 5.0)
    assert (wx[0] == 0).any() and (wx[0] != 0).any()
    # ---- binary
    na, nb = 3000, 20
    table2 = _rand_table(6110, (na, nb), 9000, drop_every=7)
    table2[:90, 0] = 17                                                # a long column
    a = (W.softmax_rows(W.normal(6111, batch * na).reshape(batch, na)) * (na * 1.2)).astype(np.float32)
    b = (W.softmax_rows(W.normal(6112, batch * nb).reshape(batch, nb)) * 3.0).astype(np.float32)
    tri = oracle.dense_to_triples(table2)
    syms2, want2, pre2, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    assert (pre2 > 1).any() and (pre2 < 1).any()
    f2 = dol.FnTable.create_dense(table2)
    assert f2.kernel_fwd == "damp_apply2_fwd_staged_kernel"
    abuf = torch.zeros((batch, na + 1), device="cuda")
    abuf[:, :na] = dev(a)
    bbuf = torch.zeros((batch, nb + 2), device="cuda")
    bbuf[:, :nb] = dev(b)
    da, db = dol.Dist(np.arange(na), abuf[:, :na]), dol.Dist(np.arange(nb), bbuf[:, :nb])
    out2 = dol.Dist.empty(f2.out_syms, batch)
    dol.apply2(da, db, f2, None, out2)
    np.testing.assert_array_equal(out2.sym_ids, syms2)
    assert_close(host(out2.prob), want2, "wide binary forward")
    np.testing.assert_array_equal(host(out2.prob) == 1.0, pre2 >= 1.0)
    # ---- binary with a short second operand: the per-j map kernels with the long row (forward) and the gated
    # gradient row (backward) in LDS; columns where some j occurs twice go through their tuple lists
    nb3 = 7
    table3 = _rand_table(6120, (na, nb3), 2500, drop_every=7)
    b3 = (W.softmax_rows(W.normal(6122, batch * nb3).reshape(batch, nb3)) * 1.1).astype(np.float32)
    tri3 = oracle.dense_to_triples(table3)
    syms3, want3, pre3, _ = oracle.damp_apply2_fwd(tri3, na, nb3, a, b3, want_pre=True)
    assert (pre3 > 1).any() and (pre3 < 1).any()
    f3 = dol.FnTable.create_dense(table3)
    assert (f3.kernel_fwd, f3.kernel_bwd) == ("damp_byj_fwd_staged_kernel", "damp_byj_bwd_row_kernel")
    db3 = dol.Dist(np.arange(nb3), dev(b3))
    out3 = dol.Dist.empty(f3.out_syms, batch)
    dol.apply2(da, db3, f3, None, out3)
    assert_close(host(out3.prob), want3, "wide per-j forward")
    np.testing.assert_array_equal(host(out3.prob) == 1.0, pre3 >= 1.0)
    g3 = np.abs(W.normal(6123, batch * syms3.size).astype(np.float32).reshape(batch, -1)) + np.float32(0.5)
    wa3, wb3 = oracle.damp_apply2_bwd(tri3, na, nb3, a, b3, g3)
    ga3 = torch.full((batch, na + 1), 5.0, device="cuda")
    gb3 = torch.empty((batch, nb3), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db3, out3, f=f3), dev(g3), ga3, gb3)
    assert_close(host(ga3)[:, :na], wa3, "wide per-j grad a")
    assert_close(host(gb3), wb3, "wide per-j grad b")
    assert np.all(host(ga3)[:, na:] == 5.0)


def test_apply_k_two_operands_equal_apply2_bit_for_bit(dol):
    B = 150
    table = W.hashed_table(41, 30, 20, 64)
    a = (W.softmax_rows(W.normal(42, B * 30).reshape(B, 30)) * 2).astype(np.float32)
    b = (W.softmax_rows(W.normal(43, B * 20).reshape(B, 20)) * 2).astype(np.float32)
    da, db = dol.Dist(np.arange(30), dev(a)), dol.Dist(np.arange(20), dev(b))
    f2, fk = dol.FnTable.create_dense(table), dol.FnkTable.create_dense(table)
    np.testing.assert_array_equal(f2.out_syms, fk.out_syms)
    o2, ok = dol.Dist.empty(f2.out_syms, B), dol.Dist.empty(fk.out_syms, B)
    dol.apply2(da, db, f2, None, o2)
    dol.apply_k([da, db], fk, None, ok)
    np.testing.assert_array_equal(host(o2.prob), host(ok.prob))


def test_apply_if_table(dol):
    B, na, nb = 90, 12, 9
    table = W.hashed_table(51, na, nb, 16)
    cond = ((np.arange(na)[:, None] + np.arange(nb)[None, :]) % 3 != 1)
    a = W.softmax_rows(W.normal(52, B * na).reshape(B, na))
    b = W.softmax_rows(W.normal(53, B * nb).reshape(B, nb))
    tri = oracle.dense_to_triples(np.where(cond, table, -1))
    syms, want = oracle.damp_apply2_fwd(tri, na, nb, a, b)
    g = W.normal(54, B * syms.size).astype(np.float32).reshape(B, -1)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    junk = np.where(cond, table, -7).astype(np.int32)               # entries the condition rejects are never read
    f = dol.FnTable.create_if(junk, cond)
    np.testing.assert_array_equal(f.out_syms, syms)
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    out = dol.Dist.empty(f.out_syms, B)
    dol.apply2(da, db, f, None, out)
    assert_close(host(out.prob), want, "apply_if forward")
    ga, gb = torch.empty((B, na), device="cuda"), torch.empty((B, nb), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, out, f=f), dev(g), ga, gb)
    assert_close(host(ga), wa, "apply_if grad a")
    assert_close(host(gb), wb, "apply_if grad b")
    with pytest.raises(dol.DolError):
        dol.FnTable.create_if(np.full((2, 2), -1, np.int32), np.ones((2, 2), np.uint8))


@pytest.mark.parametrize("k", [1, 3, 8])
def test_apply_k_dtkp(dol, k):
    """Three operands with multi-proof tags and exclusion groups, then a unary Apply that merges symbols."""
    B, nv = 60, 4
    fp = np.concatenate([W.softmax_rows(W.normal(60 + t, B * nv).reshape(B, nv)) for t in range(4)], axis=1)
    grp = np.repeat(np.arange(4), nv).astype(np.int32)
    prov = dol.Prov(dol.DTKP, k, dev(fp), grp)
    o_tags, g_tags = [], []
    for t in range(4):
        o_tags.append(oracle.dtkp_init(np.arange(nv) + nv * t, fp, k)[0])
        d = dol.Dist.empty(np.arange(nv), B, k=k)
        dol.dtkp_init(d, np.arange(nv) + nv * t, prov)
        g_tags.append(d)
    # operand 0: sum of slots 0 and 1 (several proofs per symbol)
    sum_t = np.add.outer(np.arange(nv), np.arange(nv)).astype(np.int32)
    s0, m0, p0, _ = oracle.dtkp_apply2(oracle.dense_to_triples(sum_t), nv, nv, k, grp, fp, o_tags[0], o_tags[1])
    f0 = dol.FnTable.create_dense(sum_t)
    a = dol.Dist.empty(f0.out_syms, B, k=k)
    dol.apply2(g_tags[0], g_tags[1], f0, prov, a)
    table = _rand_table(70, (s0.size, nv, nv), 9, drop_every=6)
    idx, to = oracle.dense_to_tuples(table)
    syms, om, op, opr = oracle.dtkp_applyk(idx, to, k, grp, fp, [m0, o_tags[2], o_tags[3]])
    f = dol.FnkTable.create_dense(table)
    np.testing.assert_array_equal(f.out_syms, syms)
    out = dol.Dist.empty(f.out_syms, B, k=k)
    dol.apply_k([a, g_tags[2], g_tags[3]], f, prov, out)
    np.testing.assert_array_equal(host(out.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(out.proof_prob), op)
    assert_close(host(out.prob), opr, "dtkp apply_k")
    # the same call with the operands' stored proof probabilities withheld
    bare = [dol.Dist(d.sym_ids, d.prob, d.proof_mask, None) for d in (a, g_tags[2], g_tags[3])]
    out_b = dol.Dist.empty(f.out_syms, B, k=k)
    dol.apply_k(bare, f, prov, out_b)
    np.testing.assert_array_equal(host(out_b.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(out_b.proof_prob), op)
    # unary Apply over the result
    f1 = (np.arange(syms.size) % 3).astype(np.int32)
    f1[2] = -1
    idx1, to1 = oracle.dense_to_tuples(f1)
    s1, m1, p1, pr1 = oracle.dtkp_applyk(idx1, to1, k, grp, fp, [om])
    fu = dol.FnkTable.create_dense(f1)
    np.testing.assert_array_equal(fu.out_syms, s1)
    out1 = dol.Dist.empty(fu.out_syms, B, k=k)
    dol.apply_k([out], fu, prov, out1)
    np.testing.assert_array_equal(host(out1.proof_mask).view(np.uint64), m1)
    np.testing.assert_array_equal(host(out1.proof_prob), p1)
    assert_close(host(out1.prob), pr1, "dtkp unary apply")
    if k > 1:
        assert (m1[:, :, 1] != oracle.ABSENT).any()


def test_apply_k_argument_errors_and_empty(dol):
    with pytest.raises(dol.DolError):
        dol.FnkTable([3, 3], [[0, 0], [0, 0]], [1, 2])              # one index tuple twice
    with pytest.raises(dol.DolError):
        dol.FnkTable([3, 3], [[0, 3]], [1])                         # position outside the operand
    with pytest.raises(dol.DolError):
        dol.FnkTable([2] * 7, np.zeros((1, 7), np.int32), [1])      # too many operands
    f = dol.FnkTable.create_dense(np.arange(6, dtype=np.int32).reshape(2, 3))
    a, b = dol.Dist(np.arange(2), torch.ones((4, 2), device="cuda")), dol.Dist(np.arange(3), torch.ones((4, 3), device="cuda"))
    with pytest.raises(dol.DolError) as ei:
        dol.apply_k([a, b], f, None, dol.Dist.empty(np.arange(5), 4))
    assert ei.value.status == 2
    with pytest.raises(dol.DolError):
        dol.apply_k([b, a], f, None, dol.Dist.empty(f.out_syms, 4))
    with pytest.raises(dol.DolError):
        dol.apply_k([a], f, None, dol.Dist.empty(f.out_syms, 4))
    none = dol.FnkTable.create_dense(np.full((2, 3), -1, np.int32))
    assert none.n_out == 0
    o0 = dol.Dist.empty(none.out_syms, 4)
    dol.apply_k([a, b], none, None, o0)
    ga = torch.full((4, 2), 3.0, device="cuda")
    dol.apply_k_backward([a, b], none, o0, torch.empty((4, 0), device="cuda"), [ga, None])
    assert np.all(host(ga) == 0)
    e = dol.Dist.empty(f.out_syms, 0)
    dol.apply_k([dol.Dist(np.arange(2), torch.ones((0, 2), device="cuda")), dol.Dist(np.arange(3), torch.ones((0, 3), device="cuda"))], f, None, e)


# ---------------------------------------------------------------- Product-N fold (irregular growing symbol sets)

@pytest.mark.parametrize("batch,n", [(64, 4), (256, 8), (33, 11)])
def test_product_chain(gp, batch, n):
    """The fold of Fig. 2 with f = x * y: tables without structure, a zero column that every row feeds (summed by a
    wavefront once it is long), operand rows longer than a thread's share in the backward pass."""
    w = W.product_workload(batch=batch, n_digits=n, seed=n)
    ref = OP.product_chain_fwd_bwd(w)
    prog = gp.ProductChain(w)
    prog.step()
    np.testing.assert_array_equal(prog.accs[-1].sym_ids, ref["syms"])
    for t in range(1, n):
        assert_close(host(prog.accs[t].prob), ref["accs"][t], "product stage %d" % t)
    assert_close(host(prog.g_acc[-1]), ref["g_out"], "loss gradient")
    assert_close(host(prog.grad_p), ref["grad_p"], "product chain grad")


def test_long_column_near_the_clamp_takes_the_defining_order(dol):
    """A column of 3000 tuples whose sum lies within rounding of 1: the clamp decision (seen through backward) must be
    the one of the sequential float sum, on either side of 1."""
    B, na = 48, 3000
    table = np.zeros((na, 1), np.int32)                      # every symbol maps to 0: one long column
    a = W.uniform01(81, B * na).astype(np.float32).reshape(B, na)
    a = (a / a.sum(1, keepdims=True, dtype=np.float64)).astype(np.float32)       # rows sum to 1 up to rounding
    a[::3] *= np.float32(1.0 + 2e-7)
    b = np.ones((B, 1), np.float32)
    tri = oracle.dense_to_triples(table)
    syms, want, pre32, pre64 = oracle.damp_apply2_fwd(tri, na, 1, a, b, want_pre=True)
    assert (pre32 > 1).any() and (pre32 <= 1).any() and np.abs(pre64 - 1).max() < 1e-5
    g = np.ones((B, 1), np.float32)
    wa, wb = oracle.damp_apply2_bwd(tri, na, 1, a, b, g)
    f = dol.FnTable.create_dense(table)
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(1), dev(b))
    out = dol.Dist.empty(f.out_syms, B)
    dol.apply2(da, db, f, None, out)
    assert_close(host(out.prob), want, "long column forward")
    ga, gb = torch.empty((B, na), device="cuda"), torch.empty((B, 1), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, out, f=f), dev(g), ga, gb)
    np.testing.assert_array_equal(host(ga), wa)              # 0 or 1 per sample: the decision itself
    assert_close(host(gb), wb, "long column grad b")


# ---------------------------------------------------------------- formula pipeline (filter -> chained apply -> unary apply)

@pytest.mark.parametrize("batch,length", [(64, 7), (33, 5), (5, 1)])
def test_formula_pipeline_damp(gp, batch, length):
    w = W.hwf_workload(batch=batch, length=length, seed=length)
    ref = OP.hwf_pipeline_damp(w)
    prog = gp.HwfPipeline(w, "damp")
    prog.step()
    np.testing.assert_array_equal(prog.out.sym_ids, ref["syms"])
    for t in range(1, length):
        assert_close(host(prog.accs[t].prob), ref["accs"][t], "formula stage %d" % t)
    assert_close(host(prog.out.prob), ref["out"], "formula values")
    assert_close(host(prog.grad_p), ref["grad_p"], "formula grad")


@pytest.mark.parametrize("batch,length,k", [(64, 7, 3), (20, 5, 1), (9, 3, 8)])
def test_formula_pipeline_dtkp(gp, batch, length, k):
    w = W.hwf_workload(batch=batch, length=length, k=k, seed=40 + length)
    ref = OP.hwf_pipeline_dtkp(w)
    prog = gp.HwfPipeline(w, "dtkp")
    prog.step()
    np.testing.assert_array_equal(host(prog.fact_prob), ref["fact_prob"])
    for t in range(1, length):
        m, pp, pr = ref["stages"][t - 1]
        np.testing.assert_array_equal(host(prog.accs[t].proof_mask).view(np.uint64), m)
        np.testing.assert_array_equal(host(prog.accs[t].proof_prob), pp)
    np.testing.assert_array_equal(host(prog.out.proof_mask).view(np.uint64), ref["mask"])
    np.testing.assert_array_equal(host(prog.out.proof_prob), ref["pprob"])
    assert_close(host(prog.out.prob), ref["prob"], "formula value probabilities")
    assert_close(host(prog.gfact), ref["gfact"], "formula fact gradient")
    assert_close(host(prog.grad_p), ref["grad_p"], "formula class gradient")


def test_apply_k_long_columns(dol):
    """Columns of hundreds to thousands of tuples (summed by a wavefront): a unary map onto one symbol whose sum lies
    within rounding of 1, where the clamp decision must still be the sequential float sum's, and a three-operand
    function with two images."""
    B, n = 40, 3000
    x = W.uniform01(91, B * n).astype(np.float32).reshape(B, n)
    x = (x / x.sum(1, keepdims=True, dtype=np.float64)).astype(np.float32)
    x[::3] *= np.float32(1.0 + 2e-7)
    idx, to = oracle.dense_to_tuples(np.zeros(n, np.int32))
    syms, want, pre32, pre64 = oracle.damp_applyk_fwd(idx, to, [x], want_pre=True)
    assert (pre32 > 1).any() and (pre32 <= 1).any() and np.abs(pre64 - 1).max() < 1e-5
    (wg,) = oracle.damp_applyk_bwd(idx, to, [x], np.ones((B, 1), np.float32))
    f = dol.FnkTable.create_dense(np.zeros(n, np.int32))
    d = dol.Dist(np.arange(n), dev(x))
    out = dol.Dist.empty(f.out_syms, B)
    dol.apply_k([d], f, None, out)
    assert_close(host(out.prob), want, "long unary column")
    gx = torch.empty((B, n), device="cuda")
    dol.apply_k_backward([d], f, out, torch.ones((B, 1), device="cuda"), [gx])
    np.testing.assert_array_equal(host(gx), wg)
    # three operands, two images: columns of about 500 tuples, one side of them over 1
    shape = (40, 5, 5)
    table = _rand_table(95, shape, 2)
    ins = [(W.softmax_rows(W.normal(96 + l, B * m).reshape(B, m)) * (1.3 if l == 0 else 1.0)).astype(np.float32)
           for l, m in enumerate(shape)]
    idx, to = oracle.dense_to_tuples(table)
    syms, want, pre32, _ = oracle.damp_applyk_fwd(idx, to, ins, want_pre=True)
    g = np.abs(W.normal(99, B * 2)).astype(np.float32).reshape(B, 2)
    wants = oracle.damp_applyk_bwd(idx, to, ins, g)
    f3 = dol.FnkTable.create_dense(table)
    d3 = [dol.Dist(np.arange(m), dev(v)) for m, v in zip(shape, ins)]
    out3 = dol.Dist.empty(f3.out_syms, B)
    dol.apply_k(d3, f3, None, out3)
    assert_close(host(out3.prob), want, "long three-operand columns")
    grads = [torch.empty((B, m), device="cuda") for m in shape]
    dol.apply_k_backward(d3, f3, out3, dev(g), grads)
    for l in range(3):
        assert_close(host(grads[l]), wants[l], "long three-operand grad %d" % l)


def test_short_second_operand_tables_near_the_clamp(dol):
    """f(i, j) = i + 2j over 800 x 4 symbols: columns of four tuples whose defining order (ascending i) is the
    reverse of the order the per-j kernel adds them in, with sums within rounding of 1; clamp decisions (seen
    through backward) must be those of the defining order."""
    B, na, nb = 96, 800, 4
    table = (np.arange(na)[:, None] + 2 * np.arange(nb)[None, :]).astype(np.int32)
    a = np.ones((B, na), np.float32)
    b = W.softmax_rows(W.normal(71, B * nb).reshape(B, nb))
    b[::4] *= np.float32(1.0 + 1.2e-7)
    tri = oracle.dense_to_triples(table)
    syms, want, pre32, pre64 = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    inner = pre32[:, 6:na]
    assert (inner > 1).any() and (inner <= 1).any() and np.abs(pre64[:, 6:na] - 1).max() < 1e-6
    g = np.abs(W.normal(72, B * syms.size)).astype(np.float32).reshape(B, -1)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    f = dol.FnTable.create_dense(table)
    assert f.kernel_fwd == "damp_byj_fwd_kernel" and f.kernel_bwd == "damp_byj_bwd_kernel"
    da, db = dol.Dist(np.arange(na), dev(a)), dol.Dist(np.arange(nb), dev(b))
    out = dol.Dist.empty(f.out_syms, B)
    dol.apply2(da, db, f, None, out)
    assert_close(host(out.prob), want, "per-j forward")
    ga, gb = torch.empty((B, na), device="cuda"), torch.empty((B, nb), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, out, f=f), dev(g), ga, gb)
    assert_close(host(ga), wa, "per-j grad a")
    assert_close(host(gb), wb, "per-j grad b")


# ---------------------------------------------------------------- seeded random tables over every kernel choice

@pytest.mark.parametrize("seed", range(24))
def test_random_tables_differential(dol, seed):
    """Random table shapes, densities, image counts, batch sizes and paddings (drawn from a seeded stream), so that
    every kernel the library can pick for dol_apply2 / dol_backward (LDS gather, per-j maps with and without the
    workgroup-per-sample backward, tuple lists, wavefront columns and rows) meets the oracle on shapes nobody chose
    by hand.  One-signed upstream gradient (see the module docstring)."""
    r = W.splitmix64(5000 + seed, np.arange(16)).astype(np.uint64)
    pick = lambda k, lo, hi: int(lo + r[k] % np.uint64(hi - lo + 1))
    na = [pick(0, 1, 40), pick(0, 100, 700), pick(0, 1025, 3000)][seed % 3]
    nb = [pick(1, 1, 16), pick(1, 17, 60), pick(1, 1, 4)][(seed // 3) % 3]
    n_ids = max(1, [pick(2, 1, 8), pick(2, na // 2 + 1, na + nb), pick(2, 2 * na, 3 * na)][(seed // 9) % 3])
    batch = pick(3, 1, 70)
    table = (W.splitmix64(6000 + seed, np.arange(na * nb)) % np.uint64(n_ids)).astype(np.int32).reshape(na, nb)
    drop = pick(4, 0, 3)
    if drop:
        table.reshape(-1)[::drop + 1] = -1
    scale = [1.0, 1.0, float(max(1.0, 0.7 * n_ids))][pick(5, 0, 2)]
    a = (W.softmax_rows(W.normal(7000 + seed, batch * na).reshape(batch, na)) * scale).astype(np.float32)
    b = W.softmax_rows(W.normal(8000 + seed, batch * nb).reshape(batch, nb))
    tri = oracle.dense_to_triples(table)
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, na, nb, a, b, want_pre=True)
    g = np.abs(W.normal(9000 + seed, batch * max(syms.size, 1))).astype(np.float32).reshape(batch, -1)[:, :syms.size]
    g = np.ascontiguousarray(g)
    wa, wb = oracle.damp_apply2_bwd(tri, na, nb, a, b, g)
    f = dol.FnTable.create_dense(table)
    np.testing.assert_array_equal(f.out_syms, syms)
    pad = pick(6, 0, 5)
    abuf = torch.zeros((batch, na + pad), device="cuda")
    abuf[:, :na] = dev(a)
    da, db = dol.Dist(np.arange(na), abuf[:, :na]), dol.Dist(np.arange(nb), dev(b))
    out = dol.Dist.empty(f.out_syms, batch)
    dol.apply2(da, db, f, None, out)
    what = "seed %d: %d x %d -> %d, batch %d, %s / %s" % (seed, na, nb, syms.size, batch, f.kernel_fwd, f.kernel_bwd)
    assert_close(host(out.prob), want, what + " forward")
    ga = torch.full((batch, na + pad), 3.0, device="cuda")
    gb = torch.empty((batch, nb), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, out, f=f), dev(g), ga, gb)
    assert_close(host(ga)[:, :na], wa, what + " grad a")
    assert np.all(host(ga)[:, na:] == 3.0)
    assert_close(host(gb), wb, what + " grad b")


@pytest.mark.parametrize("seed", range(8))
def test_random_tables_differential_dtkp(dol, seed):
    """The same under DTKP-AM: multi-proof operands (results of earlier applies over shared exclusion groups), few
    images so that columns run from a handful to hundreds of tuples (thread and wavefront kernels), k from 1 to 5;
    also the K-operand call on the same table."""
    r = W.splitmix64(5100 + seed, np.arange(8)).astype(np.uint64)
    k = [1, 2, 3, 5][seed % 4]
    B, nv = int(3 + r[0] % np.uint64(40)), 6
    fp = np.concatenate([W.softmax_rows(W.normal(5200 + seed * 4 + t, B * nv).reshape(B, nv)) for t in range(4)], axis=1)
    grp = np.repeat(np.arange(4), nv).astype(np.int32)
    prov = dol.Prov(dol.DTKP, k, dev(fp), grp)
    o_ops, g_ops = [], []
    for side in range(2):
        n_mid = int(8 + r[1 + side] % np.uint64(25))
        tab = (W.splitmix64(5300 + seed * 2 + side, np.arange(nv * nv)) % np.uint64(n_mid)).astype(np.int32).reshape(nv, nv)
        m0 = oracle.dtkp_init(np.arange(nv) + nv * (2 * side), fp, k)[0]
        m1 = oracle.dtkp_init(np.arange(nv) + nv * (2 * side + 1), fp, k)[0]
        s, m, p, _ = oracle.dtkp_apply2(oracle.dense_to_triples(tab), nv, nv, k, grp, fp, m0, m1)
        d0, d1 = dol.Dist.empty(np.arange(nv), B, k=k), dol.Dist.empty(np.arange(nv), B, k=k)
        dol.dtkp_init(d0, np.arange(nv) + nv * (2 * side), prov)
        dol.dtkp_init(d1, np.arange(nv) + nv * (2 * side + 1), prov)
        ft = dol.FnTable.create_dense(tab)
        d = dol.Dist.empty(ft.out_syms, B, k=k)
        dol.apply2(d0, d1, ft, prov, d)
        o_ops.append((s, m)); g_ops.append(d)
    na, nb = o_ops[0][0].size, o_ops[1][0].size
    n_ids = int(1 + r[3] % np.uint64(6))
    table = (W.splitmix64(5400 + seed, np.arange(na * nb)) % np.uint64(n_ids)).astype(np.int32).reshape(na, nb)
    table.reshape(-1)[::7] = -1
    tri = oracle.dense_to_triples(table)
    syms, om, op, opr = oracle.dtkp_apply2(tri, na, nb, k, grp, fp, o_ops[0][1], o_ops[1][1])
    f = dol.FnTable.create_dense(table)
    out = dol.Dist.empty(f.out_syms, B, k=k)
    dol.apply2(g_ops[0], g_ops[1], f, prov, out)
    np.testing.assert_array_equal(out.sym_ids, syms)
    np.testing.assert_array_equal(host(out.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(out.proof_prob), op)
    assert_close(host(out.prob), opr, "dtkp random table, seed %d" % seed)
    fk = dol.FnkTable.create_dense(table)
    outk = dol.Dist.empty(fk.out_syms, B, k=k)
    dol.apply_k(g_ops, fk, prov, outk)
    np.testing.assert_array_equal(host(outk.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(outk.proof_prob), op)
    gsym = W.normal(5500 + seed, B * syms.size).astype(np.float32).reshape(B, -1)
    want = oracle.dtkp_prob_bwd(om, fp, gsym)
    gf = torch.empty((B, fp.shape[1]), device="cuda")
    dol.dtkp_backward(out, prov, dev(gsym), gf)
    assert_close(host(gf), want, "dtkp random table gradient, seed %d" % seed)


@pytest.mark.parametrize("k", [1, 3])
def test_dtkp_apply2_input_equals_init_then_apply2(dol, k):
    """The second operand given by its facts: bit for bit what dol_dtkp_init + dol_apply2 give, on a table with
    columns of every length, a first operand with several proofs per symbol, shared exclusion groups."""
    B, nv = 50, 6
    fp = np.concatenate([W.softmax_rows(W.normal(5600 + t, B * nv).reshape(B, nv)) for t in range(3)], axis=1)
    grp = np.repeat(np.arange(3), nv).astype(np.int32)
    prov = dol.Prov(dol.DTKP, k, dev(fp), grp)
    d0, d1, d2 = (dol.Dist.empty(np.arange(nv), B, k=k) for _ in range(3))
    for t, d in enumerate((d0, d1, d2)):
        dol.dtkp_init(d, np.arange(nv) + nv * t, prov)
    tab = (W.splitmix64(5700, np.arange(nv * nv)) % np.uint64(9)).astype(np.int32).reshape(nv, nv)
    ft = dol.FnTable.create_dense(tab)
    a = dol.Dist.empty(ft.out_syms, B, k=k)
    dol.apply2(d0, d1, ft, prov, a)
    # second operand: the facts of slot 2 in a permuted order, one of them used by two symbols, one fact of slot 1
    fact_b = np.array([14, 12, 17, 12, 13, 15, 16, 7], np.int32)
    table = (W.splitmix64(5800, np.arange(a.n_sym * fact_b.size)) % np.uint64(4)).astype(np.int32).reshape(a.n_sym, -1)
    table.reshape(-1)[::5] = -1
    f = dol.FnTable.create_dense(table)
    b = dol.Dist.empty(np.arange(fact_b.size), B, k=k)
    dol.dtkp_init(b, fact_b, prov)
    want, got = dol.Dist.empty(f.out_syms, B, k=k), dol.Dist.empty(f.out_syms, B, k=k)
    dol.apply2(a, b, f, prov, want)
    dol.dtkp_apply2_input(a, fact_b, f, prov, got)
    np.testing.assert_array_equal(host(got.proof_mask), host(want.proof_mask))
    np.testing.assert_array_equal(host(got.proof_prob), host(want.proof_prob))
    np.testing.assert_array_equal(host(got.prob), host(want.prob))
    # and against the oracle's composition
    am = oracle.dtkp_apply2(oracle.dense_to_triples(tab), nv, nv, k, grp, fp,
                            oracle.dtkp_init(np.arange(nv), fp, k)[0], oracle.dtkp_init(np.arange(nv) + nv, fp, k)[0])[1]
    _, om, op, opr = oracle.dtkp_apply2(oracle.dense_to_triples(table), a.n_sym, fact_b.size, k, grp, fp, am,
                                        oracle.dtkp_init(fact_b, fp, k)[0])
    np.testing.assert_array_equal(host(got.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(got.proof_prob), op)
    with pytest.raises(dol.DolError):
        dol.dtkp_apply2_input(a, np.full(fact_b.size, 18, np.int32), f, prov, got)


@pytest.mark.parametrize("k,nv", [(1, 6), (3, 6), (3, 20), (8, 12)])
def test_dtkp_gradient_with_impossible_facts(dol, k, nv):
    """Fact probabilities of exactly 0 and far below 1e-30 in some samples: there the product of a proof's other facts
    cannot come from dividing the proof's probability, so the kernel multiplies them out.  nv = 20 gives 400 result
    symbols (several wavefronts per sample, a ragged last group of 64); the padded gradient tensor has ld > n_sym."""
    B = 70
    fp = np.concatenate([W.softmax_rows(W.normal(5900 + t, B * nv).reshape(B, nv)) for t in range(3)], axis=1)
    fp[::3, 1:nv] = 0.0                                            # kept lists there must take impossible proofs
    fp[1::5, nv + 1] = np.float32(1e-36)
    fp[2::7, 2 * nv + 3] = np.float32(1e-41)                       # subnormal
    fp[5, :] = 0.0                                                 # every proof of this sample is impossible
    fp = np.ascontiguousarray(fp, np.float32)
    grp = np.repeat(np.arange(3), nv).astype(np.int32)
    prov = dol.Prov(dol.DTKP, k, dev(fp), grp)
    d = [dol.Dist.empty(np.arange(nv), B, k=k) for _ in range(3)]
    for t in range(3):
        dol.dtkp_init(d[t], np.arange(nv) + nv * t, prov)
    # a: pairs of (slot 0, slot 1) facts folded onto few symbols, so that symbols keep several proofs
    tab = (W.splitmix64(5950, np.arange(nv * nv)) % np.uint64(nv)).astype(np.int32).reshape(nv, nv)
    ft = dol.FnTable.create_dense(tab)
    a = dol.Dist.empty(ft.out_syms, B, k=k)
    dol.apply2(d[0], d[1], ft, prov, a)
    # out: one symbol per (a symbol, slot 2 fact)
    table = np.arange(a.n_sym * nv, dtype=np.int32).reshape(a.n_sym, nv)
    f = dol.FnTable.create_dense(table)
    out = dol.Dist.empty(f.out_syms, B, k=k)
    dol.apply2(a, d[2], f, prov, out)
    inits = [oracle.dtkp_init(np.arange(nv) + nv * t, fp, k)[0] for t in range(3)]
    _, am, _, _ = oracle.dtkp_apply2(oracle.dense_to_triples(tab), nv, nv, k, grp, fp, inits[0], inits[1])
    _, om, op, opr = oracle.dtkp_apply2(oracle.dense_to_triples(table), a.n_sym, nv, k, grp, fp, am, inits[2])
    np.testing.assert_array_equal(host(out.proof_mask).view(np.uint64), om)
    np.testing.assert_array_equal(host(out.proof_prob), op)
    S = om.shape[1]
    gsym = W.normal(5960 + k, B * S).astype(np.float32).reshape(B, S)
    want = oracle.dtkp_prob_bwd(om, fp, gsym)
    assert np.abs(want[::3, 1:nv]).max() > 0                       # the zero facts do receive gradient
    gpad = torch.zeros((B, S + 5), device="cuda")
    gpad[:, :S] = dev(gsym)
    gf = torch.full((B, fp.shape[1]), 3.0, device="cuda")
    dol.dtkp_backward(out, prov, gpad, gf)
    assert_close(host(gf), want, "dtkp gradient with impossible facts, k=%d" % k)


@pytest.mark.parametrize("m,nb,batch", [(1, 1, 5), (16, 16, 257), (7, 3, 256), (16, 1, 1000), (10, 10, 255), (3, 16, 513)])
def test_sum_shaped_apply_with_short_first_operand(dol, m, nb, batch):
    """The thread-per-sample forward kernel: every width up to 16, whole and partial tiles of 256 samples, tags that
    clamp; backward (through the tile / loop kernels) on the same result."""
    a = (W.uniform01(100 + m, batch * m) * 0.9).astype(np.float32).reshape(batch, m)
    b = (W.uniform01(200 + nb, batch * nb) * 0.9).astype(np.float32).reshape(batch, nb)
    table = W.sum_table(np.arange(m), np.arange(nb))
    tri = oracle.dense_to_triples(table)
    syms, want, pre32, _ = oracle.damp_apply2_fwd(tri, m, nb, a, b, want_pre=True)
    f = dol.FnTable.create_dense(table)
    assert f.kernel_fwd.startswith("damp_conv_fwd_small_kernel")
    da, db = dol.Dist(np.arange(m), dev(a)), dol.Dist(np.arange(nb), dev(b))
    out = dol.Dist.empty(f.out_syms, batch)
    dol.apply2(da, db, f, None, out)
    assert_close(host(out.prob), want, "short first operand forward")
    if min(m, nb) >= 3:
        assert (pre32 > 1).any()
    g = np.abs(W.normal(300 + m, batch * syms.size)).astype(np.float32).reshape(batch, -1)
    wa, wb = oracle.damp_apply2_bwd(tri, m, nb, a, b, g)
    ga, gb = torch.empty((batch, m), device="cuda"), torch.empty((batch, nb), device="cuda")
    dol.backward(dol.OpRecord(dol.OP_APPLY2, da, db, out, f=f), dev(g), ga, gb)
    assert_close(host(ga), wa, "short first operand grad a")
    assert_close(host(gb), wb, "short first operand grad b")
