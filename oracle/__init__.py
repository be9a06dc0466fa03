"""CPU oracle for the Dolphin hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin numpy/ctypes front for ``dol_oracle.c`` (plain C, double accumulation).
Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package; the HIP library and its Python binding never do.

Each function mirrors one C routine; see the C file for the definitions and the
passages of the paper they restate.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DOL_ORACLE_SRC: build and load another copy of the C source instead (the planted-mistake test points it at a
# patched copy in a temporary folder; the library is then built next to that copy)
_SRC = os.environ.get("DOL_ORACLE_SRC") or os.path.join(_HERE, "dol_oracle.c")
_LIB = os.path.join(os.path.dirname(_SRC), "libdol_oracle.so")
_lib = None

ABSENT = np.uint64(0xFFFFFFFFFFFFFFFF)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over the batch).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=os.path.dirname(_SRC))
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def set_threads(n: int) -> int:
    return int(lib().orc_set_threads(C.c_int(n)))


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == 2
    return a


def _chk(rc, what):
    if rc != 0:
        raise ValueError("%s failed with oracle status %d" % (what, rc))


def dense_to_triples(table):
    """All (i, j) of a dense int32 [na,nb] symbol table whose entry is >= 0, in (i,j) order."""
    t = _i32(table)
    i, j = np.nonzero(t >= 0)
    return _i32(i), _i32(j), _i32(t[i, j])


def out_syms(tri_o):
    o = _i32(tri_o)
    buf = np.empty(max(o.size, 1), np.int32)
    s = lib().orc_out_syms(C.c_int64(o.size), _p(o, C.c_int32), _p(buf, C.c_int32))
    return buf[:s].copy()


def damp_apply2_fwd(tri, na, nb, a, b, want_pre=False):
    """Returns (out_syms[S], out[B,S]) and, if want_pre, (pre32[B,S], pre64[B,S])."""
    ti, tj, to = map(_i32, tri)
    a, b = _f32(a), _f32(b)
    B = a.shape[0]
    syms = out_syms(to)
    S = syms.size
    out = np.empty((B, S), np.float32)
    pre32 = np.empty((B, S), np.float32)
    pre64 = np.empty((B, S), np.float64)
    rc = lib().orc_damp_apply2_fwd(
        C.c_int(B), C.c_int64(ti.size), _p(ti, C.c_int32), _p(tj, C.c_int32), _p(to, C.c_int32),
        C.c_int(na), C.c_int(nb), C.c_int(S), _p(syms, C.c_int32),
        _p(a, C.c_float), C.c_int64(a.shape[1]), _p(b, C.c_float), C.c_int64(b.shape[1]),
        _p(out, C.c_float), C.c_int64(S), _p(pre32, C.c_float), _p(pre64, C.c_double))
    _chk(rc, "damp_apply2_fwd")
    return (syms, out, pre32, pre64) if want_pre else (syms, out)


def damp_apply2_bwd(tri, na, nb, a, b, g):
    """Returns (ga[B,na], gb[B,nb])."""
    ti, tj, to = map(_i32, tri)
    a, b, g = _f32(a), _f32(b), _f32(g)
    B = a.shape[0]
    syms = out_syms(to)
    S = syms.size
    assert g.shape == (B, S)
    ga = np.empty((B, na), np.float32)
    gb = np.empty((B, nb), np.float32)
    rc = lib().orc_damp_apply2_bwd(
        C.c_int(B), C.c_int64(ti.size), _p(ti, C.c_int32), _p(tj, C.c_int32), _p(to, C.c_int32),
        C.c_int(na), C.c_int(nb), C.c_int(S), _p(syms, C.c_int32),
        _p(a, C.c_float), C.c_int64(a.shape[1]), _p(b, C.c_float), C.c_int64(b.shape[1]),
        _p(g, C.c_float), C.c_int64(S),
        _p(ga, C.c_float), C.c_int64(na), _p(gb, C.c_float), C.c_int64(nb))
    _chk(rc, "damp_apply2_bwd")
    return ga, gb


def filter_plan(syms, pred):
    syms = _i32(syms)
    pred = np.ascontiguousarray(pred, np.uint8)
    os_ = np.empty(max(syms.size, 1), np.int32)
    ki = np.empty(max(syms.size, 1), np.int32)
    m = lib().orc_filter_plan(C.c_int(syms.size), _p(syms, C.c_int32), _p(pred, C.c_uint8),
                              _p(os_, C.c_int32), _p(ki, C.c_int32))
    return os_[:m].copy(), ki[:m].copy()


def damp_filter_fwd(pred, x):
    pred = np.ascontiguousarray(pred, np.uint8)
    x = _f32(x)
    K = int(pred.astype(bool).sum())
    out = np.empty((x.shape[0], K), np.float32)
    _chk(lib().orc_damp_filter_fwd(C.c_int(x.shape[0]), C.c_int(pred.size), _p(pred, C.c_uint8),
                                   _p(x, C.c_float), C.c_int64(x.shape[1]), _p(out, C.c_float), C.c_int64(K)),
         "damp_filter_fwd")
    return out


def damp_filter_bwd(pred, g):
    pred = np.ascontiguousarray(pred, np.uint8)
    g = _f32(g)
    gi = np.empty((g.shape[0], pred.size), np.float32)
    _chk(lib().orc_damp_filter_bwd(C.c_int(g.shape[0]), C.c_int(pred.size), _p(pred, C.c_uint8),
                                   _p(g, C.c_float), C.c_int64(g.shape[1]), _p(gi, C.c_float), C.c_int64(pred.size)),
         "damp_filter_bwd")
    return gi


def union_plan(sa, sb):
    sa, sb = _i32(sa), _i32(sb)
    n = max(sa.size + sb.size, 1)
    os_, ia, ib = (np.empty(n, np.int32) for _ in range(3))
    m = lib().orc_union_plan(C.c_int(sa.size), _p(sa, C.c_int32), C.c_int(sb.size), _p(sb, C.c_int32),
                             _p(os_, C.c_int32), _p(ia, C.c_int32), _p(ib, C.c_int32))
    return os_[:m].copy(), ia[:m].copy(), ib[:m].copy()


def damp_union_fwd(ia, ib, a, b):
    ia, ib = _i32(ia), _i32(ib)
    a, b = _f32(a), _f32(b)
    out = np.empty((a.shape[0], ia.size), np.float32)
    _chk(lib().orc_damp_union_fwd(C.c_int(a.shape[0]), C.c_int(ia.size), _p(ia, C.c_int32), _p(ib, C.c_int32),
                                  _p(a, C.c_float), C.c_int64(a.shape[1]), _p(b, C.c_float), C.c_int64(b.shape[1]),
                                  _p(out, C.c_float), C.c_int64(ia.size)), "damp_union_fwd")
    return out


def damp_union_bwd(ia, ib, a, b, g):
    ia, ib = _i32(ia), _i32(ib)
    a, b, g = _f32(a), _f32(b), _f32(g)
    ga = np.zeros_like(a)
    gb = np.zeros_like(b)
    _chk(lib().orc_damp_union_bwd(C.c_int(a.shape[0]), C.c_int(ia.size), _p(ia, C.c_int32), _p(ib, C.c_int32),
                                  _p(a, C.c_float), C.c_int64(a.shape[1]), _p(b, C.c_float), C.c_int64(b.shape[1]),
                                  _p(g, C.c_float), C.c_int64(g.shape[1]),
                                  _p(ga, C.c_float), C.c_int64(a.shape[1]), _p(gb, C.c_float), C.c_int64(b.shape[1])),
         "damp_union_bwd")
    return ga, gb


def reach_fwd(n, eu, ev, src, rounds, p):
    """Returns hist[rounds+1, B, n]; hist[-1] is the result."""
    eu, ev = _i32(eu), _i32(ev)
    p = _f32(p)
    hist = np.empty((rounds + 1, p.shape[0], n), np.float32)
    _chk(lib().orc_reach_fwd(C.c_int(p.shape[0]), C.c_int(n), C.c_int(eu.size), _p(eu, C.c_int32), _p(ev, C.c_int32),
                             C.c_int(src), C.c_int(rounds), _p(p, C.c_float), C.c_int64(p.shape[1]),
                             _p(hist, C.c_float)), "reach_fwd")
    return hist


def reach_bwd(n, eu, ev, rounds, p, hist, g):
    eu, ev = _i32(eu), _i32(ev)
    p, g = _f32(p), _f32(g)
    hist = np.ascontiguousarray(hist, np.float32)
    gp = np.empty_like(p)
    _chk(lib().orc_reach_bwd(C.c_int(p.shape[0]), C.c_int(n), C.c_int(eu.size), _p(eu, C.c_int32), _p(ev, C.c_int32),
                             C.c_int(rounds), _p(p, C.c_float), C.c_int64(p.shape[1]), _p(hist, C.c_float),
                             _p(g, C.c_float), C.c_int64(g.shape[1]), _p(gp, C.c_float), C.c_int64(p.shape[1])),
         "reach_bwd")
    return gp


def dtkp_init(fact_of_sym, fact_prob, k):
    """Returns (mask[B,n,k] u64, pprob[B,n,k] f32, prob[B,n] f32)."""
    fos = _i32(fact_of_sym)
    fp = _f32(fact_prob)
    B, n = fp.shape[0], fos.size
    mask = np.empty((B, n, k), np.uint64)
    pp = np.empty((B, n, k), np.float32)
    prob = np.empty((B, n), np.float32)
    _chk(lib().orc_dtkp_init(C.c_int(B), C.c_int(n), C.c_int(k), C.c_int(fp.shape[1]), _p(fos, C.c_int32),
                             _p(fp, C.c_float), _p(mask, C.c_uint64), _p(pp, C.c_float), _p(prob, C.c_float),
                             C.c_int64(n)), "dtkp_init")
    return mask, pp, prob


def dtkp_apply2(tri, na, nb, k, fact_group, fact_prob, am, bm):
    """Returns (out_syms, mask[B,S,k], pprob[B,S,k], prob[B,S])."""
    ti, tj, to = map(_i32, tri)
    fp = _f32(fact_prob)
    grp = None if fact_group is None else _i32(fact_group)
    am = np.ascontiguousarray(am, np.uint64)
    bm = np.ascontiguousarray(bm, np.uint64)
    B = fp.shape[0]
    assert am.shape == (B, na, k) and bm.shape == (B, nb, k)
    syms = out_syms(to)
    S = syms.size
    om = np.empty((B, S, k), np.uint64)
    op = np.empty((B, S, k), np.float32)
    pr = np.empty((B, S), np.float32)
    _chk(lib().orc_dtkp_apply2(
        C.c_int(B), C.c_int64(ti.size), _p(ti, C.c_int32), _p(tj, C.c_int32), _p(to, C.c_int32),
        C.c_int(na), C.c_int(nb), C.c_int(S), _p(syms, C.c_int32),
        C.c_int(k), C.c_int(fp.shape[1]), _p(grp, C.c_int32), _p(fp, C.c_float),
        _p(am, C.c_uint64), _p(bm, C.c_uint64), _p(om, C.c_uint64), _p(op, C.c_float), _p(pr, C.c_float),
        C.c_int64(S)), "dtkp_apply2")
    return syms, om, op, pr


def dtkp_union(ia, ib, am, ap, bm, bp):
    ia, ib = _i32(ia), _i32(ib)
    am = np.ascontiguousarray(am, np.uint64)
    bm = np.ascontiguousarray(bm, np.uint64)
    ap = np.ascontiguousarray(ap, np.float32)
    bp = np.ascontiguousarray(bp, np.float32)
    B, na, k = am.shape
    nb = bm.shape[1]
    S = ia.size
    om = np.empty((B, S, k), np.uint64)
    op = np.empty((B, S, k), np.float32)
    pr = np.empty((B, S), np.float32)
    _chk(lib().orc_dtkp_union(C.c_int(B), C.c_int(S), _p(ia, C.c_int32), _p(ib, C.c_int32), C.c_int(na), C.c_int(nb),
                              C.c_int(k), _p(am, C.c_uint64), _p(ap, C.c_float), _p(bm, C.c_uint64), _p(bp, C.c_float),
                              _p(om, C.c_uint64), _p(op, C.c_float), _p(pr, C.c_float), C.c_int64(S)), "dtkp_union")
    return om, op, pr


def dtkp_prob_bwd(mask, fact_prob, g):
    """Gradient of the tag probabilities w.r.t. the fact probabilities: returns gfact[B,n_facts]."""
    mask = np.ascontiguousarray(mask, np.uint64)
    fp, g = _f32(fact_prob), _f32(g)
    B, n, k = mask.shape
    assert g.shape == (B, n) and fp.shape[0] == B
    out = np.empty((B, fp.shape[1]), np.float32)
    _chk(lib().orc_dtkp_prob_bwd(C.c_int(B), C.c_int(n), C.c_int(k), C.c_int(fp.shape[1]), _p(mask, C.c_uint64),
                                 _p(fp, C.c_float), _p(g, C.c_float), C.c_int64(n), _p(out, C.c_float)), "dtkp_prob_bwd")
    return out


def dtkp_filter(pred, im, ip, iprob):
    pred = np.ascontiguousarray(pred, np.uint8)
    im = np.ascontiguousarray(im, np.uint64)
    ip = np.ascontiguousarray(ip, np.float32)
    iprob = _f32(iprob)
    B, n, k = im.shape
    K = int(pred.astype(bool).sum())
    om = np.empty((B, K, k), np.uint64)
    op = np.empty((B, K, k), np.float32)
    pr = np.empty((B, K), np.float32)
    _chk(lib().orc_dtkp_filter(C.c_int(B), C.c_int(n), C.c_int(k), _p(pred, C.c_uint8), _p(im, C.c_uint64),
                               _p(ip, C.c_float), _p(iprob, C.c_float), C.c_int64(iprob.shape[1]),
                               _p(om, C.c_uint64), _p(op, C.c_float), _p(pr, C.c_float), C.c_int64(K)), "dtkp_filter")
    return om, op, pr


def _ptr_array(arrs, ct):
    return (C.POINTER(ct) * len(arrs))(*[_p(a, ct) for a in arrs])


def dense_to_tuples(table):
    """All index tuples of a dense int32 K-dimensional symbol table whose entry is >= 0, ascending: (idx[n,K], ids[n])."""
    t = np.ascontiguousarray(table, np.int32)
    idx = np.argwhere(t >= 0).astype(np.int32).reshape(-1, t.ndim)
    return np.ascontiguousarray(idx), _i32(t[tuple(idx.T)])


def damp_applyk_fwd(idx, to, ins, want_pre=False):
    """Apply over K = len(ins) Distributions.  idx [n,K], to [n]; returns as damp_apply2_fwd."""
    ins = [_f32(x) for x in ins]
    K, B = len(ins), ins[0].shape[0]
    idx = np.ascontiguousarray(idx, np.int32).reshape(-1, K)
    to = _i32(to)
    syms = out_syms(to)
    S = syms.size
    n_sym = _i32([x.shape[1] for x in ins])
    ld = np.asarray([x.shape[1] for x in ins], np.int64)
    out = np.empty((B, S), np.float32)
    pre32 = np.empty((B, S), np.float32)
    pre64 = np.empty((B, S), np.float64)
    _chk(lib().orc_damp_applyk_fwd(
        C.c_int(B), C.c_int(K), C.c_int64(to.size), _p(idx, C.c_int32), _p(to, C.c_int32), _p(n_sym, C.c_int32),
        C.c_int(S), _p(syms, C.c_int32), _ptr_array(ins, C.c_float), _p(ld, C.c_int64),
        _p(out, C.c_float), C.c_int64(S), _p(pre32, C.c_float), _p(pre64, C.c_double)), "damp_applyk_fwd")
    return (syms, out, pre32, pre64) if want_pre else (syms, out)


def damp_applyk_bwd(idx, to, ins, g):
    """Returns the list of gradients, one [B, n_l] per operand."""
    ins = [_f32(x) for x in ins]
    g = _f32(g)
    K, B = len(ins), ins[0].shape[0]
    idx = np.ascontiguousarray(idx, np.int32).reshape(-1, K)
    to = _i32(to)
    syms = out_syms(to)
    S = syms.size
    assert g.shape == (B, S)
    n_sym = _i32([x.shape[1] for x in ins])
    ld = np.asarray([x.shape[1] for x in ins], np.int64)
    gin = [np.empty_like(x) for x in ins]
    _chk(lib().orc_damp_applyk_bwd(
        C.c_int(B), C.c_int(K), C.c_int64(to.size), _p(idx, C.c_int32), _p(to, C.c_int32), _p(n_sym, C.c_int32),
        C.c_int(S), _p(syms, C.c_int32), _ptr_array(ins, C.c_float), _p(ld, C.c_int64),
        _p(g, C.c_float), C.c_int64(S), _ptr_array(gin, C.c_float), _p(ld, C.c_int64)), "damp_applyk_bwd")
    return gin


def dtkp_applyk(idx, to, k, fact_group, fact_prob, masks):
    """Returns (out_syms, mask[B,S,k], pprob[B,S,k], prob[B,S]); masks: one [B,n_l,k] per operand."""
    masks = [np.ascontiguousarray(m, np.uint64) for m in masks]
    fp = _f32(fact_prob)
    grp = None if fact_group is None else _i32(fact_group)
    K, B = len(masks), fp.shape[0]
    idx = np.ascontiguousarray(idx, np.int32).reshape(-1, K)
    to = _i32(to)
    syms = out_syms(to)
    S = syms.size
    for m in masks:
        assert m.shape[0] == B and m.shape[2] == k
    n_sym = _i32([m.shape[1] for m in masks])
    om = np.empty((B, S, k), np.uint64)
    op = np.empty((B, S, k), np.float32)
    pr = np.empty((B, S), np.float32)
    _chk(lib().orc_dtkp_applyk(
        C.c_int(B), C.c_int(K), C.c_int64(to.size), _p(idx, C.c_int32), _p(to, C.c_int32), _p(n_sym, C.c_int32),
        C.c_int(S), _p(syms, C.c_int32), C.c_int(k), C.c_int(fp.shape[1]), _p(grp, C.c_int32), _p(fp, C.c_float),
        _ptr_array(masks, C.c_uint64), _p(om, C.c_uint64), _p(op, C.c_float), _p(pr, C.c_float), C.c_int64(S)),
        "dtkp_applyk")
    return syms, om, op, pr
