"""Seeded input generators (numpy only).  No operator/provenance arithmetic here.

Random streams are counter based: element n of stream `seed` is
finalise(seed + GOLDEN * (n + 1)) with the public-domain splitmix64 finaliser,
so any element can be produced independently and the same bytes come out on
every machine.  Normals use Box-Muller in float64; probabilities are a float64
softmax rounded once to float32; Beta(2,2) draws are the median of three
uniforms (the 2nd order statistic of 3 uniforms has exactly that law).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Any

from fractions import Fraction

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, index) -> np.ndarray:
    """Element(s) `index` (0-based, array ok) of the splitmix64 stream `seed`."""
    idx = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GOLDEN * (idx + np.uint64(1))
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        x = x ^ (x >> np.uint64(31))
    return x


def uniform01(seed: int, n: int) -> np.ndarray:
    """n float64 uniforms in (0,1): top 53 bits, shifted half a step off zero."""
    u = splitmix64(seed, np.arange(n, dtype=np.uint64)) >> np.uint64(11)
    return (u.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, n: int, sigma: float = 1.0) -> np.ndarray:
    """n float64 N(0, sigma^2) draws by Box-Muller on consecutive uniform pairs."""
    m = (n + 1) // 2
    u = uniform01(seed, 2 * m)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    th = 2.0 * np.pi * u[1::2]
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = r * np.cos(th)
    z[1::2] = r * np.sin(th)
    return z[:n] * sigma


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """Row softmax in float64, rounded to float32 (the neural front-end's job)."""
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def beta22(seed: int, n: int) -> np.ndarray:
    """n float32 Beta(2,2) draws: median of three consecutive uniforms."""
    u = uniform01(seed, 3 * n).reshape(n, 3)
    return np.median(u, axis=1).astype(np.float32)


def hashed_table(seed: int, na: int, nb: int, n_out: int) -> np.ndarray:
    """f(i,j) = splitmix64 stream `seed` at index i*nb+j, mod n_out; int32 [na,nb]."""
    idx = np.arange(na * nb, dtype=np.uint64)
    return (splitmix64(seed, idx) % np.uint64(n_out)).astype(np.int32).reshape(na, nb)


def keep_mask(seed: int, n: int) -> np.ndarray:
    """uint8 [n]: low bit of stream `seed` at index s (about half kept)."""
    return (splitmix64(seed, np.arange(n, dtype=np.uint64)) & np.uint64(1)).astype(np.uint8)


def sum_table(sym_a: np.ndarray, sym_b: np.ndarray) -> np.ndarray:
    """Symbol table of the user function f(x,y)=x+y over two id lists; int32 [na,nb]."""
    return (np.asarray(sym_a, np.int32)[:, None] + np.asarray(sym_b, np.int32)[None, :]).astype(np.int32)


def grid_edges(side: int):
    """Undirected 4-neighbour grid edges.  Ids: all horizontal edges row-major
    ((r,c)-(r,c+1) -> r*(side-1)+c), then all vertical ((r,c)-(r+1,c) ->
    side*(side-1) + r*side + c).  Returns (u[E], v[E]) node ids with u < v."""
    us, vs = [], []
    for r in range(side):
        for c in range(side - 1):
            us.append(r * side + c)
            vs.append(r * side + c + 1)
    for r in range(side - 1):
        for c in range(side):
            us.append(r * side + c)
            vs.append((r + 1) * side + c)
    return np.asarray(us, np.int32), np.asarray(vs, np.int32)


def grid_reach_triples(side: int):
    """Symbol-side table of one reachability round as (i, j, out) triples.

    Operand A ranges over the side*side node symbols, operand B over E+1 symbols:
    the E undirected edge symbols followed by one "stay" symbol (id E) whose tag
    is the conjunction identity.  Node u combined with edge {u,v} yields node v
    (both directions), node v combined with "stay" yields v.  Sorted by (i, j)."""
    u, v = grid_edges(side)
    e = np.arange(u.size, dtype=np.int32)
    n = side * side
    i = np.concatenate([u, v, np.arange(n, dtype=np.int32)])
    j = np.concatenate([e, e, np.full(n, u.size, np.int32)])
    o = np.concatenate([v, u, np.arange(n, dtype=np.int32)])
    order = np.lexsort((j, i))
    return i[order].astype(np.int32), j[order].astype(np.int32), o[order].astype(np.int32)


def random_digraph(seed: int, n_nodes: int, n_edges: int):
    """n_edges distinct directed edges (u != v) on n_nodes nodes, as ascending symbol ids u * n_nodes + v and the
    (u, v) arrays in that order."""
    ids, k = [], 0
    while len(ids) < n_edges:
        x = int(splitmix64(seed, np.array([k], dtype=np.uint64))[0] % np.uint64(n_nodes * n_nodes))
        k += 1
        if x // n_nodes != x % n_nodes and x not in ids:
            ids.append(x)
    ids = np.array(sorted(ids), np.int32)
    return ids, (ids // n_nodes).astype(np.int32), (ids % n_nodes).astype(np.int32)


def join_triples(path_ids, edge_ids, n_nodes: int):
    """Symbol-side table of one step of a transitive closure: path (x, y) at position i joined with edge (y, z)
    at position j yields the path with id x * n_nodes + z.  Tuples in ascending (i, j)."""
    ti, tj, to = [], [], []
    for i, p in enumerate(np.asarray(path_ids).tolist()):
        for j, e in enumerate(np.asarray(edge_ids).tolist()):
            if p % n_nodes == e // n_nodes:
                ti.append(i); tj.append(j); to.append((p // n_nodes) * n_nodes + e % n_nodes)
    return np.array(ti, np.int32), np.array(tj, np.int32), np.array(to, np.int32)


def closure_workload(batch: int = 64, n_nodes: int = 10, n_edges: int = 16, scale: float = 0.5, seed: int = 0) -> "Workload":
    """A seeded random directed graph with one probability per edge and sample, and an upstream gradient over the
    n_nodes^2 possible paths (the program uses the columns of the paths it derives)."""
    ids, u, v = random_digraph(_sd(seed, 6, 0), n_nodes, n_edges)
    p = (uniform01(_sd(seed, 6, 1), batch * n_edges) * scale).astype(np.float32).reshape(batch, n_edges)
    g = normal(_sd(seed, 6, 2), batch * n_nodes * n_nodes).astype(np.float32).reshape(batch, n_nodes * n_nodes)
    return Workload("transitive_closure_damp_fwd_bwd", dict(batch=batch, n_nodes=n_nodes, n_edges=n_edges),
                    dict(p=p, g=g, edge_ids=ids, edge_u=u, edge_v=v))


def product_stage_tables(n_digits: int):
    """Symbol side of the fold apply(D_res, D_i, lambda x, y: x * y) over digit Distributions (the Product-N
    program of the appendix on combinatorial explosions).  The symbols of stage t are the distinct products of
    t + 1 digits; they are interned as their rank in the last stage's sorted value list (every earlier stage's
    values occur there, since multiplying by 1 keeps a value), because the values outgrow 32 bits.
    Returns (values, stage_ids, tables): the last stage's values (Python ints), per stage the ascending id list
    int32 [m_t], and per apply the dense table int32 [m_t, 10] of produced ids."""
    stages = [list(range(10))]
    for _ in range(1, n_digits):
        stages.append(sorted({v * d for v in stages[-1] for d in range(10)}))
    values = stages[-1]
    rank = {v: r for r, v in enumerate(values)}
    stage_ids = [np.asarray([rank[v] for v in st], np.int32) for st in stages]
    tables = [np.asarray([[rank[v * d] for d in range(10)] for v in stages[t]], np.int32) for t in range(n_digits - 1)]
    return values, stage_ids, tables


def product_workload(batch: int = 256, n_digits: int = 16, seed: int = 0) -> "Workload":
    """Product-N chain: n_digits digit Distributions (softmax of N(0, variance 2) logits) and a target column of
    the last stage per sample."""
    p = np.stack([
        softmax_rows(normal(_sd(seed, 7, t), batch * 10, sigma=np.sqrt(2.0)).reshape(batch, 10))
        for t in range(n_digits)])
    values, stage_ids, tables = product_stage_tables(n_digits)
    tgt = (splitmix64(_sd(seed, 7, 100), np.arange(batch, dtype=np.uint64)) % np.uint64(len(values))).astype(np.int32)
    w = Workload("product%d_damp_chain_fwd_bwd" % n_digits, dict(batch=batch, n_digits=n_digits, values=values,
                                                                 stage_ids=stage_ids, tables=tables),
                 dict(p=p, target=tgt))
    return w


# ---- a formula-evaluation pipeline in the shape of the hand-written-formula task (App. on the HWF model): symbols of
# 14 classes per position (digits 0-9 and + - * /), digits kept at even positions and operators at odd ones, the
# formula built by one Apply per position over host-interned formula states, one unary Apply evaluating it.

HWF_OPS = "+-*/"
_HWF_NAN = ("nan",)


def _hwf_add_digit(state, d):
    """User function of the digit positions.  A state is () | (T,) | (A, s, T) | one of these plus a trailing
    operator, T the term in progress, A the folded prefix, s in '+-'; products and quotients are folded as they
    complete, sums and differences as soon as the next operator shows that precedence allows it."""
    if state == _HWF_NAN:
        return _HWF_NAN
    if state == ():
        return (Fraction(d),)
    op = state[-1]
    if op in "+-":
        return state + (Fraction(d),)
    if op == "/" and d == 0:
        return _HWF_NAN
    return state[:-2] + (state[-2] * d if op == "*" else state[-2] / d,)


def _hwf_add_op(state, op):
    if state == _HWF_NAN:
        return _HWF_NAN
    if op in "+-" and len(state) == 3:
        a, s, t = state
        state = (a + t if s == "+" else a - t,)
    return state + (op,)


def _hwf_value(state):
    if state == _HWF_NAN:
        return None
    if len(state) == 3:
        a, s, t = state
        return a + t if s == "+" else a - t
    return state[0]


def hwf_symbol_tables(length: int):
    """Symbol side of the pipeline for formulas of `length` positions (odd).  Returns
    (states, tables, values, final_map): per position the list of formula states (interned id = index, sorted by
    their printed form), per position >= 1 the dense int32 table [states before, kept symbols of the position] of
    next-state ids, the sorted list of distinct formula values (None = division by zero, last), and int32
    [last states] mapping a state to its value's index."""
    assert length % 2 == 1

    def key(st):
        return " ".join(str(x) for x in st)

    states = [sorted({_hwf_add_digit((), d) for d in range(10)}, key=key)]
    tables = []
    for pos in range(1, length):
        step, alphabet = (_hwf_add_digit, range(10)) if pos % 2 == 0 else (_hwf_add_op, HWF_OPS)
        nxt = [[step(st, x) for x in alphabet] for st in states[-1]]
        new_states = sorted({v for row in nxt for v in row}, key=key)
        idx = {st: i for i, st in enumerate(new_states)}
        tables.append(np.asarray([[idx[v] for v in row] for row in nxt], np.int32))
        states.append(new_states)
    vals = {_hwf_value(st) for st in states[-1]}
    values = sorted(v for v in vals if v is not None) + ([None] if None in vals else [])
    vidx = {v: i for i, v in enumerate(values)}
    final_map = np.asarray([vidx[_hwf_value(st)] for st in states[-1]], np.int32)
    return states, tables, values, final_map


def hwf_workload(batch: int = 64, length: int = 7, k: int = 3, seed: int = 0) -> "Workload":
    """Per position a softmax of N(0,1) logits over the 14 classes, and an N(0,1) upstream gradient over the
    distinct formula values."""
    p = softmax_rows(normal(_sd(seed, 8, 0), batch * length * 14).reshape(batch * length, 14)).reshape(batch, length, 14)
    states, tables, values, final_map = hwf_symbol_tables(length)
    g = normal(_sd(seed, 8, 1), batch * len(values)).astype(np.float32).reshape(batch, len(values))
    keep = [(np.arange(14) < 10 if pos % 2 == 0 else np.arange(14) >= 10).astype(np.uint8) for pos in range(length)]
    return Workload("hwf%d_filter_concat_eval" % length,
                    dict(batch=batch, length=length, k=k, states=states, tables=tables, values=values, keep=keep),
                    dict(p=p, g=g, final_map=final_map))


@dataclass
class Workload:
    """A named bundle of input arrays plus the scalar parameters of a config."""
    name: str
    params: Dict[str, Any] = field(default_factory=dict)
    arrays: Dict[str, np.ndarray] = field(default_factory=dict)

    def __getitem__(self, k):
        return self.arrays[k] if k in self.arrays else self.params[k]


def _sd(seed: int, config_id: int, tensor_index: int) -> int:
    return (seed * 1000003 + config_id * 1000 + tensor_index) & 0xFFFFFFFFFFFFFFFF


def config1(batch: int = 64, seed: int = 0) -> Workload:
    """Sum-2: two digit Distributions, softmax of N(0,1) logits."""
    pa = softmax_rows(normal(_sd(seed, 1, 0), batch * 10).reshape(batch, 10))
    pb = softmax_rows(normal(_sd(seed, 1, 1), batch * 10).reshape(batch, 10))
    d = np.arange(10, dtype=np.int32)
    return Workload("sum2_damp_fwd", dict(batch=batch),
                    dict(pa=pa, pb=pb, sym=d, table=sum_table(d, d)))


def config2(batch: int = 4096, n_digits: int = 15, seed: int = 0) -> Workload:
    """Sum-N chain: n_digits digit Distributions (softmax of N(0, variance 2)
    logits) and an integer target sum per sample, uniform over 0..9*n_digits."""
    p = np.stack([
        softmax_rows(normal(_sd(seed, 2, t), batch * 10, sigma=np.sqrt(2.0)).reshape(batch, 10))
        for t in range(n_digits)])
    n_out = 9 * n_digits + 1
    tgt = (splitmix64(_sd(seed, 2, 100), np.arange(batch, dtype=np.uint64)) % np.uint64(n_out)).astype(np.int32)
    return Workload("sum%d_damp_chain_fwd_bwd" % n_digits, dict(batch=batch, n_digits=n_digits),
                    dict(p=p, target=tgt, sym=np.arange(10, dtype=np.int32)))


def config3(batch: int = 16384, na: int = 64, nb: int = 64, n_out: int = 256, seed: int = 0) -> Workload:
    """Hashed apply + filter + union: inputs over na and nb symbols, hashed table
    into n_out symbols, ~50% keep-mask, a second Distribution over all n_out
    symbols, and an N(0,1) upstream gradient over the union's output."""
    pa = softmax_rows(normal(_sd(seed, 3, 0), batch * na).reshape(batch, na))
    pb = softmax_rows(normal(_sd(seed, 3, 1), batch * nb).reshape(batch, nb))
    p2 = softmax_rows(normal(_sd(seed, 3, 2), batch * n_out).reshape(batch, n_out))
    g = normal(_sd(seed, 3, 3), batch * n_out).astype(np.float32).reshape(batch, n_out)
    return Workload("hashed_apply_filter_union_damp_fwd_bwd", dict(batch=batch, na=na, nb=nb, n_out=n_out),
                    dict(pa=pa, pb=pb, p2=p2, g=g,
                         table=hashed_table(_sd(seed, 3, 4), na, nb, n_out),
                         keep=keep_mask(_sd(seed, 3, 5), n_out)))


def config4(batch: int = 1024, n_digits: int = 5, k: int = 3, seed: int = 0) -> Workload:
    """DTKP sum-N: n_digits digit Distributions; fact 10*n+d is "digit n is d";
    facts of one digit slot form one exclusion group."""
    p = np.stack([
        softmax_rows(normal(_sd(seed, 4, t), batch * 10).reshape(batch, 10))
        for t in range(n_digits)])
    fact_prob = np.ascontiguousarray(p.transpose(1, 0, 2).reshape(batch, n_digits * 10))
    group = (np.arange(n_digits * 10) // 10).astype(np.int32)
    return Workload("dtkp_top%d_sum%d_fwd" % (k, n_digits), dict(batch=batch, n_digits=n_digits, k=k),
                    dict(p=p, fact_prob=fact_prob, fact_group=group, sym=np.arange(10, dtype=np.int32)))


def config5(batch: int = 256, side: int = 32, rounds: int = 64, seed: int = 0) -> Workload:
    """Grid reachability: Beta(2,2) probability per undirected edge, N(0,1)
    upstream gradient over all nodes' final reach probabilities."""
    u, v = grid_edges(side)
    n_e = u.size
    p = beta22(_sd(seed, 5, 0), batch * n_e).reshape(batch, n_e)
    g = normal(_sd(seed, 5, 1), batch * side * side).astype(np.float32).reshape(batch, side * side)
    ti, tj, to = grid_reach_triples(side)
    return Workload("grid%d_reach_damp_fwd_bwd" % side, dict(batch=batch, side=side, rounds=rounds, src=0),
                    dict(p=p, g=g, edge_u=u, edge_v=v, tri_i=ti, tri_j=tj, tri_o=to))


CONFIG_NAMES = {1: "sum2_damp_fwd", 2: "sum15_damp_chain_fwd_bwd", 3: "hashed_apply_filter_union_damp_fwd_bwd",
                4: "dtkp_top3_sum5_fwd", 5: "grid32_reach_damp_fwd_bwd",
                6: "product16_damp_chain_fwd_bwd", 7: "hwf7_filter_concat_eval_dtkp_top3",
                8: "hwf7_filter_concat_eval_damp"}


def make_config(cid: int, **kw) -> Workload:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: product_workload, 7: hwf_workload,
            8: hwf_workload}[cid](**kw)
