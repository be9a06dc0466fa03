"""The benchmark programs as sequences of library calls (the chain driver).

Each class uploads one workload, builds the symbol-side plans once (the user
function is evaluated once per batch, Sec. 3.1.2 / App. B), allocates every
intermediate Distribution up front, and lists its launches.  ``forward()`` /
``backward()`` / ``step()`` then only issue asynchronous ``dol_*`` calls on the
current stream, so a step can be captured into a HIP graph.  No arithmetic
happens in Python.

Every launch carries the name of the kernel it runs and its algorithmic cost:
bytes the operator must move (each input element read once, each output element
written once, 4 bytes per tag, 12 bytes per DTKP proof slot) and
multiply-accumulates.  The bench turns these into roofline fractions.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List

import numpy as np
import torch

from . import binding as dol


@dataclass
class Launch:
    kernel: str                 # name of the HIP kernel the call launches
    call: Callable[[], None]
    bytes: int                  # algorithmic HBM bytes of this launch
    macs: int                   # multiply-accumulates (DAMP) or candidate proofs (DTKP)
    phase: str                  # "fwd" or "bwd"


def _dev(x: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


def sum_table_of(sym_a, sym_b) -> np.ndarray:
    """Symbol side of apply(D_a, D_b, lambda x, y: x + y): the ids are the integers themselves."""
    return (np.asarray(sym_a, np.int32)[:, None] + np.asarray(sym_b, np.int32)[None, :]).astype(np.int32)


def _n_tuples(table: np.ndarray) -> int:
    return int((np.asarray(table) >= 0).sum())


class Program:
    launches: List[Launch]
    sample_ops: int
    batch: int

    def forward(self):
        for l in self.launches:
            if l.phase == "fwd":
                l.call()

    def backward(self):
        for l in self.launches:
            if l.phase == "bwd":
                l.call()

    def step(self):
        for l in self.launches:
            l.call()

    def algorithmic_bytes(self) -> int:
        """Sum over the launches of what each must move by itself (operands in, results out)."""
        return sum(l.bytes for l in self.launches)

    # Bytes the whole step must move if nothing but the program's inputs and results touched HBM (every
    # intermediate Distribution and gradient kept on chip): set by each program from its shapes.
    min_bytes: int = 0
    flops: int = 0                      # 2 per multiply-add of the step (DAMP); 0 for DTKP (compare / select work)


def _apply_fwd(a, b, f, out, n_tup, prov=None, dtkp_k=0):
    B = a.batch
    if dtkp_k:
        return Launch("dtkp_apply2_kernel", lambda: dol.apply2(a, b, f, prov, out),
                      B * (12 * dtkp_k * (a.n_sym + b.n_sym + out.n_sym) + 4 * out.n_sym), B * n_tup * dtkp_k, "fwd")
    return Launch(f.kernel_at(False, B), lambda: dol.apply2(a, b, f, None, out),
                  4 * B * (a.n_sym + b.n_sym + out.n_sym), B * n_tup, "fwd")


def _apply_bwd(rec, g, ga, gb, n_tup):
    a, b, out = rec.a, rec.b, rec.out
    n_w = (a.n_sym if ga is not None else 0) + (b.n_sym if gb is not None else 0)
    return Launch(rec.f.kernel_at(True, a.batch), lambda: dol.backward(rec, g, ga, gb),
                  4 * a.batch * (a.n_sym + b.n_sym + out.n_sym + n_w), 2 * a.batch * n_tup, "bwd")


class Sum2Forward(Program):
    """Config 1 (Fig. 2 with two digits): one DAMP apply."""

    def __init__(self, w, device="cuda"):
        self.table = dol.FnTable.create_dense(w["table"])
        self.a = dol.Dist(w["sym"], _dev(w["pa"], device))
        self.b = dol.Dist(w["sym"], _dev(w["pb"], device))
        self.batch = self.a.batch
        self.out = dol.Dist.empty(self.table.out_syms, self.batch, device)
        self.launches = [_apply_fwd(self.a, self.b, self.table, self.out, _n_tuples(w["table"]))]
        self.sample_ops = self.batch
        self.min_bytes = self.launches[0].bytes
        self.flops = 2 * self.launches[0].macs


class SumChain(Program):
    """Config 2 (Fig. 2): left fold of DAMP apply over N digit Distributions, then the reverse sweep of
    vector-Jacobian products from the harness-supplied gradient of -log p[target]."""

    @staticmethod
    def stage_table(w, t, acc_syms, sym):
        """Symbol side of stage t: the user function over the accumulator's and the digit's symbols."""
        return sum_table_of(acc_syms, sym)

    def __init__(self, w, device="cuda"):
        p = w["p"]
        self.n, self.batch = p.shape[0], p.shape[1]
        sym = np.arange(10, dtype=np.int32) if "sym" not in w.arrays else np.asarray(w["sym"], np.int32)
        self.p_dev = _dev(p, device)                         # [n, B, 10]
        self.digits = [dol.Dist(sym, self.p_dev[t]) for t in range(self.n)]
        self.tables: List[dol.FnTable] = []
        self.accs: List[dol.Dist] = [self.digits[0]]
        n_tup = []
        for t in range(1, self.n):
            tab = self.stage_table(w, t, self.accs[-1].sym_ids, sym)
            tb = dol.FnTable.create_dense(tab)
            n_tup.append(_n_tuples(tab))
            self.tables.append(tb)
            self.accs.append(dol.Dist.empty(tb.out_syms, self.batch, device))
        self.records = [dol.OpRecord(dol.OP_APPLY2, self.accs[t - 1], self.digits[t], self.accs[t], f=self.tables[t - 1])
                        for t in range(1, self.n)]
        self.target = _dev(w["target"].astype(np.int32), device)     # column of the last stage (for sums: the sum itself)
        self.grad_p = torch.empty_like(self.p_dev)           # [n, B, 10]
        self.g_acc = [torch.empty((self.batch, d.n_sym), dtype=torch.float32, device=device) for d in self.accs]
        self.launches = [_apply_fwd(self.accs[t - 1], self.digits[t], self.tables[t - 1], self.accs[t], n_tup[t - 1])
                         for t in range(1, self.n)]
        last = self.accs[-1]
        # harness side: d(-log p[target]) / d p
        self.launches.append(Launch("nll_grad_flat_kernel", lambda: dol.nll_grad(last, self.target, self.g_acc[-1]),
                                    4 * self.batch * (2 + last.n_sym), 0, "bwd"))     # the target and its tag in, a row out
        for t in range(self.n - 1, 0, -1):
            ga = self.g_acc[t - 1] if t > 1 else self.grad_p[0]
            self.launches.append(_apply_bwd(self.records[t - 1], self.g_acc[t], ga, self.grad_p[t], n_tup[t - 1]))
        self.sample_ops = 2 * (self.n - 1) * self.batch
        n_in = sum(d.n_sym for d in self.digits)         # inputs in, their gradients and the result out, the target
        self.min_bytes = 4 * self.batch * (2 * n_in + last.n_sym + 1)
        self.flops = 2 * sum(l.macs for l in self.launches)


class ProductChain(SumChain):
    """Product-N (appendix on combinatorial explosions): the same fold with f(x, y) = x * y; the product values
    outgrow 32 bits, so the workload interns them and carries the id table of every stage."""

    @staticmethod
    def stage_table(w, t, acc_syms, sym):
        assert np.array_equal(acc_syms, w["stage_ids"][t - 1])
        return w["tables"][t - 1]


class SumChainFused(Program):
    """Config 2 through dol_fold_apply2: the whole fold, the loss gradient and the reverse sweep in one launch."""

    def __init__(self, w, device="cuda"):
        p = w["p"]
        self.n, self.batch = p.shape[0], p.shape[1]
        sym = np.asarray(w["sym"], np.int32)
        self.p_dev = _dev(p, device)
        self.digits = [dol.Dist(sym, self.p_dev[t]) for t in range(self.n)]
        self.tables, syms, macs = [], sym, 0
        for t in range(1, self.n):
            tab = sum_table_of(syms, sym)
            tb = dol.FnTable.create_dense(tab)
            self.tables.append(tb)
            syms = tb.out_syms
            macs += 3 * _n_tuples(tab)
        self.out = dol.Dist.empty(syms, self.batch, device)
        self.target = _dev(w["target"].astype(np.int32), device)
        self.grad_p = torch.empty_like(self.p_dev)
        self.fold = dol.Fold(self.digits, self.tables, out=self.out, target_col=self.target,
                             grad_inputs=[self.grad_p[t] for t in range(self.n)])
        n_in = sum(d.n_sym for d in self.digits)
        self.launches = [Launch(dol.fold_kernel(self.fold), lambda: dol.fold_apply2(self.fold),
                                4 * self.batch * (2 * n_in + self.out.n_sym + 1), self.batch * macs, "fwd")]
        self.sample_ops = 2 * (self.n - 1) * self.batch
        self.min_bytes = self.launches[0].bytes
        self.flops = 2 * self.launches[0].macs


class HashedPipeline(Program):
    """Config 3: apply with a hashed symbol table, filter by a keep-mask over the produced ids, union with a
    second Distribution over all ids; backward through all three."""

    def __init__(self, w, device="cuda"):
        B = w["pa"].shape[0]
        self.batch = B
        self.table = dol.FnTable.create_dense(w["table"])
        n_tup = _n_tuples(w["table"])
        self.a = dol.Dist(np.arange(w["na"]), _dev(w["pa"], device))
        self.b = dol.Dist(np.arange(w["nb"]), _dev(w["pb"], device))
        self.o1 = dol.Dist.empty(self.table.out_syms, B, device)
        self.pred = np.ascontiguousarray(w["keep"][self.table.out_syms], np.uint8)   # predicate on the symbols present
        self.o2 = dol.Dist.empty(dol.filter_plan(self.o1, self.pred), B, device)
        self.p2 = dol.Dist(np.arange(w["n_out"]), _dev(w["p2"], device))
        self.o3 = dol.Dist.empty(dol.union_plan(self.o2, self.p2), B, device)
        self.g3 = _dev(w["g"][:, :self.o3.n_sym], device)
        self.g2 = torch.empty((B, self.o2.n_sym), dtype=torch.float32, device=device)
        self.gp2 = torch.empty((B, self.p2.n_sym), dtype=torch.float32, device=device)
        self.g1 = torch.empty((B, self.o1.n_sym), dtype=torch.float32, device=device)
        self.ga = torch.empty((B, self.a.n_sym), dtype=torch.float32, device=device)
        self.gb = torch.empty((B, self.b.n_sym), dtype=torch.float32, device=device)
        self.rec1 = dol.OpRecord(dol.OP_APPLY2, self.a, self.b, self.o1, f=self.table)
        self.rec2 = dol.OpRecord(dol.OP_FILTER, self.o1, None, self.o2, pred_mask=self.pred)
        self.rec3 = dol.OpRecord(dol.OP_UNION, self.o2, self.p2, self.o3)
        n1, n2, n3, np2 = self.o1.n_sym, self.o2.n_sym, self.o3.n_sym, self.p2.n_sym
        self.launches = [
            _apply_fwd(self.a, self.b, self.table, self.o1, n_tup),
            Launch("damp_rows_gather_kernel", lambda: dol.filter(self.o1, self.pred, None, self.o2),
                   4 * B * (n1 + n2), 0, "fwd"),
            Launch("damp_rows_union_fwd_kernel", lambda: dol.union(self.o2, self.p2, None, self.o3),
                   4 * B * (n2 + np2 + n3), 0, "fwd"),
            Launch("damp_rows_union_bwd_kernel", lambda: dol.backward(self.rec3, self.g3, self.g2, self.gp2),
                   4 * B * (n3 + 2 * n2 + 2 * np2), 0, "bwd"),
            Launch("damp_rows_gather_kernel", lambda: dol.backward(self.rec2, self.g2, self.g1, None),
                   4 * B * (n2 + n1), 0, "bwd"),
            _apply_bwd(self.rec1, self.g1, self.ga, self.gb, n_tup),
        ]
        self.sample_ops = 6 * B
        # pa, pb, p2 and the upstream gradient in; the result and the three input gradients out
        self.min_bytes = 4 * B * (2 * (self.a.n_sym + self.b.n_sym + np2) + 2 * n3)
        self.flops = 2 * 3 * B * n_tup


class HashedPipelineFused(HashedPipeline):
    """Config 3 with filter and union as one launch each way (dol_filter_union): the filtered Distribution and its
    gradient are never materialised."""

    def __init__(self, w, device="cuda"):
        super().__init__(w, device)
        B = self.batch
        assert list(dol.filter_union_plan(self.o1, self.pred, self.p2)) == list(self.o3.sym_ids)
        self.rec23 = dol.OpRecord(dol.OP_FILTER_UNION, self.o1, self.p2, self.o3, pred_mask=self.pred)
        n1, n3, np2 = self.o1.n_sym, self.o3.n_sym, self.p2.n_sym
        self.launches = [
            self.launches[0],
            Launch("damp_rows_union_fwd_kernel", lambda: dol.filter_union(self.o1, self.pred, self.p2, None, self.o3),
                   4 * B * (n1 + np2 + n3), 0, "fwd"),
            Launch("damp_rows_union_bwd_kernel", lambda: dol.backward(self.rec23, self.g3, self.g1, self.gp2),
                   4 * B * (n3 + 2 * n1 + 2 * np2), 0, "bwd"),
            self.launches[-1],
        ]


class HashedPipelineMerged(Program):
    """Config 3 through dol_apply2_filter_union: Apply, Filter and Union in one launch, their reverse in another;
    only the program's inputs and results touch HBM (plus one word per sample that says whether a clamp acted)."""

    def __init__(self, w, device="cuda", one_launch=False):
        B = w["pa"].shape[0]
        self.batch = B
        self.table = dol.FnTable.create_dense(w["table"])
        n_tup = _n_tuples(w["table"])
        self.a = dol.Dist(np.arange(w["na"]), _dev(w["pa"], device))
        self.b = dol.Dist(np.arange(w["nb"]), _dev(w["pb"], device))
        self.pred = np.ascontiguousarray(w["keep"][self.table.out_syms], np.uint8)   # predicate on the symbols present
        self.p2 = dol.Dist(np.arange(w["n_out"]), _dev(w["p2"], device))
        o1 = dol.Dist(self.table.out_syms, None, batch=B)                             # symbols only: never materialised
        self.o3 = dol.Dist.empty(dol.filter_union_plan(o1, self.pred, self.p2), B, device)
        self.g3 = _dev(w["g"][:, :self.o3.n_sym], device)
        self.gp2 = torch.empty((B, self.p2.n_sym), dtype=torch.float32, device=device)
        self.ga = torch.empty((B, self.a.n_sym), dtype=torch.float32, device=device)
        self.gb = torch.empty((B, self.b.n_sym), dtype=torch.float32, device=device)
        self.saved = torch.empty((B,), dtype=torch.int32, device=device)
        self.merge = dol.ApplyMerge(self.a, self.b, self.table, self.pred, self.p2, self.o3, self.saved)
        na, nb, np2, n3 = self.a.n_sym, self.b.n_sym, self.p2.n_sym, self.o3.n_sym
        self.launches = [
            Launch("damp_table_merge_fwd_kernel", lambda: dol.apply2_filter_union(self.merge),
                   4 * B * (na + nb + np2 + n3), B * n_tup, "fwd"),
            Launch("damp_table_merge_bwd_kernel",
                   lambda: dol.apply2_filter_union_backward(self.merge, self.g3, self.ga, self.gb, self.gp2),
                   4 * B * (n3 + 2 * (na + nb) + np2), 2 * B * n_tup, "bwd"),
        ]
        if one_launch:                       # dol_apply2_filter_union_forward_backward: the gradient is an input
            self.launches = [Launch("damp_table_merge_fwd_bwd_kernel",
                                    lambda: dol.apply2_filter_union_forward_backward(self.merge, self.g3, self.ga, self.gb, self.gp2),
                                    4 * B * (2 * (na + nb + np2) + 2 * n3), 3 * B * n_tup, "fwd+bwd")]
        self.sample_ops = 6 * B
        self.min_bytes = 4 * B * (2 * (na + nb + np2) + 2 * n3)
        self.flops = 2 * 3 * B * n_tup


class DtkpSumChain(Program):
    """Config 4: the sum fold under DTKP-AM with k proofs per tag; fact 10*n+d says "digit n is d"."""

    def __init__(self, w, device="cuda"):
        p = w["p"]
        self.n, self.batch, self.k = p.shape[0], p.shape[1], w["k"]
        k, B = self.k, self.batch
        sym = np.asarray(w["sym"], np.int32)
        self.fact_prob = _dev(w["fact_prob"], device)
        self.prov = dol.Prov(dol.DTKP, k, self.fact_prob, w["fact_group"])
        self.digits = [dol.Dist.empty(sym, B, device, k=k) for _ in range(self.n)]
        self.facts = [10 * t + np.arange(10, dtype=np.int32) for t in range(self.n)]
        self.tables, self.accs = [], [self.digits[0]]
        self.launches = []
        for t in range(self.n):
            d, f = self.digits[t], self.facts[t]
            self.launches.append(Launch("dtkp_init_kernel", lambda d=d, f=f: dol.dtkp_init(d, f, self.prov),
                                        B * 10 * (4 + 12 * k + 4), 0, "fwd"))
        for t in range(1, self.n):
            tab = sum_table_of(self.accs[-1].sym_ids, sym)
            tb = dol.FnTable.create_dense(tab)
            self.tables.append(tb)
            out = dol.Dist.empty(tb.out_syms, B, device, k=k)
            self.launches.append(_apply_fwd(self.accs[-1], self.digits[t], tb, out, _n_tuples(tab), self.prov, k))
            self.accs.append(out)
        self.sample_ops = (self.n - 1) * B
        # the fact probabilities in; the last Distribution's proofs and tag probabilities out
        self.min_bytes = B * (4 * int(self.fact_prob.shape[1]) + self.accs[-1].n_sym * (12 * k + 4))


class DtkpSumChainFused(Program):
    """Config 4 through dol_dtkp_fold_apply2: initialisation and every apply in one launch."""

    def __init__(self, w, device="cuda", with_gradient=False):
        p = w["p"]
        self.n, self.batch, self.k = p.shape[0], p.shape[1], w["k"]
        k, B = self.k, self.batch
        sym = np.asarray(w["sym"], np.int32)
        self.fact_prob = _dev(w["fact_prob"], device)
        self.prov = dol.Prov(dol.DTKP, k, self.fact_prob, w["fact_group"])
        self.digits = [dol.Dist(sym, torch.empty((B, sym.size), device=device)) for _ in range(self.n)]
        self.facts = [10 * t + np.arange(10, dtype=np.int32) for t in range(self.n)]
        self.tables, syms, slots = [], sym, 0
        for t in range(1, self.n):
            tab = sum_table_of(syms, sym)
            tb = dol.FnTable.create_dense(tab)
            self.tables.append(tb)
            syms = tb.out_syms
            slots += _n_tuples(tab) * (1 if t == 1 else k)      # proof pairs a tuple can offer
        self.candidate_slots = B * slots
        self.out = dol.Dist.empty(syms, B, device, k=k)
        self.target = self.grad_fact = None
        if with_gradient:
            self.target = _dev((np.arange(B) % syms.size).astype(np.int32), device)
            self.grad_fact = torch.empty_like(self.fact_prob)
        self.fold = dol.DtkpFold(self.digits, self.facts, self.tables, self.out, target_col=self.target,
                                 grad_fact_prob=self.grad_fact)
        n_facts = self.fact_prob.shape[1]
        self.launches = [Launch("dtkp_fold_kernel<%d>" % k, lambda: dol.dtkp_fold_apply2(self.fold, self.prov),
                                B * (4 * n_facts + syms.size * (12 * k + 4)), 0, "fwd")]
        self.sample_ops = (self.n - 1) * B
        self.min_bytes = self.launches[0].bytes


class GridReach(Program):
    """Config 5: fixed-round single-source reachability on a 4-neighbour grid (App. B, transitive closure
    restricted to one source).  One round is one apply over (node, edge-or-stay) tuples: node u with edge
    {u,v} yields v, node v with the "stay" symbol (tag 1, the conjunction identity) yields v; the
    disjunction over the tuples of v is min(1, r[v] + sum r[u] p(u,v))."""

    def __init__(self, w, device="cuda"):
        B, side = w["p"].shape[0], w["side"]
        self.batch, self.rounds, n = B, w["rounds"], side * side
        E = w["edge_u"].size
        self.table = dol.FnTable.create_sparse(n, E + 1, w["tri_i"], w["tri_j"], w["tri_o"])
        assert self.table.n_out == n
        n_tup = int(w["tri_i"].size)
        pe = torch.ones((B, E + 1), dtype=torch.float32, device=device)
        pe[:, :E] = _dev(w["p"], device)
        self.edges = dol.Dist(np.arange(E + 1), pe)
        self.hist = torch.zeros((self.rounds + 1, B, n), dtype=torch.float32, device=device)
        self.hist[0, :, w["src"]] = 1.0
        nodes = np.arange(n)
        self.r = [dol.Dist(nodes, self.hist[t]) for t in range(self.rounds + 1)]
        # the edge Distribution is used by every round: its gradient is the sum over rounds (accumulate bit 1),
        # started by the first call of the reverse sweep, which overwrites
        self.records = [dol.OpRecord(dol.OP_APPLY2, self.r[t], self.edges, self.r[t + 1], f=self.table,
                                     accumulate=0 if t == self.rounds - 1 else 2) for t in range(self.rounds)]
        self.g_out = _dev(w["g"], device)
        self.g_r = [torch.empty((B, n), dtype=torch.float32, device=device) for _ in range(2)]
        self.g_e = torch.zeros((B, E + 1), dtype=torch.float32, device=device)
        self.grad_p = self.g_e[:, :E]                        # the last column belongs to the "stay" symbol
        self.launches = [_apply_fwd(self.r[t], self.edges, self.table, self.r[t + 1], n_tup)
                         for t in range(self.rounds)]
        g = self.g_out
        for t in range(self.rounds - 1, -1, -1):
            gn = self.g_r[t % 2]
            self.launches.append(_apply_bwd(self.records[t], g, gn, self.g_e, n_tup))
            g = gn
        self.sample_ops = 2 * self.rounds * B
        # edge probabilities and the upstream gradient in; the last round's result and the edge gradient out
        self.min_bytes = 4 * B * (2 * E + 2 * n)
        self.flops = 2 * 3 * B * self.rounds * n_tup


class GridReachFused(Program):
    """Config 5 through dol_iterate_apply2_ckpt / dol_iterate_backward_ckpt: all rounds of a sweep in one launch; only
    the last round and a checkpoint every `ckpt_every` rounds leave the chip, the reverse sweep replays the rounds in
    between in LDS.  ckpt_every = 0: the full history goes through HBM instead (dol_iterate_apply2 / _backward)."""

    def __init__(self, w, device="cuda", ckpt_every=None, one_launch=False):
        B, side = w["p"].shape[0], w["side"]
        self.batch, self.rounds, n = B, w["rounds"], side * side
        E = w["edge_u"].size
        self.E = E
        self.table = dol.FnTable.create_sparse(n, E + 1, w["tri_i"], w["tri_j"], w["tri_o"])
        if ckpt_every is None:               # the fewest segments whose rows fit the LDS a workgroup gets at this batch
            ckpt_every = dol.iterate_ckpt_every(self.table, B, max(w["rounds"], 1))
        n_tup = int(w["tri_i"].size)
        pe = torch.ones((B, E + 1), dtype=torch.float32, device=device)
        pe[:, :E] = _dev(w["p"], device)
        self.edges = dol.Dist(np.arange(E + 1), pe)
        r0 = torch.zeros((B, n), dtype=torch.float32, device=device)
        r0[:, w["src"]] = 1.0
        self.r0 = dol.Dist(np.arange(n), r0)
        self.g_out = _dev(w["g"], device)
        self.g_e = torch.empty((B, E + 1), dtype=torch.float32, device=device)
        self.grad_p = self.g_e[:, :E]
        R = self.rounds
        self.ckpt_every = ckpt_every
        if ckpt_every:
            self.out = dol.Dist.empty(np.arange(n), B, device)
            n_ck = dol.iterate_ckpt_count(R, ckpt_every)
            self.ckpt = torch.empty((n_ck, B, n), dtype=torch.float32, device=device) if n_ck else None
            fwd = lambda: dol.iterate_apply2_ckpt(self.r0, self.edges, self.table, R, ckpt_every, self.out, self.ckpt)
            bwd = lambda: dol.iterate_backward_ckpt(self.r0, self.edges, self.table, R, ckpt_every, self.ckpt,
                                                    self.g_out, None, self.g_e)
        else:
            self.hist = torch.empty((R + 1, B, n), dtype=torch.float32, device=device)
            self.out = dol.Dist(np.arange(n), self.hist[R])
            fwd = lambda: dol.iterate_apply2(self.r0, self.edges, self.table, R, self.hist)
            bwd = lambda: dol.iterate_backward(self.edges, self.table, R, self.hist, self.g_out, None, self.g_e)
        self.launches = [
            Launch("damp_iterate_fwd_kernel", fwd, 4 * B * (n + E + 1 + n), B * R * n_tup, "fwd"),     # r_0 and e in, r_R out
            Launch("damp_iterate_bwd_kernel", bwd, 4 * B * (n + 2 * (E + 1)), 2 * B * R * n_tup, "bwd"),  # gradient and e in, gradient of e out
        ]                                    # (what the sweeps keep of the rounds in between is not algorithmic)
        # dol_iterate_apply2_backward: both sweeps in one launch.  (For a batch above 512 that call issues the same two
        # kernels as the two calls above, back to back: the program then keeps the two calls, so each is timed by itself.)
        if one_launch and B <= 512:
            assert ckpt_every, "the one-launch form keeps checkpoints"
            both = lambda: dol.iterate_apply2_backward(self.r0, self.edges, self.table, R, ckpt_every, self.out, self.ckpt,
                                                       None, self.g_out, None, self.g_e)
            self.launches = [Launch("damp_iterate_fwd_bwd_kernel", both, 4 * B * (3 * n + 3 * (E + 1)), 3 * B * R * n_tup, "fwd+bwd")]
        self.sample_ops = 2 * R * B
        self.min_bytes = 4 * B * (2 * E + 2 * n)
        self.flops = 2 * 3 * B * R * n_tup


class TransitiveClosure(Program):
    """All-pairs transitive closure (App. B, Fig. 9): new = apply_if(paths, edges, join), merged = union(paths, new),
    repeated until the merge adds no symbol.  The symbol side (which paths exist after each step, the join table of
    each step) is worked out on the host when the program is built; a step of the program is then a fixed list of
    dol_apply2 / dol_union launches followed by the reverse sweep of dol_backward calls, in which a Distribution
    used twice (paths feed both the join and the union) sums the gradients of its uses through the accumulate flags."""

    def __init__(self, w, join_triples, device="cuda"):
        n, B = w["n_nodes"], w["p"].shape[0]
        self.batch = B
        eids = np.asarray(w["edge_ids"], np.int32)
        self.edges = dol.Dist(eids, _dev(w["p"], device))
        paths, self.rounds, fwd = self.edges, [], []
        while True:
            tri = join_triples(paths.sym_ids, eids, n)
            table = dol.FnTable.create_sparse(paths.n_sym, eids.size, *tri)
            new = dol.Dist.empty(table.out_syms, B, device)
            merged = dol.Dist.empty(dol.union_plan(paths, new), B, device)
            self.rounds.append((paths, table, new, merged, int(tri[0].size)))
            fwd.append(_apply_fwd(paths, self.edges, table, new, int(tri[0].size)))
            fwd.append(Launch("damp_union_fwd", lambda a=paths, b=new, o=merged: dol.union(a, b, None, o),
                              4 * B * (paths.n_sym + new.n_sym + merged.n_sym), 0, "fwd"))
            grew = merged.n_sym != paths.n_sym
            paths = merged
            if not grew:
                break
        self.out = paths
        self.g_out = _dev(np.ascontiguousarray(w["g"][:, paths.sym_ids]), device)
        self.grad_p = torch.empty_like(self.edges.prob)
        bwd, g, first = [], self.g_out, True
        for a, table, new, merged, n_tup in reversed(self.rounds):
            g_a = torch.empty((B, a.n_sym), dtype=torch.float32, device=device)
            g_new = torch.empty((B, new.n_sym), dtype=torch.float32, device=device)
            rec_u = dol.OpRecord(dol.OP_UNION, a, new, merged)
            rec_a = dol.OpRecord(dol.OP_APPLY2, a, self.edges, new, f=table, accumulate=1 if first else 3)
            bwd.append(Launch("damp_union_bwd", lambda r=rec_u, g=g, x=g_a, y=g_new: dol.backward(r, g, x, y),
                              4 * B * (merged.n_sym + 2 * a.n_sym + 2 * new.n_sym), 0, "bwd"))
            bwd.append(_apply_bwd(rec_a, g_new, g_a, self.grad_p, n_tup))
            g, first = g_a, False
        # the first paths are the edges themselves: their gradient joins the edges' (an all-true filter's backward adds)
        keep_all = np.ones(self.edges.n_sym, np.uint8)
        rec_id = dol.OpRecord(dol.OP_FILTER, self.edges, None, self.edges, pred_mask=keep_all, accumulate=1)
        bwd.append(Launch("damp_rows_gather_kernel", lambda r=rec_id, g=g: dol.backward(r, g, self.grad_p, None),
                          4 * B * 3 * self.edges.n_sym, 0, "bwd"))
        self.launches = fwd + bwd
        self.sample_ops = 4 * len(self.rounds) * B


class HwfPipeline(Program):
    """Formula pipeline (appendix on the HWF model): Filter every position's 14 classes to the admissible ones
    (digits at even positions, operators at odd ones), fold Apply over the positions with the formula-building
    function over host-interned formula states, evaluate with a unary Apply.  provenance "damp": reverse sweep of
    vector-Jacobian products down to the class probabilities; "dtkp": the kept classes are the input facts (tags
    initialised after the Filter), one dol_dtkp_backward on the result, then the Filters' transposes."""

    def __init__(self, w, provenance="damp", device="cuda"):
        p = w["p"]
        B, L = p.shape[0], p.shape[1]
        self.batch, self.L, self.provenance = B, L, provenance
        dtkp = provenance == "dtkp"
        k = w["k"] if dtkp else 0
        self.p_dev = _dev(p, device)                                   # [B, L, 14]
        self.grad_p = torch.empty_like(self.p_dev)
        self.g = _dev(w["g"], device)
        self.pos = [dol.Dist(np.arange(14), self.p_dev[:, t, :]) for t in range(L)]
        self.keep = [np.ascontiguousarray(m, np.uint8) for m in w["keep"]]
        kept = [dol.filter_plan(self.pos[t], self.keep[t]) for t in range(L)]
        off = np.concatenate([[0], np.cumsum([len(x) for x in kept])]).astype(np.int64)
        self.launches = []
        if dtkp:
            self.fact_prob = torch.empty((B, int(off[-1])), dtype=torch.float32, device=device)
            self.gfact = torch.empty_like(self.fact_prob)
            grp = np.concatenate([np.full(len(x), t, np.int32) for t, x in enumerate(kept)])
            self.prov = dol.Prov(dol.DTKP, k, self.fact_prob, grp)
            self.xs = [dol.Dist(kept[t], self.fact_prob[:, off[t]:off[t + 1]]) for t in range(L)]
            self.tags = [dol.Dist.empty(kept[0], B, device, k=k)]
        else:
            self.prov = None
            self.xs = [dol.Dist.empty(kept[t], B, device) for t in range(L)]
            self.tags = self.xs
        self.filters = [dol.OpRecord(dol.OP_FILTER, self.pos[t], None, self.xs[t], pred_mask=self.keep[t]) for t in range(L)]
        for t in range(L):
            self.launches.append(Launch("damp_gather_cols_kernel", lambda t=t: dol.filter(self.pos[t], self.keep[t], None, self.xs[t]),
                                        4 * B * (14 + self.xs[t].n_sym), 0, "fwd"))
        facts = [np.arange(off[t], off[t + 1], dtype=np.int32) for t in range(L)]
        if dtkp:                                     # only position 0 needs stored tags: the later positions enter
            self.launches.append(Launch("dtkp_init_kernel", lambda: dol.dtkp_init(self.tags[0], facts[0], self.prov),
                                        B * self.tags[0].n_sym * (4 + 12 * k + 4), 0, "fwd"))   # as input operands
        self.tables, self.accs, n_tup = [], [self.tags[0]], []
        for t in range(1, L):
            tb = dol.FnTable.create_dense(w["tables"][t - 1])
            self.tables.append(tb)
            n_tup.append(_n_tuples(w["tables"][t - 1]))
            out = dol.Dist.empty(tb.out_syms, B, device, k=k)
            if dtkp:
                a = self.accs[-1]
                self.launches.append(Launch("dtkp_apply2_kernel",
                                            lambda a=a, t=t, tb=tb, out=out: dol.dtkp_apply2_input(a, facts[t], tb, self.prov, out),
                                            B * (12 * k * (a.n_sym + out.n_sym) + 4 * (self.xs[t].n_sym + out.n_sym)),
                                            B * n_tup[-1] * k, "fwd"))
            else:
                self.launches.append(_apply_fwd(self.accs[-1], self.tags[t], tb, out, n_tup[-1], self.prov, k))
            self.accs.append(out)
        self.final = dol.FnkTable.create_dense(w["final_map"])
        self.out = dol.Dist.empty(self.final.out_syms, B, device, k=k)
        last = self.accs[-1]
        per = 12 * k + 4 if dtkp else 4
        self.launches.append(Launch("dtkp_applyk_kernel" if dtkp else self.final.kernel_fwd,
                                    lambda: dol.apply_k([last], self.final, self.prov, self.out),
                                    B * per * (last.n_sym + self.out.n_sym), B * last.n_sym * max(k, 1), "fwd"))
        n_ops = 2 * L + (1 if dtkp else 0)
        if dtkp:
            self.launches.append(Launch("dtkp_prob_bwd_kernel", lambda: dol.dtkp_backward(self.out, self.prov, self.g, self.gfact),
                                        B * (self.out.n_sym * (12 * k + 4) + 8 * int(off[-1])), 0, "bwd"))
            for t in range(L):
                self.launches.append(Launch("damp_gather_cols_kernel",
                                            lambda t=t: dol.backward(self.filters[t], self.gfact[:, off[t]:off[t + 1]], self.grad_p[:, t, :], None),
                                            4 * B * (14 + self.xs[t].n_sym), 0, "bwd"))
            n_ops += 1 + L
        else:
            self.g_acc = [torch.empty((B, d.n_sym), dtype=torch.float32, device=device) for d in self.accs]
            self.g_x = [torch.empty((B, d.n_sym), dtype=torch.float32, device=device) for d in self.xs]
            self.g_acc[0] = self.g_x[0]                                # the first accumulator is position 0 itself
            self.launches.append(Launch(self.final.kernel_bwd,
                                        lambda: dol.apply_k_backward([last], self.final, self.out, self.g, [self.g_acc[-1]]),
                                        4 * B * (last.n_sym + 2 * self.out.n_sym), B * last.n_sym, "bwd"))   # out, g in; gx out
            self.records = [dol.OpRecord(dol.OP_APPLY2, self.accs[t - 1], self.xs[t], self.accs[t], f=self.tables[t - 1])
                            for t in range(1, L)]
            for t in range(L - 1, 0, -1):
                self.launches.append(_apply_bwd(self.records[t - 1], self.g_acc[t], self.g_acc[t - 1], self.g_x[t], n_tup[t - 1]))
            for t in range(L):
                self.launches.append(Launch("damp_gather_cols_kernel",
                                            lambda t=t: dol.backward(self.filters[t], self.g_x[t], self.grad_p[:, t, :], None),
                                            4 * B * (14 + self.xs[t].n_sym), 0, "bwd"))
            n_ops += 2 * L
        self.sample_ops = n_ops * B


def make_program(config_id: int, workload, device="cuda") -> Program:
    if config_id in (7, 8):
        return HwfPipeline(workload, "dtkp" if config_id == 7 else "damp", device)
    return {1: Sum2Forward, 2: SumChain, 3: HashedPipeline, 4: DtkpSumChain, 5: GridReach,
            6: ProductChain}[config_id](workload, device)
