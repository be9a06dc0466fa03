"""The benchmark programs as sequences of library calls (the chain driver).

Each class uploads one workload, builds the symbol-side plans once (the user
function is evaluated once per batch, Sec. 3.1.2 / App. B), allocates every
intermediate Distribution up front, and then ``forward()`` / ``backward()`` only
issue asynchronous ``dol_*`` calls on the current stream, so a step can be
captured into a HIP graph.  No arithmetic happens in Python.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as dol


def _dev(x: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


def sum_table_of(sym_a, sym_b) -> np.ndarray:
    """Symbol side of apply(D_a, D_b, lambda x, y: x + y): the ids are the integers themselves."""
    return (np.asarray(sym_a, np.int32)[:, None] + np.asarray(sym_b, np.int32)[None, :]).astype(np.int32)


class Sum2Forward:
    """Config 1 (Fig. 2 with two digits): one DAMP apply."""

    def __init__(self, w, device="cuda"):
        self.table = dol.FnTable.create_dense(w["table"])
        self.a = dol.Dist(w["sym"], _dev(w["pa"], device))
        self.b = dol.Dist(w["sym"], _dev(w["pb"], device))
        self.out = dol.Dist.empty(self.table.out_syms, self.a.batch, device)
        self.sample_ops = self.a.batch

    def forward(self):
        dol.apply2(self.a, self.b, self.table, None, self.out)
        return self.out


class SumChain:
    """Config 2 (Fig. 2): left fold of DAMP apply over N digit Distributions, then the reverse sweep of
    vector-Jacobian products from the harness-supplied gradient of -log p[target]."""

    def __init__(self, w, device="cuda"):
        p = w["p"]
        self.n, self.batch = p.shape[0], p.shape[1]
        sym = np.asarray(w["sym"], np.int32)
        self.p_dev = _dev(p, device)                         # [n, B, 10]
        self.digits = [dol.Dist(sym, self.p_dev[t]) for t in range(self.n)]
        self.tables: List[dol.FnTable] = []
        self.accs: List[dol.Dist] = [self.digits[0]]
        for t in range(1, self.n):
            tb = dol.FnTable.create_dense(sum_table_of(self.accs[-1].sym_ids, sym))
            self.tables.append(tb)
            self.accs.append(dol.Dist.empty(tb.out_syms, self.batch, device))
        self.records = [dol.OpRecord(dol.OP_APPLY2, self.accs[t - 1], self.digits[t], self.accs[t], f=self.tables[t - 1])
                        for t in range(1, self.n)]
        self.target = _dev(w["target"].astype(np.int32), device)     # column index = the sum itself
        self.grad_p = torch.empty_like(self.p_dev)           # [n, B, 10]
        self.g_acc = [torch.empty((self.batch, d.n_sym), dtype=torch.float32, device=device) for d in self.accs]
        self.sample_ops = 2 * (self.n - 1) * self.batch

    def forward(self):
        for t in range(1, self.n):
            dol.apply2(self.accs[t - 1], self.digits[t], self.tables[t - 1], None, self.accs[t])
        return self.accs[-1]

    def loss_grad(self):
        """Harness side: d(-log p[target]) / d p, written into the last gradient buffer."""
        dol.nll_grad(self.accs[-1], self.target, self.g_acc[-1])
        return self.g_acc[-1]

    def backward(self):
        for t in range(self.n - 1, 0, -1):
            ga = self.g_acc[t - 1] if t > 1 else self.grad_p[0]
            dol.backward(self.records[t - 1], self.g_acc[t], ga, self.grad_p[t])
        return self.grad_p

    def step(self):
        self.forward()
        self.loss_grad()
        return self.backward()


class HashedPipeline:
    """Config 3: apply with a hashed symbol table, filter by a keep-mask over the produced ids, union with a
    second Distribution over all ids; backward through all three."""

    def __init__(self, w, device="cuda"):
        B = w["pa"].shape[0]
        self.batch = B
        self.table = dol.FnTable.create_dense(w["table"])
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
        self.sample_ops = 6 * B

    def forward(self):
        dol.apply2(self.a, self.b, self.table, None, self.o1)
        dol.filter(self.o1, self.pred, None, self.o2)
        dol.union(self.o2, self.p2, None, self.o3)
        return self.o3

    def backward(self):
        dol.backward(self.rec3, self.g3, self.g2, self.gp2)
        dol.backward(self.rec2, self.g2, self.g1, None)
        dol.backward(self.rec1, self.g1, self.ga, self.gb)
        return self.ga, self.gb, self.gp2

    def step(self):
        self.forward()
        return self.backward()


class DtkpSumChain:
    """Config 4: the sum fold under DTKP-AM with k proofs per tag; fact 10*n+d says "digit n is d"."""

    def __init__(self, w, device="cuda"):
        p = w["p"]
        self.n, self.batch, self.k = p.shape[0], p.shape[1], w["k"]
        sym = np.asarray(w["sym"], np.int32)
        self.fact_prob = _dev(w["fact_prob"], device)
        self.prov = dol.Prov(dol.DTKP, self.k, self.fact_prob, w["fact_group"])
        self.digits = [dol.Dist.empty(sym, self.batch, device, k=self.k) for _ in range(self.n)]
        self.facts = [10 * t + np.arange(10, dtype=np.int32) for t in range(self.n)]
        self.tables, self.accs = [], [self.digits[0]]
        for t in range(1, self.n):
            tb = dol.FnTable.create_dense(sum_table_of(self.accs[-1].sym_ids, sym))
            self.tables.append(tb)
            self.accs.append(dol.Dist.empty(tb.out_syms, self.batch, device, k=self.k))
        self.sample_ops = (self.n - 1) * self.batch

    def forward(self):
        for t in range(self.n):
            dol.dtkp_init(self.digits[t], self.facts[t], self.prov)
        for t in range(1, self.n):
            dol.apply2(self.accs[t - 1], self.digits[t], self.tables[t - 1], self.prov, self.accs[t])
        return self.accs[-1]

    def step(self):
        return self.forward()


class GridReach:
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
        self.E = E
        self.sample_ops = 2 * self.rounds * B

    def forward(self):
        for t in range(self.rounds):
            dol.apply2(self.r[t], self.edges, self.table, None, self.r[t + 1])
        return self.r[-1]

    def backward(self):
        g = self.g_out
        for t in range(self.rounds - 1, -1, -1):
            gn = self.g_r[t % 2]
            dol.backward(self.records[t], g, gn, self.g_e)
            g = gn
        return self.grad_p

    def step(self):
        self.forward()
        return self.backward()
