"""ctypes binding of libdolphin_hip.so: argument marshalling only.

Every function here has the name of the C entry point it calls (minus the
``dol_`` prefix where a class wraps a handle).  Device memory and the stream
come from PyTorch-ROCm; all arithmetic runs in the library's HIP kernels.
There is no fallback: if the shared library is missing, import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdolphin_hip.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libdolphin_hip.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'` "
        "or `python paper_2410_03348_amd/build.py`; there is no CPU fallback." % LIB_PATH)

_lib = C.CDLL(LIB_PATH)

DAMP, DTKP = 0, 1
OP_APPLY2, OP_FILTER, OP_UNION, OP_FILTER_UNION = 0, 1, 2, 3
MAX_K, MAX_FACTS, MAX_SYMBOLS = 8, 63, 65535
ABSENT_PROOF = 0xFFFFFFFFFFFFFFFF
STATUS_NAMES = {0: "DOL_OK", 1: "DOL_EINVAL", 2: "DOL_ESHAPE", 3: "DOL_ENOMEM", 4: "DOL_EHIP", 5: "DOL_EUNSUPPORTED"}


class DolError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, str(status)), message))
        self.status = status


class _Prov(C.Structure):
    _fields_ = [("kind", C.c_int32), ("k", C.c_int32), ("n_facts", C.c_int32),
                ("fact_group", C.POINTER(C.c_int32)), ("fact_prob", C.c_void_p)]


class _Dist(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_sym", C.c_int32), ("ld", C.c_int64),
                ("sym_ids", C.POINTER(C.c_int32)), ("prob", C.c_void_p),
                ("proof_mask", C.c_void_p), ("proof_prob", C.c_void_p)]


class _OpRecord(C.Structure):
    _fields_ = [("op", C.c_int32), ("a", C.POINTER(_Dist)), ("b", C.POINTER(_Dist)), ("out", C.POINTER(_Dist)),
                ("f", C.c_void_p), ("pred_mask", C.POINTER(C.c_uint8)), ("prov", C.POINTER(_Prov)),
                ("accumulate", C.c_int32)]


_i32p = C.POINTER(C.c_int32)
_u8p = C.POINTER(C.c_uint8)
_lib.dol_fn_table_create_dense.argtypes = [C.c_int32, C.c_int32, _i32p, C.POINTER(C.c_void_p)]
_lib.dol_fn_table_create_sparse.argtypes = [C.c_int32, C.c_int32, C.c_int64, _i32p, _i32p, _i32p, C.POINTER(C.c_void_p)]
_lib.dol_fn_table_create_if.argtypes = [C.c_int32, C.c_int32, _i32p, _u8p, C.POINTER(C.c_void_p)]
_lib.dol_fnk_table_create.argtypes = [C.c_int32, _i32p, C.c_int64, _i32p, _i32p, C.POINTER(C.c_void_p)]
_lib.dol_fnk_table_n_out.argtypes = [C.c_void_p]
_lib.dol_fnk_table_n_out.restype = C.c_int32
_lib.dol_fnk_table_out_syms.argtypes = [C.c_void_p]
_lib.dol_fnk_table_out_syms.restype = _i32p
_lib.dol_fnk_table_kernel.argtypes = [C.c_void_p, C.c_int32]
_lib.dol_fnk_table_kernel.restype = C.c_char_p
_lib.dol_fnk_table_destroy.argtypes = [C.c_void_p]
_lib.dol_fnk_table_destroy.restype = None
_lib.dol_apply_k.argtypes = [C.c_int32, C.POINTER(C.POINTER(_Dist)), C.c_void_p, C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_apply_k_backward.argtypes = [C.c_int32, C.POINTER(C.POINTER(_Dist)), C.c_void_p, C.POINTER(_Dist), C.c_void_p,
                                      C.c_int64, C.POINTER(C.c_void_p), C.c_void_p]
_lib.dol_fn_table_n_out.argtypes = [C.c_void_p]
_lib.dol_fn_table_n_out.restype = C.c_int32
_lib.dol_fn_table_out_syms.argtypes = [C.c_void_p]
_lib.dol_fn_table_out_syms.restype = _i32p
_lib.dol_fn_table_kernel.argtypes = [C.c_void_p, C.c_int32]
_lib.dol_fn_table_kernel.restype = C.c_char_p
_lib.dol_fn_table_kernel_at.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
_lib.dol_fn_table_kernel_at.restype = C.c_char_p
_lib.dol_fn_table_destroy.argtypes = [C.c_void_p]
_lib.dol_fn_table_destroy.restype = None
_lib.dol_apply2.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_dtkp_apply2_input.argtypes = [C.POINTER(_Dist), _i32p, C.c_void_p, C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_filter_plan.argtypes = [C.POINTER(_Dist), _u8p, _i32p, _i32p]
_lib.dol_filter.argtypes = [C.POINTER(_Dist), _u8p, C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_union_plan.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), _i32p, _i32p]
_lib.dol_union.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_filter_union_plan.argtypes = [C.POINTER(_Dist), _u8p, C.POINTER(_Dist), _i32p, _i32p]
_lib.dol_filter_union.argtypes = [C.POINTER(_Dist), _u8p, C.POINTER(_Dist), C.POINTER(_Prov), C.POINTER(_Dist), C.c_void_p]
_lib.dol_dtkp_init.argtypes = [C.POINTER(_Dist), _i32p, C.POINTER(_Prov), C.c_void_p]
_lib.dol_backward.argtypes = [C.POINTER(_OpRecord), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.dol_dtkp_backward.argtypes = [C.POINTER(_Dist), C.POINTER(_Prov), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
_lib.dol_nll_grad.argtypes = [C.POINTER(_Dist), C.c_void_p, C.c_void_p, C.c_void_p]
_lib.dol_last_error.restype = C.c_char_p
_lib.dol_version.restype = C.c_char_p


def last_error() -> str:
    return _lib.dol_last_error().decode()


def version() -> str:
    return _lib.dol_version().decode()


def _check(status: int):
    if status != 0:
        raise DolError(status, last_error())


def _np_i32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.int32)


def _ptr(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _stream(stream) -> C.c_void_p:
    """A torch stream, a raw handle, or None = torch's current stream."""
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


class Prov:
    """dol_prov.  fact_prob: float32 device tensor [batch, n_facts]; fact_group: host ints or None."""

    def __init__(self, kind: int = DAMP, k: int = 0, fact_prob: Optional[torch.Tensor] = None, fact_group=None):
        self.kind, self.k = kind, k
        self.fact_prob = fact_prob
        self._grp = None if fact_group is None else _np_i32(fact_group)
        n_facts = 0
        if fact_prob is not None:
            assert fact_prob.dtype == torch.float32 and fact_prob.is_contiguous() and fact_prob.dim() == 2
            n_facts = fact_prob.shape[1]
        if self._grp is not None:
            assert self._grp.size == n_facts
        self.c = _Prov(kind, k, n_facts, _ptr(self._grp, C.c_int32),
                       C.c_void_p(fact_prob.data_ptr()) if fact_prob is not None else None)

    def ref(self):
        return C.byref(self.c)


class Dist:
    """dol_dist over caller-owned torch tensors.  prob: float32 [batch, ld>=n_sym] (row stride = ld)."""

    def __init__(self, sym_ids, prob: Optional[torch.Tensor], proof_mask: Optional[torch.Tensor] = None,
                 proof_prob: Optional[torch.Tensor] = None, batch: Optional[int] = None):
        self.sym_ids = _np_i32(sym_ids)
        n = self.sym_ids.size
        self.prob, self.proof_mask, self.proof_prob = prob, proof_mask, proof_prob
        ld = n
        if prob is not None:
            assert prob.dtype == torch.float32 and prob.dim() == 2 and (prob.shape[1] == 0 or prob.stride(1) == 1)
            assert prob.shape[1] == n
            batch = prob.shape[0]
            ld = max(int(prob.stride(0)), n)
        for t, dt in ((proof_mask, (torch.int64, torch.uint64)), (proof_prob, (torch.float32,))):
            if t is not None:
                assert t.dtype in dt and t.is_contiguous() and t.dim() == 3 and t.shape[1] == n
                batch = t.shape[0] if batch is None else batch
        assert batch is not None
        self.batch, self.n_sym, self.ld = batch, n, ld
        self.c = _Dist(batch, n, ld, _ptr(self.sym_ids, C.c_int32),
                       C.c_void_p(prob.data_ptr()) if prob is not None else None,
                       C.c_void_p(proof_mask.data_ptr()) if proof_mask is not None else None,
                       C.c_void_p(proof_prob.data_ptr()) if proof_prob is not None else None)

    def ref(self):
        return C.byref(self.c)

    @staticmethod
    def empty(sym_ids, batch: int, device="cuda", k: int = 0, ld: Optional[int] = None) -> "Dist":
        """Allocate uninitialised tag tensors (torch is the allocator)."""
        n = len(sym_ids)
        ld = n if ld is None else ld
        prob = torch.empty((batch, ld), dtype=torch.float32, device=device)[:, :n] if ld != n else \
            torch.empty((batch, n), dtype=torch.float32, device=device)
        pm = pp = None
        if k > 0:
            pm = torch.empty((batch, n, k), dtype=torch.int64, device=device)
            pp = torch.empty((batch, n, k), dtype=torch.float32, device=device)
        return Dist(sym_ids, prob, pm, pp, batch=batch)


class FnTable:
    """dol_fn_table handle."""

    def __init__(self, handle: C.c_void_p, na: int, nb: int):
        self._h, self.na, self.nb = handle, na, nb
        self.n_out = int(_lib.dol_fn_table_n_out(handle))
        p = _lib.dol_fn_table_out_syms(handle)
        self.out_syms = np.ctypeslib.as_array(p, shape=(self.n_out,)).copy() if self.n_out else np.empty(0, np.int32)
        self.kernel_fwd = _lib.dol_fn_table_kernel(handle, 0).decode()
        self.kernel_bwd = _lib.dol_fn_table_kernel(handle, 1).decode()

    def kernel_at(self, backward: bool, batch: int) -> str:
        """Name of the DAMP kernel launched for a batch of this size with contiguous, aligned tensors."""
        return _lib.dol_fn_table_kernel_at(self._h, 1 if backward else 0, batch).decode()

    @staticmethod
    def create_dense(out_id) -> "FnTable":
        t = _np_i32(out_id)
        assert t.ndim == 2
        h = C.c_void_p()
        _check(_lib.dol_fn_table_create_dense(t.shape[0], t.shape[1], _ptr(t, C.c_int32), C.byref(h)))
        return FnTable(h, t.shape[0], t.shape[1])

    @staticmethod
    def create_if(out_id, cond) -> "FnTable":
        """ApplyIf: the table of out_id restricted to the tuples where cond is non-zero."""
        t = _np_i32(out_id)
        c = np.ascontiguousarray(cond, dtype=np.uint8)
        assert t.ndim == 2 and c.shape == t.shape
        h = C.c_void_p()
        _check(_lib.dol_fn_table_create_if(t.shape[0], t.shape[1], _ptr(t, C.c_int32), _ptr(c, C.c_uint8), C.byref(h)))
        return FnTable(h, t.shape[0], t.shape[1])

    @staticmethod
    def create_sparse(na: int, nb: int, i, j, out_id) -> "FnTable":
        i, j, o = _np_i32(i), _np_i32(j), _np_i32(out_id)
        assert i.shape == j.shape == o.shape and i.ndim == 1
        h = C.c_void_p()
        _check(_lib.dol_fn_table_create_sparse(na, nb, i.size, _ptr(i, C.c_int32), _ptr(j, C.c_int32),
                                               _ptr(o, C.c_int32), C.byref(h)))
        return FnTable(h, na, nb)

    def destroy(self):
        if self._h is not None:
            _lib.dol_fn_table_destroy(self._h)
            self._h = None

    def __del__(self):
        # The collector may run this at any moment, also while a stream is being captured into a HIP graph, where
        # releasing device memory and code is not allowed: such handles wait for the next release outside a capture.
        try:
            if self._h is None:
                return
            if torch.cuda.is_available() and torch.cuda.is_current_stream_capturing():
                _deferred_tables.append(self._h)
                self._h = None
                return
            self.destroy()
            while _deferred_tables:
                _lib.dol_fn_table_destroy(_deferred_tables.pop())
        except Exception:
            pass


_deferred_tables = []


def apply2(a: Dist, b: Dist, f: FnTable, prov: Optional[Prov], out: Dist, stream=None):
    _check(_lib.dol_apply2(a.ref(), b.ref(), f._h, prov.ref() if prov else None, out.ref(), _stream(stream)))


class FnkTable:
    """dol_fnk_table handle: the admitted tuples of a function over K Distributions."""

    def __init__(self, n_sym, idx, out_id):
        n_sym, o = _np_i32(n_sym), _np_i32(out_id)
        self.K = int(n_sym.size)
        idx = _np_i32(idx).reshape(-1, self.K)
        assert idx.shape[0] == o.size
        h = C.c_void_p()
        _check(_lib.dol_fnk_table_create(self.K, _ptr(n_sym, C.c_int32), o.size, _ptr(idx, C.c_int32),
                                         _ptr(o, C.c_int32), C.byref(h)))
        self._h, self.n_sym = h, n_sym
        self.n_out = int(_lib.dol_fnk_table_n_out(h))
        self.kernel_fwd = _lib.dol_fnk_table_kernel(h, 0).decode()
        self.kernel_bwd = _lib.dol_fnk_table_kernel(h, 1).decode()
        p = _lib.dol_fnk_table_out_syms(h)
        self.out_syms = np.ctypeslib.as_array(p, shape=(self.n_out,)).copy() if self.n_out else np.empty(0, np.int32)

    @staticmethod
    def create_dense(out_id, cond=None) -> "FnkTable":
        """out_id: int array with one axis per operand; entries < 0, or where cond is zero, are rejected tuples."""
        t = _np_i32(out_id)
        if cond is not None:
            t = np.where(np.asarray(cond) != 0, t, -1).astype(np.int32)
        idx = np.argwhere(t >= 0).astype(np.int32).reshape(-1, t.ndim)
        return FnkTable(t.shape, idx, t[tuple(idx.T)])

    def destroy(self):
        if self._h is not None:
            _lib.dol_fnk_table_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _dist_array(dists):
    return (C.POINTER(_Dist) * len(dists))(*[C.pointer(d.c) for d in dists])


def apply_k(ins, f: FnkTable, prov: Optional[Prov], out: Dist, stream=None):
    _check(_lib.dol_apply_k(len(ins), _dist_array(ins), f._h, prov.ref() if prov else None, out.ref(), _stream(stream)))


def apply_k_backward(ins, f: FnkTable, out: Dist, grad_out: torch.Tensor, grad_in, stream=None):
    """grad_out [batch, >= n_out] (row stride = its stride(0)); grad_in: one tensor (rows of stride ins[l].ld) or None per operand."""
    assert grad_out.dtype == torch.float32 and grad_out.dim() == 2 and grad_out.stride(1) == 1
    ptrs = (C.c_void_p * len(ins))(*[None if g is None else g.data_ptr() for g in grad_in])
    _check(_lib.dol_apply_k_backward(len(ins), _dist_array(ins), f._h, out.ref(), _dptr(grad_out),
                                     max(int(grad_out.stride(0)), grad_out.shape[1]), ptrs, _stream(stream)))


def dtkp_apply2_input(a: Dist, fact_of_sym_b, f: FnTable, prov: Prov, out: Dist, stream=None):
    """dol_apply2 whose second operand is an input Distribution: symbol j of it is fact fact_of_sym_b[j]."""
    fb = _np_i32(fact_of_sym_b)
    assert fb.size == f.nb
    _check(_lib.dol_dtkp_apply2_input(a.ref(), _ptr(fb, C.c_int32), f._h, prov.ref(), out.ref(), _stream(stream)))


def filter_plan(d: Dist, pred_mask):
    pm = np.ascontiguousarray(pred_mask, dtype=np.uint8)
    n = C.c_int32()
    syms = np.empty(max(d.n_sym, 1), np.int32)
    _check(_lib.dol_filter_plan(d.ref(), _ptr(pm, C.c_uint8), C.byref(n), _ptr(syms, C.c_int32)))
    return syms[:n.value].copy()


def filter(d: Dist, pred_mask, prov: Optional[Prov], out: Dist, stream=None):  # noqa: A001 (the operator's name)
    pm = np.ascontiguousarray(pred_mask, dtype=np.uint8)
    _check(_lib.dol_filter(d.ref(), _ptr(pm, C.c_uint8), prov.ref() if prov else None, out.ref(), _stream(stream)))


def union_plan(a: Dist, b: Dist):
    n = C.c_int32()
    syms = np.empty(max(a.n_sym + b.n_sym, 1), np.int32)
    _check(_lib.dol_union_plan(a.ref(), b.ref(), C.byref(n), _ptr(syms, C.c_int32)))
    return syms[:n.value].copy()


def union(a: Dist, b: Dist, prov: Optional[Prov], out: Dist, stream=None):
    _check(_lib.dol_union(a.ref(), b.ref(), prov.ref() if prov else None, out.ref(), _stream(stream)))


def filter_union_plan(d: Dist, pred_mask, c: Dist):
    pm = np.ascontiguousarray(pred_mask, dtype=np.uint8)
    n = C.c_int32()
    syms = np.empty(max(d.n_sym + c.n_sym, 1), np.int32)
    _check(_lib.dol_filter_union_plan(d.ref(), _ptr(pm, C.c_uint8), c.ref(), C.byref(n), _ptr(syms, C.c_int32)))
    return syms[:n.value].copy()


def filter_union(d: Dist, pred_mask, c: Dist, prov: Optional[Prov], out: Dist, stream=None):
    pm = np.ascontiguousarray(pred_mask, dtype=np.uint8)
    _check(_lib.dol_filter_union(d.ref(), _ptr(pm, C.c_uint8), c.ref(), prov.ref() if prov else None, out.ref(),
                                 _stream(stream)))


class _ApplyMerge(C.Structure):
    _fields_ = [("a", C.POINTER(_Dist)), ("b", C.POINTER(_Dist)), ("f", C.c_void_p), ("pred_mask", _u8p),
                ("c", C.POINTER(_Dist)), ("out", C.POINTER(_Dist)), ("saved", C.c_void_p)]


_lib.dol_apply2_filter_union.argtypes = [C.POINTER(_ApplyMerge), C.c_void_p]
_lib.dol_apply2_filter_union_backward.argtypes = [C.POINTER(_ApplyMerge), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_int32, C.c_void_p]
_lib.dol_apply2_filter_union_forward_backward.argtypes = _lib.dol_apply2_filter_union_backward.argtypes


class ApplyMerge:
    """dol_apply_merge: union(filter(apply2(a, b, f), pred_mask), c) described once, for the forward and reverse calls."""

    def __init__(self, a: Dist, b: Dist, f: FnTable, pred_mask, c: Dist, out: Dist, saved: Optional[torch.Tensor] = None):
        self._keep = (a, b, f, c, out, saved)
        self._pred = np.ascontiguousarray(pred_mask, dtype=np.uint8)
        assert self._pred.shape == (f.n_out,)
        assert saved is None or (saved.dtype == torch.int32 and saved.is_contiguous() and saved.shape == (a.batch,))
        self.c = _ApplyMerge(C.pointer(a.c), C.pointer(b.c), f._h, _ptr(self._pred, C.c_uint8), C.pointer(c.c), C.pointer(out.c),
                             C.c_void_p(saved.data_ptr()) if saved is not None else None)


def apply2_filter_union(m: ApplyMerge, stream=None):
    _check(_lib.dol_apply2_filter_union(C.byref(m.c), _stream(stream)))


def apply2_filter_union_backward(m: ApplyMerge, grad_out: torch.Tensor, grad_a: Optional[torch.Tensor],
                                 grad_b: Optional[torch.Tensor], grad_c: Optional[torch.Tensor], accumulate: int = 0,
                                 stream=None):
    assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
    _check(_lib.dol_apply2_filter_union_backward(C.byref(m.c), _dptr(grad_out), int(grad_out.stride(0)), _dptr(grad_a),
                                                 _dptr(grad_b), _dptr(grad_c), accumulate, _stream(stream)))


def apply2_filter_union_forward_backward(m: ApplyMerge, grad_out: torch.Tensor, grad_a: Optional[torch.Tensor],
                                         grad_b: Optional[torch.Tensor], grad_c: Optional[torch.Tensor], accumulate: int = 0,
                                         stream=None):
    """Forward and backward of union(filter(apply2(a, b, f)), c) in one launch (grad_out is an input)."""
    assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
    _check(_lib.dol_apply2_filter_union_forward_backward(C.byref(m.c), _dptr(grad_out), int(grad_out.stride(0)), _dptr(grad_a),
                                                         _dptr(grad_b), _dptr(grad_c), accumulate, _stream(stream)))


def dtkp_init(d: Dist, fact_of_sym, prov: Prov, stream=None):
    fos = _np_i32(fact_of_sym)
    _check(_lib.dol_dtkp_init(d.ref(), _ptr(fos, C.c_int32), prov.ref(), _stream(stream)))


class OpRecord:
    """dol_op_record; keeps its operands alive."""

    def __init__(self, op: int, a: Dist, b: Optional[Dist], out: Dist, f: Optional[FnTable] = None, pred_mask=None,
                 prov: Optional[Prov] = None, accumulate: int = 0):
        self.a, self.b, self.out, self.f, self.prov = a, b, out, f, prov
        self.pred = None if pred_mask is None else np.ascontiguousarray(pred_mask, dtype=np.uint8)
        self.c = _OpRecord(op, C.pointer(a.c), C.pointer(b.c) if b is not None else None, C.pointer(out.c),
                           f._h if f is not None else None, _ptr(self.pred, C.c_uint8),
                           C.pointer(prov.c) if prov is not None else None, accumulate)


def _dptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def backward(rec: OpRecord, grad_out: torch.Tensor, grad_a: Optional[torch.Tensor], grad_b: Optional[torch.Tensor],
             stream=None):
    """grad_out rows have stride rec.out.ld, grad_a rows rec.a.ld, grad_b rows rec.b.ld."""
    _check(_lib.dol_backward(C.byref(rec.c), _dptr(grad_out), _dptr(grad_a), _dptr(grad_b), _stream(stream)))


def dtkp_backward(d: Dist, prov: Prov, grad_prob: torch.Tensor, grad_fact_prob: torch.Tensor, stream=None):
    """grad_prob [batch, >= n_sym] (row stride = its stride(0)); grad_fact_prob [batch, n_facts] contiguous, overwritten."""
    assert grad_prob.dtype == torch.float32 and grad_prob.dim() == 2 and grad_prob.stride(1) == 1
    assert grad_fact_prob.dtype == torch.float32 and grad_fact_prob.is_contiguous()
    _check(_lib.dol_dtkp_backward(d.ref(), prov.ref(), _dptr(grad_prob), max(int(grad_prob.stride(0)), grad_prob.shape[1]),
                                  _dptr(grad_fact_prob), _stream(stream)))


class _Fold(C.Structure):
    _fields_ = [("n_inputs", C.c_int32), ("inputs", C.POINTER(C.POINTER(_Dist))), ("tables", C.POINTER(C.c_void_p)),
                ("out", C.POINTER(_Dist)), ("target_col", C.c_void_p), ("grad_out", C.c_void_p),
                ("grad_out_ld", C.c_int64), ("grad_inputs", C.POINTER(C.c_void_p))]


_lib.dol_fold_apply2.argtypes = [C.POINTER(_Fold), C.c_void_p]
_lib.dol_fold_kernel.argtypes = [C.POINTER(_Fold)]
_lib.dol_fold_kernel.restype = C.c_char_p


class Fold:
    """dol_fold: a left fold of DAMP applies run forward (and backward) in one launch.  Keeps its operands alive."""

    def __init__(self, inputs, tables, out: Optional[Dist] = None, target_col: Optional[torch.Tensor] = None,
                 grad_out: Optional[torch.Tensor] = None, grad_inputs=None):
        n = len(inputs)
        assert len(tables) == n - 1
        self.keep = (inputs, tables, out, target_col, grad_out, grad_inputs)
        self._in = (C.POINTER(_Dist) * n)(*[C.pointer(d.c) for d in inputs])
        self._tb = (C.c_void_p * max(n - 1, 1))(*[t._h for t in tables])
        self._gi = None
        if grad_inputs is not None:
            assert len(grad_inputs) == n
            self._gi = (C.c_void_p * n)(*[None if g is None else g.data_ptr() for g in grad_inputs])
        if target_col is not None:
            assert target_col.dtype == torch.int32 and target_col.is_contiguous()
        ldg = 0
        if grad_out is not None:
            assert grad_out.dtype == torch.float32 and grad_out.dim() == 2 and grad_out.stride(1) == 1
            ldg = max(int(grad_out.stride(0)), grad_out.shape[1])
        self.c = _Fold(n, self._in, self._tb, C.pointer(out.c) if out is not None else None,
                       _dptr(target_col), _dptr(grad_out), ldg,
                       C.cast(self._gi, C.POINTER(C.c_void_p)) if self._gi is not None else None)


def fold_apply2(fold: Fold, stream=None):
    _check(_lib.dol_fold_apply2(C.byref(fold.c), _stream(stream)))


def fold_kernel(fold: Fold) -> str:
    return _lib.dol_fold_kernel(C.byref(fold.c)).decode()


class _DtkpFold(C.Structure):
    _fields_ = [("n_inputs", C.c_int32), ("inputs", C.POINTER(C.POINTER(_Dist))), ("fact_of_sym", C.POINTER(_i32p)),
                ("tables", C.POINTER(C.c_void_p)), ("out", C.POINTER(_Dist)), ("target_col", C.c_void_p),
                ("grad_out", C.c_void_p), ("grad_out_ld", C.c_int64), ("grad_fact_prob", C.c_void_p)]


_lib.dol_dtkp_fold_apply2.argtypes = [C.POINTER(_DtkpFold), C.POINTER(_Prov), C.c_void_p]


class DtkpFold:
    """dol_dtkp_fold: a left fold of DTKP applies over naturally initialised inputs, one launch.  Keeps its operands alive."""

    def __init__(self, inputs, facts, tables, out: Dist, target_col: Optional[torch.Tensor] = None,
                 grad_out: Optional[torch.Tensor] = None, grad_fact_prob: Optional[torch.Tensor] = None):
        n = len(inputs)
        assert len(tables) == n - 1 and len(facts) == n
        self._facts = [_np_i32(f) for f in facts]
        self.keep = (inputs, tables, out, target_col, grad_out, grad_fact_prob)
        self._in = (C.POINTER(_Dist) * n)(*[C.pointer(d.c) for d in inputs])
        self._fo = (_i32p * n)(*[_ptr(f, C.c_int32) for f in self._facts])
        self._tb = (C.c_void_p * max(n - 1, 1))(*[t._h for t in tables])
        if target_col is not None:
            assert target_col.dtype == torch.int32 and target_col.is_contiguous()
        ldg = 0
        if grad_out is not None:
            assert grad_out.dtype == torch.float32 and grad_out.dim() == 2 and grad_out.stride(1) == 1
            ldg = max(int(grad_out.stride(0)), grad_out.shape[1])
        if grad_fact_prob is not None:
            assert grad_fact_prob.dtype == torch.float32 and grad_fact_prob.is_contiguous()
        self.c = _DtkpFold(n, self._in, self._fo, self._tb, C.pointer(out.c), _dptr(target_col), _dptr(grad_out), ldg,
                           _dptr(grad_fact_prob))


def dtkp_fold_apply2(fold: DtkpFold, prov: Prov, stream=None):
    _check(_lib.dol_dtkp_fold_apply2(C.byref(fold.c), prov.ref(), _stream(stream)))


_lib.dol_iterate_apply2.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
_lib.dol_iterate_backward.argtypes = [C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_void_p, C.c_void_p]


def iterate_apply2(r0: Dist, e: Dist, f: FnTable, rounds: int, hist: torch.Tensor, stream=None):
    """hist: float32 [rounds+1, batch, na] contiguous; receives r_0 .. r_rounds."""
    assert hist.dtype == torch.float32 and hist.is_contiguous() and hist.shape == (rounds + 1, r0.batch, f.na)
    _check(_lib.dol_iterate_apply2(r0.ref(), e.ref(), f._h, rounds, _dptr(hist), _stream(stream)))


def iterate_backward(e: Dist, f: FnTable, rounds: int, hist: torch.Tensor, grad_out: torch.Tensor,
                     grad_r0: Optional[torch.Tensor], grad_e: Optional[torch.Tensor], stream=None):
    """grad_out rows: stride grad_out.stride(0); grad_r0 [batch, na] contiguous; grad_e rows have stride e.ld."""
    assert hist.dtype == torch.float32 and hist.is_contiguous() and hist.shape == (rounds + 1, e.batch, f.na)
    assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
    assert grad_r0 is None or grad_r0.is_contiguous()
    _check(_lib.dol_iterate_backward(e.ref(), f._h, rounds, _dptr(hist), _dptr(grad_out),
                                     max(int(grad_out.stride(0)), grad_out.shape[1]), _dptr(grad_r0), _dptr(grad_e),
                                     _stream(stream)))


_lib.dol_iterate_ckpt_count.argtypes = [C.c_int32, C.c_int32]
_lib.dol_iterate_ckpt_count.restype = C.c_int32
_lib.dol_iterate_ckpt_every.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
_lib.dol_iterate_ckpt_every.restype = C.c_int32
_lib.dol_iterate_apply2_ckpt.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_int32,
                                         C.POINTER(_Dist), C.c_void_p, C.c_void_p]
_lib.dol_iterate_backward_ckpt.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]


def iterate_ckpt_count(rounds: int, ckpt_every: int) -> int:
    return int(_lib.dol_iterate_ckpt_count(rounds, ckpt_every))


def iterate_ckpt_every(f: FnTable, batch: int, rounds: int) -> int:
    """The checkpoint interval the library favours for this table, batch and round count."""
    return int(_lib.dol_iterate_ckpt_every(f._h, batch, rounds))


def iterate_apply2_ckpt(r0: Dist, e: Dist, f: FnTable, rounds: int, ckpt_every: int, out: Dist,
                        ckpt: Optional[torch.Tensor], stream=None):
    """ckpt: float32 [iterate_ckpt_count(rounds, ckpt_every), batch, na] contiguous (None when that count is 0)."""
    n = iterate_ckpt_count(rounds, ckpt_every)
    assert n == 0 or (ckpt.dtype == torch.float32 and ckpt.is_contiguous() and ckpt.shape == (n, r0.batch, f.na))
    _check(_lib.dol_iterate_apply2_ckpt(r0.ref(), e.ref(), f._h, rounds, ckpt_every, out.ref(), _dptr(ckpt),
                                        _stream(stream)))


def iterate_backward_ckpt(r0: Dist, e: Dist, f: FnTable, rounds: int, ckpt_every: int, ckpt: Optional[torch.Tensor],
                          grad_out: torch.Tensor, grad_r0: Optional[torch.Tensor], grad_e: Optional[torch.Tensor],
                          stream=None):
    assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
    assert grad_r0 is None or grad_r0.is_contiguous()
    _check(_lib.dol_iterate_backward_ckpt(r0.ref(), e.ref(), f._h, rounds, ckpt_every, _dptr(ckpt), _dptr(grad_out),
                                          max(int(grad_out.stride(0)), grad_out.shape[1]), _dptr(grad_r0), _dptr(grad_e),
                                          _stream(stream)))


_lib.dol_iterate_apply2_backward.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_int32,
                                             C.POINTER(_Dist), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                             C.c_void_p, C.c_void_p]


def iterate_apply2_backward(r0: Dist, e: Dist, f: FnTable, rounds: int, ckpt_every: int, out: Dist,
                            ckpt: Optional[torch.Tensor], target_col: Optional[torch.Tensor], grad_out: Optional[torch.Tensor],
                            grad_r0: Optional[torch.Tensor], grad_e: Optional[torch.Tensor], stream=None):
    """Forward rounds and reverse sweep in one call (one launch up to 512 samples); exactly one of target_col (int32 [batch])
    and grad_out."""
    ldg = 0
    if grad_out is not None:
        assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
        ldg = max(int(grad_out.stride(0)), grad_out.shape[1])
    if target_col is not None:
        assert target_col.dtype == torch.int32 and target_col.is_contiguous()
    assert grad_r0 is None or grad_r0.is_contiguous()
    _check(_lib.dol_iterate_apply2_backward(r0.ref(), e.ref(), f._h, rounds, ckpt_every, out.ref(), _dptr(ckpt), _dptr(target_col),
                                            _dptr(grad_out), ldg, _dptr(grad_r0), _dptr(grad_e), _stream(stream)))


_lib.dol_iterate_backward_noalloc.argtypes = [C.POINTER(_Dist), C.POINTER(_Dist), C.c_void_p, C.c_int32, C.c_void_p,
                                              C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]


def iterate_backward_noalloc(r0: Dist, e: Dist, f: FnTable, rounds: int, grad_out: torch.Tensor,
                             grad_r0: Optional[torch.Tensor], grad_e: Optional[torch.Tensor], stream=None):
    """The reverse sweep with the library's built-in workspace: no allocation, forward sweep replayed inside."""
    assert grad_out.dtype == torch.float32 and grad_out.stride(1) == 1
    assert grad_r0 is None or grad_r0.is_contiguous()
    _check(_lib.dol_iterate_backward_noalloc(r0.ref(), e.ref(), f._h, rounds, _dptr(grad_out),
                                             max(int(grad_out.stride(0)), grad_out.shape[1]), _dptr(grad_r0),
                                             _dptr(grad_e), _stream(stream)))


def nll_grad(d: Dist, target_col: torch.Tensor, grad: torch.Tensor, stream=None):
    """target_col: int32 device tensor [batch]; grad rows have stride d.ld."""
    assert target_col.dtype == torch.int32 and target_col.is_contiguous()
    _check(_lib.dol_nll_grad(d.ref(), _dptr(target_col), _dptr(grad), _stream(stream)))
