"""dol_iterate_backward_noalloc (the entry point that allocates nothing) against dol_iterate_apply2_ckpt +
dol_iterate_backward_ckpt, through the C ABI: two calls in a row, the second on a smaller input."""
import ctypes as C
import gc

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def host(t):
    return t.detach().cpu().numpy()


def _reference(dol, gp, w):
    prog = gp.GridReachFused(w, ckpt_every=8)
    prog.step()
    g0 = torch.empty((prog.batch, prog.r0.n_sym), device="cuda")
    dol.iterate_backward_ckpt(prog.r0, prog.edges, prog.table, prog.rounds, 8, prog.ckpt, prog.g_out, g0, None)
    torch.cuda.synchronize()
    return prog, host(g0).copy(), host(prog.g_e).copy()


def test_no_alloc_entry_point_matches_the_workspace_one():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2410_03348_amd import binding as dol, programs as gp
    lib = dol._lib
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for batch, side, rounds in [(96, 16, 40), (10, 5, 11)]:           # the second call is smaller than the first
        w = W.config5(batch=batch, side=side, rounds=rounds, seed=9)
        prog, want_g0, want_ge = _reference(dol, gp, w)
        n, nb = side * side, prog.edges.n_sym
        g0 = torch.full((batch, n), -7.0, device="cuda")
        ge = torch.full((batch, nb), -7.0, device="cuda")
        gc.collect()                        # (tensors of earlier tests must not be released in between)
        gc.disable()
        try:
            before = torch.cuda.memory_allocated()
            st = lib.dol_iterate_backward_noalloc(prog.r0.ref(), prog.edges.ref(), prog.table._h, rounds,
                                                  C.c_void_p(prog.g_out.data_ptr()), prog.g_out.stride(0),
                                                  C.c_void_p(g0.data_ptr()), C.c_void_p(ge.data_ptr()), stream)
            assert st == 0, dol.last_error()
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
        finally:
            gc.enable()
        np.testing.assert_array_equal(host(g0), want_g0)               # same kernels, same order: bit for bit
        np.testing.assert_array_equal(host(ge), want_ge)
    # beyond the built-in workspace: a clear error, outputs untouched
    big = dol.FnTable.create_sparse(4096, 2, np.arange(4096, dtype=np.int32), np.zeros(4096, np.int32),
                                    np.arange(4096, dtype=np.int32))
    B = 600
    r0 = dol.Dist(np.arange(4096), torch.zeros((B, 4096), device="cuda"))
    e = dol.Dist(np.arange(2), torch.ones((B, 2), device="cuda"))
    g = torch.zeros((B, 4096), device="cuda")
    out = torch.full((B, 4096), 3.0, device="cuda")
    st = lib.dol_iterate_backward_noalloc(r0.ref(), e.ref(), big._h, 64, C.c_void_p(g.data_ptr()), 4096,
                                          C.c_void_p(out.data_ptr()), None, stream)
    assert st == 5 and "workspace" in dol.last_error()
    assert float(out.min()) == 3.0
