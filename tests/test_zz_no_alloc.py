"""prefixkv_select_static, the entry point for callers that cannot allocate: through the C ABI, its
outputs equal prefixkv_select's bit for bit on two calls in a row (the second on a smaller input, so
the built-in scratch array still holds the first call's words), and the calls allocate nothing."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2412_03409_amd as P
from paper_2412_03409_amd import binding as Bd
from pkv_workloads import synthetic_importance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def alloc_out(B, L, N):
    return P.SelectResult(
        order=torch.full((B, L, N), -7, dtype=torch.int32, device=DEV),
        cum=torch.full((B, L, N), -7, dtype=torch.int64, device=DEV),
        prefix=torch.full((B, L, N), -7.0, dtype=torch.float32, device=DEV),
        lengths=torch.full((B, L), -7, dtype=torch.int32, device=DEV),
        p=torch.full((B,), -7.0, dtype=torch.float64, device=DEV),
        iters=torch.full((B,), -7, dtype=torch.int32, device=DEV),
        raw_total=torch.full((B,), -7, dtype=torch.int64, device=DEV),
        status=torch.full((B,), -7, dtype=torch.int32, device=DEV))


def raw_static_call(imp, budget, out, tol=0, max_iters=64, fixup=1):
    """The C entry point itself, through ctypes: plain device pointers and sizes."""
    lib = P.load()
    B, L, N = imp.shape
    prm = Bd._SelectParams(int(budget), int(tol), int(max_iters), int(fixup))
    vp = lambda t: C.c_void_p(t.data_ptr())
    return lib.prefixkv_select_static(B, L, N, vp(imp), C.byref(prm), vp(out.order), vp(out.cum), vp(out.prefix),
                                      vp(out.lengths), vp(out.p), vp(out.iters), vp(out.raw_total), vp(out.status),
                                      C.c_void_p(torch.cuda.current_stream().cuda_stream))


def same(a: P.SelectResult, b: P.SelectResult, status_zero_only_rows=None):
    st = a.status.cpu().numpy()
    np.testing.assert_array_equal(st, b.status.cpu().numpy())
    ok = st == 0          # order/cum/prefix of a rejected sequence are unspecified
    for f in ("lengths", "p", "iters", "raw_total"):
        np.testing.assert_array_equal(getattr(a, f).cpu().numpy(), getattr(b, f).cpu().numpy(), err_msg=f)
    for f in ("order", "cum", "prefix"):
        np.testing.assert_array_equal(getattr(a, f).cpu().numpy()[ok], getattr(b, f).cpu().numpy()[ok], err_msg=f)


def test_static_select_equals_select_on_two_calls_in_a_row():
    assert P.prefixkv_static_scratch_segments() == 65536
    cases = [(3, 32, 680, 4352, 0), (2, 5, 100, 77, 3)]      # the second call is smaller
    inputs = []
    for i, (B, L, N, budget, tol) in enumerate(cases):
        imp = synthetic_importance(B, L, N, seed=900 + i, ties=bool(i))
        if i == 0:
            imp[1, 4, 9] = float("nan")                      # one rejected sequence: its status words are non-zero
        imp = torch.from_numpy(imp).to(DEV) if isinstance(imp, np.ndarray) else imp.to(DEV)
        inputs.append((imp, budget, tol, alloc_out(B, L, N), alloc_out(B, L, N)))
    # reference results from the existing entry point (this one may allocate its workspace)
    for imp, budget, tol, ref, _ in inputs:
        P.prefixkv_select(imp, budget, tol_tokens=tol, out=ref)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    for imp, budget, tol, _, got in inputs:                  # two calls in a row, no synchronisation between them
        assert raw_static_call(imp, budget, got, tol=tol) == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    for imp, budget, tol, ref, got in inputs:
        same(ref, got)
        st = got.status.cpu().numpy()
        L, N = imp.shape[1], imp.shape[2]
        if L < budget < L * N:
            assert (got.lengths.cpu().numpy()[st == 0].sum(-1) == budget).all()
    assert inputs[0][4].status.cpu().numpy().tolist() == [0, 1, 0]


def test_static_select_through_the_binding_and_size_limit():
    B, L, N = 2, 40, 680
    imp = synthetic_importance(B, L, N, seed=77)
    imp = torch.from_numpy(imp).to(DEV) if isinstance(imp, np.ndarray) else imp.to(DEV)
    ref = P.prefixkv_select(imp, 5440)
    got = P.prefixkv_select_static(imp, 5440, alloc_out(B, L, N))
    torch.cuda.synchronize()
    same(ref, got)
    # more segments than the built-in array holds: refused, nothing enqueued
    lib = P.load()
    prm = Bd._SelectParams(10, 0, 64, 1)
    fake = C.c_void_p(0x1000)
    assert lib.prefixkv_select_static(1025, 64, 8, fake, C.byref(prm), fake, fake, None, fake, fake, fake, fake,
                                      fake, None) == 5
