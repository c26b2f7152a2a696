"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments synchronously (no launch happens on these paths)."""
import ctypes as C
import os
import re

import pytest

import paper_2412_03409_amd as P
from paper_2412_03409_amd import binding as Bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "prefixkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(prefixkv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load()
    names = declared_symbols()
    assert {"prefixkv_importance", "prefixkv_select", "prefixkv_compact", "prefixkv_decode_attn"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert P.prefixkv_version() >= 100
    assert P.prefixkv_status_string(0) == "ok"


def test_workspace_queries():
    dt = P.PKV_BF16
    # bf16: one row of N column sums per (head, workgroup of the head); a workgroup holds 12 pairs of 32-row
    # tiles, so 680 positions (22 tiles, 11 pairs) are one workgroup and 8192 positions (128 pairs) are 11
    per = (1 * 32 * 32 * 680 * 4 + 255) // 256 * 256
    assert P.prefixkv_workspace_bytes(Bd.OP_IMPORTANCE, 1, 32, 32, 32, 680, 128, dt) == per
    assert P.prefixkv_workspace_bytes(Bd.OP_IMPORTANCE, 1, 32, 32, 32, 680, 128, dt, has_lse=True) == per
    assert P.prefixkv_workspace_bytes(Bd.OP_IMPORTANCE, 4, 32, 32, 8, 8192, 128, dt) == 4 * 32 * 32 * 11 * 8192 * 4
    f32 = (1 * 4 * 2 * 128 * 4 + 255) // 256 * 256
    assert P.prefixkv_workspace_bytes(Bd.OP_IMPORTANCE, 1, 4, 2, 2, 128, 64, P.PKV_F32) == 2 * f32
    assert P.prefixkv_workspace_bytes(Bd.OP_IMPORTANCE, 1, 4, 2, 2, 128, 64, P.PKV_F32, has_lse=True) == f32
    # a status word per (sequence, layer), padded to 256 bytes, then 256 ints of tabulated lengths per layer
    assert P.prefixkv_workspace_bytes(Bd.OP_SELECT, 2, 32, 32, 32, 680, 128, dt) == 256 + 2 * 32 * 1024
    assert P.select_workspace_bytes(2, 32, 680) == 256 + 2 * 32 * 1024
    assert P.select_workspace_bytes(1, 5, 9) == 256 + 5 * 1024
    assert P.prefixkv_workspace_bytes(Bd.OP_DECODE, 1, 32, 32, 32, 680, 128, dt) == 0
    # invalid shapes give 0
    assert P.prefixkv_workspace_bytes(Bd.OP_SELECT, 2, 65, 32, 32, 680, 128, dt) == 0
    assert P.prefixkv_workspace_bytes(Bd.OP_SELECT, 2, 32, 32, 32, 680, 96, dt) == 0
    assert P.prefixkv_workspace_bytes(Bd.OP_SELECT, 2, 32, 32, 5, 680, 128, dt) == 0
    assert P.prefixkv_workspace_bytes(9, 2, 32, 32, 32, 680, 128, dt) == 0
    assert P.prefixkv_cache_tokens_upper_bound(16, 4352, 32, 512) == 16 * (4352 + 32 * 512)


def _shape(**kw):
    d = dict(B=1, L=4, H=2, Hkv=2, N=128, D=64, dtype=P.PKV_F32)
    d.update(kw)
    return Bd._Shape(*[d[k] for k in ("B", "L", "H", "Hkv", "N", "D", "dtype")])


FAKE = C.c_void_p(0x1000)  # never dereferenced: every call below fails validation first


def test_importance_argument_errors():
    lib = P.load()
    st = Bd._Strides(4 * 2 * 128 * 64, 2 * 128 * 64, 128 * 64, 64)
    call = lambda s, q=FAKE, k=FAKE, sc=FAKE, out=FAKE, qs=st, ws=FAKE, wsb=1 << 30: lib.prefixkv_importance(
        C.byref(s), q, qs, k, st, sc, None, out, ws, wsb, None)
    assert call(_shape(), q=None) == 1
    assert call(_shape(), out=None) == 1
    assert call(_shape(L=0)) == 2
    assert call(_shape(L=65)) == 2
    assert call(_shape(N=8193)) == 2
    assert call(_shape(D=96)) == 2
    assert call(_shape(H=3, Hkv=2)) == 2
    assert call(_shape(dtype=7)) == 3
    assert call(_shape(), qs=Bd._Strides(1, 1, 1, 63)) == 4
    assert call(_shape(), q=C.c_void_p(0x1004)) == 4
    assert call(_shape(), ws=None) == 5
    assert call(_shape(), wsb=16) == 5


def test_select_argument_errors():
    lib = P.load()
    def call(B=1, L=4, N=128, imp=FAKE, budget=10, tol=0, iters=64, lengths=FAKE, ws=FAKE, wsb=1 << 20):
        prm = Bd._SelectParams(budget, tol, iters, 1)
        return lib.prefixkv_select(B, L, N, imp, C.byref(prm), FAKE, FAKE, None, lengths, FAKE, FAKE, FAKE,
                                   FAKE, ws, wsb, None)
    assert call(imp=None) == 1
    assert call(lengths=None) == 1
    assert call(L=65) == 2
    assert call(N=0) == 2
    assert call(N=8193) == 2
    assert call(budget=0) == 6
    assert call(tol=-1) == 6
    assert call(iters=0) == 6
    assert call(ws=None) == 5
    assert call(wsb=3) == 5
    assert call(ws=C.c_void_p(0x1004)) == 5       # the table of tabulated lengths is read 16 bytes at a time


def test_select_static_argument_errors():
    lib = P.load()
    def call(B=1, L=4, N=128, imp=FAKE, budget=10, tol=0, iters=64, lengths=FAKE):
        prm = Bd._SelectParams(budget, tol, iters, 1)
        return lib.prefixkv_select_static(B, L, N, imp, C.byref(prm), FAKE, FAKE, None, lengths, FAKE, FAKE, FAKE,
                                          FAKE, None)
    assert lib.prefixkv_static_scratch_segments() == 65536
    assert call(imp=None) == 1
    assert call(lengths=None) == 1
    assert call(L=65) == 2
    assert call(N=8193) == 2
    assert call(budget=0) == 6
    assert call(iters=0) == 6
    assert call(B=65536 // 4 + 1) == 5      # one sequence more than the built-in scratch array holds


def test_rank_and_offline_config_argument_errors():
    lib = P.load()
    rank = lambda B=1, L=4, N=128, imp=FAKE, st=FAKE, ws=FAKE, wsb=1 << 20: lib.prefixkv_rank(
        B, L, N, imp, FAKE, FAKE, None, st, ws, wsb, None)
    assert rank(imp=None) == 1
    assert rank(st=None) == 1
    assert rank(L=0) == 2
    assert rank(N=8193) == 2
    assert rank(ws=None) == 5
    assert rank(wsb=15) == 5
    off = lambda S=3, L=4, N=128, sl=FAKE, budget=100, Bo=2, out=FAKE: lib.prefixkv_offline_config(
        S, L, N, sl, budget, Bo, out, None)
    assert off(sl=None) == 1
    assert off(out=None) == 1
    assert off(S=0) == 2
    assert off(S=65537) == 2
    assert off(L=65) == 2
    assert off(Bo=0) == 2
    assert off(budget=0) == 6


def test_prefill_argument_errors():
    lib = P.load()
    st = Bd._Strides(4 * 2 * 128 * 64, 2 * 128 * 64, 128 * 64, 64)
    bf = _shape(dtype=P.PKV_BF16)
    pf = lambda q=FAKE, lse=FAKE, sh=bf, qs=st: lib.prefixkv_prefill_attn(
        C.byref(sh), q, qs, FAKE, st, FAKE, st, FAKE, FAKE, lse, None)
    assert pf(q=None) == 1
    assert pf(lse=None) == 1
    assert pf(sh=_shape(D=32, dtype=P.PKV_BF16)) == 2
    assert pf(sh=_shape()) == 7               # fp32 storage is not provided
    assert pf(qs=Bd._Strides(0, 0, 0, 6)) == 4
    assert pf(q=C.c_void_p(0x1004)) == 4


def test_gini_and_merge_argument_errors():
    lib = P.load()
    assert lib.prefixkv_gini(1, 4, 128, None, FAKE, None) == 1
    assert lib.prefixkv_gini(1, 4, 128, FAKE, None, None) == 1
    assert lib.prefixkv_gini(1, 65, 128, FAKE, FAKE, None) == 2
    assert lib.prefixkv_gini(1, 4, 0, FAKE, FAKE, None) == 2
    st = Bd._Strides(4 * 2 * 128 * 64, 2 * 128 * 64, 128 * 64, 64)
    mg = lambda k=FAKE, kp=FAKE, sh=_shape(), ks=st: lib.prefixkv_merge_position(
        C.byref(sh), k, ks, FAKE, st, FAKE, FAKE, kp, FAKE, FAKE, FAKE, None)
    assert mg(k=None) == 1
    assert mg(kp=None) == 1
    assert mg(sh=_shape(D=32)) == 2
    assert mg(sh=_shape(dtype=7)) == 3
    assert mg(ks=Bd._Strides(0, 0, 0, 6)) == 4
    assert mg(k=C.c_void_p(0x1004)) == 4


def test_merge_feature_argument_errors():
    lib = P.load()
    st = Bd._Strides(4 * 2 * 128 * 64, 2 * 128 * 64, 128 * 64, 64)
    bf = _shape(dtype=P.PKV_BF16)
    need = lib.prefixkv_workspace_bytes(P.binding.OP_MERGE_FEATURE, C.byref(bf), 0)
    assert need == 2 * bf.B * bf.L * bf.Hkv * ((bf.N + 63) // 64 * 64) * 4
    mf = lambda k=FAKE, mt=FAKE, sh=bf, ks=st, ws=FAKE, nb=need: lib.prefixkv_merge_feature(
        C.byref(sh), k, ks, FAKE, st, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, mt, ws, nb, None)
    assert mf(k=None) == 1
    assert mf(mt=None) == 1
    assert mf(sh=_shape(D=32, dtype=P.PKV_BF16)) == 2
    assert mf(sh=_shape(dtype=7)) == 3
    assert mf(sh=_shape()) == 7                      # fp32 storage is not provided
    assert mf(ks=Bd._Strides(0, 0, 0, 6)) == 4
    assert mf(ks=Bd._Strides(0, 0, 0, 1 << 24)) == 7  # rows beyond 31-bit element offsets
    assert mf(ws=None) == 5
    assert mf(nb=need - 1) == 5


def test_compact_and_decode_argument_errors():
    lib = P.load()
    st = Bd._Strides(4 * 2 * 128 * 64, 2 * 128 * 64, 128 * 64, 64)
    s = _shape()
    comp = lambda k=FAKE, cap=8, sh=s, ks=st: lib.prefixkv_compact(
        C.byref(sh), k, ks, FAKE, st, FAKE, FAKE, cap, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None)
    assert comp(k=None) == 1
    assert comp(cap=-1) == 2
    assert comp(cap=(1 << 20) - 128) == 2     # N + decode_capacity reaches 2^20 slots per segment
    assert comp(cap=(1 << 20) - 129, ks=Bd._Strides(0, 0, 0, 6)) == 4   # one below the bound passes the size check
    assert comp(sh=_shape(D=32)) == 2
    assert comp(ks=Bd._Strides(0, 0, 0, 6)) == 4
    dec = lambda l0=0, l1=4, q=FAKE, kn=FAKE, vn=FAKE, sh=s: lib.prefixkv_decode_attn(
        C.byref(sh), l0, l1, q, kn, vn, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None)
    assert dec(q=None) == 1
    assert dec(kn=None) == 1          # k_new without v_new
    assert dec(l0=2, l1=2) == 2
    assert dec(l1=5) == 2
    assert dec(sh=_shape(H=4096, Hkv=2)) == 2
    assert dec(q=C.c_void_p(0x1008)) == 4
    gqa = _shape(H=32, Hkv=8, dtype=P.PKV_BF16)   # grouped-query bf16: the work list lives in the workspace
    need = P.prefixkv_workspace_bytes(Bd.OP_DECODE, gqa.B, gqa.L, gqa.H, gqa.Hkv, gqa.N, gqa.D, gqa.dtype)
    assert need > 0
    assert dec(sh=gqa) == 5
    assert lib.prefixkv_decode_attn(C.byref(gqa), 0, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                    FAKE, need - 1, None) == 5
    ev = lambda t=1, d=4, kn=FAKE, base=FAKE, kp=None, sh=s: lib.prefixkv_decode_attn_evict(
        C.byref(sh), 0, 4, FAKE, kn, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, base, FAKE, kp, t, d, FAKE, None, 0,
        None)
    assert ev(kn=None) == 1           # the pruning step always stores a token
    assert ev(base=None) == 1
    assert ev(t=0) == 2
    assert ev(d=0) == 2
    assert ev(d=65536) == 2
    assert ev(sh=_shape(D=32)) == 2


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(ValueError):
        P.prefixkv_select(torch.ones(1, 2, 8), 4)
