"""ctypes front end of the PrefixKV CPU oracle (``prefixkv_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module, and this
module never imports the product package.

All functions take and return NumPy arrays on the host.  Floating inputs are fp32 arrays whose
values are already representable in the workload's storage dtype.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "prefixkv_oracle.c"
_LIB = _HERE / "libprefixkv_oracle.so"

NONFINITE, NEGATIVE, ZERO_LAYER, RANGE = 1, 2, 4, 8


_LIB_SAN = _HERE / "libprefixkv_oracle_san.so"
# PKV_ORACLE_SANITIZE=1 makes lib() load the build with AddressSanitizer and UndefinedBehaviorSanitizer
# (the process must then run with the gcc sanitizer runtime preloaded; tests/test_oracle_sanitized.py does).
_SANITIZE = os.environ.get("PKV_ORACLE_SANITIZE", "0") == "1"


def build(force: bool = False, sanitize: bool = False) -> Path:
    """Compile the oracle with gcc (fp64 arithmetic must stay in source order: no -ffast-math).
    sanitize=True builds the checked variant (-fsanitize=address,undefined -O1) beside it."""
    out = _LIB_SAN if sanitize else _LIB
    if force or not out.exists() or out.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = out.with_suffix(".so.tmp%d" % os.getpid())
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
        subprocess.check_call(["gcc", *opt, "-std=c99", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, out)
    return out


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime, to be preloaded by a process that loads the checked build."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(str(build(sanitize=_SANITIZE)))
        _lib.pkvo_threads.restype = C.c_int
        _lib.pkvo_decode_attn.restype = C.c_int
        _lib.pkvo_sort_prefix_layer.restype = C.c_int
        _lib.pkvo_decode_attn_evict.restype = C.c_int
    return _lib


def threads() -> int:
    return int(lib().pkvo_threads())


def _p(a, ty=C.c_void_p):
    return None if a is None else a.ctypes.data_as(ty)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def importance(q, k, scale, want_lse: bool = False, m_lo: int = 0):
    """q [B,L,H,N,D], k [B,L,Hkv,N,D], scale [L] -> importance [B,L,N] f32 (and lse [B,L,H,N] f64).
    m_lo > 0: only query rows m >= m_lo are processed; columns n >= m_lo are complete, the rest NaN."""
    q, k, scale = _f32(q), _f32(k), _f32(scale)
    B, L, H, N, D = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, L, Hkv, N, D) and H % Hkv == 0 and scale.shape == (L,)
    imp = np.empty((B, L, N), dtype=np.float32)
    lse = np.empty((B, L, H, N), dtype=np.float64) if want_lse else None
    lib().pkvo_importance(B, L, H, Hkv, N, D, _p(q), _p(k), _p(scale), _p(imp), _p(lse), int(m_lo))
    return (imp, lse) if want_lse else imp


def prefill_attn(q, k, v, scale, out_bf16: bool = False):
    """Causal attention of the whole prompt: q [B,L,H,N,D], k/v [B,L,Hkv,N,D], scale [L]
    -> (out [B,L,H,N,D] f32, lse [B,L,H,N] f64)."""
    q, k, v, scale = _f32(q), _f32(k), _f32(v), _f32(scale)
    B, L, H, N, D = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, L, Hkv, N, D) and v.shape == k.shape and H % Hkv == 0 and scale.shape == (L,)
    out = np.empty((B, L, H, N, D), dtype=np.float32)
    lse = np.empty((B, L, H, N), dtype=np.float64)
    lib().pkvo_prefill_attn(B, L, H, Hkv, N, D, _p(q), _p(k), _p(v), _p(scale), _p(out), _p(lse), int(out_bf16))
    return out, lse


def sort_prefix_layer(imp):
    """One layer: importance [N] -> (status, order [N] i32, cum [N] u64, prefix [N] f32)."""
    imp = _f32(imp)
    N = imp.shape[0]
    order = np.zeros(N, dtype=np.int32)
    cum = np.zeros(N, dtype=np.uint64)
    prefix = np.zeros(N, dtype=np.float32)
    st = lib().pkvo_sort_prefix_layer(N, _p(imp), _p(order), _p(cum), _p(prefix))
    return int(st), order, cum, prefix


def search(cum, budget_tokens: int, tol_tokens: int = 0, max_iters: int = 64, fixup: bool = True):
    """One sequence: cum [L,N] u64 -> (lengths [L] i32, p, iters, raw_total)."""
    cum = np.ascontiguousarray(cum, dtype=np.uint64)
    L, N = cum.shape
    assert max_iters >= 1
    lengths = np.zeros(L, dtype=np.int32)
    p = C.c_double(0.0)
    it = C.c_int32(0)
    raw = C.c_int64(0)
    lib().pkvo_search(L, N, _p(cum), C.c_int64(budget_tokens), C.c_int64(tol_tokens), max_iters,
                      int(bool(fixup)), _p(lengths), C.byref(p), C.byref(it), C.byref(raw))
    return lengths, p.value, it.value, raw.value


def select(imp, budget_tokens: int, tol_tokens: int = 0, max_iters: int = 64, fixup: bool = True):
    """importance [B,L,N] -> dict(order, cum, prefix, lengths, p, iters, raw_total, status)."""
    imp = _f32(imp)
    B, L, N = imp.shape
    assert max_iters >= 1
    out = dict(order=np.zeros((B, L, N), np.int32), cum=np.zeros((B, L, N), np.uint64),
               prefix=np.zeros((B, L, N), np.float32), lengths=np.zeros((B, L), np.int32),
               p=np.zeros(B, np.float64), iters=np.zeros(B, np.int32),
               raw_total=np.zeros(B, np.int64), status=np.zeros(B, np.int32))
    lib().pkvo_select(B, L, N, _p(imp), C.c_int64(budget_tokens), C.c_int64(tol_tokens), max_iters,
                      int(bool(fixup)), _p(out["order"]), _p(out["cum"]), _p(out["prefix"]),
                      _p(out["lengths"]), _p(out["p"]), _p(out["iters"]), _p(out["raw_total"]),
                      _p(out["status"]))
    return out


def rank(imp):
    """Stage 2 only: importance [B,L,N] -> dict(order, cum, prefix, status[B]) (no search)."""
    imp = _f32(imp)
    B, L, N = imp.shape
    out = dict(order=np.zeros((B, L, N), np.int32), cum=np.zeros((B, L, N), np.uint64),
               prefix=np.zeros((B, L, N), np.float32), status=np.zeros(B, np.int32))
    for b in range(B):
        for l in range(L):
            st, o, c, pf = sort_prefix_layer(imp[b, l])
            out["status"][b] |= st
            out["order"][b, l], out["cum"][b, l], out["prefix"][b, l] = o, c, pf
    return out


def offline_config(sample_lengths, N: int, budget_tokens: int):
    """sample_lengths [S,L] i32 from S calibration sequences -> shared lengths [L] i32."""
    sl = np.ascontiguousarray(sample_lengths, dtype=np.int32)
    S, L = sl.shape
    out = np.zeros(L, dtype=np.int32)
    lib().pkvo_offline_config(S, L, int(N), _p(sl), C.c_int64(budget_tokens), _p(out))
    return out


def compact(k, v, order, lengths, decode_capacity: int):
    """k,v [B,L,Hkv,N,D]; order [B,L,N]; lengths [B,L] -> ragged cache dict.
    kc/vc are flat f32 arrays of sum(caps)*Hkv*D elements (segment (b,l) = [Hkv][cap][D] at token
    offset seg_off[b,l]); slots that hold nothing are NaN."""
    k, v = _f32(k), _f32(v)
    B, L, Hkv, N, D = k.shape
    order = np.ascontiguousarray(order, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    total = int(lengths.sum()) + B * L * decode_capacity
    out = dict(seg_off=np.zeros((B, L), np.int64), caps=np.zeros((B, L), np.int32),
               kc=np.full(total * Hkv * D, np.nan, np.float32),
               vc=np.full(total * Hkv * D, np.nan, np.float32),
               kept_pos=np.full(total, -1, np.int32), lens=np.zeros((B, L), np.int32),
               Hkv=Hkv, D=D)
    lib().pkvo_compact(B, L, Hkv, N, D, _p(k), _p(v), _p(order), _p(lengths), decode_capacity,
                       _p(out["seg_off"]), _p(out["caps"]), _p(out["kc"]), _p(out["vc"]),
                       _p(out["kept_pos"]), _p(out["lens"]))
    return out


def decode_attn(cache, q, k_new, v_new, scale, l0=None, l1=None, out_bf16: bool = False):
    """One decode step over layers [l0,l1) on a cache dict from compact(); mutates the cache
    (append) and returns out [B,L,H,D] f32 (layers outside the range are NaN)."""
    q, scale = _f32(q), _f32(scale)
    B, L, H, D = q.shape
    Hkv = cache["Hkv"]
    l0 = 0 if l0 is None else l0
    l1 = L if l1 is None else l1
    if k_new is not None:
        k_new, v_new = _f32(k_new), _f32(v_new)
        assert k_new.shape == (B, L, Hkv, D) and v_new.shape == (B, L, Hkv, D)
    out = np.full((B, L, H, D), np.nan, np.float32)
    rc = lib().pkvo_decode_attn(B, L, H, Hkv, D, l0, l1, _p(q), _p(k_new), _p(v_new), _p(scale),
                                _p(cache["kc"]), _p(cache["vc"]), _p(cache["seg_off"]),
                                _p(cache["caps"]), _p(cache["lens"]), _p(out), int(out_bf16))
    if rc != 0:
        raise ValueError("append exceeds segment capacity")
    return out


def decode_attn_evict(cache, base_lens, q, k_new, v_new, scale, N: int, t: int, d: int, l0=None, l1=None,
                      out_bf16: bool = False):
    """Decode step t (1-based) with pruning at distance d on a cache dict from compact(); the cache
    must have been built with decode_capacity >= d+1 (+ room for survivors).  base_lens [B,L] are the
    prefill lengths.  Mutates kc/vc/kept_pos/lens (lens = permanent entries); returns out [B,L,H,D]."""
    q, scale, k_new, v_new = _f32(q), _f32(scale), _f32(k_new), _f32(v_new)
    B, L, H, D = q.shape
    Hkv = cache["Hkv"]
    l0 = 0 if l0 is None else l0
    l1 = L if l1 is None else l1
    base_lens = np.ascontiguousarray(base_lens, dtype=np.int32)
    assert base_lens.shape == (B, L) and k_new.shape == (B, L, Hkv, D) and v_new.shape == (B, L, Hkv, D)
    out = np.full((B, L, H, D), np.nan, np.float32)
    rc = lib().pkvo_decode_attn_evict(B, L, H, Hkv, int(N), D, l0, l1, _p(q), _p(k_new), _p(v_new), _p(scale),
                                      _p(cache["kc"]), _p(cache["vc"]), _p(cache["kept_pos"]),
                                      _p(cache["seg_off"]), _p(cache["caps"]), _p(base_lens),
                                      _p(cache["lens"]), int(t), int(d), _p(out), int(out_bf16))
    if rc != 0:
        raise ValueError("distance < 1, or the segment capacity cannot hold the ring and the survivors")
    return out


def gini(cum):
    """cum [B,L,N] u64 (from select/rank) -> Gini coefficient of every layer's priority sequence [B,L] f64."""
    cum = np.ascontiguousarray(cum, dtype=np.uint64)
    B, L, N = cum.shape
    out = np.zeros((B, L), dtype=np.float64)
    lib().pkvo_gini(C.c_long(B * L), N, _p(cum), _p(out))
    return out


def merge_position(cache, k, v, storage_bf16: bool = False):
    """Average every pruned position into the nearest kept one, in place on a cache dict from compact()
    (before any decode step).  k, v [B,L,Hkv,N,D] are the uncompressed tensors."""
    k, v = _f32(k), _f32(v)
    B, L, Hkv, N, D = k.shape
    assert v.shape == k.shape and cache["Hkv"] == Hkv and cache["D"] == D
    lib().pkvo_merge_position(B, L, Hkv, N, D, _p(k), _p(v), _p(cache["seg_off"]), _p(cache["caps"]),
                              _p(cache["kept_pos"]), _p(cache["lens"]), _p(cache["kc"]), _p(cache["vc"]),
                              int(storage_bf16))
    return cache


def feature_match(cache, x):
    """Feature-similarity matching of one tensor x [B,L,Hkv,N,D] (keys or values) against the retained set of a
    cache dict from compact(): match [B,L,Hkv,N] i32 (slot for a pruned position, -1 for a retained one) and the
    cosine of that best pair [B,L,Hkv,N] f64."""
    x = _f32(x)
    B, L, Hkv, N, D = x.shape
    assert cache["Hkv"] == Hkv and cache["D"] == D
    match = np.zeros((B, L, Hkv, N), np.int32)
    best = np.zeros((B, L, Hkv, N), np.float64)
    lib().pkvo_feature_match(B, L, Hkv, N, D, _p(x), _p(cache["seg_off"]), _p(cache["kept_pos"]),
                             _p(cache["lens"]), _p(match), _p(best))
    return match, best


def match_cosine(cache, x, match):
    """Cosine of every pruned position of x with the retained vector that `match` assigns it to (1 where -1)."""
    x = _f32(x)
    B, L, Hkv, N, D = x.shape
    match = np.ascontiguousarray(match, dtype=np.int32)
    assert match.shape == (B, L, Hkv, N)
    out = np.zeros((B, L, Hkv, N), np.float64)
    lib().pkvo_match_cosine(B, L, Hkv, N, D, _p(x), _p(cache["seg_off"]), _p(cache["kept_pos"]), _p(match), _p(out))
    return out


def merge_by_match(cache, name: str, x, match, storage_bf16: bool = False):
    """Replace every retained vector of cache[name] ('kc' or 'vc') by the average of itself and the pruned
    vectors of x that `match` assigns to its slot; in place."""
    x = _f32(x)
    B, L, Hkv, N, D = x.shape
    match = np.ascontiguousarray(match, dtype=np.int32)
    assert match.shape == (B, L, Hkv, N) and name in ("kc", "vc")
    lib().pkvo_merge_by_match(B, L, Hkv, N, D, _p(x), _p(cache["seg_off"]), _p(cache["caps"]),
                              _p(cache["kept_pos"]), _p(cache["lens"]), _p(match), _p(cache[name]),
                              int(storage_bf16))
    return cache


def merge_feature(cache, k, v, storage_bf16: bool = False):
    """Feature-similarity merging of keys (by key cosine) and values (by value cosine), in place on a cache dict
    from compact(); returns the two assignments."""
    mk, _ = feature_match(cache, k)
    mv, _ = feature_match(cache, v)
    merge_by_match(cache, "kc", k, mk, storage_bf16)
    merge_by_match(cache, "vc", v, mv, storage_bf16)
    return mk, mv


def segment(cache, name: str, b: int, l: int):
    """View of segment (b,l) of 'kc'/'vc' as [Hkv, cap, D], or of 'kept_pos' as [cap]."""
    off = int(cache["seg_off"][b, l])
    cap = int(cache["caps"][b, l])
    if name == "kept_pos":
        return cache["kept_pos"][off:off + cap]
    Hkv, D = cache["Hkv"], cache["D"]
    return cache[name][off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)
