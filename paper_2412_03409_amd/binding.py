"""ctypes binding of include/prefixkv.h.  Argument marshalling only.

The wrappers have the names of the C entry points.  Tensors must live on the GPU; outputs and the
workspace are allocated here with torch (the library itself never allocates) unless passed in.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import torch

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libprefixkv.so"

PKV_F32, PKV_BF16 = 0, 1
OP_IMPORTANCE, OP_SELECT, OP_COMPACT, OP_DECODE, OP_MERGE_FEATURE = 0, 1, 2, 3, 4


class PrefixKVError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: status {code} ({prefixkv_status_string(code)})")
        self.code = code


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "L", "H", "Hkv", "N", "D", "dtype")]


class _Strides(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("b", "l", "h", "n")]


class _SelectParams(C.Structure):
    _fields_ = [("budget_tokens", C.c_int64), ("tol_tokens", C.c_int64), ("max_iters", C.c_int32),
                ("fixup", C.c_int32)]


_lib = None


def lib_path() -> Path:
    return _LIB_PATH


def load(path: Optional[str] = None) -> C.CDLL:
    """Load libprefixkv.so (or another build of it at `path`); raises if it has not been built
    (no fallback exists)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("PKV_LIB_PATH")   # an alternative build of the same library
    lib_file = Path(path) if path else _LIB_PATH
    if not lib_file.exists():
        raise ImportError(f"{lib_file} is missing: build it with `python -m paper_2412_03409_amd.build` "
                          "(hipcc, gfx950); there is no CPU path")
    L = C.CDLL(str(lib_file))
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    L.prefixkv_version.restype = C.c_int
    L.prefixkv_status_string.restype = C.c_char_p
    L.prefixkv_status_string.argtypes = [C.c_int]
    L.prefixkv_workspace_bytes.restype = sz
    L.prefixkv_workspace_bytes.argtypes = [i32, C.POINTER(_Shape), i32]
    L.prefixkv_importance.restype = C.c_int
    L.prefixkv_importance.argtypes = [C.POINTER(_Shape), vp, _Strides, vp, _Strides, vp, vp, vp, vp, sz, vp]
    L.prefixkv_prefill_attn.restype = C.c_int
    L.prefixkv_prefill_attn.argtypes = [C.POINTER(_Shape), vp, _Strides, vp, _Strides, vp, _Strides, vp, vp, vp, vp]
    L.prefixkv_select.restype = C.c_int
    L.prefixkv_select.argtypes = [i32, i32, i32, vp, C.POINTER(_SelectParams), vp, vp, vp, vp, vp, vp, vp,
                                  vp, vp, sz, vp]
    L.prefixkv_select_static.restype = C.c_int
    L.prefixkv_select_static.argtypes = [i32, i32, i32, vp, C.POINTER(_SelectParams), vp, vp, vp, vp, vp, vp, vp,
                                         vp, vp]
    L.prefixkv_static_scratch_segments.restype = C.c_int
    L.prefixkv_rank.restype = C.c_int
    L.prefixkv_rank.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    L.prefixkv_offline_config.restype = C.c_int
    L.prefixkv_offline_config.argtypes = [i32, i32, i32, vp, i64, i32, vp, vp]
    L.prefixkv_gini.restype = C.c_int
    L.prefixkv_gini.argtypes = [i32, i32, i32, vp, vp, vp]
    L.prefixkv_merge_position.restype = C.c_int
    L.prefixkv_merge_position.argtypes = [C.POINTER(_Shape), vp, _Strides, vp, _Strides, vp, vp, vp, vp, vp, vp, vp]
    L.prefixkv_merge_feature.restype = C.c_int
    L.prefixkv_merge_feature.argtypes = [C.POINTER(_Shape), vp, _Strides, vp, _Strides, vp, vp, vp, vp, vp, vp, vp,
                                         vp, sz, vp]
    L.prefixkv_compact.restype = C.c_int
    L.prefixkv_compact.argtypes = [C.POINTER(_Shape), vp, _Strides, vp, _Strides, vp, vp, i32, vp, vp, vp,
                                   vp, vp, vp, vp, sz, vp]
    L.prefixkv_cache_tokens_upper_bound.restype = i64
    L.prefixkv_cache_tokens_upper_bound.argtypes = [i32, i64, i32, i32]
    L.prefixkv_decode_attn.restype = C.c_int
    L.prefixkv_decode_attn.argtypes = [C.POINTER(_Shape), i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                       vp, sz, vp]
    L.prefixkv_decode_attn_evict.restype = C.c_int
    L.prefixkv_decode_attn_evict.argtypes = [C.POINTER(_Shape), i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                             vp, vp, i32, i32, vp, vp, sz, vp]
    L.prefixkv_calibration_copy.restype = C.c_int
    L.prefixkv_calibration_copy.argtypes = [vp, vp, sz, vp]
    _lib = L
    return L


def prefixkv_version() -> int:
    return int(load().prefixkv_version())


def prefixkv_status_string(code: int) -> str:
    return load().prefixkv_status_string(int(code)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PKV_F32
    if t.dtype == torch.bfloat16:
        return PKV_BF16
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def _shape(B, L, H, Hkv, N, D, dtype) -> _Shape:
    return _Shape(B, L, H, Hkv, N, D, dtype)


def _strides5(t: torch.Tensor) -> _Strides:
    if t.stride(4) != 1:
        raise ValueError("the head dimension must be contiguous")
    return _Strides(t.stride(0), t.stride(1), t.stride(2), t.stride(3))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must be on the GPU")


def _ws(nbytes: int, device, ws: Optional[torch.Tensor]) -> torch.Tensor:
    if ws is not None:
        if ws.numel() * ws.element_size() < nbytes:
            raise ValueError("workspace too small")
        return ws
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def prefixkv_workspace_bytes(op: int, B, L, H, Hkv, N, D, dtype, has_lse: bool = False) -> int:
    s = _shape(B, L, H, Hkv, N, D, dtype)
    return int(load().prefixkv_workspace_bytes(op, C.byref(s), int(has_lse)))


def select_workspace_bytes(B: int, L: int, N: int) -> int:
    # stages 2 and 3 do not depend on the head geometry: any valid one serves for the size query
    s = _shape(B, L, 1, 1, N, 128, PKV_BF16)
    return int(load().prefixkv_workspace_bytes(OP_SELECT, C.byref(s), 0))


def prefixkv_cache_tokens_upper_bound(B: int, budget_tokens: int, L: int, decode_capacity: int) -> int:
    return int(load().prefixkv_cache_tokens_upper_bound(B, budget_tokens, L, decode_capacity))


def prefixkv_importance(q: torch.Tensor, k: torch.Tensor, scale: torch.Tensor,
                        lse: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                        ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q [B,L,H,N,D], k [B,L,Hkv,N,D] (bf16 or f32), scale [L] f32, optional lse [B,L,H,N] f32
    -> importance [B,L,N] f32."""
    _need_cuda(q, k, scale, lse, out, ws)
    B, L, H, N, D = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, L, Hkv, N, D) or k.dtype != q.dtype:
        raise ValueError("k must be [B,L,Hkv,N,D] with q's dtype")
    if scale.dtype != torch.float32 or scale.shape != (L,) or not scale.is_contiguous():
        raise ValueError("scale must be contiguous f32 [L]")
    if lse is not None and (lse.dtype != torch.float32 or lse.shape != (B, L, H, N) or not lse.is_contiguous()):
        raise ValueError("lse must be contiguous f32 [B,L,H,N]")
    s = _shape(B, L, H, Hkv, N, D, _dtype_code(q))
    if out is None:
        out = torch.empty((B, L, N), dtype=torch.float32, device=q.device)
    nbytes = load().prefixkv_workspace_bytes(OP_IMPORTANCE, C.byref(s), int(lse is not None))
    w = _ws(nbytes, q.device, ws)
    rc = load().prefixkv_importance(C.byref(s), _ptr(q), _strides5(q), _ptr(k), _strides5(k), _ptr(scale),
                                    _ptr(lse), _ptr(out), _ptr(w), w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_importance")
    return out


def prefixkv_prefill_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: torch.Tensor,
                          out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None):
    """Causal attention over the prompt: q [B,L,H,N,D], k/v [B,L,Hkv,N,D] (bf16), scale [L] f32
    -> (out [B,L,H,N,D] bf16, lse [B,L,H,N] f32, ready to be passed to prefixkv_importance)."""
    _need_cuda(q, k, v, scale, out, lse)
    B, L, H, N, D = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, L, Hkv, N, D) or v.shape != k.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("k, v must be [B,L,Hkv,N,D] with q's dtype")
    if scale.dtype != torch.float32 or scale.shape != (L,) or not scale.is_contiguous():
        raise ValueError("scale must be contiguous f32 [L]")
    if out is None:
        out = torch.empty((B, L, H, N, D), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, L, H, N), dtype=torch.float32, device=q.device)
    s = _shape(B, L, H, Hkv, N, D, _dtype_code(q))
    rc = load().prefixkv_prefill_attn(C.byref(s), _ptr(q), _strides5(q), _ptr(k), _strides5(k), _ptr(v),
                                      _strides5(v), _ptr(scale), _ptr(out), _ptr(lse), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_prefill_attn")
    return out, lse


@dataclass
class SelectResult:
    order: torch.Tensor      # [B,L,N] i32
    cum: torch.Tensor        # [B,L,N] i64 holding the u64 bit pattern
    prefix: Optional[torch.Tensor]  # [B,L,N] f32
    lengths: torch.Tensor    # [B,L] i32
    p: torch.Tensor          # [B] f64
    iters: torch.Tensor      # [B] i32
    raw_total: torch.Tensor  # [B] i64
    status: torch.Tensor     # [B] i32


def prefixkv_select(importance: torch.Tensor, budget_tokens: int, tol_tokens: int = 0,
                    max_iters: int = 64, fixup: bool = True, want_prefix: bool = True,
                    out: Optional[SelectResult] = None, ws: Optional[torch.Tensor] = None) -> SelectResult:
    """importance [B,L,N] f32 -> SelectResult (all on the device; nothing is read back)."""
    _need_cuda(importance, ws)
    if importance.dtype != torch.float32 or importance.dim() != 3 or not importance.is_contiguous():
        raise ValueError("importance must be contiguous f32 [B,L,N]")
    B, L, N = importance.shape
    dev = importance.device
    if out is None:
        out = SelectResult(
            order=torch.empty((B, L, N), dtype=torch.int32, device=dev),
            cum=torch.empty((B, L, N), dtype=torch.int64, device=dev),
            prefix=torch.empty((B, L, N), dtype=torch.float32, device=dev) if want_prefix else None,
            lengths=torch.empty((B, L), dtype=torch.int32, device=dev),
            p=torch.empty(B, dtype=torch.float64, device=dev),
            iters=torch.empty(B, dtype=torch.int32, device=dev),
            raw_total=torch.empty(B, dtype=torch.int64, device=dev),
            status=torch.empty(B, dtype=torch.int32, device=dev))
    prm = _SelectParams(int(budget_tokens), int(tol_tokens), int(max_iters), int(bool(fixup)))
    w = _ws(select_workspace_bytes(B, L, N), dev, ws)
    rc = load().prefixkv_select(B, L, N, _ptr(importance), C.byref(prm), _ptr(out.order), _ptr(out.cum),
                                _ptr(out.prefix), _ptr(out.lengths), _ptr(out.p), _ptr(out.iters),
                                _ptr(out.raw_total), _ptr(out.status), _ptr(w),
                                w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_select")
    return out


def prefixkv_select_static(importance: torch.Tensor, budget_tokens: int, out: SelectResult, tol_tokens: int = 0,
                           max_iters: int = 64, fixup: bool = True) -> SelectResult:
    """prefixkv_select without a workspace and without any allocation: `out` must be pre-allocated
    (all eight tensors; prefix may be None).  B*L <= prefixkv_static_scratch_segments()."""
    _need_cuda(importance, out.order, out.cum, out.prefix, out.lengths, out.p, out.iters, out.raw_total, out.status)
    if importance.dtype != torch.float32 or importance.dim() != 3 or not importance.is_contiguous():
        raise ValueError("importance must be contiguous f32 [B,L,N]")
    B, L, N = importance.shape
    prm = _SelectParams(int(budget_tokens), int(tol_tokens), int(max_iters), int(bool(fixup)))
    rc = load().prefixkv_select_static(B, L, N, _ptr(importance), C.byref(prm), _ptr(out.order), _ptr(out.cum),
                                       _ptr(out.prefix), _ptr(out.lengths), _ptr(out.p), _ptr(out.iters),
                                       _ptr(out.raw_total), _ptr(out.status), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_select_static")
    return out


def prefixkv_static_scratch_segments() -> int:
    return int(load().prefixkv_static_scratch_segments())


@dataclass
class RankResult:
    order: torch.Tensor      # [B,L,N] i32
    cum: torch.Tensor        # [B,L,N] i64 holding the u64 bit pattern
    prefix: Optional[torch.Tensor]  # [B,L,N] f32
    status: torch.Tensor     # [B] i32


def prefixkv_rank(importance: torch.Tensor, want_prefix: bool = True, out: Optional[RankResult] = None,
                  ws: Optional[torch.Tensor] = None) -> RankResult:
    """importance [B,L,N] f32 -> per-layer ranking and cumulative priority, without the search."""
    _need_cuda(importance, ws)
    if importance.dtype != torch.float32 or importance.dim() != 3 or not importance.is_contiguous():
        raise ValueError("importance must be contiguous f32 [B,L,N]")
    B, L, N = importance.shape
    dev = importance.device
    if out is None:
        out = RankResult(
            order=torch.empty((B, L, N), dtype=torch.int32, device=dev),
            cum=torch.empty((B, L, N), dtype=torch.int64, device=dev),
            prefix=torch.empty((B, L, N), dtype=torch.float32, device=dev) if want_prefix else None,
            status=torch.empty(B, dtype=torch.int32, device=dev))
    w = _ws(select_workspace_bytes(B, L, N), dev, ws)
    rc = load().prefixkv_rank(B, L, N, _ptr(importance), _ptr(out.order), _ptr(out.cum), _ptr(out.prefix),
                              _ptr(out.status), _ptr(w), w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_rank")
    return out


def prefixkv_offline_config(sample_lengths: torch.Tensor, N: int, budget_tokens: int, B_out: int = 1,
                            out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """sample_lengths [S,L] i32 (device) -> shared per-layer lengths, repeated: [B_out,L] i32."""
    _need_cuda(sample_lengths, out)
    if sample_lengths.dtype != torch.int32 or sample_lengths.dim() != 2 or not sample_lengths.is_contiguous():
        raise ValueError("sample_lengths must be contiguous i32 [S,L]")
    S, L = sample_lengths.shape
    if out is None:
        out = torch.empty((B_out, L), dtype=torch.int32, device=sample_lengths.device)
    elif out.dtype != torch.int32 or out.shape != (B_out, L) or not out.is_contiguous():
        raise ValueError("out must be contiguous i32 [B_out,L]")
    rc = load().prefixkv_offline_config(S, L, int(N), _ptr(sample_lengths), int(budget_tokens), int(B_out),
                                        _ptr(out), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_offline_config")
    return out


@dataclass
class CompactResult:
    kc: torch.Tensor         # flat [cache_tokens*Hkv*D] storage dtype
    vc: torch.Tensor
    kept_pos: torch.Tensor   # [cache_tokens] i32
    seg_off: torch.Tensor    # [B,L] i64 (tokens)
    caps: torch.Tensor       # [B,L] i32
    lens: torch.Tensor       # [B,L] i32
    cache_tokens: int
    Hkv: int
    D: int


def prefixkv_compact(k: torch.Tensor, v: torch.Tensor, order: torch.Tensor, lengths: torch.Tensor,
                     decode_capacity: int, cache_tokens: int,
                     out: Optional[CompactResult] = None) -> CompactResult:
    """k,v [B,L,Hkv,N,D]; order [B,L,N] i32; lengths [B,L] i32 -> ragged compressed cache.
    cache_tokens: token slots to allocate (prefixkv_cache_tokens_upper_bound)."""
    _need_cuda(k, v, order, lengths)
    B, L, Hkv, N, D = k.shape
    if v.shape != k.shape or v.dtype != k.dtype:
        raise ValueError("v must match k")
    if order.dtype != torch.int32 or order.shape != (B, L, N) or not order.is_contiguous():
        raise ValueError("order must be contiguous i32 [B,L,N]")
    if lengths.dtype != torch.int32 or lengths.shape != (B, L) or not lengths.is_contiguous():
        raise ValueError("lengths must be contiguous i32 [B,L]")
    dev = k.device
    if out is None:
        out = CompactResult(
            kc=torch.empty(cache_tokens * Hkv * D, dtype=k.dtype, device=dev),
            vc=torch.empty(cache_tokens * Hkv * D, dtype=k.dtype, device=dev),
            kept_pos=torch.empty(cache_tokens, dtype=torch.int32, device=dev),
            seg_off=torch.empty((B, L), dtype=torch.int64, device=dev),
            caps=torch.empty((B, L), dtype=torch.int32, device=dev),
            lens=torch.empty((B, L), dtype=torch.int32, device=dev),
            cache_tokens=int(cache_tokens), Hkv=Hkv, D=D)
    s = _shape(B, L, Hkv, Hkv, N, D, _dtype_code(k))
    rc = load().prefixkv_compact(C.byref(s), _ptr(k), _strides5(k), _ptr(v), _strides5(v), _ptr(order),
                                 _ptr(lengths), int(decode_capacity), _ptr(out.seg_off), _ptr(out.caps),
                                 _ptr(out.kc), _ptr(out.vc), _ptr(out.kept_pos), _ptr(out.lens), None, 0,
                                 _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_compact")
    return out


def prefixkv_merge_position(cache: CompactResult, k: torch.Tensor, v: torch.Tensor) -> CompactResult:
    """Average every pruned position into the nearest kept one, in place on a freshly compacted cache."""
    _need_cuda(k, v)
    B, L, Hkv, N, D = k.shape
    if v.shape != k.shape or v.dtype != k.dtype or k.dtype != cache.kc.dtype or D != cache.D or Hkv != cache.Hkv:
        raise ValueError("k, v must be the [B,L,Hkv,N,D] tensors the cache was compacted from")
    s = _shape(B, L, Hkv, Hkv, N, D, _dtype_code(k))
    rc = load().prefixkv_merge_position(C.byref(s), _ptr(k), _strides5(k), _ptr(v), _strides5(v),
                                        _ptr(cache.seg_off), _ptr(cache.caps), _ptr(cache.kept_pos),
                                        _ptr(cache.lens), _ptr(cache.kc), _ptr(cache.vc), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_merge_position")
    return cache


def prefixkv_merge_feature(cache: CompactResult, k: torch.Tensor, v: torch.Tensor,
                           match: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Average every pruned vector into the most similar (cosine) retained vector of its head, keys by key
    similarity and values by value similarity, in place on a freshly compacted bf16 cache.  Returns the
    assignment match [2,B,L,Hkv,N] i32 (plane 0 keys, 1 values; -1 at retained positions)."""
    _need_cuda(k, v, match, ws)
    B, L, Hkv, N, D = k.shape
    if v.shape != k.shape or v.dtype != k.dtype or k.dtype != cache.kc.dtype or D != cache.D or Hkv != cache.Hkv:
        raise ValueError("k, v must be the [B,L,Hkv,N,D] tensors the cache was compacted from")
    if match is None:
        match = torch.empty((2, B, L, Hkv, N), dtype=torch.int32, device=k.device)
    elif match.dtype != torch.int32 or tuple(match.shape) != (2, B, L, Hkv, N) or not match.is_contiguous():
        raise ValueError("match must be contiguous i32 [2,B,L,Hkv,N]")
    s = _shape(B, L, Hkv, Hkv, N, D, _dtype_code(k))
    w = _ws(load().prefixkv_workspace_bytes(OP_MERGE_FEATURE, C.byref(s), 0), k.device, ws)
    rc = load().prefixkv_merge_feature(C.byref(s), _ptr(k), _strides5(k), _ptr(v), _strides5(v),
                                       _ptr(cache.seg_off), _ptr(cache.caps), _ptr(cache.kept_pos),
                                       _ptr(cache.lens), _ptr(cache.kc), _ptr(cache.vc), _ptr(match), _ptr(w),
                                       w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_merge_feature")
    return match


def prefixkv_gini(cum: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """cum [B,L,N] (i64 holding the u64 sums of prefixkv_select / prefixkv_rank) -> Gini coefficients [B,L] f64."""
    _need_cuda(cum, out)
    if cum.dtype != torch.int64 or cum.dim() != 3 or not cum.is_contiguous():
        raise ValueError("cum must be contiguous i64 [B,L,N]")
    B, L, N = cum.shape
    if out is None:
        out = torch.empty((B, L), dtype=torch.float64, device=cum.device)
    rc = load().prefixkv_gini(B, L, N, _ptr(cum), _ptr(out), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_gini")
    return out


def prefixkv_decode_attn(cache: CompactResult, q: torch.Tensor, k_new: Optional[torch.Tensor],
                         v_new: Optional[torch.Tensor], scale: torch.Tensor, N: int,
                         l0: int = 0, l1: Optional[int] = None,
                         out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decode step over layers [l0,l1): q [B,L,H,D], k_new/v_new [B,L,Hkv,D] or None
    -> out [B,L,H,D].  Appends in place and advances cache.lens on the device."""
    _need_cuda(q, k_new, v_new, scale, out)
    B, L, H, D = q.shape
    l1 = L if l1 is None else l1
    if not q.is_contiguous() or q.dtype != cache.kc.dtype or D != cache.D:
        raise ValueError("q must be contiguous [B,L,H,D] in the cache dtype")
    for t in (k_new, v_new):
        if t is not None and (t.shape != (B, L, cache.Hkv, D) or not t.is_contiguous() or t.dtype != q.dtype):
            raise ValueError("k_new/v_new must be contiguous [B,L,Hkv,D] in the cache dtype")
    if scale.dtype != torch.float32 or scale.shape != (L,) or not scale.is_contiguous():
        raise ValueError("scale must be contiguous f32 [L]")
    if out is None:
        out = torch.empty((B, L, H, D), dtype=q.dtype, device=q.device)
    s = _shape(B, L, H, cache.Hkv, N, D, _dtype_code(q))
    w = _ws(load().prefixkv_workspace_bytes(OP_DECODE, C.byref(s), 0), q.device, ws)
    rc = load().prefixkv_decode_attn(C.byref(s), int(l0), int(l1), _ptr(q), _ptr(k_new), _ptr(v_new),
                                     _ptr(scale), _ptr(cache.kc), _ptr(cache.vc), _ptr(cache.seg_off),
                                     _ptr(cache.caps), _ptr(cache.lens), _ptr(out), _ptr(w),
                                     w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_decode_attn")
    return out


def prefixkv_decode_attn_evict(cache: CompactResult, base_lens: torch.Tensor, q: torch.Tensor,
                               k_new: torch.Tensor, v_new: torch.Tensor, scale: torch.Tensor, N: int, t: int,
                               distance: int, l0: int = 0, l1: Optional[int] = None,
                               track_positions: bool = True, out: Optional[torch.Tensor] = None,
                               ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Decode step t (1-based) with pruning at `distance` from the newest token; cache.lens counts the
    permanent entries.  base_lens [B,L] i32 = the lengths the cache was compacted with."""
    _need_cuda(q, k_new, v_new, scale, base_lens, out)
    B, L, H, D = q.shape
    l1 = L if l1 is None else l1
    if not q.is_contiguous() or q.dtype != cache.kc.dtype or D != cache.D:
        raise ValueError("q must be contiguous [B,L,H,D] in the cache dtype")
    for x in (k_new, v_new):
        if x.shape != (B, L, cache.Hkv, D) or not x.is_contiguous() or x.dtype != q.dtype:
            raise ValueError("k_new/v_new must be contiguous [B,L,Hkv,D] in the cache dtype")
    if scale.dtype != torch.float32 or scale.shape != (L,) or not scale.is_contiguous():
        raise ValueError("scale must be contiguous f32 [L]")
    if base_lens.dtype != torch.int32 or base_lens.shape != (B, L) or not base_lens.is_contiguous():
        raise ValueError("base_lens must be contiguous i32 [B,L]")
    if out is None:
        out = torch.empty((B, L, H, D), dtype=q.dtype, device=q.device)
    s = _shape(B, L, H, cache.Hkv, N, D, _dtype_code(q))
    w = _ws(load().prefixkv_workspace_bytes(OP_DECODE, C.byref(s), 0), q.device, ws)
    rc = load().prefixkv_decode_attn_evict(
        C.byref(s), int(l0), int(l1), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(scale), _ptr(cache.kc),
        _ptr(cache.vc), _ptr(cache.seg_off), _ptr(cache.caps), _ptr(base_lens), _ptr(cache.lens),
        _ptr(cache.kept_pos) if track_positions else None, int(t), int(distance), _ptr(out), _ptr(w),
        w.numel() * w.element_size(), _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_decode_attn_evict")
    return out


def prefixkv_calibration_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain copy kernel of src's size into dst (byte-counter calibration aid)."""
    _need_cuda(dst, src)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst too small")
    rc = load().prefixkv_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream())
    if rc != 0:
        raise PrefixKVError(rc, "prefixkv_calibration_copy")
