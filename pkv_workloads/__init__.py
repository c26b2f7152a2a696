"""Seeded synthetic workloads for the PrefixKV hot path.

This module only draws random tensors with the shapes and the coarse structure of the
paper's LLaVA-style runs (per-layer attention concentration that differs from layer to
layer, a few "sink" keys that attract most attention).  It holds none of the method's
arithmetic: no softmax, no sort, no search.  Both the CPU oracle tests and the HIP path
consume its outputs; neither of them is imported here.

Draw order for one workload (all from generators seeded with ``seed_base + index``):
  1. ``s_l ~ U[s_lo, s_hi]`` per layer (host generator), ``scale_l = s_l / sqrt(D)``
  2. sink positions (host generator)
  3. per sequence b: Q, K, V ~ N(0,1) in fp32 (generator on the target device), the sink
     structure is applied, then the tensors are rounded to the storage dtype (RNE)
  4. decode-step tensors q_t, k_t, v_t ~ N(0,1)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch

SEED_BASE = 412034090


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    L: int
    H: int
    Hkv: int
    D: int
    N: int
    B: int
    dtype: str  # "f32" | "bf16"  (storage dtype of Q/K/V and of the decode output)
    s_lo: float
    s_hi: float
    sink: Optional[str]  # "q0mean": k[...,0,:] = 4*mean_m q ; "frac": a fraction of key rows x4
    sink_frac: float
    budget: float  # fraction of the L*N cached positions that may be kept
    decode_steps: int

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def budget_tokens(self, r: Optional[float] = None) -> int:
        """Integer per-sequence budget: round-half-away of r*L*N."""
        r = self.budget if r is None else r
        return int(math.floor(r * self.L * self.N + 0.5))

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    # BASELINE configs[0]
    "tiny": Workload("tiny", 0, L=4, H=2, Hkv=2, D=64, N=128, B=1, dtype="f32",
                     s_lo=0.5, s_hi=3.0, sink="q0mean", sink_frac=0.0, budget=0.5, decode_steps=8),
    # BASELINE configs[1] -- the configuration the headline metric is quoted on
    "llava7b_b1": Workload("llava7b_b1", 1, L=32, H=32, Hkv=32, D=128, N=680, B=1, dtype="bf16",
                           s_lo=0.5, s_hi=3.0, sink="frac", sink_frac=0.01, budget=0.2, decode_steps=256),
    # BASELINE configs[2]
    "llava7b_b16": Workload("llava7b_b16", 2, L=32, H=32, Hkv=32, D=128, N=680, B=16, dtype="bf16",
                            s_lo=0.5, s_hi=3.0, sink="frac", sink_frac=0.01, budget=0.2, decode_steps=512),
    # BASELINE configs[3]
    "llava13b_b8": Workload("llava13b_b8", 3, L=40, H=40, Hkv=40, D=128, N=680, B=8, dtype="bf16",
                            s_lo=0.3, s_hi=4.0, sink=None, sink_frac=0.0, budget=0.2, decode_steps=256),
    # BASELINE configs[4]
    "gqa_long": Workload("gqa_long", 4, L=32, H=32, Hkv=8, D=128, N=8192, B=4, dtype="bf16",
                         s_lo=0.5, s_hi=3.0, sink="frac", sink_frac=0.01, budget=0.1, decode_steps=512),
}


def _host_gen(w: Workload, stream: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + w.index + 1000003 * stream)
    return g


def layer_scales(w: Workload) -> torch.Tensor:
    """scale[L] fp32 (host): s_l / sqrt(D) with s_l ~ U[s_lo, s_hi]."""
    g = _host_gen(w, 1)
    s = torch.rand(w.L, generator=g, dtype=torch.float64) * (w.s_hi - w.s_lo) + w.s_lo
    return (s / math.sqrt(w.D)).to(torch.float32)


def sink_positions(w: Workload) -> torch.Tensor:
    """Sorted int64 positions of the sink keys, shared by all layers, heads and sequences."""
    if w.sink != "frac":
        return torch.zeros(0, dtype=torch.int64)
    cnt = max(1, int(round(w.sink_frac * w.N)))
    g = _host_gen(w, 2)
    rest = torch.randperm(w.N - 1, generator=g)[: cnt - 1] + 1
    return torch.sort(torch.cat([torch.zeros(1, dtype=torch.int64), rest])).values


def make_prefill(w: Workload, device: str = "cpu", want_v: bool = True):
    """Returns dict(q[B,L,H,N,D], k[B,L,Hkv,N,D], v[...], scale[L]) in the storage dtype on
    `device`.  Values are a pure function of (workload, device type)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_BASE + w.index)
    dt = w.torch_dtype
    q = torch.empty((w.B, w.L, w.H, w.N, w.D), dtype=dt, device=dev)
    k = torch.empty((w.B, w.L, w.Hkv, w.N, w.D), dtype=dt, device=dev)
    v = torch.empty((w.B, w.L, w.Hkv, w.N, w.D), dtype=dt, device=dev) if want_v else None
    sinks = sink_positions(w).to(dev)
    grp = w.H // w.Hkv
    # one layer at a time bounds the fp32 staging memory for the long-context shape
    for b in range(w.B):
        for l in range(w.L):
            qf = torch.randn((w.H, w.N, w.D), generator=g, device=dev, dtype=torch.float32)
            kf = torch.randn((w.Hkv, w.N, w.D), generator=g, device=dev, dtype=torch.float32)
            if w.sink == "q0mean":
                # key 0 of each kv head points along the mean query of its head group
                qm = qf.view(w.Hkv, grp, w.N, w.D).mean(dim=(1, 2))
                kf[:, 0, :] = 4.0 * qm
            elif w.sink == "frac":
                kf[:, sinks, :] *= 4.0
            q[b, l].copy_(qf)
            k[b, l].copy_(kf)
            if want_v:
                vf = torch.randn((w.Hkv, w.N, w.D), generator=g, device=dev, dtype=torch.float32)
                v[b, l].copy_(vf)
    out = {"q": q, "k": k, "scale": layer_scales(w).to(dev)}
    if want_v:
        out["v"] = v
    return out


def make_decode(w: Workload, steps: Optional[int] = None, device: str = "cpu"):
    """Decode-step tensors q_t[T,B,L,H,D], k_t, v_t[T,B,L,Hkv,D] in the storage dtype."""
    dev = torch.device(device)
    T = w.decode_steps if steps is None else steps
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_BASE + w.index + 7919)
    dt = w.torch_dtype
    q = torch.empty((T, w.B, w.L, w.H, w.D), dtype=dt, device=dev)
    k = torch.empty((T, w.B, w.L, w.Hkv, w.D), dtype=dt, device=dev)
    v = torch.empty((T, w.B, w.L, w.Hkv, w.D), dtype=dt, device=dev)
    for t in range(T):
        q[t].copy_(torch.randn(q.shape[1:], generator=g, device=dev, dtype=torch.float32))
        k[t].copy_(torch.randn(k.shape[1:], generator=g, device=dev, dtype=torch.float32))
        v[t].copy_(torch.randn(v.shape[1:], generator=g, device=dev, dtype=torch.float32))
    return {"q": q, "k": k, "v": v}


def synthetic_importance(B: int, L: int, N: int, seed: int, ties: bool = False,
                         device: str = "cpu") -> torch.Tensor:
    """A stand-alone importance-like tensor [B,L,N] fp32 >= 0 whose rows sum to about N, with a
    per-layer concentration that differs across layers (heavy-tailed, a few dominant positions).
    With ties=True values are quantised coarsely so that many equal keys occur."""
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + 500 + seed)
    conc = torch.rand((B, L, 1), generator=g, dtype=torch.float64) * 3.5 + 0.5
    z = torch.randn((B, L, N), generator=g, dtype=torch.float64)
    x = torch.exp(conc * z)
    x = x / x.sum(dim=-1, keepdim=True) * N
    if ties:
        x = torch.round(x * 8.0) / 8.0
    return x.to(torch.float32).to(device)
