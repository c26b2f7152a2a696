"""Pre-allocated driver of the whole hot path for one workload shape: importance -> select ->
compact -> T decode steps.  Only buffer management and call sequencing; every step runs in the
HIP library.  Used by the benchmark, the smoke check and the end-to-end tests."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B_


class HotPath:
    def __init__(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: torch.Tensor,
                 budget_tokens: int, decode_steps: int, tol_tokens: int = 0, max_iters: int = 64,
                 fixup: bool = True, evict_distance: Optional[int] = None):
        self.q, self.k, self.v, self.scale = q, k, v, scale
        self.B, self.L, self.H, self.N, self.D = q.shape
        self.Hkv = k.shape[2]
        self.budget_tokens, self.T = int(budget_tokens), int(decode_steps)
        self.tol_tokens, self.max_iters, self.fixup = tol_tokens, max_iters, fixup
        # append-only decode needs one slot per step; pruning at a fixed distance needs the ring plus
        # room for the survivors (never more than one per step)
        self.evict_distance = evict_distance
        self.decode_capacity = self.T if evict_distance is None else evict_distance + 1 + self.T
        dev, dt = q.device, q.dtype
        Bn, L, H, N, D, Hkv = self.B, self.L, self.H, self.N, self.D, self.Hkv
        code = B_.PKV_F32 if dt == torch.float32 else B_.PKV_BF16
        self.importance = torch.empty((Bn, L, N), dtype=torch.float32, device=dev)
        self.imp_ws = torch.empty(B_.prefixkv_workspace_bytes(B_.OP_IMPORTANCE, Bn, L, H, Hkv, N, D, code),
                                  dtype=torch.uint8, device=dev)
        self.sel = B_.SelectResult(
            order=torch.empty((Bn, L, N), dtype=torch.int32, device=dev),
            cum=torch.empty((Bn, L, N), dtype=torch.int64, device=dev),
            prefix=torch.empty((Bn, L, N), dtype=torch.float32, device=dev),
            lengths=torch.empty((Bn, L), dtype=torch.int32, device=dev),
            p=torch.empty(Bn, dtype=torch.float64, device=dev),
            iters=torch.empty(Bn, dtype=torch.int32, device=dev),
            raw_total=torch.empty(Bn, dtype=torch.int64, device=dev),
            status=torch.empty(Bn, dtype=torch.int32, device=dev))
        self.sel_ws = torch.empty(max(256, B_.select_workspace_bytes(Bn, L, N)), dtype=torch.uint8, device=dev)
        budget_cap = min(self.budget_tokens, L * N)
        self.cache_tokens = B_.prefixkv_cache_tokens_upper_bound(Bn, budget_cap, L, self.decode_capacity)
        self.cache = B_.CompactResult(
            kc=torch.empty(self.cache_tokens * Hkv * D, dtype=dt, device=dev),
            vc=torch.empty(self.cache_tokens * Hkv * D, dtype=dt, device=dev),
            kept_pos=torch.empty(self.cache_tokens, dtype=torch.int32, device=dev),
            seg_off=torch.empty((Bn, L), dtype=torch.int64, device=dev),
            caps=torch.empty((Bn, L), dtype=torch.int32, device=dev),
            lens=torch.empty((Bn, L), dtype=torch.int32, device=dev),
            cache_tokens=self.cache_tokens, Hkv=Hkv, D=D)
        self.out = torch.empty((max(self.T, 1), Bn, L, H, D), dtype=dt, device=dev)
        self.dec_ws = torch.empty(max(256, B_.prefixkv_workspace_bytes(B_.OP_DECODE, Bn, L, H, Hkv, N, D, code)),
                                  dtype=torch.uint8, device=dev)
        self._graph: Optional[torch.cuda.CUDAGraph] = None

    # ---- the four C-ABI calls, on pre-allocated buffers ------------------------------------------
    def run_importance(self, lse: Optional[torch.Tensor] = None):
        return B_.prefixkv_importance(self.q, self.k, self.scale, lse=lse, out=self.importance, ws=self.imp_ws)

    def run_select(self):
        return B_.prefixkv_select(self.importance, self.budget_tokens, self.tol_tokens, self.max_iters,
                                  self.fixup, out=self.sel, ws=self.sel_ws)

    def run_compact(self):
        return B_.prefixkv_compact(self.k, self.v, self.sel.order, self.sel.lengths, self.decode_capacity,
                                   self.cache_tokens, out=self.cache)

    def run_decode_step(self, t: int, dq, dk, dv):
        if self.evict_distance is not None:
            return B_.prefixkv_decode_attn_evict(self.cache, self.sel.lengths, dq[t], dk[t], dv[t], self.scale,
                                                 self.N, t + 1, self.evict_distance, out=self.out[t], ws=self.dec_ws)
        return B_.prefixkv_decode_attn(self.cache, dq[t], dk[t], dv[t], self.scale, self.N, out=self.out[t],
                                       ws=self.dec_ws)

    def run_decode_loop(self, dq, dk, dv):
        for t in range(self.T):
            self.run_decode_step(t, dq, dk, dv)

    # ---- the decode loop as one HIP graph (T launches, no host work between them) -----------
    def capture_decode_loop(self, dq, dk, dv):
        self.run_compact()            # a valid cache state for the capture-time launches
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run_decode_loop(dq, dk, dv)
        self._graph = g
        return g

    def replay_decode_loop(self):
        self._graph.replay()
