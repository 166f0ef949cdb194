"""Device buffers for the calls of the library, sized as include/moe_mi355x.h says (N*k expert rows), and the
configuration of a workload.  Plumbing for the tests and the benchmark: allocation only, no arithmetic."""
from __future__ import annotations

import torch

from . import binding as moe

DT_BF16 = moe.DT_BF16


def tdtype(w):
    return torch.bfloat16 if w.dtype == DT_BF16 else torch.float32


def capacity_of(w) -> int:
    """T of a workload through the library's own moe_capacity (0 = nothing dropped, the paper's f = *)."""
    return 0 if w.f is None else moe.moe_capacity(w.N, w.E, w.k, w.f)


def make_cfg(w, capacity=None, accumulate=0):
    cap = capacity_of(w) if capacity is None else capacity
    return moe.MoeConfig.make(w.N, w.M, w.E, w.H, w.k, cap, w.dtype, w.act, w.renormalize, w.add_residual, accumulate)


class Buffers:
    """Device buffers for every output of the path."""

    def __init__(self, w, cfg, dev="cuda"):
        N, M, E, H, k = w.N, w.M, w.E, w.H, w.k
        A = N * k
        dt = tdtype(w)
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        el = dict(dtype=dt, device=dev)
        ws_bytes, saved_bytes = moe.moe_workspace_bytes(cfg)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.saved = torch.empty(saved_bytes, dtype=torch.uint8, device=dev)
        self.logits = torch.empty(N, E, **f32); self.probs = torch.empty(N, E, **f32)
        self.topk_idx = torch.empty(N, k, **i32); self.topk_w = torch.empty(N, k, **f32)
        self.pos = torch.empty(N, k, **i32); self.row_of = torch.empty(N, k, **i32)
        self.count = torch.empty(E, **i32); self.offsets = torch.empty(E + 1, **i32)
        self.src_of_row = torch.empty(A, **i32)
        self.xe = torch.empty(A, M, **el); self.q = torch.empty(A, M, **el)
        self.a1 = torch.empty(A, H, **el); self.hh = torch.empty(A, H, **el)
        self.a3 = torch.empty(A, H, **el) if w.gated else None
        self.y = torch.empty(N, M, **el); self.dx = torch.empty(N, M, **el)
        self.dq = torch.empty(A, M, **el); self.dxe = torch.empty(A, M, **el)
        self.dtopk_w = torch.empty(N, k, **f32)
        self.dw_gate = torch.empty(M, E, **el); self.db_gate = torch.empty(E, **f32)
        self.dw1 = torch.empty(E, M, H, **el); self.dw2 = torch.empty(E, H, M, **el)
        self.dw3 = torch.empty(E, M, H, **el) if w.gated else None
