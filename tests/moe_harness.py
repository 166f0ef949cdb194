"""Shared plumbing for the GPU parity tests: move seeded inputs to the device, call the C-ABI through
the Python binding, bring results back as fp64 numpy, and run the oracle on the same stored inputs."""
from __future__ import annotations

import numpy as np
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from oracle import moe_oracle as O

TOL = {S.DT_BF16: 2e-2, S.DT_F32: 1e-5}   # max |gpu - oracle| / max |oracle| per tensor


def tdtype(w):
    return torch.bfloat16 if w.dtype == S.DT_BF16 else torch.float32


def to_dev(a, dev="cuda"):
    """numpy (fp32 / int32 / uint16 bf16 bits) -> device tensor of the matching torch dtype."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def store(a64, w):
    """fp64 oracle tensor -> the workload's storage format (numpy), for use as an input of a later call."""
    a32 = np.asarray(a64, np.float32)
    return S.f32_to_bf16_bits(a32) if w.dtype == S.DT_BF16 else a32


def to_np(t):
    """device tensor -> fp64 numpy (ints stay ints)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def rel_err(got, want):
    want = np.asarray(want, np.float64)
    got = np.asarray(got, np.float64)
    scale = float(np.max(np.abs(want))) if want.size else 0.0
    if want.size == 0:
        return 0.0
    return float(np.max(np.abs(got - want))) / max(scale, 1e-30)


def cap_of(w):
    return 0 if w.f is None else O.capacity(w.N, w.E, w.k, w.f)


def make_cfg(w, capacity=None, accumulate=0):
    cap = cap_of(w) if capacity is None else capacity
    return moe.MoeConfig.make(w.N, w.M, w.E, w.H, w.k, cap, w.dtype, w.act, w.renormalize, w.add_residual, accumulate)


def f64_inputs(d):
    return {k: (None if v is None else S.to_f64(v)) for k, v in d.items()}


def oracle_layer(w, d, capacity=None):
    """Full oracle forward + backward on the stored inputs (widened exactly to fp64)."""
    f = f64_inputs(d)
    cap = cap_of(w) if capacity is None else capacity
    fwd = O.layer_fwd(f["x"], f["w_gate"], f["b_gate"], f["w1"], f["w3"], f["w2"], w.k, cap, w.act, w.renormalize,
                      w.add_residual)
    bwd = O.layer_bwd(f["dy"], f["x"], f["w_gate"], f["b_gate"], f["w1"], f["w3"], f["w2"], fwd, w.act, w.renormalize,
                      w.add_residual)
    return f, fwd, bwd


class Buffers:
    """Device buffers for every output of the path, sized as the header says (N*k expert rows)."""

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


def dev_inputs(d):
    return {k: to_dev(v) for k, v in d.items()}


def run_layer(w, d, capacity=None, accumulate=0, bufs=None, dd=None):
    """moe_layer_fwd + moe_layer_bwd through the binding; returns (cfg, buffers)."""
    cfg = make_cfg(w, capacity, accumulate)
    b = bufs or Buffers(w, cfg)
    dd = dd or dev_inputs(d)
    moe.moe_layer_fwd(cfg, dd["x"], dd["w_gate"], dd["b_gate"], dd["w1"], dd["w3"], dd["w2"], b.y, b.saved, b.ws)
    moe.moe_layer_bwd(cfg, dd["dy"], dd["x"], dd["w_gate"], dd["w1"], dd["w3"], dd["w2"], b.saved, b.dx, b.dw_gate,
                      b.db_gate if d["b_gate"] is not None else None, b.dw1, b.dw3, b.dw2, b.ws)
    torch.cuda.synchronize()
    return cfg, b


def saved_np(cfg, b, name, dtype):
    return to_np(moe.saved_view(cfg, b.saved, name, dtype))


ROUTING_INT = ["topk_idx", "pos", "count", "offsets", "row_of", "src_of_row"]


def assert_routing_equal(got: dict, want: dict):
    for name in ROUTING_INT:
        g, o = np.asarray(got[name]).reshape(-1), np.asarray(want[name]).reshape(-1)
        assert g.shape == o.shape, name
        bad = np.nonzero(g != o)[0]
        assert bad.size == 0, f"{name}: {bad.size} mismatches, first at {bad[:5]} gpu={g[bad[:5]]} oracle={o[bad[:5]]}"
