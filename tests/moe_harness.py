"""Shared plumbing for the GPU parity tests: move seeded inputs to the device, call the C-ABI through
the Python binding, bring results back as fp64 numpy, and run the oracle on the same stored inputs."""
from __future__ import annotations

import numpy as np
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from oracle import moe_oracle as O
from paper_2501_10714_amd.buffers import Buffers, capacity_of, make_cfg, tdtype  # noqa: F401  (no oracle in there)

TOL = {S.DT_BF16: 2e-2, S.DT_F32: 1e-5}   # max |gpu - oracle| / max |oracle| per tensor


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


def violations(got, want, tol):
    """Number of elements with |got - want| > tol * |want| + tol * rms(want): the element-wise companion of
    rel_err, which guards the small entries of a tensor that the max-norm measure does not see."""
    want = np.asarray(want, np.float64)
    got = np.asarray(got, np.float64)
    if want.size == 0:
        return 0
    rms = float(np.sqrt(np.mean(want * want)))
    return int(np.count_nonzero(np.abs(got - want) > tol * np.abs(want) + tol * rms))


# Share of the elements of a tensor that may miss the element-wise bound.  The bound is 2 % of the element plus 2 %
# of the tensor's rms.  A bf16 result carries one rounding (2^-9 of its own size) plus the roundings of the bf16
# intermediates it was formed from (a1, a3, hh, dq, da1, da3); measured, the rms of the error is 0.3 - 0.4 % of the
# tensor's rms.  For sums over thousands of rows the error is Gaussian and 2 % is never reached; a weight gradient
# of an expert with a few dozen rows is dominated by single rows whose error is a product of three rounded factors
# (heavy-tailed), and a few elements in 10^4 reach 2 - 2.5 % of the rms (seen: 5 of 32768 for an expert of 23 rows).
# A mis-addressed row or column tile, the mistake this measure is for, puts 10 % or more of a sampled tensor outside
# the bound, so the bar sits two orders of magnitude below that and one above what rounding produces.
VIOLATION_SHARE = 1e-3


def check(got, want, tol, name=""):
    """Both measures of parity on one tensor: max |gpu - oracle| / max |oracle| <= tol, and at most
    VIOLATION_SHARE of the elements outside |d| <= tol |oracle| + tol rms(oracle)."""
    r = rel_err(got, want)
    assert r <= tol, f"{name}: max relative error {r:.3e} > {tol:.1e}"
    n = violations(got, want, tol)
    size = int(np.asarray(want).size)
    assert n <= int(VIOLATION_SHARE * size), f"{name}: {n} of {size} elements outside rtol = atol/rms = {tol:.1e}"
    return r, n


def gate_logits_are_exact(w):
    """Which gate kernel a workload takes: fp32 inputs, more than 64 experts and expert choice go through the fp64
    product (every logit is the fp32 rounding of an fp64 sum, bit-equal to the oracle's); bf16 with up to 64 experts
    goes through the matrix cores with exact logits only for the tokens whose top-k decision is close."""
    return w.dtype != S.DT_BF16 or w.E > 64 or w.renormalize == 3


def check_logits(got, want, w, x64, wg64):
    """Gate logits against the oracle's.  Exact path: bit-equal.  Matrix-core path: every logit within an eighth of
    the bound the kernel's decision rule relies on, eps[t,e] = 2^-17 |x_t|_2 |w_e|_2 (it assumes every addition inside
    a chain of 64 products rounds, doubled), plus one fp32 rounding: the margin is the evidence that the assumed bound
    on the matrix cores' internal rounding holds with room to spare."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if gate_logits_are_exact(w):
        assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} logits differ in bits"
        return
    eps = 2.0 ** -17 * np.sqrt((x64 * x64).sum(1))[:, None] * np.sqrt((wg64 * wg64).sum(0))[None, :]
    d = np.abs(got - want)
    bound = eps / 8 + 2.0 ** -23 * np.abs(want)
    bad = np.nonzero(~(d <= bound))
    assert bad[0].size == 0, (f"{bad[0].size} logits outside eps/8; worst ratio {np.nanmax(d / bound):.3g} "
                              f"at {bad[0][:3]}, {bad[1][:3]}")
    scale = float(np.max(np.abs(want)))
    assert float(d.max()) <= 1e-5 * scale, "logits differ by more than 1e-5 of the largest"


def cap_of(w):
    """Capacity of a workload: the product's moe_capacity, which must agree with the oracle's formula."""
    cap = capacity_of(w)
    assert cap == (0 if w.f is None else O.capacity(w.N, w.E, w.k, w.f)), "moe_capacity differs from the oracle"
    return cap


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
