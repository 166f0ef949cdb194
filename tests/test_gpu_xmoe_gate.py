"""The X-MoE gate of FSMoE Sec. 2.1 (cosine scores after a low-rank projection) through the C ABI against the
oracle: projection, scores and routing bit-exact, gate weights and gradients within the float tolerances."""
import numpy as np
import pytest
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from moe_harness import check, TOL, Buffers, assert_routing_equal, cap_of, make_cfg, rel_err, store, to_dev, to_np
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu
W = S.WORKLOADS

# (workload, d_proj): several 64-token tiles with a ragged tail, E below / at / above a register chunk,
# d_proj below and above 32 (the padded width of the bf16 products) and not a multiple of it
CASES = {
    "xmoe_bf16_topk": (S.scaled(W["mixtral"], N=1000, M=256, H=64, E=8, k=2, renormalize=1, seed=51), 64),
    "xmoe_bf16_drops": (S.scaled(W["finegrained"], N=700, M=128, H=64, E=16, k=4, f=1.0, seed=52), 24),
    "xmoe_bf16_wide": (S.scaled(W["switch"], N=450, M=192, H=64, E=64, k=1, f=1.25, seed=53), 136),
    "xmoe_f32_sigmoid": (S.scaled(W["tiny"], N=333, M=72, H=64, E=5, k=2, f=1.2, renormalize=2, seed=54), 12),
    "xmoe_f32_all": (S.scaled(W["tiny"], N=130, M=40, H=64, E=9, k=3, renormalize=0, seed=55), 4),
    "xmoe_f32_max_d": (S.scaled(W["tiny"], N=100, M=32, H=64, E=12, k=2, renormalize=1, seed=56), 256),
}


@pytest.mark.parametrize("name", list(CASES))
def test_xmoe_route_forward_and_backward(name):
    w, d = CASES[name]
    cfg = make_cfg(w)
    b = Buffers(w, cfg)
    x, wp, wg, dtw = S.draw_x(w), S.draw_w_proj(w, d), S.draw_w_embed(w, d), S.draw_dtopk_w(w)
    f = lambda a: S.to_f64(a)
    cap = cap_of(w)
    ref = O.route_xmoe(f(x), f(wp), f(wg), w.k, cap, w.renormalize)
    ws = torch.empty(moe.moe_route_xmoe_workspace_bytes(cfg, d), dtype=torch.uint8, device="cuda")
    proj = torch.empty(w.N, d, dtype=torch.float32, device="cuda")
    moe.moe_route_xmoe(cfg, to_dev(x), to_dev(wp), to_dev(wg), d, proj, b.logits, b.probs, b.topk_idx, b.topk_w, b.pos,
                       b.row_of, b.count, b.offsets, b.src_of_row, ws)
    torch.cuda.synchronize()
    assert np.array_equal(proj.cpu().numpy(), ref["proj"])
    got = b.logits.cpu().numpy()
    assert np.array_equal(got, ref["logits"]), f"{np.count_nonzero(got != ref['logits'])} scores differ in bits"
    assert np.abs(got).max() <= 1.0
    assert_routing_equal({n: to_np(getattr(b, n)) for n in ("topk_idx", "pos", "count", "offsets", "row_of", "src_of_row")}, ref)
    check(to_np(b.probs), ref["probs"], 1e-5)
    check(to_np(b.topk_w), ref["topk_w"], 1e-5)

    # backward from the oracle's forward tensors (rounded to what the call takes)
    ds, dwp, dwg, dx = O.gate_bwd_xmoe(f(x), f(wp), f(wg), ref["proj"], ref["logits"], ref["topk_idx"], ref["pos"],
                                       dtw.astype(np.float64), w.renormalize)
    base = store(0.25 * f(S.draw_dy(w)), w)      # something already in dx: the call accumulates
    b.dx.copy_(to_dev(base))
    dw_proj = torch.empty(w.M, d, dtype=b.dw_gate.dtype, device="cuda")
    dw_gate = torch.empty(d, w.E, dtype=b.dw_gate.dtype, device="cuda")
    moe.moe_route_xmoe_bwd(cfg, to_dev(x), to_dev(wp), to_dev(wg), d, to_dev(ref["proj"]),
                           to_dev(ref["probs"].astype(np.float32)), to_dev(ref["topk_idx"]), to_dev(ref["pos"]), to_dev(dtw),
                           dw_proj, dw_gate, b.dx, ws)
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    check(to_np(dw_proj), dwp, tol)
    check(to_np(dw_gate), dwg, tol)
    check(to_np(b.dx), S.to_f64(base) + dx, tol)
    # a second call on a smaller problem with the same workspace: nothing of the first may leak
    if name == "xmoe_bf16_topk":
        w2 = S.scaled(w, N=200)
        cfg2 = make_cfg(w2)
        b2 = Buffers(w2, cfg2)
        x2 = S.draw_x(w2)
        ref2 = O.route_xmoe(f(x2), f(wp), f(wg), w2.k, cap_of(w2), w2.renormalize)
        proj2 = torch.empty(w2.N, d, dtype=torch.float32, device="cuda")
        moe.moe_route_xmoe(cfg2, to_dev(x2), to_dev(wp), to_dev(wg), d, proj2, b2.logits, b2.probs, b2.topk_idx, b2.topk_w,
                           b2.pos, b2.row_of, b2.count, b2.offsets, b2.src_of_row, ws)
        torch.cuda.synchronize()
        assert np.array_equal(b2.logits.cpu().numpy(), ref2["logits"])
        assert_routing_equal({n: to_np(getattr(b2, n)) for n in ("topk_idx", "pos", "count", "offsets", "row_of", "src_of_row")}, ref2)


def test_xmoe_argument_checks():
    w, d = CASES["xmoe_f32_all"]
    cfg = make_cfg(w)
    with pytest.raises(moe.MoeError, match="d_proj"):
        moe.moe_route_xmoe_workspace_bytes(cfg, 6)
    with pytest.raises(moe.MoeError, match="d_proj"):
        moe.moe_route_xmoe_workspace_bytes(cfg, 260)
    b = Buffers(w, cfg)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    proj = torch.empty(w.N, d, dtype=torch.float32, device="cuda")
    x, wp, wg = to_dev(S.draw_x(w)), to_dev(S.draw_w_proj(w, d)), to_dev(S.draw_w_embed(w, d))
    with pytest.raises(moe.MoeError, match="workspace"):
        moe.moe_route_xmoe(cfg, x, wp, wg, d, proj, b.logits, b.probs, b.topk_idx, b.topk_w, b.pos, b.row_of, b.count,
                           b.offsets, b.src_of_row, small)


@pytest.mark.parametrize("name", ["xmoe_bf16_topk", "xmoe_f32_sigmoid"])
def test_xmoe_layer_through_the_stage_calls(name):
    """A whole MoE layer with the X-MoE gate, forward and backward, chained from the per-stage entry points
    (route -> ordering -> experts -> I-ordering and back), against the same chain of oracle functions."""
    w, d = CASES[name]
    cfg = make_cfg(w)
    b = Buffers(w, cfg)
    f = lambda a: None if a is None else S.to_f64(a)
    x, wp, wg = S.draw_x(w), S.draw_w_proj(w, d), S.draw_w_embed(w, d)
    dw = S.draw_all(w)
    w1, w3, w2, dy = dw["w1"], dw["w3"], dw["w2"], dw["dy"]
    # ---- oracle
    r = O.route_xmoe(f(x), f(wp), f(wg), w.k, cap_of(w), w.renormalize)
    n_rows = int(r["offsets"][-1])
    xe = O.order(f(x), r["row_of"], n_rows)
    q, saved = O.expert_ffn(xe, r["offsets"], f(w1), f(w3), f(w2), w.act)
    y = O.inverse_order(q, r["topk_w"], r["row_of"], f(x) if w.add_residual else None)
    dq, dtw = O.inverse_order_bwd(f(dy), q, r["topk_w"], r["row_of"])
    dxe, dw1, dw3, dw2 = O.expert_ffn_bwd(dq, xe, r["offsets"], f(w1), f(w3), f(w2), saved, w.act)
    dx = O.order_bwd(dxe, r["row_of"], f(dy) if w.add_residual else None)
    _, dwp, dwg, dx_gate = O.gate_bwd_xmoe(f(x), f(wp), f(wg), r["proj"], r["logits"], r["topk_idx"], r["pos"], dtw,
                                           w.renormalize)
    # ---- the library, stage by stage
    ws_x = torch.empty(moe.moe_route_xmoe_workspace_bytes(cfg, d), dtype=torch.uint8, device="cuda")
    proj = torch.empty(w.N, d, dtype=torch.float32, device="cuda")
    xd, wpd, wgd, w1d, w3d, w2d, dyd = (None if a is None else to_dev(a) for a in (x, wp, wg, w1, w3, w2, dy))
    moe.moe_route_xmoe(cfg, xd, wpd, wgd, d, proj, b.logits, b.probs, b.topk_idx, b.topk_w, b.pos, b.row_of, b.count,
                       b.offsets, b.src_of_row, ws_x)
    moe.moe_dispatch(cfg, xd, b.row_of, b.xe)
    moe.moe_expert_ffn_fwd(cfg, b.xe, b.offsets, w1d, w3d, w2d, b.q, b.a1, b.a3, b.hh, b.ws)
    moe.moe_combine(cfg, b.q, b.topk_w, b.row_of, xd if w.add_residual else None, b.y)
    moe.moe_combine_bwd(cfg, dyd, b.q, b.topk_w, b.row_of, b.dq, b.dtopk_w)
    moe.moe_expert_ffn_bwd(cfg, b.dq, b.xe, b.offsets, w1d, w3d, w2d, b.a1, b.a3, b.hh, b.dxe, b.dw1, b.dw3, b.dw2, b.ws)
    moe.moe_dispatch_bwd(cfg, b.dxe, b.row_of, dyd if w.add_residual else None, b.dx)
    dw_proj = torch.empty(w.M, d, dtype=b.dw_gate.dtype, device="cuda")
    dw_gate = torch.empty(d, w.E, dtype=b.dw_gate.dtype, device="cuda")
    moe.moe_route_xmoe_bwd(cfg, xd, wpd, wgd, d, proj, b.probs, b.topk_idx, b.pos, b.dtopk_w, dw_proj, dw_gate, b.dx, ws_x)
    torch.cuda.synchronize()
    assert_routing_equal({n: to_np(getattr(b, n)) for n in ("topk_idx", "pos", "count", "offsets", "row_of", "src_of_row")}, r)
    tol = TOL[w.dtype]
    check(to_np(b.y), y, tol)
    check(to_np(b.dx), dx + dx_gate, tol)
    check(to_np(dw_proj), dwp, tol)
    check(to_np(dw_gate), dwg, tol)
    check(to_np(b.dw1), dw1, tol)
    check(to_np(b.dw2), dw2, tol)
    if w.gated:
        check(to_np(b.dw3), dw3, tol)
