"""GPU parity at the full benchmark shapes, through the fused layer calls in the configuration
bench.py times.  The GPT-2 shape is checked against the full oracle.  The three larger shapes are
checked on what the oracle can compute one by one: the routing in full (bit exact), y / dx / dtopk_w
for a seeded sample of tokens, columns of every expert's weight gradients over all of its rows, and
dW_g / db_g in full through a second backward pass whose dy is zero outside the sampled tokens."""
import numpy as np
import pytest
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from oracle import moe_oracle as O
from moe_harness import (check, check_logits, TOL, Buffers, assert_routing_equal, cap_of, dev_inputs, make_cfg, oracle_layer, rel_err,
                         run_layer, saved_np, to_dev, to_np)

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
ROUTING = ("topk_idx", "pos", "count", "offsets", "row_of", "src_of_row")


def test_gpt2_shape_full_oracle():
    w = S.WORKLOADS["gpt2"]
    d = S.draw_all(w)
    f, fwd, bwd = oracle_layer(w, d)
    cfg, b = run_layer(w, d)
    got = {n: saved_np(cfg, b, n, torch.int32).reshape(np.asarray(fwd[n]).shape) for n in ROUTING}
    assert_routing_equal(got, fwd)
    assert int(fwd["count"].max()) <= 1229     # balanced gate: the capacity is not reached at this shape
    check_logits(saved_np(cfg, b, "logits", torch.float32).reshape(w.N, w.E), fwd["logits"], w, f["x"], f["w_gate"])
    tol = TOL[w.dtype]
    for name, want in (("y", fwd["y"]), ("dx", bwd["dx"]), ("dw_gate", bwd["dw_gate"]), ("dw1", bwd["dw1"]),
                       ("dw2", bwd["dw2"])):
        check(to_np(getattr(b, name)), want, tol, str(name))


N_TOKENS, N_COLS = 256, 16      # sampled tokens; sampled hidden columns of every expert's weight gradients


@pytest.mark.parametrize("name", ["mixtral", "finegrained", "switch"])
def test_large_shapes_sampled(name):
    w = S.WORKLOADS[name]
    d = S.draw_all(w)
    tol = TOL[w.dtype]
    x, dy, wg = S.to_f64(d["x"]), S.to_f64(d["dy"]), S.to_f64(d["w_gate"])
    bg = None if d["b_gate"] is None else d["b_gate"].astype(np.float64)
    cap = cap_of(w)
    r = O.route(x, wg, bg, w.k, cap, w.renormalize)

    dd = dev_inputs(d)
    cfg, b = run_layer(w, d, dd=dd)
    got = {n: saved_np(cfg, b, n, torch.int32).reshape(np.asarray(r[n]).shape) for n in ROUTING}
    assert_routing_equal(got, r)
    check_logits(saved_np(cfg, b, "logits", torch.float32).reshape(w.N, w.E), r["logits"], w, x, wg)
    count = np.asarray(r["count"])
    print(f"\n{name}: rows per expert min {count.min()} max {count.max()}, capacity {cap}, "
          f"{int((count % 256 != 0).sum())} experts end in a partial row tile")
    if w.f is None:
        assert int(r["offsets"][-1]) == w.N * w.k            # f = *: nothing dropped
    else:
        # the skewed gates fill some experts to the cap (tokens dropped) and leave others far below the mean
        assert int(count.max()) == cap and (r["pos"] < 0).any() and int(count.min()) < w.N * w.k // w.E // 2

    # ---- sampled tokens: y, dx, dtopk_w
    toks = S.sample_indices(w, N_TOKENS, w.N)
    cache = {}

    def expert_weight(which, e):
        if (which, e) not in cache:
            if len(cache) >= 3:
                cache.clear()
            cache[(which, e)] = S.to_f64(d[which][e])
        return cache[(which, e)]

    s = O.layer_tokens(toks, x, dy, wg, r, expert_weight, w.act, w.renormalize, w.add_residual, bg is not None)
    cache.clear()
    check(to_np(b.y[torch.from_numpy(toks).cuda()]), s["y"], tol, "y")
    check(to_np(b.dx[torch.from_numpy(toks).cuda()]), s["dx"], tol, "dx")

    # ---- weight-gradient columns over all rows of EVERY expert (the fullest, the emptiest and every partial last
    #      row tile among them)
    for e in range(w.E):
        cols = S.sample_indices(w, N_COLS, w.H, part=100 + int(e))
        c1, c3, c2 = O.expert_wgrad_columns(int(e), cols, x, dy, r, S.to_f64(d["w1"][e]),
                                            S.to_f64(d["w3"][e]) if w.gated else None, S.to_f64(d["w2"][e]), w.act)
        ct = torch.from_numpy(cols).cuda()
        check(to_np(b.dw1[e][:, ct]), c1, tol, f"dw1[{e}]")
        check(to_np(b.dw2[e][ct, :]), c2, tol, f"dw2[{e}]")
        if w.gated:
            check(to_np(b.dw3[e][:, ct]), c3, tol, f"dw3[{e}]")

    # ---- one whole expert in full: every stored activation and every weight-gradient element of expert 0
    if name == "mixtral":
        e = 0
        lo, hi = int(r["offsets"][e]), int(r["offsets"][e + 1])
        src = np.asarray(r["src_of_row"][lo:hi]).astype(np.int64)
        t, j = src // w.k, src % w.k
        w1, w3, w2 = (S.to_f64(d[n][e]) for n in ("w1", "w3", "w2"))
        q, a1, a3, hh = O.expert_rows_fwd(x[t], w1, w3, w2, w.act)
        sv = lambda n: to_np(moe.saved_view(cfg, b.saved, n, torch.bfloat16).view(w.N * w.k, -1)[lo:hi])
        check(sv("a1"), a1, tol, "a1 of expert 0")
        check(sv("a3"), a3, tol, "a3 of expert 0")
        check(sv("hh"), hh, tol, "hh of expert 0")
        check(sv("q"), q, tol, "q of expert 0")
        dq = np.asarray(r["topk_w"])[t, j][:, None] * dy[t]
        dxe, g1, g3, g2 = O.expert_rows_bwd(dq, x[t], a1, a3, hh, w1, w3, w2, w.act)
        del a1, a3, hh, dxe
        check(to_np(b.dw1[e]), g1, tol, "dw1 of expert 0")
        check(to_np(b.dw3[e]), g3, tol, "dw3 of expert 0")
        check(to_np(b.dw2[e]), g2, tol, "dw2 of expert 0")
        del g1, g2, g3, w1, w2, w3

    # ---- gate gradients in full: backward with dy zero outside the sampled tokens
    dy_m = np.zeros_like(d["dy"])
    dy_m[toks] = d["dy"][toks]
    dd["dy"] = to_dev(dy_m)
    moe.moe_layer_bwd(cfg, dd["dy"], dd["x"], dd["w_gate"], dd["w1"], dd["w3"], dd["w2"], b.saved, b.dx, b.dw_gate,
                      b.db_gate if bg is not None else None, b.dw1, b.dw3, b.dw2, b.ws)
    torch.cuda.synchronize()
    dl = s["dlogits"]                                        # rows of the sampled tokens; zero elsewhere
    check(to_np(b.dw_gate), x[toks].T @ dl, tol, "dw_gate")
    if bg is not None:
        check(to_np(b.db_gate), dl.sum(0), tol, "db_gate")
    others = np.setdiff1d(np.arange(w.N), toks)[:4096]
    assert torch.count_nonzero(b.dx[torch.from_numpy(others).cuda()]).item() == 0   # no gradient without dy


def _timed(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def test_xmoe_gate_at_the_mixtral_token_shape():
    """X-MoE gate (Sec. 2.1) at N, M, E, k of the Mixtral shape with a 256-wide projection: projection, scores and
    routing bit exact in full, gradients in full within the bf16 tolerance."""
    w = S.scaled(S.WORKLOADS["mixtral"], H=64, seed=61)
    d_proj = 256
    cfg = make_cfg(w)
    b = Buffers(w, cfg)
    x, wp, wg, dtw = S.draw_x(w), S.draw_w_proj(w, d_proj), S.draw_w_embed(w, d_proj), S.draw_dtopk_w(w)
    ref = O.route_xmoe(S.to_f64(x), S.to_f64(wp), S.to_f64(wg), w.k, cap_of(w), w.renormalize)
    ws = torch.empty(moe.moe_route_xmoe_workspace_bytes(cfg, d_proj), dtype=torch.uint8, device="cuda")
    proj = torch.empty(w.N, d_proj, dtype=torch.float32, device="cuda")
    xd, wpd, wgd = to_dev(x), to_dev(wp), to_dev(wg)
    fwd = lambda: moe.moe_route_xmoe(cfg, xd, wpd, wgd, d_proj, proj, b.logits, b.probs, b.topk_idx, b.topk_w, b.pos,
                                     b.row_of, b.count, b.offsets, b.src_of_row, ws)
    t_fwd = _timed(fwd)
    assert np.array_equal(proj.cpu().numpy(), ref["proj"])
    assert np.array_equal(b.logits.cpu().numpy(), ref["logits"])
    assert_routing_equal({n: to_np(getattr(b, n)) for n in ROUTING}, ref)
    check(to_np(b.topk_w), ref["topk_w"], 1e-5)

    ds, dwp, dwg, dx = O.gate_bwd_xmoe(S.to_f64(x), S.to_f64(wp), S.to_f64(wg), ref["proj"], ref["logits"], ref["topk_idx"],
                                       ref["pos"], dtw.astype(np.float64), w.renormalize)
    dw_proj = torch.empty(w.M, d_proj, dtype=b.dw_gate.dtype, device="cuda")
    dw_gate = torch.empty(d_proj, w.E, dtype=b.dw_gate.dtype, device="cuda")
    args = (to_dev(ref["proj"]), to_dev(ref["probs"].astype(np.float32)), to_dev(ref["topk_idx"]), to_dev(ref["pos"]), to_dev(dtw))

    def bwd():
        b.dx.zero_()
        moe.moe_route_xmoe_bwd(cfg, xd, wpd, wgd, d_proj, *args, dw_proj, dw_gate, b.dx, ws)
    t_bwd = _timed(bwd)
    tol = TOL[w.dtype]
    check(to_np(dw_proj), dwp, tol)
    check(to_np(dw_gate), dwg, tol)
    check(to_np(b.dx), dx, tol)
    print(f"\nX-MoE gate, N={w.N} M={w.M} D={d_proj} E={w.E}: forward {t_fwd:.3f} ms, backward (with dx clear) {t_bwd:.3f} ms")


def test_expert_choice_gate_at_the_mixtral_token_shape():
    """Expert choice (Sec. 2.1) at N, M, E of the Mixtral shape, every expert keeping N/4 tokens: routing bit exact
    in full, weights and gate gradients in full."""
    w = S.scaled(S.WORKLOADS["mixtral"], H=64, k=8, f=0.25, renormalize=3, seed=62)
    cfg = make_cfg(w)
    assert cfg.capacity == w.N // 4
    b = Buffers(w, cfg)
    x, wg = S.draw_x(w), S.draw_w_gate(w)
    dtw = S.draw_dtopk_w(w)
    ref = O.route(S.to_f64(x), S.to_f64(wg), None, w.k, cap_of(w), w.renormalize)
    xd, wgd = to_dev(x), to_dev(wg)
    fwd = lambda: moe.moe_route(cfg, xd, wgd, None, b.logits, b.probs, b.topk_idx, b.topk_w, b.pos, b.row_of, b.count,
                                b.offsets, b.src_of_row, b.ws)
    t_fwd = _timed(fwd)
    assert np.array_equal(b.logits.cpu().numpy(), ref["logits"])
    assert_routing_equal({n: to_np(getattr(b, n)) for n in ROUTING}, ref)
    check(to_np(b.topk_w), ref["topk_w"], 1e-5)
    check(to_np(b.probs), ref["probs"], 1e-5)

    dl, dwg, _, dx = O.gate_bwd(S.to_f64(x), S.to_f64(wg), ref["logits"], ref["topk_idx"], ref["pos"], dtw.astype(np.float64),
                                w.renormalize, False)
    args = (to_dev(ref["probs"].astype(np.float32)), to_dev(ref["topk_idx"]), to_dev(ref["pos"]), to_dev(dtw))

    def bwd():
        b.dx.zero_()
        moe.moe_route_bwd(cfg, xd, wgd, *args, b.dw_gate, None, b.dx, b.ws)
    t_bwd = _timed(bwd)
    tol = TOL[w.dtype]
    check(to_np(b.dw_gate), dwg, tol)
    check(to_np(b.dx), dx, tol)
    print(f"\nexpert-choice gate, N={w.N} M={w.M} E={w.E}, {cfg.capacity} tokens per expert: forward {t_fwd:.3f} ms, "
          f"backward (with dx clear) {t_bwd:.3f} ms")
