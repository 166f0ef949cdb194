"""Pins for the CPU oracle: each part is checked against something other than itself.

Brute force on tiny inputs, closed forms, the dense one-hot ("GShard ordering", paper Sec. 2.1)
formulation of the ordering functions, reduction to a dense FFN, hand-computed textbook values,
central finite differences and adjoint identities.  No GPU, no HIP library.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import moe_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ACTS = [O.ACT_RELU, O.ACT_GELU_TANH, O.ACT_SWIGLU, O.ACT_GELU_ERF]


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- gate logits

def test_logits_match_exact_rational_dot():
    r = rng(1)
    x = r.standard_normal((5, 7)).astype(np.float32)
    w = r.standard_normal((7, 3)).astype(np.float32)
    b = r.standard_normal(3).astype(np.float32)
    got = O.gate_logits(x, w, b)
    assert got.dtype == np.float32
    for t in range(5):
        for e in range(3):
            exact = sum(Fraction(float(x[t, m])) * Fraction(float(w[m, e])) for m in range(7)) + Fraction(float(b[e]))
            assert got[t, e] == np.float32(float(exact))


def test_logits_special_cases():
    r = rng(2)
    x = r.standard_normal((9, 4))
    assert np.all(O.gate_logits(x, np.zeros((4, 5))) == 0)
    b = np.arange(5, dtype=np.float32)
    assert np.array_equal(O.gate_logits(x, np.zeros((4, 5)), b), np.tile(b, (9, 1)))
    # E = 1: the logit is a plain dot product, and transposing operands would change the shape
    w = r.standard_normal((4, 1))
    assert np.allclose(O.gate_logits(x, w)[:, 0], [float(np.dot(x[t], w[:, 0])) for t in range(9)], rtol=1e-6)


# ----------------------------------------------------------------------------- top-k and gate weights

@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_topk_matches_full_sort(k):
    r = rng(3 + k)
    logits = r.standard_normal((200, 5)).astype(np.float32)
    logits[::7, 1] = logits[::7, 3]           # plant exact ties
    logits[::11] = 0.25                       # all-equal rows
    idx = O.keep_top_k(logits, k)
    for t in range(200):
        want = sorted(range(5), key=lambda e: (-float(logits[t, e]), e))[:k]
        assert list(idx[t]) == want


def test_tie_goes_to_lower_index():
    idx = O.keep_top_k(np.array([[1.0, 3.0, 3.0, 3.0]], np.float32), 2)
    assert list(idx[0]) == [1, 2]


def keep_topk_then_softmax_literal(logit_row, k):
    """The paper's formula spelled out: non-top-k entries become -inf, then a softmax over all E."""
    order = sorted(range(len(logit_row)), key=lambda e: (-float(logit_row[e]), e))[:k]
    v = [(-math.inf if e not in order else float(logit_row[e])) for e in range(len(logit_row))]
    m = max(v)
    z = [math.exp(a - m) if a != -math.inf else 0.0 for a in v]
    s = sum(z)
    return [a / s for a in z]


@pytest.mark.parametrize("k", [1, 2, 4])
def test_renormalised_weights_equal_softmax_of_keeptopk(k):
    r = rng(10 + k)
    logits = (2 * r.standard_normal((50, 6))).astype(np.float32)
    idx = O.keep_top_k(logits, k)
    w = O.gate_weights(logits, idx, 1)
    p = O.softmax_all(logits)
    for t in range(50):
        lit = keep_topk_then_softmax_literal(logits[t], k)
        dense = np.zeros(6)
        dense[idx[t]] = w[t]
        assert np.allclose(dense, lit, rtol=1e-13, atol=0)
        assert sum(1 for a in lit if a == 0.0) == 6 - k            # dropped entries are exactly zero
        assert np.allclose(w[t], p[t, idx[t]] / p[t, idx[t]].sum(), rtol=1e-12)  # closed form
    assert np.allclose(w.sum(1), 1.0, rtol=1e-14)
    if k == 1:
        assert np.all(w == 1.0)


def test_unrenormalised_weights_are_selected_probabilities():
    r = rng(20)
    logits = (3 * r.standard_normal((40, 7))).astype(np.float32)
    p = O.softmax_all(logits)
    assert np.allclose(p.sum(1), 1.0, rtol=1e-14)
    for t in range(40):                                            # textbook softmax, written out
        z = [math.exp(float(a)) for a in logits[t]]
        assert np.allclose(p[t], [a / sum(z) for a in z], rtol=1e-12)
    idx = O.keep_top_k(logits, 3)
    w = O.gate_weights(logits, idx, 0)
    for t in range(40):
        assert np.array_equal(w[t], p[t, idx[t]])
        assert w[t, 0] >= w[t, 1] >= w[t, 2]
    # k = E: both variants coincide
    idx_all = O.keep_top_k(logits, 7)
    assert np.allclose(O.gate_weights(logits, idx_all, 0), O.gate_weights(logits, idx_all, 1), rtol=1e-12)


# ----------------------------------------------------------------------------- capacity

def test_capacity_golden():
    for line in open(os.path.join(GOLD, "capacity.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, e, k, f, t = line.split()
        assert O.capacity(int(n), int(e), int(k), float(f)) == int(t)
    assert O.capacity(100, 4, 2, None) == 0


# ----------------------------------------------------------------------------- positions: brute force

def brute_positions(idx, n_experts, cap):
    """For each expert list its (j, t) assignments in lexicographic order and keep the first T."""
    n, k = idx.shape
    pos = -np.ones((n, k), np.int32)
    count = np.zeros(n_experts, np.int32)
    for e in range(n_experts):
        mine = sorted((j, t) for t in range(n) for j in range(k) if idx[t, j] == e)
        kept = mine if cap <= 0 else mine[:cap]
        for p, (j, t) in enumerate(kept):
            pos[t, j] = p
        count[e] = len(kept)
    return pos, count


def test_positions_exhaustive_tiny():
    # every routing of 4 tokens to 3 experts with k = 2 distinct choices, capacities 1..3 and unlimited
    pairs = [(a, b) for a in range(3) for b in range(3) if a != b]
    for combo in itertools.product(pairs, repeat=4):
        idx = np.array(combo, np.int32)
        for cap in (0, 1, 2, 3):
            pos, count, offsets, row_of, src = O.assign_positions(idx, 3, cap)
            bp, bc = brute_positions(idx, 3, cap)
            assert np.array_equal(pos, bp) and np.array_equal(count, bc)


@pytest.mark.parametrize("n,e,k,cap", [(300, 5, 2, 70), (257, 8, 3, 0), (64, 4, 1, 10), (100, 3, 3, 1000)])
def test_position_invariants(n, e, k, cap):
    r = rng(n + e)
    logits = r.standard_normal((n, e)).astype(np.float32) + np.linspace(0, 1.5, e, dtype=np.float32)
    idx = O.keep_top_k(logits, k)
    pos, count, offsets, row_of, src = O.assign_positions(idx, e, cap)
    bp, bc = brute_positions(idx, e, cap)
    assert np.array_equal(pos, bp) and np.array_equal(count, bc)
    if cap > 0:
        assert count.max() <= cap
    total = np.bincount(idx.ravel(), minlength=e)
    assert np.array_equal(count, np.minimum(total, cap) if cap > 0 else total)
    assert offsets[0] == 0 and np.array_equal(np.diff(offsets), count)
    a = int(offsets[-1])
    kept = row_of[row_of >= 0]
    assert len(kept) == a and len(set(kept.tolist())) == a and set(kept.tolist()) == set(range(a))
    assert np.all(src[a:] == -1)
    for rrow in range(a):                                          # src_of_row inverts row_of
        t, j = divmod(int(src[rrow]), k)
        assert row_of[t, j] == rrow
        ex = idx[t, j]
        assert offsets[ex] <= rrow < offsets[ex + 1]
    for ex in range(e):                                            # rows of an expert are ordered by (j, t)
        keys = [(int(s) % k, int(s) // k) for s in src[offsets[ex]:offsets[ex + 1]]]
        assert keys == sorted(keys)


# ----------------------------------------------------------------------------- ordering: dense one-hot formulation

def dense_masks(idx, pos, w, n_experts, cap_dim):
    n, k = idx.shape
    disp = np.zeros((n, n_experts, cap_dim))
    comb = np.zeros((n, n_experts, cap_dim))
    for t in range(n):
        for j in range(k):
            if pos[t, j] >= 0:
                disp[t, idx[t, j], pos[t, j]] = 1.0
                comb[t, idx[t, j], pos[t, j]] = w[t, j]
    return disp, comb


@pytest.mark.parametrize("cap", [0, 6])
def test_order_and_inverse_order_match_dense_einsum(cap):
    r = rng(31)
    n, m, e, k = 24, 5, 4, 2
    x = r.standard_normal((n, m))
    logits = r.standard_normal((n, e)).astype(np.float32)
    idx = O.keep_top_k(logits, k)
    w = O.gate_weights(logits, idx, 0)
    pos, count, offsets, row_of, src = O.assign_positions(idx, e, cap)
    cap_dim = int(count.max())
    disp, comb = dense_masks(idx, pos, w, e, cap_dim)
    padded = np.einsum("tec,tm->ecm", disp, x)                     # (E, T, M) layout of the paper
    xe = O.order(x, row_of, int(offsets[-1]))
    for ex in range(e):
        assert np.array_equal(xe[offsets[ex]:offsets[ex + 1]], padded[ex, :count[ex]])
        assert np.all(padded[ex, count[ex]:] == 0)
    qpad = r.standard_normal((e, cap_dim, m))
    q = np.concatenate([qpad[ex, :count[ex]] for ex in range(e)])
    y = O.inverse_order(q, w, row_of)
    assert np.allclose(y, np.einsum("tec,ecm->tm", comb, qpad), rtol=1e-13, atol=1e-15)
    if cap:
        dropped_all = np.all(pos < 0, axis=1)
        assert dropped_all.any() or (pos < 0).any()
        assert np.all(y[dropped_all] == 0)
    assert np.array_equal(O.inverse_order(q, w, row_of, x), y + x)


def test_inverse_order_reverses_order():
    r = rng(32)
    x = r.standard_normal((40, 6))
    idx = r.integers(0, 5, (40, 1)).astype(np.int32)
    pos, count, offsets, row_of, src = O.assign_positions(idx, 5, 0)
    xe = O.order(x, row_of, 40)
    assert np.array_equal(O.inverse_order(xe, np.ones((40, 1)), row_of), x)


# ----------------------------------------------------------------------------- experts

def test_activation_golden_values():
    fn = {"gelu_tanh": lambda z: O.activation(z, O.ACT_GELU_TANH), "gelu_erf": lambda z: O.activation(z, O.ACT_GELU_ERF),
          "relu": lambda z: O.activation(z, O.ACT_RELU), "silu": O.silu}
    for line in open(os.path.join(GOLD, "activations.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, z, v = line.split()
        assert abs(float(fn[name](np.array([float(z)]))[0]) - float(v)) < 1e-14


@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_GELU_TANH, O.ACT_GELU_ERF])
def test_activation_grad_fd(act):
    z = np.linspace(-3, 3, 61) + 0.013
    h = 1e-6
    fd = (O.activation(z + h, act) - O.activation(z - h, act)) / (2 * h)
    assert np.allclose(O.activation_grad(z, act), fd, atol=1e-8)
    fd = (O.silu(z + h) - O.silu(z - h)) / (2 * h)
    assert np.allclose(O.silu_grad(z), fd, atol=1e-8)


def test_activation_limits():
    big = np.array([30.0])
    for act in (O.ACT_RELU, O.ACT_GELU_TANH, O.ACT_GELU_ERF):
        assert np.allclose(O.activation(big, act), big) and np.allclose(O.activation(-big, act), 0, atol=1e-12)
    assert np.allclose(O.silu(big), big) and np.allclose(O.silu(-big), 0, atol=1e-10)


def dense_ffn_by_loops(x, w1, w3, w2, act):
    """Textbook FFN on one matrix, element by element (no matmul), for tiny shapes."""
    n, m = x.shape
    h = w1.shape[1]
    y = np.zeros((n, w2.shape[1]))
    for t in range(n):
        hid = np.zeros(h)
        for c in range(h):
            a = sum(x[t, i] * w1[i, c] for i in range(m))
            if act == O.ACT_SWIGLU:
                b = sum(x[t, i] * w3[i, c] for i in range(m))
                hid[c] = a / (1 + math.exp(-a)) * b
            elif act == O.ACT_RELU:
                hid[c] = max(a, 0.0)
            elif act == O.ACT_GELU_TANH:
                hid[c] = 0.5 * a * (1 + math.tanh(math.sqrt(2 / math.pi) * (a + 0.044715 * a ** 3)))
            else:
                hid[c] = 0.5 * a * (1 + math.erf(a / math.sqrt(2)))
        for o in range(w2.shape[1]):
            y[t, o] = sum(hid[c] * w2[c, o] for c in range(h))
    return y


@pytest.mark.parametrize("act", ACTS)
def test_identical_experts_all_selected_reduce_to_dense_ffn(act):
    r = rng(40 + act)
    n, m, h, e = 12, 5, 7, 3
    x = r.standard_normal((n, m))
    wg = r.standard_normal((m, e))
    w1 = np.tile(r.standard_normal((1, m, h)), (e, 1, 1))
    w3 = np.tile(r.standard_normal((1, m, h)), (e, 1, 1))
    w2 = np.tile(r.standard_normal((1, h, m)), (e, 1, 1))
    for renorm in (0, 1):
        out = O.layer_fwd(x, wg, None, w1, w3, w2, e, 0, act, renorm, 0)
        assert np.allclose(out["y"], dense_ffn_by_loops(x, w1[0], w3[0], w2[0], act), rtol=1e-11, atol=1e-12)
        assert int(out["offsets"][-1]) == n * e


@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_SWIGLU])
def test_distinct_experts_match_per_token_definition(act):
    r = rng(50 + act)
    n, m, h, e, k = 10, 4, 6, 3, 2
    x = r.standard_normal((n, m)); wg = r.standard_normal((m, e)); bg = r.standard_normal(e)
    w1 = r.standard_normal((e, m, h)); w3 = r.standard_normal((e, m, h)); w2 = r.standard_normal((e, h, m))
    out = O.layer_fwd(x, wg, bg, w1, w3, w2, k, 0, act, 0, 0)
    p = O.softmax_all(out["logits"])
    for t in range(n):
        top = sorted(range(e), key=lambda i: (-float(out["logits"][t, i]), i))[:k]
        want = sum(p[t, i] * dense_ffn_by_loops(x[t:t + 1], w1[i], w3[i], w2[i], act)[0] for i in top)
        assert np.allclose(out["y"][t], want, rtol=1e-11, atol=1e-12)


def test_dropped_tokens_contribute_zero():
    r = rng(60)
    n, m, h, e = 30, 4, 5, 3
    x = r.standard_normal((n, m)); wg = np.zeros((m, e)); bg = np.array([2.0, 0.0, -2.0])   # everyone picks expert 0
    w1 = r.standard_normal((e, m, h)); w2 = r.standard_normal((e, h, m))
    out = O.layer_fwd(x, wg, bg, w1, None, w2, 1, 4, O.ACT_RELU, 0, 0)
    assert list(out["count"]) == [4, 0, 0]
    assert np.all(out["pos"][:4, 0] == np.arange(4)) and np.all(out["pos"][4:] == -1)
    assert np.all(out["y"][4:] == 0) and np.any(out["y"][:4] != 0)
    out_r = O.layer_fwd(x, wg, bg, w1, None, w2, 1, 4, O.ACT_RELU, 0, 1)
    assert np.array_equal(out_r["y"][4:], x[4:])
    dy = r.standard_normal((n, m))
    g = O.layer_bwd(dy, x, wg, bg, w1, None, w2, out, O.ACT_RELU, 0, 0)
    assert np.all(g["dx"][4:] == 0) and np.all(g["dtopk_w"][4:] == 0) and np.all(g["dlogits"][4:] == 0)
    g_r = O.layer_bwd(dy, x, wg, bg, w1, None, w2, out_r, O.ACT_RELU, 0, 1)
    assert np.array_equal(g_r["dx"][4:], dy[4:])


# ----------------------------------------------------------------------------- backward: finite differences

def _loss_and_grads(params, dy, k, cap, act, renorm, resid):
    x, wg, bg, w1, w3, w2 = params
    fwd = O.layer_fwd(x, wg, bg, w1, w3, w2, k, cap, act, renorm, resid, logit_dtype=np.float64)
    g = O.layer_bwd(dy, x, wg, bg, w1, w3, w2, fwd, act, renorm, resid)
    return fwd, g


@pytest.mark.parametrize("act,k,cap,renorm,resid", [
    (O.ACT_RELU, 1, 5, 0, 0), (O.ACT_GELU_TANH, 2, 7, 0, 1), (O.ACT_SWIGLU, 2, 0, 1, 0),
    (O.ACT_SWIGLU, 3, 8, 0, 0), (O.ACT_GELU_ERF, 2, 0, 1, 1), (O.ACT_GELU_TANH, 1, 0, 1, 0),
    (O.ACT_SWIGLU, 2, 0, O.GATE_SIGMOID, 0), (O.ACT_GELU_TANH, 3, 6, O.GATE_SIGMOID, 1),
    (O.ACT_SWIGLU, 4, 5, O.GATE_EXPERT_CHOICE, 0), (O.ACT_GELU_TANH, 4, 9, O.GATE_EXPERT_CHOICE, 1)])
def test_layer_backward_matches_central_differences(act, k, cap, renorm, resid):
    r = rng(70 + act + 10 * k)
    n, m, h, e = 14, 4, 5, 4
    x = r.standard_normal((n, m)); wg = r.standard_normal((m, e)); bg = r.standard_normal(e)
    w1 = 0.7 * r.standard_normal((e, m, h)); w2 = 0.7 * r.standard_normal((e, h, m))
    w3 = 0.7 * r.standard_normal((e, m, h)) if act == O.ACT_SWIGLU else None
    dy = r.standard_normal((n, m))
    params = [x, wg, bg, w1, w3, w2]
    fwd, g = _loss_and_grads(params, dy, k, cap, act, renorm, resid)
    if cap:
        assert (fwd["pos"] < 0).any()          # the case really drops something
    names = ["dx", "dw_gate", "db_gate", "dw1", "dw3", "dw2"]
    eps = 1e-6
    for p, name in zip(params, names):
        if p is None:
            assert g[name] is None
            continue
        flat = p.reshape(-1)
        picks = r.choice(flat.size, size=min(flat.size, 25), replace=False)
        for i in picks:
            old = flat[i]
            flat[i] = old + eps
            fp = O.layer_fwd(*params, k, cap, act, renorm, resid, logit_dtype=np.float64)
            flat[i] = old - eps
            fm = O.layer_fwd(*params, k, cap, act, renorm, resid, logit_dtype=np.float64)
            flat[i] = old
            assert np.array_equal(fp["topk_idx"], fwd["topk_idx"]) and np.array_equal(fm["topk_idx"], fwd["topk_idx"])
            assert np.array_equal(fp["pos"], fwd["pos"]) and np.array_equal(fm["pos"], fwd["pos"])
            fd = float(((fp["y"] - fm["y"]) * dy).sum() / (2 * eps))
            an = float(g[name].reshape(-1)[i])
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (name, i, fd, an)
    if renorm and k == 1:
        assert np.all(g["dw_gate"] == 0) and np.all(fwd["topk_w"] == 1.0)   # degenerate case of the literal formula


def test_backward_adjoint_identity_and_expert_flop_ratio():
    # <dy, J v> = <J^T dy, v> for the expert block (linear in dq for fixed activations)
    r = rng(80)
    a, m, h = 9, 4, 6
    xe = r.standard_normal((a, m)); w1 = r.standard_normal((1, m, h)); w3 = r.standard_normal((1, m, h)); w2 = r.standard_normal((1, h, m))
    off = np.array([0, a], np.int32)
    q, saved = O.expert_ffn(xe, off, w1, w3, w2, O.ACT_SWIGLU)
    dq = r.standard_normal((a, m)); v = r.standard_normal((a, m))
    dxe, dw1, dw3, dw2 = O.expert_ffn_bwd(dq, xe, off, w1, w3, w2, saved, O.ACT_SWIGLU)
    eps = 1e-6
    qp, _ = O.expert_ffn(xe + eps * v, off, w1, w3, w2, O.ACT_SWIGLU)
    qm, _ = O.expert_ffn(xe - eps * v, off, w1, w3, w2, O.ACT_SWIGLU)
    assert abs(float(((qp - qm) / (2 * eps) * dq).sum()) - float((dxe * v).sum())) < 1e-6
    # backward runs two products per forward product (Sec. 4.4): 3 forward, 6 backward for the gated FFN
    fwd_products = 3
    bwd_products = 6    # dHh, dW2, dXe via W1, dXe via W3, dW1, dW3
    assert bwd_products == 2 * fwd_products


# ----------------------------------------------------------------------------- sampled evaluation agrees with the full one

@pytest.mark.parametrize("act,renorm,resid,cap", [(O.ACT_SWIGLU, 1, 0, 0), (O.ACT_GELU_TANH, 0, 1, 20)])
def test_sampled_functions_match_full(act, renorm, resid, cap):
    r = rng(90 + act)
    n, m, h, e, k = 60, 6, 8, 4, 2
    x = r.standard_normal((n, m)); wg = r.standard_normal((m, e)); bg = r.standard_normal(e)
    w1 = r.standard_normal((e, m, h)); w3 = r.standard_normal((e, m, h)) if act == O.ACT_SWIGLU else None
    w2 = r.standard_normal((e, h, m)); dy = r.standard_normal((n, m))
    fwd = O.layer_fwd(x, wg, bg, w1, w3, w2, k, cap, act, renorm, resid)
    g = O.layer_bwd(dy, x, wg, bg, w1, w3, w2, fwd, act, renorm, resid)
    toks = np.array([0, 3, 17, 33, 59])
    ws = {"w1": w1, "w3": w3, "w2": w2}
    s = O.layer_tokens(toks, x, dy, wg, fwd, lambda name, ex: ws[name][ex], act, renorm, resid, True)
    assert np.allclose(s["y"], fwd["y"][toks], rtol=1e-12, atol=1e-13)
    assert np.allclose(s["dx"], g["dx"][toks], rtol=1e-12, atol=1e-13)
    assert np.allclose(s["dtopk_w"], g["dtopk_w"][toks], rtol=1e-12, atol=1e-13)
    assert np.allclose(s["dlogits"], g["dlogits"][toks], rtol=1e-12, atol=1e-13)
    cols = np.array([1, 4, 6])
    for ex in range(e):
        c1, c3, c2 = O.expert_wgrad_columns(ex, cols, x, dy, fwd, w1[ex], w3[ex] if w3 is not None else None, w2[ex], act)
        assert np.allclose(c1, g["dw1"][ex][:, cols], rtol=1e-12, atol=1e-13)
        assert np.allclose(c2, g["dw2"][ex][cols, :], rtol=1e-12, atol=1e-13)
        if w3 is not None:
            assert np.allclose(c3, g["dw3"][ex][:, cols], rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- the layer in chunks (Sec. 4.2)

@pytest.mark.parametrize("r", [1, 2, 3, 5, 16])
def test_chunk_bounds_partition_every_expert(r):
    """Chunks of an expert are consecutive, disjoint, cover its rows, and differ in size by at most one row;
    checked against a brute-force assignment of every row to the chunk c with c*n <= i*r < (c+1)*n... by counting."""
    counts = np.array([0, 1, 2, 7, 16, 17, 255, 256, 1000])
    offsets = np.concatenate([[0], np.cumsum(counts)])
    begin, end = O.chunk_bounds(offsets, r)
    for e, n in enumerate(counts):
        assert begin[0, e] == offsets[e] and end[r - 1, e] == offsets[e + 1]
        assert (end[:-1, e] == begin[1:, e]).all()
        sizes = end[:, e] - begin[:, e]
        assert sizes.sum() == n and sizes.max() - sizes.min() <= 1
        # row i (0-based) of n lies in chunk c iff floor(c n / r) <= i < floor((c+1) n / r); brute force over rows
        for c in range(r):
            rows = [i for i in range(n) if (c * n) // r <= i < ((c + 1) * n) // r]
            assert len(rows) == sizes[c]
            if rows:
                assert offsets[e] + rows[0] == begin[c, e] and offsets[e] + rows[-1] + 1 == end[c, e]


@pytest.mark.parametrize("act,k,cap,r", [(O.ACT_SWIGLU, 2, 0, 3), (O.ACT_GELU_TANH, 1, 4, 2), (O.ACT_RELU, 3, 5, 16)])
def test_chunked_layer_equals_whole_layer(act, k, cap, r):
    """Sec. 4.2: cutting the capacity dimension into r chunks does not change what the layer computes."""
    g = rng(200 + r)
    n, m, h, e = 23, 6, 7, 4
    x = g.standard_normal((n, m)); wg = g.standard_normal((m, e)); bg = g.standard_normal(e)
    w1 = g.standard_normal((e, m, h)); w2 = g.standard_normal((e, h, m))
    w3 = g.standard_normal((e, m, h)) if act == O.ACT_SWIGLU else None
    whole = O.layer_fwd(x, wg, bg, w1, w3, w2, k, cap, act, 1, 0)
    parts = O.layer_fwd_chunked(x, wg, bg, w1, w3, w2, k, cap, act, 1, 0, r)
    for name in ("topk_idx", "pos", "row_of", "offsets"):
        assert np.array_equal(whole[name], parts[name])
    for name in ("xe", "q", "y"):
        np.testing.assert_allclose(parts[name], whole[name], rtol=1e-12, atol=1e-12)
    for a, b in zip(whole["saved"], parts["saved"]):
        if a is not None:
            np.testing.assert_allclose(b, a, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- sigmoid gate (Sec. 2.1)

def test_sigmoid_gate_values():
    """Sec. 2.1: with the sigmoid gate the expert output is scaled by sigma(H_i); closed-form values, and the
    choices stay those of the k largest logits."""
    logits = np.array([[0.0, math.log(3.0), -math.log(3.0), 40.0], [-40.0, 2.0, 1.0, 0.5]])
    idx = O.keep_top_k(logits, 2)
    assert idx.tolist() == [[3, 1], [1, 2]]
    w = O.gate_weights(logits, idx, O.GATE_SIGMOID)
    want = [[1.0 / (1.0 + math.exp(-40.0)), 0.75], [1.0 / (1.0 + math.exp(-2.0)), 1.0 / (1.0 + math.exp(-1.0))]]
    np.testing.assert_allclose(w, want, rtol=1e-15)
    dense = O.gate_dense(logits, idx, O.GATE_SIGMOID)
    np.testing.assert_allclose(dense[0], [0.5, 0.75, 0.25, want[0][0]], rtol=1e-15)
    # unlike the softmax gates the weights of a token do not sum to one and do not depend on each other
    l2 = logits.copy(); l2[0, 1] += 1.0
    w2 = O.gate_weights(l2, O.keep_top_k(l2, 2), O.GATE_SIGMOID)
    assert w2[0, 0] == w[0, 0] and w2[0, 1] > w[0, 1]


# ----------------------------------------------------------------------------- noisy gate (Sec. 2.1)

def test_softplus_values():
    z = np.array([0.0, math.log(math.e - 1.0), -800.0, 800.0, -1.0])
    want = [math.log(2.0), 1.0, 0.0, 800.0, math.log1p(math.exp(-1.0))]
    np.testing.assert_allclose(O.softplus(z), want, rtol=1e-15, atol=1e-300)


def test_noisy_logits_special_cases():
    """Zero noise gives the plain gate; with W_noise = 0 every Softplus is ln 2, so H = I.W_g + ln2 * noise."""
    g = rng(300)
    x = g.standard_normal((9, 5)); wg = g.standard_normal((5, 4)); wn = g.standard_normal((5, 4)); bg = g.standard_normal(4)
    z = g.standard_normal((9, 4))
    h0, nl = O.gate_logits_noisy(x, wg, bg, wn, np.zeros((9, 4)), np.float64)
    assert np.array_equal(h0, O.gate_logits(x, wg, bg, np.float64))
    np.testing.assert_allclose(nl, x @ wn, rtol=1e-14)
    h1, _ = O.gate_logits_noisy(x, wg, bg, np.zeros((5, 4)), z, np.float64)
    np.testing.assert_allclose(h1, x @ wg + bg + math.log(2.0) * z, rtol=1e-14)
    # one entry by hand
    h2, _ = O.gate_logits_noisy(x, wg, None, wn, z, np.float64)
    t, e = 3, 2
    want = sum(x[t, m] * wg[m, e] for m in range(5)) + z[t, e] * math.log1p(math.exp(sum(x[t, m] * wn[m, e] for m in range(5))))
    assert h2[t, e] == pytest.approx(want, rel=1e-13)


@pytest.mark.parametrize("renorm,k,cap", [(1, 2, 0), (0, 3, 6), (O.GATE_SIGMOID, 2, 0)])
def test_noisy_gate_backward_matches_central_differences(renorm, k, cap):
    """L = sum_{kept (t,j)} c[t,j] * gate weight: its gradient with respect to W_g, b_g, W_noise and x, noise draws
    and routing held fixed, against central differences."""
    g = rng(310 + k)
    n, m, e = 12, 5, 6
    x = g.standard_normal((n, m)); wg = g.standard_normal((m, e)); wn = 0.5 * g.standard_normal((m, e))
    bg = g.standard_normal(e); z = g.standard_normal((n, e)); c = g.standard_normal((n, k))
    r0 = O.route_noisy(x, wg, bg, wn, z, k, cap, renorm, np.float64)

    def loss(x_, wg_, bg_, wn_):
        lg, _ = O.gate_logits_noisy(x_, wg_, bg_, wn_, z, np.float64)
        w = O.gate_weights(lg, r0["topk_idx"], renorm)       # the decision of the unperturbed point
        return float((c * w * (r0["pos"] >= 0)).sum())

    dl, dwg, dbg, dwn, dx = O.gate_bwd_noisy(x, wg, wn, z, r0["noise_logits"], r0["logits"], r0["topk_idx"], r0["pos"], c,
                                             renorm, True)
    eps = 1e-6
    for arr, grad, which in ((x, dx, 0), (wg, dwg, 1), (bg, dbg, 2), (wn, dwn, 3)):
        flat = arr.reshape(-1)
        for i in g.choice(flat.size, size=min(flat.size, 20), replace=False):
            args = [x.copy(), wg.copy(), bg.copy(), wn.copy()]
            args[which].reshape(-1)[i] += eps
            up = loss(*args)
            args[which].reshape(-1)[i] -= 2 * eps
            dn = loss(*args)
            assert grad.reshape(-1)[i] == pytest.approx((up - dn) / (2 * eps), rel=2e-5, abs=2e-8)


# ----------------------------------------------------------------------------- X-MoE gate (Sec. 2.1)

def test_xmoe_scores_are_cosines():
    """Hand values: cos((3,4),(4,3)) = 24/25, cos((1,0),(1,1)) = 1/sqrt 2, opposite vectors give -1, orthogonal 0;
    every entry against the definition written with loops; and the invariances of a cosine."""
    x = np.array([[3.0, 4.0], [1.0, 0.0], [-2.0, -2.0], [1.0, -1.0]])
    wp = np.eye(2)
    wg = np.array([[4.0, 1.0], [3.0, 1.0]])            # expert embeddings are the columns (4,3) and (1,1)
    s, p = O.gate_logits_xmoe(x, wp, wg, np.float64)
    assert np.array_equal(p, x)
    want = np.array([[24 / 25, 7 / (5 * math.sqrt(2))], [4 / 5, 1 / math.sqrt(2)], [-7 / (5 * math.sqrt(2)), -1.0],
                     [1 / (5 * math.sqrt(2)), 0.0]])
    np.testing.assert_allclose(s, want, rtol=1e-14, atol=1e-16)

    g = rng(400)
    n, m, d, e = 7, 6, 3, 5
    x = g.standard_normal((n, m)); wp = g.standard_normal((m, d)); wg = g.standard_normal((d, e))
    s, p = O.gate_logits_xmoe(x, wp, wg, np.float64)
    for t in range(n):
        pr = [sum(x[t, i] * wp[i, j] for i in range(m)) for j in range(d)]
        for i in range(e):
            dot = sum(pr[j] * wg[j, i] for j in range(d))
            na = math.sqrt(sum(v * v for v in pr)); nb = math.sqrt(sum(wg[j, i] ** 2 for j in range(d)))
            assert s[t, i] == pytest.approx(dot / (na * nb), rel=1e-12, abs=1e-15)
    assert np.all(np.abs(s) <= 1.0 + 1e-15)
    # a cosine ignores the length of either vector: scaling tokens, the projection, or single embeddings
    s2, _ = O.gate_logits_xmoe(x * g.uniform(0.5, 3.0, (n, 1)), 4.0 * wp, wg * g.uniform(0.5, 3.0, (1, e)), np.float64)
    np.testing.assert_allclose(s2, s, rtol=1e-12, atol=1e-15)
    # a rotation of the projected space applied to both sides leaves every score unchanged
    rot, _ = np.linalg.qr(g.standard_normal((d, d)))
    s3, _ = O.gate_logits_xmoe(x, wp @ rot, rot.T @ wg, np.float64)
    np.testing.assert_allclose(s3, s, rtol=1e-12, atol=1e-14)
    # unit tokens, identity projection, unit embeddings: the scores are the plain gate product
    xu = x / np.linalg.norm(x, axis=1, keepdims=True); wu = g.standard_normal((m, e)); wu /= np.linalg.norm(wu, axis=0)
    s4, _ = O.gate_logits_xmoe(xu, np.eye(m), wu, np.float64)
    np.testing.assert_allclose(s4, O.gate_logits(xu, wu, None, np.float64), rtol=1e-12, atol=1e-15)


def test_xmoe_route_is_route_on_the_scores():
    """The decision and the layout come from the scores exactly as route() takes them from I.W_g: with unit tokens,
    identity projection and unit embeddings the two routes agree in every integer output."""
    g = rng(401)
    n, m, e, k = 40, 8, 6, 2
    x = g.standard_normal((n, m)); x /= np.linalg.norm(x, axis=1, keepdims=True)
    wg = g.standard_normal((m, e)); wg /= np.linalg.norm(wg, axis=0)
    a = O.route_xmoe(x, np.eye(m), wg, k, 9, 1, np.float64)
    b = O.route(x, wg, None, k, 9, 1, np.float64)
    for key in ("topk_idx", "pos", "count", "offsets", "row_of", "src_of_row"):
        assert np.array_equal(a[key], b[key]), key
    np.testing.assert_allclose(a["topk_w"], b["topk_w"], rtol=1e-12)


@pytest.mark.parametrize("renorm,k,cap", [(1, 2, 0), (0, 3, 7), (O.GATE_SIGMOID, 2, 0)])
def test_xmoe_gate_backward_matches_central_differences(renorm, k, cap):
    """L = sum_{kept (t,j)} c[t,j] * gate weight, as a function of x, W_proj and W_g with the routing held fixed."""
    g = rng(410 + k)
    n, m, d, e = 11, 6, 4, 5
    x = g.standard_normal((n, m)); wp = g.standard_normal((m, d)); wg = g.standard_normal((d, e)); c = g.standard_normal((n, k))
    r0 = O.route_xmoe(x, wp, wg, k, cap, renorm, np.float64)

    def loss(x_, wp_, wg_):
        s, _ = O.gate_logits_xmoe(x_, wp_, wg_, np.float64)
        w = O.gate_weights(s, r0["topk_idx"], renorm)
        return float((c * w * (r0["pos"] >= 0)).sum())

    ds, dwp, dwg, dx = O.gate_bwd_xmoe(x, wp, wg, r0["proj"], r0["logits"], r0["topk_idx"], r0["pos"], c, renorm)
    eps = 1e-6
    for arr, grad, which in ((x, dx, 0), (wp, dwp, 1), (wg, dwg, 2)):
        flat = arr.reshape(-1)
        for i in g.choice(flat.size, size=min(flat.size, 20), replace=False):
            args = [x.copy(), wp.copy(), wg.copy()]
            args[which].reshape(-1)[i] += eps
            up = loss(*args)
            args[which].reshape(-1)[i] -= 2 * eps
            dn = loss(*args)
            assert grad.reshape(-1)[i] == pytest.approx((up - dn) / (2 * eps), rel=2e-5, abs=2e-8)
    # the scores do not depend on the length of an embedding or of a projected token, so the gradient has no
    # component along either: <dW_g[:,i], W_g[:,i]> = 0 and <dx[t], x[t]> = 0 (x scales its projection)
    assert np.abs((dwg * wg).sum(axis=0)).max() < 1e-12
    assert np.abs((dx * x).sum(axis=1)).max() < 1e-12
    assert np.abs((dwp * wp).sum()) < 1e-12


# ----------------------------------------------------------------------------- expert choice (Sec. 2.1)

@pytest.mark.parametrize("n,e,k", [(17, 3, 5), (12, 4, 1), (9, 2, 9), (7, 3, 20)])
def test_expert_choice_matches_sorted_columns_and_the_printed_formula(n, e, k):
    g = rng(500 + n)
    x = g.standard_normal((n, 6)); wg = g.standard_normal((6, e)); bg = g.standard_normal(e)
    r = O.route_expert_choice(x, wg, bg, k, np.float64)
    h = x @ wg + bg
    kk = min(k, n)
    for i in range(e):
        # brute force: sort the tokens of the column by (logit descending, token ascending), keep the first k
        want = sorted(sorted(range(n), key=lambda t: (-h[t, i], t))[:kk])
        got = [t for t in range(n) if r["pos"][t, i] >= 0]
        assert got == want
        assert [int(r["pos"][t, i]) for t in got] == list(range(kk))       # rows in token order
        # Softmax(KeepTopK(H^T, k)) spelled out: -inf outside the kept entries of the expert's row of H^T
        row = np.full(n, -np.inf); row[want] = h[want, i]
        z = np.exp(row - row.max()); lit = z / z.sum()
        np.testing.assert_allclose(r["topk_w"][:, i], lit, rtol=1e-13, atol=0)
        assert r["topk_w"][:, i].sum() == pytest.approx(1.0, abs=1e-14)
    assert np.array_equal(r["count"], np.full(e, kk)) and np.array_equal(r["offsets"], np.arange(e + 1) * kk)
    assert np.array_equal(r["topk_idx"], np.tile(np.arange(e), (n, 1)))
    assert np.array_equal(r["probs"], r["topk_w"])
    np.testing.assert_allclose(O.expert_choice_dense(h, r["pos"]), r["probs"], rtol=1e-13, atol=0)
    # the two index maps are inverse to each other and cover exactly the rows 0 .. E k - 1
    rows = r["row_of"][r["row_of"] >= 0]
    assert sorted(rows.tolist()) == list(range(e * kk))
    for t in range(n):
        for i in range(e):
            if r["row_of"][t, i] >= 0:
                assert r["src_of_row"][r["row_of"][t, i]] == t * e + i
                assert r["row_of"][t, i] == r["offsets"][i] + r["pos"][t, i]
    assert np.all(r["src_of_row"][e * kk:] == -1)


def test_expert_choice_tie_goes_to_the_earlier_token():
    x = np.array([[1.0], [2.0], [2.0], [0.5], [2.0]])
    r = O.route_expert_choice(x, np.array([[1.0, -1.0]]), None, 2, np.float64)
    assert [t for t in range(5) if r["pos"][t, 0] >= 0] == [1, 2]           # three equal maxima: the first two
    assert [t for t in range(5) if r["pos"][t, 1] >= 0] == [0, 3]           # column of -x: the two smallest x
    np.testing.assert_allclose(r["topk_w"][[1, 2], 0], [0.5, 0.5])


def test_expert_choice_with_every_token_kept_is_a_dense_mixture():
    """k >= N: every expert processes every token, weighted by the softmax over the tokens of its column; with
    identical experts the layer is (sum of the token's weights) * FFN(token)."""
    g = rng(510)
    n, m, h, e = 6, 4, 5, 3
    x = g.standard_normal((n, m)); wg = g.standard_normal((m, e))
    w1 = np.repeat(g.standard_normal((1, m, h)), e, axis=0); w2 = np.repeat(g.standard_normal((1, h, m)), e, axis=0)
    out = O.layer_fwd(x, wg, None, w1, None, w2, e, n, O.ACT_GELU_TANH, O.GATE_EXPERT_CHOICE, 0, np.float64)
    hh = x @ wg
    col = np.exp(hh - hh.max(axis=0)); col /= col.sum(axis=0)
    np.testing.assert_allclose(out["topk_w"], col, rtol=1e-13)
    dense = dense_ffn_by_loops(x, w1[0], None, w2[0], O.ACT_GELU_TANH)
    np.testing.assert_allclose(out["y"], col.sum(axis=1, keepdims=True) * dense, rtol=1e-12, atol=1e-14)


def test_expert_choice_backward_is_the_token_choice_jacobian_on_the_transposed_problem():
    """Softmax(KeepTopK(.)) along the tokens of H^T: the logit gradient must equal what the token-choice gate
    gives when experts and tokens swap roles."""
    g = rng(520)
    n, m, e, k = 15, 5, 4, 6
    x = g.standard_normal((n, m)); wg = g.standard_normal((m, e)); bg = g.standard_normal(e)
    r = O.route_expert_choice(x, wg, bg, k, np.float64)
    dtw = g.standard_normal((n, e))
    dl, dwg, dbg, dx = O.gate_bwd(x, wg, r["logits"], r["topk_idx"], r["pos"], dtw, O.GATE_EXPERT_CHOICE, True)
    kept = O.keep_top_k(r["logits"].T, k)                                  # [E,k]: the "choices" of each expert
    dt = np.stack([dtw[kept[i], i] for i in range(e)])                     # upstream gradient in that layout
    dl_t, _, _, _ = O.gate_bwd(np.zeros((e, 1)), np.zeros((1, n)), r["logits"].T, kept, np.zeros((e, k), np.int32), dt,
                               O.GATE_SOFTMAX_TOPK, False)
    np.testing.assert_allclose(dl, dl_t.T, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(dwg, x.T @ dl, rtol=1e-13)
    np.testing.assert_allclose(dbg, dl.sum(axis=0), rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(dx, dl @ wg.T, rtol=1e-13)
    assert np.abs(dl.sum(axis=0)).max() < 1e-14                            # a softmax Jacobian annihilates constants
