"""CPU oracle for one GPU's share of a Mixture-of-Experts layer (forward + backward).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
library is checked against.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it; it shares no code with the HIP path and imports
nothing from it.  All floating point runs in fp64 on inputs that were widened
exactly from their stored format (fp32 or bf16), except where noted: gate logits
are rounded once to fp32, because the top-k decision is taken on fp32 logits on
both sides (the paper fixes no precision for it).

What the paper defines and where (FSMoE, Sec. 2.1 unless noted):
  * gate:      G(I) = Softmax(KeepTopK(H(I), k)),  H(I) = I . W_g  (noise term
               left out), KeepTopK keeps the k largest entries and sets the rest
               to -inf                                   -> gate_logits, keep_top_k,
                                                            gate_weights
  * capacity:  T := k * f * B * L / E  (f = * : nothing dropped, Table 4)
                                                         -> capacity
  * ordering:  layout (B, L, M) -> (E, T, M), slab i holds expert i's tokens
                                                         -> assign_positions, order
  * experts:   Q_i = e_i(G[i,:,:]); two-layer FFN with W1 (M,H), W2 (H,M), or the
               Mixtral three-matrix FFN (Sec. 3.1 "Expert")   -> expert_ffn
  * I-order:   reverse of ordering, outputs scaled by the gate value and summed
               back into (B, L, M)                       -> inverse_order
  * backward:  every operation stores its activation and its gradient is computed
               by hand (Sec. 4.4); expert backward is twice the forward work
                                                         -> *_bwd
  * other gates of Sec. 2.1: the sigmoid gate (expert output scaled by sigma(H_i))
               -> gate_weights / gate_dense / gate_bwd with renormalize = 2;
               the noise term of H(I), with the normal draws as an argument
               -> gate_logits_noisy, route_noisy, gate_bwd_noisy;
               the X-MoE scores s_i = cos(W_proj I, W_g[:, i]) after a low-rank projection
               -> gate_logits_xmoe, route_xmoe, gate_bwd_xmoe;
               expert choice, G(I) = Softmax(KeepTopK((I.W_g)^T, k)): every expert keeps its top tokens
               -> route_expert_choice, expert_choice_dense, gate_bwd with renormalize = 3
  * chunks:    Sec. 4.2 cuts the capacity dimension into r parts that pass
               through ordering and experts one after the other
                                                         -> chunk_bounds, layer_fwd_chunked

Readings taken where the paper is silent (each is listed in the design notes):
  ties in top-k go to the lower expert index; T is rounded up; when an expert
  overflows, all first choices are served before any second choice and earlier
  tokens first; gate weights are not renormalised after a drop; a token whose
  every choice is dropped outputs zero (plus the residual when requested);
  experts have no biases; GELU is the tanh form unless the erf form is asked for;
  the sigmoid gate keeps the top-k selection on the logits; the two products of the
  noisy gate are each rounded to fp32 before H is formed from them in fp64; chunk c
  of r of an expert with n rows is rows floor(c n / r) .. floor((c+1) n / r) - 1;
  the X-MoE projection is stored [M,D] and rounded to fp32 before the cosine is formed
  in fp64, with no temperature and no epsilon; expert choice: ties go to the earlier
  token, an expert's rows are its kept tokens in token order, and the capacity argument
  is the number of tokens every expert keeps.

Parity status: every function here is pinned by tests/test_oracle_pins.py
(brute force on tiny inputs, closed forms, the dense one-hot formulation of the
ordering, dense-FFN reduction, finite differences and adjoint identities).
"""
from __future__ import annotations

import math

import numpy as np

ACT_RELU, ACT_GELU_TANH, ACT_SWIGLU, ACT_GELU_ERF = 0, 1, 2, 3


# ----------------------------------------------------------------------------- gate

def gate_logits(x, w_gate, b_gate=None, logit_dtype=np.float32):
    """H(I) = I . W_g (+ b_g), accumulated in fp64, rounded once to fp32.  [N,E] float32.

    logit_dtype=np.float64 skips the rounding; the finite-difference pins use it so that the
    layer is a smooth function of its inputs."""
    h = np.asarray(x, np.float64) @ np.asarray(w_gate, np.float64)
    if b_gate is not None:
        h = h + np.asarray(b_gate, np.float64)[None, :]
    return h.astype(logit_dtype)


def softplus(z):
    """Softplus(z) = ln(1 + e^z), evaluated as logaddexp(0, z) (no overflow for large |z|)."""
    return np.logaddexp(0.0, np.asarray(z, np.float64))


def gate_logits_noisy(x, w_gate, b_gate, w_noise, noise, logit_dtype=np.float32):
    """The noisy gate of Sec. 2.1: H(I)_i = (I.W_g)_i + N(0,1) * Softplus((I.W_noise)_i), with the standard-normal
    draws passed in (`noise`, [N,E]) so that the result is a function of its arguments.

    Reading of the precision (the paper gives none): both products are accumulated in fp64 and rounded once to
    fp32 (they are outputs of the path: the second one is kept for the backward pass); H is then formed from
    those two fp32 tensors in fp64 and rounded once to fp32.  Returns (H, I.W_noise), both [N,E]."""
    clean = gate_logits(x, w_gate, b_gate, logit_dtype)
    nl = gate_logits(x, w_noise, None, logit_dtype)
    h = clean.astype(np.float64) + np.asarray(noise, np.float64) * softplus(nl)
    return h.astype(logit_dtype), nl


def keep_top_k(logits, k):
    """Indices of the k largest logits of every token, largest first.  [N,k] int32.

    Repeated arg-max on the logits as given (fp32 in the parity path); among equal values the lower expert
    index wins (np.argmax returns the first maximum)."""
    l = np.array(logits, copy=True)
    n, e = l.shape
    idx = np.empty((n, k), np.int32)
    rows = np.arange(n)
    for j in range(k):
        a = np.argmax(l, axis=1)
        idx[:, j] = a
        l[rows, a] = -np.inf
    return idx


def softmax_all(logits):
    """Softmax over all E experts, fp64.  [N,E]."""
    l = np.asarray(logits, np.float64)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


# values of the `renormalize` argument (the gate-weight function)
GATE_SOFTMAX_ALL = 0   # softmax over all E, the selected probabilities used as they are
GATE_SOFTMAX_TOPK = 1  # Softmax(KeepTopK(H, k)) as printed in Sec. 2.1
GATE_SIGMOID = 2       # the sigmoid gate of Sec. 2.1 (BASE, StableMoE): expert output scaled by sigma(H_i)
GATE_EXPERT_CHOICE = 3  # expert choice (Sec. 2.1): every expert keeps its top tokens, Softmax(KeepTopK(H^T, k))


def sigmoid(z):
    z = np.asarray(z, np.float64)
    return 1.0 / (1.0 + np.exp(-z))


def gate_weights(logits, topk_idx, renormalize):
    """Gate value of every kept choice.  [N,k] float64.

    renormalize=1: Softmax(KeepTopK(.)) literally: the -inf entries vanish, so the
    k kept logits are soft-maxed among themselves.
    renormalize=0: softmax over all E, the selected probabilities used as they are.
    renormalize=2: sigmoid gate, sigma(H_i) of each selected logit (Sec. 2.1)."""
    l = np.asarray(logits, np.float64)
    sel = np.take_along_axis(l, topk_idx.astype(np.int64), axis=1)
    if renormalize == GATE_SIGMOID:
        return sigmoid(sel)
    if renormalize:
        z = np.exp(sel - sel[:, :1])       # choice 0 is the largest kept logit
        return z / z.sum(axis=1, keepdims=True)
    p = softmax_all(logits)
    return np.take_along_axis(p, topk_idx.astype(np.int64), axis=1)


def gate_dense(logits, topk_idx, renormalize):
    """G(I) as an [N,E] matrix: Softmax(KeepTopK(H, k)) (zeros off the top-k) when renormalize=1,
    the softmax over all E when 0, sigma(H) of every logit for the sigmoid gate."""
    if renormalize == GATE_SIGMOID:
        return sigmoid(logits)
    if not renormalize:
        return softmax_all(logits)
    g = np.zeros(np.shape(logits), np.float64)
    np.put_along_axis(g, topk_idx.astype(np.int64), gate_weights(logits, topk_idx, 1), axis=1)
    return g


# ----------------------------------------------------------------------------- capacity and ordering

def capacity(n_tokens, n_experts, top_k, f):
    """T = ceil(k * f * N / E) evaluated left to right in fp64; f=None means no limit (returns 0)."""
    if f is None:
        return 0
    return int(math.ceil(((float(top_k) * float(f)) * float(n_tokens)) / float(n_experts)))


def assign_positions(topk_idx, n_experts, cap):
    """Slot of every (token, choice) inside its expert's slab, -1 when dropped.

    Walk choice rank j = 0..k-1, and inside each rank the tokens in order; an
    assignment takes the expert's next free slot while one is left (cap <= 0: always).
    Returns pos [N,k], count [E], offsets [E+1], row_of [N,k], src_of_row [N*k]
    (entries past offsets[E] are -1); all int32.  row = offsets[e] + pos in the
    compact expert-major buffer, src = t*k + j."""
    n, k = topk_idx.shape
    pos = np.full((n, k), -1, np.int32)
    count = np.zeros(n_experts, np.int32)
    for j in range(k):
        for t in range(n):
            e = int(topk_idx[t, j])
            if cap <= 0 or count[e] < cap:
                pos[t, j] = count[e]
                count[e] += 1
    offsets = np.zeros(n_experts + 1, np.int32)
    for e in range(n_experts):
        offsets[e + 1] = offsets[e] + count[e]
    row_of = np.full((n, k), -1, np.int32)
    src_of_row = np.full(n * k, -1, np.int32)
    for t in range(n):
        for j in range(k):
            if pos[t, j] >= 0:
                r = int(offsets[topk_idx[t, j]] + pos[t, j])
                row_of[t, j] = r
                src_of_row[r] = t * k + j
    return pos, count, offsets, row_of, src_of_row


def order(x, row_of, n_rows):
    """Ordering function: Xe[row_of[t,j], :] = x[t, :] for every kept assignment.  [n_rows, M]."""
    x = np.asarray(x)
    xe = np.zeros((n_rows, x.shape[1]), x.dtype)
    n, k = row_of.shape
    for t in range(n):
        for j in range(k):
            r = row_of[t, j]
            if r >= 0:
                xe[r] = x[t]
    return xe


def inverse_order(q, topk_w, row_of, x=None):
    """I-ordering: y[t] = sum over kept j of w[t,j] * Q[row_of[t,j]]  (+ x[t] when given)."""
    n, k = row_of.shape
    y = np.zeros((n, q.shape[1]), np.float64)
    for t in range(n):
        for j in range(k):
            r = row_of[t, j]
            if r >= 0:
                y[t] += topk_w[t, j] * q[r]
    if x is not None:
        y = y + np.asarray(x, np.float64)
    return y


# ----------------------------------------------------------------------------- experts

def _erf(z):
    return np.vectorize(math.erf, otypes=[np.float64])(z)


def activation(a, act):
    """Element-wise activation of the two-layer expert."""
    if act == ACT_RELU:
        return np.maximum(a, 0.0)
    if act == ACT_GELU_TANH:
        return 0.5 * a * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (a + 0.044715 * a ** 3)))
    if act == ACT_GELU_ERF:
        return 0.5 * a * (1.0 + _erf(a / math.sqrt(2.0)))
    raise ValueError(act)


def activation_grad(a, act):
    if act == ACT_RELU:
        return (a > 0.0).astype(np.float64)
    if act == ACT_GELU_TANH:
        c = math.sqrt(2.0 / math.pi)
        u = c * (a + 0.044715 * a ** 3)
        th = np.tanh(u)
        return 0.5 * (1.0 + th) + 0.5 * a * (1.0 - th * th) * c * (1.0 + 3.0 * 0.044715 * a * a)
    if act == ACT_GELU_ERF:
        return 0.5 * (1.0 + _erf(a / math.sqrt(2.0))) + a * np.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)
    raise ValueError(act)


def silu(a):
    return a / (1.0 + np.exp(-a))


def silu_grad(a):
    s = 1.0 / (1.0 + np.exp(-a))
    return s * (1.0 + a * (1.0 - s))


def expert_rows_fwd(xe_rows, w1, w3, w2, act):
    """One expert applied to a block of its rows.  Returns (q, a1, a3, hh); a3 is None unless SwiGLU."""
    a1 = xe_rows @ w1
    if act == ACT_SWIGLU:
        a3 = xe_rows @ w3
        hh = silu(a1) * a3
    else:
        a3 = None
        hh = activation(a1, act)
    return hh @ w2, a1, a3, hh


def expert_ffn(xe, offsets, w1, w3, w2, act):
    """Q_i = e_i(G[i,:,:]) on the compact buffer: rows offsets[e]..offsets[e+1] belong to expert e.

    Returns q [A,M] and the stored activations (a1, a3, hh), each [A,H]."""
    n_rows = int(offsets[-1])
    e_cnt = len(offsets) - 1
    h = w1.shape[2]
    q = np.zeros((n_rows, xe.shape[1]), np.float64)
    a1 = np.zeros((n_rows, h), np.float64)
    a3 = np.zeros((n_rows, h), np.float64) if act == ACT_SWIGLU else None
    hh = np.zeros((n_rows, h), np.float64)
    for e in range(e_cnt):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        qe, a1e, a3e, hhe = expert_rows_fwd(xe[lo:hi], w1[e], w3[e] if a3 is not None else None, w2[e], act)
        q[lo:hi], a1[lo:hi], hh[lo:hi] = qe, a1e, hhe
        if a3 is not None:
            a3[lo:hi] = a3e
    return q, (a1, a3, hh)


def expert_rows_bwd(dq_rows, xe_rows, a1, a3, hh, w1, w3, w2, act):
    """Adjoint of expert_rows_fwd.  Returns dxe, dw1, dw3, dw2 (dw3 None unless SwiGLU)."""
    dhh = dq_rows @ w2.T
    dw2 = hh.T @ dq_rows
    if act == ACT_SWIGLU:
        da1 = dhh * a3 * silu_grad(a1)
        da3 = dhh * silu(a1)
        dxe = da1 @ w1.T + da3 @ w3.T
        return dxe, xe_rows.T @ da1, xe_rows.T @ da3, dw2
    da1 = dhh * activation_grad(a1, act)
    return da1 @ w1.T, xe_rows.T @ da1, None, dw2


def expert_ffn_bwd(dq, xe, offsets, w1, w3, w2, saved, act):
    a1, a3, hh = saved
    e_cnt = len(offsets) - 1
    dxe = np.zeros_like(xe, dtype=np.float64)
    dw1 = np.zeros_like(w1, dtype=np.float64)
    dw2 = np.zeros_like(w2, dtype=np.float64)
    dw3 = np.zeros_like(w3, dtype=np.float64) if act == ACT_SWIGLU else None
    for e in range(e_cnt):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        r = expert_rows_bwd(dq[lo:hi], xe[lo:hi], a1[lo:hi], a3[lo:hi] if a3 is not None else None,
                            hh[lo:hi], w1[e], w3[e] if dw3 is not None else None, w2[e], act)
        dxe[lo:hi], dw1[e], dw2[e] = r[0], r[1], r[3]
        if dw3 is not None:
            dw3[e] = r[2]
    return dxe, dw1, dw3, dw2


# ----------------------------------------------------------------------------- backward of ordering and gate

def inverse_order_bwd(dy, q, topk_w, row_of):
    """dQ[row] = w * dy[t];  dw[t,j] = <dy[t], Q[row]>  (0 for dropped choices)."""
    n, k = row_of.shape
    dq = np.zeros_like(q, dtype=np.float64)
    dw = np.zeros((n, k), np.float64)
    for t in range(n):
        for j in range(k):
            r = row_of[t, j]
            if r >= 0:
                dq[r] = topk_w[t, j] * dy[t]
                dw[t, j] = float(np.dot(dy[t], q[r]))
    return dq, dw


def order_bwd(dxe, row_of, dy=None):
    """dx[t] = sum over kept j of dXe[row_of[t,j]]  (+ dy[t] for the residual)."""
    n, k = row_of.shape
    dx = np.zeros((n, dxe.shape[1]), np.float64)
    for t in range(n):
        for j in range(k):
            r = row_of[t, j]
            if r >= 0:
                dx[t] += dxe[r]
    if dy is not None:
        dx = dx + dy
    return dx


def gate_bwd(x, w_gate, logits, topk_idx, pos, dtopk_w, renormalize, has_bias):
    """Adjoint of the gate with the routing decision held fixed.

    g[t,e] = dw[t,j] at e = idx[t,j] for kept j, else 0.
    renormalize=0: dl = p * (g - <g,p>), p the softmax over all E.
    renormalize=1: the same formula on the k selected entries with p -> w; other entries 0.
    renormalize=2 (sigmoid gate): dl = g * p * (1 - p), p = sigma(logits): the choices do not interact.
    renormalize=3 (expert choice): slot j of a token is expert j; dl = p * (g - sum over tokens of g * p), column-wise.
    Returns dlogits [N,E], dW_g [M,E], db_g [E] or None, and the gate's share of dx [N,M]."""
    n, k = topk_idx.shape
    e_cnt = logits.shape[1]
    g = np.zeros((n, e_cnt), np.float64)
    for t in range(n):
        for j in range(k):
            if pos[t, j] >= 0:
                g[t, topk_idx[t, j]] = dtopk_w[t, j]
    if renormalize == GATE_EXPERT_CHOICE:
        # the softmax runs over the tokens an expert kept (down a column), so the same Jacobian couples the
        # kept tokens of one expert instead of the kept experts of one token
        p = expert_choice_dense(logits, pos)
        dl = p * (g - (g * p).sum(axis=0, keepdims=True))
    else:
        p = gate_dense(logits, topk_idx, renormalize)
        if renormalize == GATE_SIGMOID:
            dl = g * p * (1.0 - p)
        else:
            dl = p * (g - (g * p).sum(axis=1, keepdims=True))
    dw_gate = x.T @ dl
    db_gate = dl.sum(axis=0) if has_bias else None
    return dl, dw_gate, db_gate, dl @ w_gate.T


def route_noisy(x, w_gate, b_gate, w_noise, noise, k, cap, renormalize, logit_dtype=np.float32):
    """route() with the noisy logits of Sec. 2.1 in place of I.W_g."""
    logits, nl = gate_logits_noisy(x, w_gate, b_gate, w_noise, noise, logit_dtype)
    idx = keep_top_k(logits, k)
    w = gate_weights(logits, idx, renormalize)
    pos, count, offsets, row_of, src_of_row = assign_positions(idx, w_gate.shape[1], cap)
    return dict(logits=logits, noise_logits=nl, probs=gate_dense(logits, idx, renormalize), topk_idx=idx, topk_w=w,
                pos=pos, count=count, offsets=offsets, row_of=row_of, src_of_row=src_of_row)


def gate_bwd_noisy(x, w_gate, w_noise, noise, noise_logits, logits, topk_idx, pos, dtopk_w, renormalize, has_bias):
    """Adjoint of the noisy gate with the routing decision and the noise draws held fixed.

    dH as in gate_bwd.  H = I.W_g + b + noise * Softplus(I.W_noise), Softplus' = sigma, so
    d(I.W_noise) = dH * noise * sigma(I.W_noise); each product then contributes x^T.d(.) to its weight and
    d(.).W^T to dx.  Returns dH, dW_g, db_g or None, dW_noise, and the gate's share of dx."""
    dl, dw_gate, db_gate, dx = gate_bwd(x, w_gate, logits, topk_idx, pos, dtopk_w, renormalize, has_bias)
    dn = dl * np.asarray(noise, np.float64) * sigmoid(noise_logits)
    return dl, dw_gate, db_gate, x.T @ dn, dx + dn @ w_noise.T


# ----------------------------------------------------------------------------- X-MoE gate (Sec. 2.1)

def unit_rows(v, axis):
    """v scaled to unit l2 length along `axis` (no epsilon: a zero vector has no direction and gives nan)."""
    v = np.asarray(v, np.float64)
    return v / np.sqrt((v * v).sum(axis=axis, keepdims=True))


def gate_logits_xmoe(x, w_proj, w_gate, logit_dtype=np.float32):
    """X-MoE routing scores of Sec. 2.1: the token is first projected to a low dimension D, projection and
    expert embeddings are l2-normalised, and s_i = cos(W_proj I, W_g[:, i]).

    Readings: w_proj is stored [M,D] and applied as I . W_proj (the same orientation as W_g [M,E] in H = I . W_g),
    w_gate is [D,E] with one expert embedding per column; no temperature and no epsilon (the formula has none).
    The projection is accumulated in fp64 and rounded once to fp32: it is an output, kept for the backward pass.
    The cosine is then formed in fp64 from that fp32 tensor and rounded once to fp32, and the top-k is taken on
    these scores.  Returns (s [N,E], projection [N,D])."""
    proj = gate_logits(x, w_proj, None, logit_dtype)
    s = unit_rows(proj, 1) @ unit_rows(w_gate, 0)
    return s.astype(logit_dtype), proj


def route_xmoe(x, w_proj, w_gate, k, cap, renormalize, logit_dtype=np.float32):
    """route() with the X-MoE scores in place of I.W_g; everything after the scores is unchanged."""
    logits, proj = gate_logits_xmoe(x, w_proj, w_gate, logit_dtype)
    idx = keep_top_k(logits, k)
    w = gate_weights(logits, idx, renormalize)
    pos, count, offsets, row_of, src_of_row = assign_positions(idx, w_gate.shape[1], cap)
    return dict(logits=logits, proj=proj, probs=gate_dense(logits, idx, renormalize), topk_idx=idx, topk_w=w,
                pos=pos, count=count, offsets=offsets, row_of=row_of, src_of_row=src_of_row)


def gate_bwd_xmoe(x, w_proj, w_gate, proj, logits, topk_idx, pos, dtopk_w, renormalize):
    """Adjoint of the X-MoE gate with the routing decision held fixed.

    ds as in gate_bwd.  s = pn . wn with pn = p / |p| (rows) and wn = w / |w| (columns), so the product gives
    d(pn) = ds . wn^T and d(wn) = pn^T . ds, and a unit-length scaling u = v / |v| has the adjoint
    dv = (du - u <u, du>) / |v|.  Then p = I . W_proj: dW_proj = x^T . dp, dx = dp . W_proj^T.
    Returns ds [N,E], dW_proj [M,D], dW_g [D,E], and the gate's share of dx [N,M]."""
    p = np.asarray(proj, np.float64)
    wg = np.asarray(w_gate, np.float64)
    pn, wn = unit_rows(p, 1), unit_rows(wg, 0)
    ds, dwn, _, dpn = gate_bwd(pn, wn, logits, topk_idx, pos, dtopk_w, renormalize, False)
    dp = (dpn - pn * (pn * dpn).sum(axis=1, keepdims=True)) / np.sqrt((p * p).sum(axis=1, keepdims=True))
    dwg = (dwn - wn * (wn * dwn).sum(axis=0, keepdims=True)) / np.sqrt((wg * wg).sum(axis=0, keepdims=True))
    x = np.asarray(x, np.float64)
    return ds, x.T @ dp, dwg, dp @ np.asarray(w_proj, np.float64).T


# ----------------------------------------------------------------------------- expert choice (Sec. 2.1)

def expert_choice_dense(logits, pos):
    """G^T as an [N,E] matrix for expert choice: down every column, the softmax over the tokens that expert
    kept (pos >= 0), zeros elsewhere."""
    l = np.asarray(logits, np.float64)
    p = np.zeros(l.shape, np.float64)
    for e in range(l.shape[1]):
        kept = np.asarray(pos)[:, e] >= 0
        if kept.any():
            z = np.exp(l[kept, e] - l[kept, e].max())
            p[kept, e] = z / z.sum()
    return p


def route_expert_choice(x, w_gate, b_gate, k_tokens, logit_dtype=np.float32):
    """Expert choice: G(I) = Softmax(KeepTopK((I.W_g)^T, k)): the logits are transposed, so KeepTopK runs along
    the tokens and every expert keeps its k_tokens largest (all N when k_tokens >= N); the softmax is over the
    kept logits of that expert, as printed.  Ties go to the earlier token.

    Layout, in the terms of the rest of the layer: a token has one slot per expert (topk_idx[t, j] = j), kept
    or not (pos = -1, weight 0); the rows of an expert are its kept tokens in token order."""
    logits = gate_logits(x, w_gate, b_gate, logit_dtype)
    n, e_cnt = logits.shape
    k = min(int(k_tokens), n)
    assert k >= 1
    kept = keep_top_k(logits.T, k)                 # [E,k] token indices, largest logit first
    w_kept = gate_weights(logits.T, kept, 1)       # Softmax over the kept logits of every expert
    pos = np.full((n, e_cnt), -1, np.int32)
    w = np.zeros((n, e_cnt), np.float64)
    for e in range(e_cnt):
        for p_, t in enumerate(sorted(int(t) for t in kept[e])):
            pos[t, e] = p_
        w[kept[e].astype(np.int64), e] = w_kept[e]
    count = np.full(e_cnt, k, np.int32)
    offsets = (np.arange(e_cnt + 1) * k).astype(np.int32)
    row_of = np.where(pos >= 0, offsets[None, :-1] + pos, -1).astype(np.int32)
    src_of_row = np.full(n * e_cnt, -1, np.int32)
    for t in range(n):
        for e in range(e_cnt):
            if row_of[t, e] >= 0:
                src_of_row[row_of[t, e]] = t * e_cnt + e
    topk_idx = np.tile(np.arange(e_cnt, dtype=np.int32), (n, 1))
    return dict(logits=logits, probs=w.copy(), topk_idx=topk_idx, topk_w=w, pos=pos, count=count, offsets=offsets,
                row_of=row_of, src_of_row=src_of_row)


# ----------------------------------------------------------------------------- whole layer

def route(x, w_gate, b_gate, k, cap, renormalize, logit_dtype=np.float32):
    if renormalize == GATE_EXPERT_CHOICE:
        assert k == w_gate.shape[1], "expert choice: a token has one slot per expert"
        return route_expert_choice(x, w_gate, b_gate, cap, logit_dtype)
    logits = gate_logits(x, w_gate, b_gate, logit_dtype)
    idx = keep_top_k(logits, k)
    w = gate_weights(logits, idx, renormalize)
    pos, count, offsets, row_of, src_of_row = assign_positions(idx, w_gate.shape[1], cap)
    return dict(logits=logits, probs=gate_dense(logits, idx, renormalize), topk_idx=idx, topk_w=w, pos=pos,
                count=count, offsets=offsets, row_of=row_of, src_of_row=src_of_row)


def layer_fwd(x, w_gate, b_gate, w1, w3, w2, k, cap, act, renormalize, add_residual, logit_dtype=np.float32):
    r = route(x, w_gate, b_gate, k, cap, renormalize, logit_dtype)
    xe = order(x, r["row_of"], int(r["offsets"][-1]))
    q, saved = expert_ffn(xe, r["offsets"], w1, w3, w2, act)
    y = inverse_order(q, r["topk_w"], r["row_of"], x if add_residual else None)
    r.update(xe=xe, q=q, saved=saved, y=y)
    return r


def layer_bwd(dy, x, w_gate, b_gate, w1, w3, w2, fwd, act, renormalize, add_residual):
    dq, dtopk_w = inverse_order_bwd(dy, fwd["q"], fwd["topk_w"], fwd["row_of"])
    dxe, dw1, dw3, dw2 = expert_ffn_bwd(dq, fwd["xe"], fwd["offsets"], w1, w3, w2, fwd["saved"], act)
    dx = order_bwd(dxe, fwd["row_of"], dy if add_residual else None)
    dl, dw_gate, db_gate, dx_gate = gate_bwd(x, w_gate, fwd["logits"], fwd["topk_idx"], fwd["pos"], dtopk_w,
                                             renormalize, b_gate is not None)
    return dict(dx=dx + dx_gate, dw_gate=dw_gate, db_gate=db_gate, dw1=dw1, dw3=dw3, dw2=dw2,
                dq=dq, dtopk_w=dtopk_w, dxe=dxe, dlogits=dl)


# ----------------------------------------------------------------------------- the layer in r chunks (Sec. 4.2)
# Sec. 4.2 / Fig. 5 cut the capacity dimension of the dispatched tensor into r parts that go through
# dispatch -> experts one after the other.  Rows are independent there, so the result is that of r = 1.

def chunk_bounds(offsets, r):
    """begin[c,e], end[c,e]: chunk c of r holds rows floor(c n / r) .. floor((c+1) n / r) - 1 of the n rows of expert e."""
    e_cnt = len(offsets) - 1
    begin = np.zeros((r, e_cnt), np.int64)
    end = np.zeros((r, e_cnt), np.int64)
    for e in range(e_cnt):
        lo, n = int(offsets[e]), int(offsets[e + 1]) - int(offsets[e])
        for c in range(r):
            begin[c, e] = lo + (c * n) // r
            end[c, e] = lo + ((c + 1) * n) // r
    return begin, end


def layer_fwd_chunked(x, w_gate, b_gate, w1, w3, w2, k, cap, act, renormalize, add_residual, r,
                      logit_dtype=np.float32):
    """layer_fwd with ordering and experts done chunk by chunk, in chunk order."""
    out = route(x, w_gate, b_gate, k, cap, renormalize, logit_dtype)
    n_rows = int(out["offsets"][-1])
    h = w1.shape[2]
    xe = np.zeros((n_rows, x.shape[1]))
    q = np.zeros((n_rows, x.shape[1]))
    a1 = np.zeros((n_rows, h))
    a3 = np.zeros((n_rows, h)) if act == ACT_SWIGLU else None
    hh = np.zeros((n_rows, h))
    begin, end = chunk_bounds(out["offsets"], r)
    for c in range(r):
        for e in range(len(out["offsets"]) - 1):
            lo, hi = int(begin[c, e]), int(end[c, e])
            if hi == lo:
                continue
            xe[lo:hi] = x[out["src_of_row"][lo:hi] // k]  # ordering function, these rows only
            qe, a1e, a3e, hhe = expert_rows_fwd(xe[lo:hi], w1[e], w3[e] if a3 is not None else None, w2[e], act)
            q[lo:hi], a1[lo:hi], hh[lo:hi] = qe, a1e, hhe
            if a3 is not None:
                a3[lo:hi] = a3e
    y = inverse_order(q, out["topk_w"], out["row_of"], x if add_residual else None)
    out.update(xe=xe, q=q, saved=(a1, a3, hh), y=y)
    return out


# ----------------------------------------------------------------------------- sampled evaluation for large shapes
# Given the (cheap, full) routing, rows are independent: outputs for a subset of tokens, and columns of
# the weight gradients for a subset of hidden units, follow from the same per-row definitions above.

def layer_tokens(tokens, x, dy, w_gate, route_out, expert_weight, act, renormalize, add_residual, has_bias):
    """y[t], dx[t], dtopk_w[t], dlogits[t] for the given tokens only.

    expert_weight(name, e) returns expert e's fp64 matrix ('w1' | 'w3' | 'w2')."""
    tokens = np.asarray(tokens)
    idx, w, row_of, pos = (route_out[n] for n in ("topk_idx", "topk_w", "row_of", "pos"))
    m = x.shape[1]
    k = idx.shape[1]
    y = np.zeros((len(tokens), m))
    dx = np.zeros((len(tokens), m))
    dtw = np.zeros((len(tokens), k))
    by_expert = {}
    for i, t in enumerate(tokens):
        for j in range(k):
            if row_of[t, j] >= 0:
                by_expert.setdefault(int(idx[t, j]), []).append((i, int(t), j))
    for e, items in sorted(by_expert.items()):
        w1 = expert_weight("w1", e)
        w3 = expert_weight("w3", e) if act == ACT_SWIGLU else None
        w2 = expert_weight("w2", e)
        ii = np.array([a[0] for a in items]); tt = np.array([a[1] for a in items]); jj = np.array([a[2] for a in items])
        xr = x[tt]
        q, a1, a3, hh = expert_rows_fwd(xr, w1, w3, w2, act)
        gw = w[tt, jj]
        np.add.at(y, ii, gw[:, None] * q)
        dtw[ii, jj] = np.einsum("rm,rm->r", dy[tt], q)
        dq = gw[:, None] * dy[tt]
        dxe = expert_rows_bwd(dq, xr, a1, a3, hh, w1, w3, w2, act)[0]
        np.add.at(dx, ii, dxe)
    if add_residual:
        y += x[tokens]
        dx += dy[tokens]
    sub = {n: route_out[n][tokens] for n in ("logits", "topk_idx", "pos")}
    dl, _, _, dx_gate = gate_bwd(x[tokens], w_gate, sub["logits"], sub["topk_idx"], sub["pos"], dtw,
                                 renormalize, has_bias)
    return dict(y=y, dx=dx + dx_gate, dtopk_w=dtw, dlogits=dl)


def expert_wgrad_columns(e, cols, x, dy, route_out, w1, w3, w2, act):
    """dW1[e][:, cols], dW3[e][:, cols], dW2[e][cols, :] over ALL rows of expert e.

    Needs only the pre-activations of the chosen hidden units: a1[:, cols] = Xe.W1[:, cols],
    dHh[:, cols] = dQ.W2[cols, :]^T."""
    offsets, src = route_out["offsets"], route_out["src_of_row"]
    k = route_out["topk_idx"].shape[1]
    lo, hi = int(offsets[e]), int(offsets[e + 1])
    s = src[lo:hi].astype(np.int64)
    t, j = s // k, s % k
    xr = x[t]
    dq = route_out["topk_w"][t, j][:, None] * dy[t]
    a1 = xr @ w1[:, cols]
    dhh = dq @ w2[cols, :].T
    if act == ACT_SWIGLU:
        a3 = xr @ w3[:, cols]
        hh = silu(a1) * a3
        da1 = dhh * a3 * silu_grad(a1)
        da3 = dhh * silu(a1)
        return xr.T @ da1, xr.T @ da3, hh.T @ dq
    hh = activation(a1, act)
    da1 = dhh * activation_grad(a1, act)
    return xr.T @ da1, None, hh.T @ dq
