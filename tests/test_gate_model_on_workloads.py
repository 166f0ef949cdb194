"""The matrix-core gate end to end as a CPU model, on the five workloads' own inputs (their d_model, experts, k, bias
and value distributions; a sample of the tokens).

Fast pass as the kernel states it (csrc/gate_mfma.hip): exact bf16 x bf16 products, fp32 sums inside chains of 64 k,
fp64 sum of the chains, fp32 norms, eps = 7.71e-6 * |x_t| * max_e |w_e|; then the kernel's decision rule and the repair
(tests/test_gate_decision_rule.py holds the same rule against adversarial perturbations).  Checked: the routing equals
the oracle's top-k on every sampled token; the fast pass stays within eps / 8 of the exact logits (the margin the GPU
parity tests hold the kernel to); only a small share of the tokens needs a repair.  The order of the additions inside a
chain is the hardware's own and not documented; the model adds in numpy's order, which is as good as any other."""
import numpy as np
import pytest

import moe_synth as S
from oracle import moe_oracle as O
from test_gate_decision_rule import rule

N_SAMPLE = 1024


def fast_pass(x, w):
    """x [n, M], w [M, E] fp64 arrays holding bf16 values -> approximate fp32 logits (before the bias) and eps per token."""
    n, M = x.shape
    pad = (-M) % 64
    x32 = np.pad(x, ((0, 0), (0, pad))).astype(np.float32)
    w32 = np.pad(w, ((0, pad), (0, 0))).astype(np.float32)
    acc = np.zeros((n, w.shape[1]), np.float64)
    for c in range(0, M + pad, 64):
        acc += (x32[:, c:c + 64] @ w32[c:c + 64, :]).astype(np.float32)  # one chain: fp32 sums of 64 exact products
    nx = (x32 * x32).sum(1, dtype=np.float32)
    nw = (w32 * w32).sum(0, dtype=np.float32)
    eps = np.float32(7.71e-6) * np.sqrt(nx * nw.max())
    return acc, eps


@pytest.mark.parametrize("name", ["tiny", "gpt2", "mixtral", "finegrained", "switch"])
def test_model_of_the_gate_routes_like_the_oracle(name):
    full = S.WORKLOADS[name]
    w = S.scaled(full, N=min(full.N, N_SAMPLE))
    x = S.to_f64(S.draw_x(w)) if w.dtype == S.DT_BF16 else S.to_f64(S.f32_to_bf16_bits(S.draw_x(w)))
    wg_raw = S.draw_w_gate(w)
    wg = S.to_f64(wg_raw) if w.dtype == S.DT_BF16 else S.to_f64(S.f32_to_bf16_bits(wg_raw))
    b = S.draw_b_gate(w)
    b64 = None if b is None else np.asarray(b, np.float64)
    exact = O.gate_logits(x, wg, b64)                       # fp32 roundings of the fp64 sums: what a repair writes
    want = O.keep_top_k(exact, w.k)
    acc, eps = fast_pass(x, wg)
    approx = (acc + (0.0 if b64 is None else b64)).astype(np.float32)
    err = np.abs(approx.astype(np.float64) - (x @ wg + (0.0 if b64 is None else b64)))
    assert (err <= eps[:, None] / 8 + 2.0 ** -23 * np.abs(exact)).all(), float((err / eps[:, None]).max())
    repaired = 0
    for t in range(w.N):
        got, marked = rule(approx[t], exact[t], float(eps[t]), w.k)
        repaired += bool(marked)
        assert got == list(want[t]), (t, marked)
    assert repaired <= 0.05 * w.N, repaired
