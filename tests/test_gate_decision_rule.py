"""The decision rule of the matrix-core gate, checked on the CPU with a model of the kernel's logic.

The kernel decides the top-k on approximate logits a[e] that differ from the exact ones t[e] by at most eps, recomputes
exactly (a) both members of every close pair of neighbours among the k selected and (b), when an unselected expert is
within reach of the k-th selected value, all experts within reach together with the k-th selected one, and decides again.
The claim: the second decision equals the decision on the exact values, for ANY perturbation within the bound.  This
test draws exact logits with many near-ties, perturbs them adversarially and at random within eps, runs the rule as
the kernel states it (csrc/gate_mfma.hip), and compares with the top-k of the exact values (ties: lower index)."""
import numpy as np
import pytest


def exact_topk(t, k):
    order = sorted(range(len(t)), key=lambda e: (-t[e], e))
    return order[:k]


def select(vals, k):
    """Repeated arg-max with the lower index winning ties, as every gate kernel selects."""
    sel, prev_v, prev_e = [], None, -1
    for j in range(k):
        be, bv = -1, 0.0
        for e, v in enumerate(vals):
            eligible = j == 0 or v < prev_v or (v == prev_v and e > prev_e)
            if eligible and (be < 0 or v > bv):
                be, bv = e, v
        sel.append(be)
        prev_v, prev_e = bv, be
    return sel


def rule(a, t32, eps, k):
    """a: approximate fp32 logits; t32: the exact logits rounded to fp32 (what a repair writes)."""
    a = np.asarray(a, np.float32).copy()
    sel = select(a, k)
    selv = [a[e] for e in sel]
    marked = set()
    for j in range(k - 1):
        x, y = np.float32(selv[j]), np.float32(selv[j + 1])
        thr = np.float32(2.0 * eps + 2.4e-7 * (abs(x) + abs(y)))
        if not (x - y > thr):
            marked.update((sel[j], sel[j + 1]))
    vk = np.float32(selv[k - 1])
    zone = vk - np.float32(2.0 * eps + 4.8e-7 * abs(vk))
    within = {e for e in range(len(a)) if not (a[e] < zone)} - set(sel)
    if within:
        marked |= within | {sel[k - 1]}
    for e in marked:
        a[e] = t32[e]
    return (select(a, k) if marked else sel), marked


@pytest.mark.parametrize("E,k", [(8, 2), (8, 1), (16, 4), (64, 6), (5, 5), (32, 1)])
def test_rule_reproduces_the_exact_top_k(E, k):
    rng = np.random.default_rng(1000 * E + k)
    eps = 1e-3
    n_marked = 0
    for trial in range(1500):
        t = rng.normal(size=E)
        # plant clusters of near-ties at the scale of eps: pairs, triples, chains across the k-th place
        for _ in range(rng.integers(0, 4)):
            src = rng.integers(E)
            for dst in rng.choice(E, size=rng.integers(1, 4), replace=False):
                t[dst] = t[src] + rng.uniform(-3, 3) * eps * rng.choice([0.0, 0.01, 0.3, 1.0, 2.0])
        t32 = t.astype(np.float32)
        want = exact_topk(t32.tolist(), k)          # the oracle decides on fp32-rounded exact logits
        for mode in range(4):
            if mode == 0:
                d = rng.uniform(-eps, eps, size=E)
            elif mode == 1:                           # push neighbours in the exact order towards each other
                order = np.argsort(-t)
                d = np.zeros(E)
                d[order[::2]] = -eps
                d[order[1::2]] = eps
            elif mode == 2:
                d = rng.choice([-eps, eps], size=E)
            else:
                d = np.zeros(E)
            a = (t + 0.999 * d).astype(np.float32)  # |a - t| <= eps also after the rounding to fp32
            got, marked = rule(a, t32, eps, k)
            n_marked += bool(marked)
            assert got == want, (trial, mode, t, a, marked)
    assert n_marked > 100                             # the repair path was exercised


def test_rule_marks_nothing_when_gaps_are_clear():
    a = np.array([3.0, 1.0, 2.0, -1.0, 0.0], np.float32)
    got, marked = rule(a, a, 1e-3, 2)
    assert got == [0, 2] and not marked


def test_rule_with_exact_ties_goes_to_the_lower_index():
    t = np.array([1.0, 2.0, 2.0, 0.5, 2.0], np.float64)
    a = (t + np.array([0, -1e-4, 1e-4, 0, 3e-4])).astype(np.float32)
    got, marked = rule(a, t.astype(np.float32), 1e-3, 2)
    assert got == [1, 2] and {1, 2, 4} <= marked
