"""Pipeline-degree selection (FSMoE Sec. 4): pins of the oracle against what the paper and the mathematics
fix, then the library's host functions against the oracle.  No GPU is involved (host code only)."""
import itertools
import math
import random

import pytest

import paper_2501_10714_amd as moe
from oracle import pipeline_oracle as P


def model(**kw):
    base = dict(alpha_a2a=0.0, beta_a2a=0.0, n_a2a=0.0, alpha_ag=0.0, beta_ag=0.0, n_ag=0.0, alpha_rs=0.0, beta_rs=0.0,
                n_rs=0.0, alpha_exp=0.0, beta_exp=0.0, n_exp=0.0, t_gar=0.0)
    base.update(kw)
    return P.Model(**base)


def random_model(g):
    # start-up times of 1..100 us, per-unit times and sizes spanning regimes where each case occurs
    u = lambda lo, hi: math.exp(g.uniform(math.log(lo), math.log(hi)))
    return P.Model(u(1, 100), u(1e-4, 1e-1), u(1e2, 1e6), u(1, 100), u(1e-4, 1e-1), u(1e2, 1e6), u(1, 100), u(1e-4, 1e-1),
                   u(1e2, 1e6), u(1, 100), u(1e-4, 1e-1), u(1e2, 1e6), g.choice([0.0, u(1, 1e5)]))


# ----------------------------------------------------------------------------- pins of the oracle

def test_closed_forms_two_printed_forms_agree():
    """Sec. 4.2 prints every t^moe_i twice (in chunk times, and with alpha, beta, n written out)."""
    g = random.Random(1)
    for _ in range(200):
        m = random_model(g)
        for r, c in itertools.product((1, 2, 3, 7, 16), (1, 2, 3, 4)):
            assert P.case_time(m, r, c) == pytest.approx(P.case_time_expanded(m, r, c), rel=1e-12)


def test_the_four_constraint_sets_partition_every_degree():
    """Every truth assignment of Q1..Q7 satisfies exactly one of the four constraint sets."""
    g = random.Random(2)
    seen = set()
    for _ in range(3000):
        m = random_model(g)
        for r in (1, 2, 5, 32):
            c = P.case_constraints(m, r)
            assert sum(c.values()) == 1
            seen.add([k for k, v in c.items() if v][0])
    assert seen == {1, 2, 3, 4}      # the sampler reaches all four regimes


def test_worked_cases():
    # only AlltoAll costs anything: Q1 holds, experts never exceed it, no AllReduce -> Case 3, 2 r t_a2a
    m = model(alpha_a2a=10.0, beta_a2a=0.01, n_a2a=1000.0)
    assert P.case_constraints(m, 4) == {1: False, 2: False, 3: True, 4: False}
    assert P.case_time(m, 4, 3) == pytest.approx(2 * 4 * (10.0 + 2.5))
    # one GPU: no communication at all -> Case 2 for every r, t = r alpha_exp + n beta: chunking only adds start-ups
    m = model(alpha_exp=5.0, beta_exp=0.002, n_exp=1e6)
    for r in (1, 2, 8):
        assert P.case_constraints(m, r)[2]
        assert P.case_time(m, r, 2) == pytest.approx(r * 5.0 + 2000.0)
    assert P.find_optimal_pipeline_degree(m, 16) == (1, pytest.approx(2005.0), 2)
    # a Gradient-AllReduce longer than everything else -> Case 1, and Case 1 grows with r: the best degree is 1
    m = model(alpha_a2a=10.0, beta_a2a=0.01, n_a2a=1000.0, alpha_exp=5.0, beta_exp=0.001, n_exp=1000.0, t_gar=1e6)
    r, t, c = P.find_optimal_pipeline_degree(m, 16)
    assert (r, c) == (1, 1) and t == pytest.approx(2 * 20.0 + 1e6)
    # intra-node collectives dominate -> Case 4
    m = model(alpha_ag=50.0, beta_ag=0.1, n_ag=1e4, alpha_rs=50.0, beta_rs=0.1, n_rs=1e4, alpha_a2a=1.0, beta_a2a=1e-4,
              n_a2a=100.0, alpha_exp=1.0, beta_exp=1e-4, n_exp=100.0)
    assert P.case_constraints(m, 2)[4]


@pytest.mark.parametrize("case", [2, 3, 4])
def test_interior_optimum_is_next_to_the_stationary_point(case):
    """f_2, f_3, f_4 have the form A r + B / r + C (convex): on a stretch of degrees that all fall into that
    case, the best integer degree is floor or ceil of sqrt(B / A)."""
    if case == 2:    # experts dominate; B = 2 n_a2a beta_a2a + n_ag beta_ag + n_rs beta_rs, A = alpha_exp
        m = model(alpha_a2a=1.0, beta_a2a=0.02, n_a2a=2e4, alpha_ag=1.0, beta_ag=0.01, n_ag=1e4, alpha_rs=1.0, beta_rs=0.01,
                  n_rs=1e4, alpha_exp=20.0, beta_exp=1.0, n_exp=1e5)
        a, b = m.alpha_exp, 2 * m.n_a2a * m.beta_a2a + m.n_ag * m.beta_ag + m.n_rs * m.beta_rs
    elif case == 3:  # AlltoAll dominates; B = n_ag beta_ag + n_rs beta_rs, A = 2 alpha_a2a
        m = model(alpha_a2a=2.0, beta_a2a=1.0, n_a2a=1e4, alpha_ag=0.5, beta_ag=0.05, n_ag=1e4, alpha_rs=0.5, beta_rs=0.05,
                  n_rs=1e4, alpha_exp=0.1, beta_exp=1e-4, n_exp=1e3)
        a, b = 2 * m.alpha_a2a, m.n_ag * m.beta_ag + m.n_rs * m.beta_rs
    else:            # AllGather / ReduceScatter dominate; B = 2 n_a2a beta_a2a, A = alpha_ag + alpha_rs
        m = model(alpha_a2a=0.1, beta_a2a=0.01, n_a2a=1e5, alpha_ag=5.0, beta_ag=1.0, n_ag=1e4, alpha_rs=5.0, beta_rs=1.0,
                  n_rs=1e4, alpha_exp=0.1, beta_exp=1e-4, n_exp=1e3)
        a, b = m.alpha_ag + m.alpha_rs, 2 * m.n_a2a * m.beta_a2a
    r_max = 64
    # (at r = 1 nothing overlaps and Q2, Q3 hold whenever experts cost anything, so r = 1 is Case 1 or 2)
    assert all(P.case_constraints(m, r)[case] for r in range(2, r_max + 1))
    r, t = P.solve(m, case, r_max)
    star = math.sqrt(b / a)
    assert 2 < star < r_max and r in (math.floor(star), math.ceil(star))
    assert t == pytest.approx(a * r + b / r + (P.case_time(m, 1, case) - a - b), rel=1e-12)


def test_algorithm_equals_exhaustive_search():
    """Algorithm 1 (four constrained solves, then arg-min) finds what trying every degree finds."""
    g = random.Random(3)
    for _ in range(500):
        m = random_model(g)
        r_max = g.choice([1, 4, 32])
        best = min(((sum(P.case_time(m, r, c) for c in (1, 2, 3, 4) if P.case_constraints(m, r)[c]), r)
                    for r in range(1, r_max + 1)))
        r, t, _ = P.find_optimal_pipeline_degree(m, r_max)
        assert t == pytest.approx(best[0], rel=1e-14) and r == best[1]


# ----------------------------------------------------------------------------- the library against the oracle

def to_c(m):
    return moe.PipelineModel(*m)


def test_library_matches_oracle():
    g = random.Random(4)
    cases = set()
    for _ in range(1000):
        m = random_model(g)
        cm = to_c(m)
        for r in (1, 2, 3, 8, 33):
            t, c = moe.moe_pipeline_time(cm, r)
            want_c = [k for k, v in P.case_constraints(m, r).items() if v][0]
            assert c == want_c
            assert t == pytest.approx(P.case_time(m, r, want_c), rel=1e-13)
        r_max = g.choice([1, 5, 64])
        got = moe.moe_find_pipeline_degree(cm, r_max)
        want = P.find_optimal_pipeline_degree(m, r_max)
        assert got[0] == want[0] and got[2] == want[2] and got[1] == pytest.approx(want[1], rel=1e-13)
        cases.add(got[2])
    assert cases == {1, 2, 3, 4}


def test_library_rejects_bad_arguments():
    m = to_c(model(alpha_exp=1.0))
    with pytest.raises(moe.MoeError):
        moe.moe_find_pipeline_degree(m, 0)
    bad = to_c(model(alpha_exp=-1.0))
    with pytest.raises(moe.MoeError):
        moe.moe_find_pipeline_degree(bad, 4)
    assert math.isnan(moe.moe_pipeline_time(bad, 2)[0])
    assert math.isnan(moe.moe_pipeline_time(m, 0.5)[0])
