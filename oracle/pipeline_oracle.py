"""Oracle for the pipeline-degree selection of FSMoE Sec. 4 (test infrastructure only; plain Python floats).

Written from Sec. 4.1 (linear performance models, Eq. 1), Sec. 4.2 (conditions Q1..Q7, Cases 1..4 with
their closed forms and constraint sets) and Sec. 4.3 (Algorithm 1, FindOptimalPipelineDegree), in the
paper's order and notation.  Reading: the degree r is a number of chunks, hence an integer, and
solve(f_i) is carried out by trying every degree 1..r_max that satisfies case i's constraint (exact),
where the paper runs SLSQP on a real-valued r.  Only tests may import this file.
"""
import math
from collections import namedtuple

Model = namedtuple("Model", "alpha_a2a beta_a2a n_a2a alpha_ag beta_ag n_ag alpha_rs beta_rs n_rs "
                            "alpha_exp beta_exp n_exp t_gar")


def chunk_times(m, r):
    """Sec. 4.1, Eq. (1): t_{a2a,r}, t_{ag,r}, t_{rs,r}, t_{exp,r}."""
    return (m.alpha_a2a + m.n_a2a / r * m.beta_a2a, m.alpha_ag + m.n_ag / r * m.beta_ag,
            m.alpha_rs + m.n_rs / r * m.beta_rs, m.alpha_exp + m.n_exp / r * m.beta_exp)


def conditions(m, r):
    """Q1..Q7 of Sec. 4.2 as a dict of booleans."""
    a2a, ag, rs, ex = chunk_times(m, r)
    return {
        1: a2a > ag,
        2: r * ex > 2 * (r - 1) * a2a,
        3: r * ex > (r - 1) * (ag + rs),
        4: m.t_gar > ag + rs,
        5: m.t_gar > r * ex - 2 * (r - 1) * a2a + ag + rs,
        6: m.t_gar > r * ag + r * rs - 2 * (r - 1) * a2a,
        7: m.t_gar > ag + rs + r * ex - 2 * (r - 1) * a2a,
    }


def case_constraints(m, r):
    """The constraint set of each of the four minimisation problems of Sec. 4.2, as printed."""
    q = conditions(m, r)
    return {
        1: (q[1] and not q[2] and q[4]) or (q[1] and q[2] and q[5]) or (not q[1] and not q[3] and q[6])
           or (not q[1] and q[3] and q[7]),
        2: (q[1] and q[2] and not q[5]) or (not q[1] and q[3] and not q[7]),
        3: q[1] and not q[2] and not q[4],
        4: not q[1] and not q[3] and not q[6],
    }


def case_time(m, r, case):
    """f_1..f_4 of Sec. 4.2 in their first printed form (in terms of the chunk times)."""
    a2a, ag, rs, ex = chunk_times(m, r)
    if case == 1:
        return 2 * r * a2a + m.t_gar
    if case == 2:
        return 2 * a2a + ag + rs + r * ex
    if case == 3:
        return 2 * r * a2a + ag + rs
    return 2 * a2a + r * ag + r * rs


def case_time_expanded(m, r, case):
    """The same four functions in their second printed form (alpha, beta, n written out)."""
    if case == 1:
        return 2 * r * m.alpha_a2a + 2 * m.n_a2a * m.beta_a2a + m.t_gar
    if case == 2:
        return (2 * m.alpha_a2a + 2 * m.n_a2a / r * m.beta_a2a + m.alpha_ag + m.n_ag / r * m.beta_ag + m.alpha_rs
                + m.n_rs / r * m.beta_rs + r * m.alpha_exp + m.n_exp * m.beta_exp)
    if case == 3:
        return (2 * r * m.alpha_a2a + 2 * m.n_a2a * m.beta_a2a + m.alpha_ag + m.n_ag / r * m.beta_ag + m.alpha_rs
                + m.n_rs / r * m.beta_rs)
    return (2 * m.alpha_a2a + 2 * m.n_a2a / r * m.beta_a2a + r * m.alpha_ag + m.n_ag * m.beta_ag + r * m.alpha_rs
            + m.n_rs * m.beta_rs)


def solve(m, case, r_max):
    """solve(f_case): the best degree in 1..r_max among those that satisfy the case's constraint.
    Returns (r, t) or (None, inf) when no degree does."""
    best_r, best_t = None, math.inf
    for r in range(1, r_max + 1):
        if case_constraints(m, r)[case]:
            t = case_time(m, r, case)
            if t < best_t:
                best_r, best_t = r, t
    return best_r, best_t


def find_optimal_pipeline_degree(m, r_max):
    """Algorithm 1: the four solves, then the arg-min of the four minima.  Returns (r, t_moe, case)."""
    candidates = [solve(m, c, r_max) for c in (1, 2, 3, 4)]
    best = None
    for c, (r, t) in zip((1, 2, 3, 4), candidates):
        if r is not None and (best is None or t < best[1] or (t == best[1] and r < best[0])):
            best = (r, t, c)
    return best
