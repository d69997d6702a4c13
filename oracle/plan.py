"""Oracle for the lower level of the parallelization planner: TEST INFRASTRUCTURE, not a product path.

Plain, slow, obviously correct: the integer programs of Sec. 4.2 (Eq. 2: layers per stage of one pipeline;
Eq. 3: micro-batches per pipeline; Eq. 1: both together) are solved by enumerating EVERY assignment, and the
relaxed problem behind Theorem 2 (Sec. 4.3.1) is solved as a linear program.  Only tests, the smoke test and the
benchmark's CPU-baseline leg may import this module; it shares no code with the library.
"""
import itertools

import numpy as np


def compositions(total, parts, caps=None):
    """Every tuple of `parts` non-negative integers summing to `total` (each at most its cap, if given)."""
    if parts == 1:
        if caps is None or caps[0] is None or total <= caps[0]:
            yield (total,)
        return
    hi = total if caps is None or caps[0] is None else min(total, caps[0])
    for first in range(hi + 1):
        for rest in compositions(total - first, parts - 1, None if caps is None else caps[1:]):
            yield (first,) + rest


def layers_bruteforce(y, L, caps=None):
    """Eq. 2: the minimum over all l in N0^n with sum L (and l_j <= cap_j) of max_j y_j l_j, and every minimiser."""
    best, arg = None, []
    for l in compositions(L, len(y), caps):
        v = max(yj * lj for yj, lj in zip(y, l))
        if best is None or v < best:
            best, arg = v, [l]
        elif v == best:
            arg.append(l)
    return best, arg


def microbatches_bruteforce(o, n_mb):
    """Eq. 3: the minimum over all m in N0^dp with sum n_mb of max_i o_i m_i, and every minimiser."""
    return layers_bruteforce(o, n_mb)


def lower_level_bruteforce(pipelines, L, n_mb, tau=1.0):
    """Eq. 1 for fixed pipelines (a list of lists of stage rates), by enumerating the JOINT assignment space: every
    combination of one layer split per pipeline and one micro-batch split.  Returns the minimum of
    max_i (max_j y_ij l_ij) m_i tau.  Exponential: tiny inputs only."""
    per_pipe = [list(compositions(L, len(y))) for y in pipelines]
    best = None
    for m in compositions(n_mb, len(pipelines)):
        for ls in itertools.product(*per_pipe):
            v = max(max(yj * lj for yj, lj in zip(y, l)) * mi for y, l, mi in zip(pipelines, ls, m)) * tau
            if best is None or v < best:
                best = v
    return best


def relaxed_time(y, L=1.0):
    """The relaxed problem of Theorem 2 for one set of groups: real-valued l_j >= 0, sum l_j = L, minimise the
    bottleneck t >= y_j l_j, as a linear program (variables l_1..l_n, t)."""
    from scipy.optimize import linprog
    n = len(y)
    c = np.zeros(n + 1)
    c[-1] = 1.0
    a_ub = np.zeros((n, n + 1))
    for j in range(n):
        a_ub[j, j] = y[j]
        a_ub[j, -1] = -1.0
    a_eq = np.ones((1, n + 1))
    a_eq[0, -1] = 0.0
    res = linprog(c, A_ub=a_ub, b_ub=np.zeros(n), A_eq=a_eq, b_eq=[L], bounds=[(0, None)] * (n + 1), method="highs")
    assert res.status == 0
    return float(res.x[-1])


def sorted_loads(y, l):
    return tuple(sorted((yj * lj for yj, lj in zip(y, l)), reverse=True))


def split_groups_bruteforce(x, sizes, rho):
    """Group splitting (Sec. 4.3.1, Appendix B.7) without the appendix's proposition: EVERY assignment of the GPUs to
    groups of the given sizes; returns the largest sum over groups of 1 / (rho_g * max x in the group)."""
    n = len(x)
    assert sum(sizes) == n
    best = None

    def rec(g, free, acc):
        nonlocal best
        if g == len(sizes):
            if best is None or acc > best:
                best = acc
            return
        for members in itertools.combinations(sorted(free), sizes[g]):
            rec(g + 1, free - set(members), acc + 1.0 / (rho[g] * max(x[i] for i in members)))
    rec(0, set(range(n)), 0.0)
    return best


def consecutive_run_candidates(n, sizes):
    """The candidate groupings of Appendix B.7 for GPUs already sorted by descending rate: one tuple of index runs per
    order of the groups."""
    out = []
    for order in sorted(set(itertools.permutations(range(len(sizes))))):
        at, runs = 0, [None] * len(sizes)
        for g in order:
            runs[g] = tuple(range(at, at + sizes[g]))
            at += sizes[g]
        out.append(tuple(runs))
    return out
