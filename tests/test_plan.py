"""The planner's lower level (include/mls_plan.h): the brute-force oracle against what the paper prints and the
mathematics fix, then the library against the oracle.  Host code only: no GPU needed."""
import math
import random

import pytest

from oracle import plan as oplan


# ---------------------------------------------------------------- the oracle against the paper and the mathematics
def test_oracle_microbatch_split_of_the_110b_case_study():
    """Sec. 7.3, Table 4, 110B under S4: the two pipelines' heaviest stages hold 21 and 22 layers on groups of the
    same kind and B/b = 64; the printed micro-batch split is (33, 31)."""
    best, arg = oplan.microbatches_bruteforce([21.0, 22.0], 64)
    assert arg == [(33, 31)] and best == 21.0 * 33


def test_oracle_microbatch_split_of_the_32b_case_study():
    """Sec. 7.3, Table 4, 32B under S5 (level-1 stragglers x = 2.62): bottlenecks 17 layers on a straggling pair,
    max(7 layers on a straggling pair, 18 on a healthy pair), 15 and 15; the printed split is (7, 17, 20, 20)."""
    o = [17 * 2.62, max(7 * 2.62, 18.0), 15.0, 15.0]
    best, arg = oplan.microbatches_bruteforce(o, 64)
    assert (7, 17, 20, 20) in arg and len(arg) == 1


def test_oracle_layer_split_of_the_110b_second_pipeline():
    """Table 4, 110B under S4, second pipeline: three pairs and three full nodes share 80 layers as (4, 5, 5, 22,
    22, 22).  With rates inversely proportional to the group size that split has bottleneck 22/8; any split with a
    smaller or equal bottleneck keeps every stage at or below floor((22/8) / y_j) layers, so enumerating under
    those caps covers all of them."""
    y = [1 / 2, 1 / 2, 1 / 2, 1 / 8, 1 / 8, 1 / 8]
    printed = (4, 5, 5, 22, 22, 22)
    assert max(a * b for a, b in zip(y, printed)) == 22 / 8
    best, arg = oplan.layers_bruteforce(y, 80, caps=[5, 5, 5, 22, 22, 22])
    assert best == 22 / 8 and printed in arg


def test_oracle_uniform_rates_give_the_uniform_plan():
    """Sec. 7.1: with all straggling rates 1 the plan is the uniform one."""
    best, arg = oplan.layers_bruteforce([1.0] * 4, 60)
    assert arg == [(15, 15, 15, 15)] and best == 15
    best, arg = oplan.microbatches_bruteforce([15.0] * 4, 64)
    assert arg == [(16, 16, 16, 16)]


def test_oracle_heavy_straggler_gets_zero_layers():
    """Sec. 4.2: a group whose rate is high enough is assigned no layers at all."""
    best, arg = oplan.layers_bruteforce([1.0, 1.0, 50.0], 12)
    assert arg == [(6, 6, 0)]


def test_oracle_capacity_limits_bind():
    """Eq. 2's memory constraint as a per-stage layer cap: a cap below the unconstrained share moves layers on."""
    best, arg = oplan.layers_bruteforce([1.0, 1.0, 1.0], 12, caps=[2, None, None])
    assert arg == [(2, 5, 5)]
    assert oplan.layers_bruteforce([1.0, 1.0], 12, caps=[2, 3])[0] is None  # cannot hold 12 layers


def test_oracle_joint_problem_separates():
    """Sec. 4.2: solving Eq. 2 per pipeline and then Eq. 3 equals the joint optimum of Eq. 1 (enumerated jointly)."""
    rng = random.Random(7)
    for _ in range(12):
        pipes = [[rng.choice([1.0, 1.0, 1.5, 2.62, 3.8]) * rng.choice([1.0, 0.5]) for _ in range(rng.randint(1, 3))]
                 for _ in range(rng.randint(1, 3))]
        L, n_mb = rng.randint(1, 6), rng.randint(0, 7)
        joint = oplan.lower_level_bruteforce(pipes, L, n_mb, tau=0.5)
        o = [oplan.layers_bruteforce(p, L)[0] for p in pipes]
        split = oplan.microbatches_bruteforce(o, n_mb)[0] * 0.5
        assert joint == pytest.approx(split, rel=1e-12)


def test_oracle_relaxed_problem_matches_theorem_2():
    """Theorem 2: under the relaxation the best time of a grouping is proportional to 1 / sum(1/y), so the ratio of
    two groupings is (sum 1/y'') / (sum 1/y').  The linear program knows nothing of that formula."""
    y1, y2 = [1.0, 1.0, 2.62, 0.5], [0.25, 3.8, 1.0]
    ratio = oplan.relaxed_time(y1) / oplan.relaxed_time(y2)
    assert ratio == pytest.approx(sum(1 / v for v in y2) / sum(1 / v for v in y1), rel=1e-9)


# ---------------------------------------------------------------- the library against the paper's printed values
def test_library_reproduces_the_case_studies():
    import paper_2410_13333_amd as mls
    m, t = mls.plan_microbatches([21.0, 22.0], 64)
    assert m == [33, 31] and t == 21.0 * 33
    m, _ = mls.plan_microbatches([17 * 2.62, max(7 * 2.62, 18.0), 15.0, 15.0], 64)
    assert m == [7, 17, 20, 20]
    l, o = mls.plan_layers([1 / 2, 1 / 2, 1 / 2, 1 / 8, 1 / 8, 1 / 8], 80)
    assert o == 22 / 8 and sorted(l) == [4, 5, 5, 22, 22, 22]  # the printed split, up to which pair holds 4


def test_library_theoretic_optimum_matches_table_3():
    """Sec. 7.2, Table 3, column R_opt: 110B under S4 on 64 GPUs (x = 5.42, 3.75, 2.57) prints 1.04; 32B under S5
    on 32 GPUs (eight x = 2.62 and one x = 3.8) prints 1.22."""
    import paper_2410_13333_amd as mls
    # the straggling rates are printed with two decimals, and so are the ratios
    assert abs(mls.theoretic_slowdown(64, [5.42, 3.75, 2.57]) - 1.04) < 0.006
    assert abs(mls.theoretic_slowdown(32, [2.62] * 8 + [3.8]) - 1.22) < 0.006
    assert mls.theoretic_slowdown(8, []) == 1.0
    assert math.isnan(mls.theoretic_slowdown(2, [1.5, 2.0, 3.0]))


# ---------------------------------------------------------------- the library against the oracle
def _rates(rng, n):
    return [rng.choice([1.0, 1.0, 1.0, 1.31, 2.62, 3.8, 5.42, 40.0]) * rng.choice([1.0, 0.5, 0.25, 0.125]) for _ in range(n)]


def test_library_layer_split_equals_enumeration():
    import paper_2410_13333_amd as mls
    rng = random.Random(11)
    for case in range(300):
        n = rng.randint(1, 5)
        y, L = _rates(rng, n), rng.randint(0, 14)
        caps = [rng.choice([None, None, rng.randint(0, 6)]) for _ in range(n)] if case % 3 == 0 else None
        best, arg = oplan.layers_bruteforce(y, L, caps)
        if best is None:
            with pytest.raises(mls.MlsError) as e:
                mls.plan_layers(y, L, caps)
            assert e.value.code == -3
            continue
        l, o = mls.plan_layers(y, L, caps)
        assert o == best and tuple(l) in arg
        # the documented tie rule: among the optima, the smallest sum of loads
        assert sum(a * b for a, b in zip(y, l)) == pytest.approx(min(sum(a * b for a, b in zip(y, c)) for c in arg), rel=1e-12)


def test_library_microbatch_split_and_lower_level_equal_enumeration():
    import paper_2410_13333_amd as mls
    rng = random.Random(13)
    for _ in range(100):
        o = [r * rng.randint(1, 30) for r in _rates(rng, rng.randint(1, 5))]
        n_mb = rng.randint(0, 16)
        best, arg = oplan.microbatches_bruteforce(o, n_mb)
        m, t = mls.plan_microbatches(o, n_mb)
        assert t == best and tuple(m) in arg
    for _ in range(20):
        pipes = [_rates(rng, rng.randint(1, 3)) for _ in range(rng.randint(1, 3))]
        L, n_mb, tau = rng.randint(1, 6), rng.randint(0, 7), 5.5e-3
        ls, m, t = mls.plan_lower_level(pipes, L, n_mb, tau)
        assert all(sum(l) == L for l in ls) and sum(m) == n_mb
        assert t == pytest.approx(oplan.lower_level_bruteforce(pipes, L, n_mb, tau), rel=1e-12)
        assert t == pytest.approx(tau * max(max(y * k for y, k in zip(p, l)) * mi for p, l, mi in zip(pipes, ls, m)))


def test_library_large_instance_properties():
    """Sizes the enumeration cannot reach: the split sums to L and stays under the caps, its bottleneck is the
    value returned, and that value is optimal by a counting certificate: the stages cannot hold L layers while
    every load stays strictly below it."""
    import paper_2410_13333_amd as mls
    rng = random.Random(17)
    for _ in range(50):
        n = rng.randint(2, 16)
        y, L = _rates(rng, n), rng.randint(50, 400)
        caps = [rng.choice([None, rng.randint(L // n, L)]) for _ in range(n)]
        l, o = mls.plan_layers(y, L, caps)
        assert sum(l) == L and all(k >= 0 and (c is None or k <= c) for k, c in zip(l, caps))
        assert o == max(a * b for a, b in zip(y, l))
        below = 0
        for yj, c in zip(y, caps):
            k = 0
            while yj * (k + 1) < o and (c is None or k + 1 <= c) and k + 1 <= L:
                k += 1
            below += k
        assert below < L


def test_library_grouping_ratio_equals_the_relaxed_lp():
    import paper_2410_13333_amd as mls
    rng = random.Random(19)
    for _ in range(10):
        y1, y2 = _rates(rng, rng.randint(1, 6)), _rates(rng, rng.randint(1, 6))
        assert mls.grouping_time_ratio(y1, y2) == pytest.approx(oplan.relaxed_time(y1) / oplan.relaxed_time(y2), rel=1e-8)
    assert math.isnan(mls.grouping_time_ratio([1.0, -1.0], [1.0]))


def test_library_rejects_bad_arguments():
    import paper_2410_13333_amd as mls
    for bad in ([0.0, 1.0], [float("inf")], [float("nan"), 1.0]):
        with pytest.raises(mls.MlsError) as e:
            mls.plan_layers(bad, 4)
        assert e.value.code == -1
    with pytest.raises(mls.MlsError):
        mls.plan_layers([1.0], -1)
    with pytest.raises(mls.MlsError):
        mls.plan_lower_level([[1.0], []], 4, 4, 1.0)


def _golden():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_case_studies.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        kind, cite, inputs, result = [p.strip() for p in line.split("|")]
        args = {k.strip(): [float(v) for v in vs.split()] for k, vs in (item.split("=") for item in inputs.split(";"))}
        yield kind, cite, args, [float(v) for v in result.split("=")[1].split()]


def test_golden_file_of_printed_values_oracle_and_library():
    """tests/golden/paper_case_studies.txt holds what the paper prints; both the enumeration and the library must
    reproduce every record."""
    import paper_2410_13333_amd as mls
    seen = 0
    for kind, cite, a, want in _golden():
        seen += 1
        if kind == "microbatches":
            best, arg = oplan.microbatches_bruteforce(a["o"], int(a["n_mb"][0]))
            assert arg == [tuple(int(v) for v in want)], cite
            assert mls.plan_microbatches(a["o"], int(a["n_mb"][0]))[0] == [int(v) for v in want], cite
        elif kind == "layers":
            L, printed = int(a["L"][0]), tuple(int(v) for v in want)
            value = max(y * l for y, l in zip(a["y"], printed))
            caps = [int(value / y) for y in a["y"]]               # any split at least as good stays under these
            best, arg = oplan.layers_bruteforce(a["y"], L, caps=caps)
            assert best == value and printed in arg, cite
            l, o = mls.plan_layers(a["y"], L)
            assert o == value and sorted(l) == sorted(printed), cite
        elif kind == "theoretic":
            assert abs(mls.theoretic_slowdown(int(a["N"][0]), a["x"]) - want[0]) < 0.006, cite
    assert seen == 5


def test_oracle_split_candidates_are_the_six_of_the_appendix():
    """Appendix B.7 lists, for 7 GPUs X1..X7 in descending rate and groups Y1, Y2, Y3 of 1, 2, 4 GPUs, exactly these
    six groupings (1-based GPU numbers as printed)."""
    printed = {((1,), (2, 3), (4, 5, 6, 7)), ((1,), (6, 7), (2, 3, 4, 5)), ((3,), (1, 2), (4, 5, 6, 7)),
               ((5,), (6, 7), (1, 2, 3, 4)), ((7,), (1, 2), (3, 4, 5, 6)), ((7,), (5, 6), (1, 2, 3, 4))}
    got = {tuple(tuple(i + 1 for i in run) for run in cand) for cand in oplan.consecutive_run_candidates(7, [1, 2, 4])}
    assert got == printed


def test_split_groups_library_matches_exhaustive_search():
    """The appendix's proposition (an optimum uses consecutive runs) and the library's pick, against the search over
    every assignment; rates include the three stragglers of the appendix's experiment (2.57, 5.42, 12.53)."""
    import paper_2410_13333_amd as mls
    rng = random.Random(23)
    cases = [([12.53, 5.42, 2.57, 1.0, 1.0, 1.0, 1.0], [1, 2, 4], [1.0, 0.55, 0.3])]
    for _ in range(40):
        sizes = rng.choice([[1, 2, 4], [1, 1, 2], [2, 2], [1, 2, 2, 2], [4, 2, 1], [1, 1, 1, 1]])
        x = [rng.choice([1.0, 1.0, 1.0, 1.31, 2.57, 2.62, 3.75, 5.42, 12.53]) for _ in range(sum(sizes))]
        rho = [{1: 1.0, 2: 0.55, 4: 0.3}[s] * rng.choice([1.0, 1.1]) for s in sizes]
        cases.append((x, sizes, rho))
    for x, sizes, rho in cases:
        want = oplan.split_groups_bruteforce(x, sizes, rho)
        group_of, inv = mls.plan_split_groups(x, sizes, rho)
        assert sorted(group_of.count(g) for g in range(len(sizes))) == sorted(sizes)
        assert [group_of.count(g) for g in range(len(sizes))] == sizes
        got = sum(1.0 / (rho[g] * max(xi for xi, gi in zip(x, group_of) if gi == g)) for g in range(len(sizes)))
        assert got == pytest.approx(inv, rel=1e-14) and inv == pytest.approx(want, rel=1e-12)
    # first case: the two heaviest stragglers share the pair, the third stands alone, the healthy four stay together
    assert mls.plan_split_groups(*cases[0])[0] == [1, 1, 0, 2, 2, 2, 2]
    with pytest.raises(mls.MlsError):
        mls.plan_split_groups([1.0, 1.0], [1, 2], [1.0, 1.0])
