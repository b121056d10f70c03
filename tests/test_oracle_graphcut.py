"""Pins of the oracle's graph-cut route (Section 4, "Submodular functions":
f(A) = sum_{v in V \\ A} sum_{v' in A} sim(v, v')) against what the definition and the mathematics
fix: closed forms on constant similarity, the cut symmetry f(A) = f(V \\ A), submodularity and
non-monotonicity, every accepted marginal value re-derived from the definition, reductions of
Algorithm 1 to a sort, a hand-simulated trace on constant similarity, exhaustive search on tiny
inputs, quota and cover invariants."""
import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as si


def mix(seed, n, d=8):
    return oracle.similarity(si.make_class(seed=seed, n=n, d=d), float(d))


def f_numpy(S, A):
    A = np.asarray(sorted(A), dtype=np.int64)
    rest = np.setdiff1d(np.arange(S.shape[0]), A)
    return float(S[np.ix_(rest, A)].astype(np.float64).sum())


def test_f_matches_numpy_and_closed_forms():
    S = mix(1, 40)
    rng = np.random.default_rng(0)
    for m in (0, 1, 7, 20, 39, 40):
        A = rng.choice(40, size=m, replace=False)
        assert oracle.f_value(S, A, "gc") == pytest.approx(f_numpy(S, A), rel=1e-12, abs=1e-12)
    # constant similarity c off the diagonal: f(A) = |A| (n - |A|) c
    n, c = 30, 0.375
    C = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(C, 1.0)
    for m in range(0, n + 1, 5):
        assert oracle.f_value(C, np.arange(m), "gc") == m * (n - m) * c
    assert oracle.f_value(S, np.arange(40), "gc") == 0.0          # f(V) = 0: not monotone
    assert oracle.f_value(S, [], "gc") == 0.0


def test_cut_symmetry_submodularity_and_a_negative_marginal():
    S = mix(2, 36)
    rng = np.random.default_rng(1)
    allv = np.arange(36)
    for _ in range(40):
        B = rng.choice(36, size=rng.integers(2, 30), replace=False)
        A = B[: rng.integers(1, len(B))]
        # symmetric similarity: the cut of A is the cut of its complement
        assert oracle.f_value(S, A, "gc") == pytest.approx(oracle.f_value(S, np.setdiff1d(allv, A), "gc"), rel=1e-12)
        v = rng.choice(np.setdiff1d(allv, B))
        gA = oracle.f_value(S, np.append(A, v), "gc") - oracle.f_value(S, A, "gc")
        gB = oracle.f_value(S, np.append(B, v), "gc") - oracle.f_value(S, B, "gc")
        assert gA >= gB - 1e-9                                     # diminishing returns
    # adding the last outsider to a nearly full set lowers f
    A = np.arange(35)
    assert oracle.f_value(S, np.arange(36), "gc") - oracle.f_value(S, A, "gc") < 0.0


def test_every_accepted_marginal_value_is_the_definitions():
    S = mix(3, 48)
    cap = oracle.quota(48, [1, 2, 3])
    out = oracle.partition_class(S, cap, trace=True, objective="gc")
    assert out["steps"] == 48
    members = {k: [] for k in range(3)}
    f = np.zeros(3)
    for t in range(48):
        k, v, g = int(out["tr_block"][t]), int(out["tr_elem"][t]), float(out["tr_gain"][t])
        # block: least f among the blocks with room, lowest index on ties
        room = [kk for kk in range(3) if len(members[kk]) < cap[kk]]
        assert k == min(room, key=lambda kk: (f[kk], kk))
        base = f_numpy(S, members[k])
        gains = {u: f_numpy(S, members[k] + [u]) - base for u in range(48) if all(u not in m for m in members.values())}
        assert g == pytest.approx(gains[v], rel=1e-10, abs=1e-10)
        assert gains[v] >= max(gains.values()) - 1e-9
        members[k].append(v)
        f[k] += g
    for k in range(3):
        assert out["obj"][k] == pytest.approx(f_numpy(S, members[k]), rel=1e-12)
        assert out["fsum"][k] == pytest.approx(out["obj"][k], rel=1e-10)
    assert np.bincount(out["assign"], minlength=3).tolist() == cap.tolist()
    assert sorted(out["order"].tolist()) == list(range(48))


def test_unit_quotas_reduce_to_a_sort_by_column_sum_without_the_diagonal():
    n = 14
    S = mix(4, n)
    out = oracle.partition_class(S, [1] * n, objective="gc")
    key = S.astype(np.float64).sum(axis=0) - np.diag(S).astype(np.float64)
    expected = np.argsort(-key, kind="stable")
    assert [int(np.flatnonzero(out["assign"] == t)[0]) for t in range(n)] == expected.tolist()


def test_constant_similarity_trace_follows_the_closed_form():
    # all marginal values tie, so the lowest free index goes next; blocks follow f = m (n - m) c
    n, c = 24, 0.5
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    cap = [4, 8, 12]
    out = oracle.partition_class(S, cap, trace=True, objective="gc")
    cnt = [0, 0, 0]
    for t in range(n):
        f = [m * (n - m) * c for m in cnt]
        room = [k for k in range(3) if cnt[k] < cap[k]]
        k = min(room, key=lambda kk: (f[kk], kk))
        assert out["tr_block"][t] == k and out["tr_elem"][t] == t
        assert out["tr_gain"][t] == (cnt[k] + 1) * (n - cnt[k] - 1) * c - cnt[k] * (n - cnt[k]) * c
        cnt[k] += 1
    assert out["obj"].tolist() == [m * (n - m) * c for m in cap]


def test_cardinality_greedy_never_beats_the_exhaustive_optimum_and_is_close():
    ratios = []
    for seed in range(6):
        n, b = 9, 4
        S = mix(10 + seed, n)
        out = oracle.partition_class(S, [b], objective="gc")
        greedy = out["obj"][0]
        opt = max(f_numpy(S, A) for A in itertools.combinations(range(n), b))
        assert greedy <= opt + 1e-9
        ratios.append(greedy / opt)
    assert min(ratios) > 0.9      # b <= n/2: the greedy stays in the increasing part of the cut function


def test_lockstep_referee_accepts_its_own_trace_and_catches_a_planted_swap():
    S = mix(5, 60)
    cap = oracle.quota(60, [1, 1, 2])
    out = oracle.partition_class(S, cap, objective="gc")
    res = oracle.lockstep(S, cap, out["order"], out["assign"], rel_tol=0.0, objective="gc")
    assert res["rc"] == 0 and res["exact"] == 60
    # the facility-location referee must not accept a graph-cut trace (different choices)
    assert oracle.lockstep(S, cap, out["order"], out["assign"], rel_tol=1e-5, objective="fl")["rc"] == 1
    # plant a mistake in the trace: swap the samples taken at steps 10 and 40
    order = out["order"].copy()
    a, b = int(np.flatnonzero(order == 10)[0]), int(np.flatnonzero(order == 40)[0])
    assign = out["assign"].copy()
    order[a], order[b] = 40, 10
    assign[a], assign[b] = assign[b], assign[a]
    assert oracle.lockstep(S, cap, order, assign, rel_tol=1e-9, objective="gc")["rc"] == 1


def test_absolute_window_of_the_referee_on_a_hand_built_trace():
    """Three samples, one block of quota 1, dyadic similarities: the marginal values from the empty block are
    g(0) = 0.5 + 0.25, g(1) = 0.5 + 0.125, g(2) = 0.25 + 0.125 (Section 4's graph-cut f with A = {u}).
    A trace that takes sample 1 is delta = 0.125 below the best: the referee must accept it exactly when
    the absolute window reaches delta, and the relative window must stay out of it (rel_tol = 0)."""
    S = np.array([[1.0, 0.5, 0.25], [0.5, 1.0, 0.125], [0.25, 0.125, 1.0]], dtype=np.float32)
    assert [f_numpy(S, [u]) for u in range(3)] == [0.75, 0.625, 0.375]
    cap = [1]
    order = np.array([-1, 0, -1], dtype=np.int32)
    assign = np.array([-1, 0, -1], dtype=np.int32)
    for abs_tol, ok in ((0.125, True), (0.5, True), (0.1249, False), (0.0, False)):
        res = oracle.lockstep(S, cap, order, assign, rel_tol=0.0, objective="gc", abs_tol=abs_tol)
        assert (res["rc"] == 0) == ok, (abs_tol, res)
        assert res["near_elem"] == (1 if ok else 0) and res["violations"] == (0 if ok else 1)
    # the relative gap reported is delta over the larger magnitude
    res = oracle.lockstep(S, cap, order, assign, rel_tol=0.0, objective="gc", abs_tol=0.0)
    assert res["worst_elem_gap"] == 0.125 / 0.75
    # the best sample itself is exact under a zero window
    best = oracle.lockstep(S, cap, np.array([0, -1, -1], dtype=np.int32), np.array([0, -1, -1], dtype=np.int32),
                           rel_tol=0.0, objective="gc", abs_tol=0.0)
    assert best["rc"] == 0 and best["exact"] == 1
    # the worst sample is 0.375 below: a window of 0.125 must not let it through
    worst = oracle.lockstep(S, cap, np.array([-1, -1, 0], dtype=np.int32), np.array([-1, -1, 0], dtype=np.int32),
                            rel_tol=0.0, objective="gc", abs_tol=0.125)
    assert worst["rc"] == 1


def test_absolute_window_applies_at_a_later_step_with_negative_marginal_values():
    """Four samples, one block of quota 3, constant similarity c = 0.5 except one pair: at the third step the
    block holds two samples and the marginal values of the remaining two are (from the definition)
    g(u) = sum_{v outside, v != u} S(v,u) - sum_{a in A} S(u,a), negative here.  The trace takes the worse one."""
    S = np.full((4, 4), 0.5, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    S[2, 3] = S[3, 2] = 0.25
    S[0, 2] = S[2, 0] = 0.75
    out = oracle.partition_class(S, [3], trace=True, objective="gc")
    # first two picks from the definition: column sums without the diagonal 1.75, 1.5, 1.5, 1.25 -> sample 0;
    # then g(1) = 0.5 + 0.5 - 0.5 = 0.5, g(2) = 0.5 + 0.25 - 0.75 = 0, g(3) = 0.5 + 0.25 - 0.5 = 0.25 -> sample 1
    assert out["tr_elem"][:2].tolist() == [0, 1] and out["tr_gain"][:2].tolist() == [1.75, 0.5]
    # third step, A = {0, 1}: g(2) = S(3,2) - S(2,0) - S(2,1) = 0.25 - 1.25 = -1.0, g(3) = 0.25 - 1.0 = -0.75
    base = f_numpy(S, [0, 1])
    assert f_numpy(S, [0, 1, 2]) - base == -1.0 and f_numpy(S, [0, 1, 3]) - base == -0.75
    assert out["tr_elem"][2] == 3 and out["tr_gain"][2] == -0.75
    order = np.array([0, 1, 2, -1], dtype=np.int32)          # the trace takes sample 2 at the third step
    assign = np.array([0, 0, 0, -1], dtype=np.int32)
    for abs_tol, ok in ((0.25, True), (0.2499, False)):
        res = oracle.lockstep(S, [3], order, assign, rel_tol=0.0, objective="gc", abs_tol=abs_tol)
        assert (res["rc"] == 0) == ok and res["checked"] == 3, (abs_tol, res)
        assert res["first_violation"] == (-1 if ok else 2)


def test_an_asymmetric_similarity_is_evaluated_as_printed_and_refused_by_the_greedy():
    """Section 4 prints f(A) = sum_{v outside A} sum_{v' in A} sim(v, v'): the first index is the outside
    sample.  The definition is evaluated that way on any matrix; the greedy and its referee read marginal
    values along rows, which is only the same thing for a symmetric matrix, and say so by refusing others."""
    S = np.array([[1.0, 0.5, 0.25], [0.125, 1.0, 0.75], [0.0625, 0.375, 1.0]], dtype=np.float32)
    # A = {0}: outside samples 1 and 2, terms S[1][0] + S[2][0] (not S[0][1] + S[0][2])
    assert oracle.f_value(S, [0], "gc") == 0.125 + 0.0625
    assert oracle.f_value(S, [1, 2], "gc") == 0.5 + 0.25
    with pytest.raises(ValueError):
        oracle.partition_class(S, [1, 1], objective="gc")
    res = oracle.lockstep(S, [1], np.array([0, -1, -1], dtype=np.int32), np.array([0, -1, -1], dtype=np.int32),
                          rel_tol=1e-5, objective="gc")
    assert res["rc"] == -2
    # made symmetric, both run
    Ssym = np.maximum(S, S.T)
    assert oracle.partition_class(Ssym, [1, 1], objective="gc")["steps"] == 2
