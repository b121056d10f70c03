"""Pins of the oracle's Algorithm-1 greedy and of its facility-location value
against closed forms, library routines, exhaustive search and the properties
the paper states (Section 3.1: partition, submodularity, monotonicity)."""
import itertools
import math

import numpy as np
import pytest

import oracle
import synth_inputs as si


def mixture_S(seed, n, d=8):
    X = si.make_class(seed=seed, n=n, d=d)
    return oracle.similarity(X, float(d))


def const_S(n, c):
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    return S


# ---------------------------------------------------------------- f itself
def test_f_matches_numpy_definition():
    S = mixture_S(1, 40)
    rng = np.random.default_rng(0)
    for m in (1, 2, 7, 40):
        A = rng.choice(40, size=m, replace=False)
        ref = S[:, A].astype(np.float64).max(axis=1).sum()
        assert oracle.f_value(S, A) == pytest.approx(ref, rel=1e-14)
    assert oracle.f_value(S, []) == 0.0


def test_f_closed_form_constant_similarity():
    n, c = 12, 0.25
    S = const_S(n, c)
    for m in range(1, n + 1):
        assert oracle.f_value(S, list(range(m))) == m + (n - m) * c   # exact: dyadic


def test_f_uses_rows_as_covered_points_and_columns_as_members():
    # an asymmetric S makes a transposed access visible
    S = np.array([[1.0, 0.5, 0.0], [0.25, 1.0, 0.0], [0.75, 0.125, 1.0]], dtype=np.float32)
    # A = {1}: sum_j S[j][1] = 0.5 + 1 + 0.125
    assert oracle.f_value(S, [1]) == 1.625
    g = oracle.gain_row(S, np.zeros(3))
    assert g.tolist() == [2.0, 1.625, 1.0]       # column sums


@pytest.mark.parametrize("seed", range(5))
def test_f_monotone_and_submodular_on_nested_subsets(seed):
    n = 30
    S = mixture_S(seed, n)
    rng = np.random.default_rng(seed)
    for _ in range(40):
        perm = rng.permutation(n)
        b = int(rng.integers(1, n - 1))
        a = int(rng.integers(0, b + 1))
        A, B, v = perm[:a], perm[:b], perm[b]
        gA = oracle.f_value(S, list(A) + [v]) - oracle.f_value(S, A)
        gB = oracle.f_value(S, list(B) + [v]) - oracle.f_value(S, B)
        assert gB >= -1e-12                     # monotone
        assert gA >= gB - 1e-12                 # diminishing returns


# ---------------------------------------------------------------- step logic
def test_every_step_is_the_definitions_argmax_and_argmin():
    """Re-derive every step of a run from f evaluated by its definition."""
    n, cap = 14, [3, 5, 6]
    S = mixture_S(7, n)
    out = oracle.partition_class(S, cap, trace=True)
    assert out["steps"] == n
    blocks = [[] for _ in cap]
    taken = set()
    for t in range(n):
        fvals = [oracle.f_value(S, b) for b in blocks]
        open_blocks = [k for k in range(len(cap)) if len(blocks[k]) < cap[k]]
        js = min(open_blocks, key=lambda k: (fvals[k], k))
        assert out["tr_block"][t] == js
        cands = [v for v in range(n) if v not in taken]
        vals = [oracle.f_value(S, blocks[js] + [v]) for v in cands]
        vs = cands[int(np.argmax(vals))]
        assert out["tr_elem"][t] == vs
        assert out["tr_gain"][t] == pytest.approx(max(vals) - fvals[js], rel=1e-10, abs=1e-12)
        blocks[js].append(vs)
        taken.add(vs)
    for k, b in enumerate(blocks):
        assert sorted(np.flatnonzero(out["assign"] == k).tolist()) == sorted(b)


def test_all_unit_quotas_reduce_to_a_sort_of_column_sums():
    n = 25
    S = mixture_S(3, n)
    out = oracle.partition_class(S, [1] * n)
    colsum = S.astype(np.float64).sum(axis=0)
    expected = np.argsort(-colsum, kind="stable")
    for t, v in enumerate(expected):
        assert out["assign"][v] == t and out["order"][v] == t


def _textbook_greedy(S, b):
    """Cardinality-constrained greedy with f from numpy's definition, no coverage vector."""
    n = S.shape[0]
    A = []
    Sd = S.astype(np.float64)
    for _ in range(b):
        best, pick = -1.0, -1
        for v in range(n):
            if v in A:
                continue
            val = Sd[:, A + [v]].max(axis=1).sum()
            if val > best:
                best, pick = val, v
        A.append(pick)
    return A


@pytest.mark.parametrize("seed,b", [(0, 3), (1, 4), (2, 5), (3, 2)])
def test_single_block_is_textbook_greedy_and_meets_its_bound(seed, b):
    n = 11
    S = mixture_S(seed, n, d=4)
    out = oracle.partition_class(S, [b], trace=True)
    assert out["tr_elem"].tolist() == _textbook_greedy(S, b)
    assert np.sum(out["assign"] == 0) == b and np.sum(out["assign"] == -1) == n - b
    opt = max(S[:, list(A)].astype(np.float64).max(axis=1).sum()
              for A in itertools.combinations(range(n), b))
    best_sum, best_min, _ = oracle.bruteforce(S, [b])
    assert best_sum == pytest.approx(opt, rel=1e-14)           # pins the enumerator too
    assert best_min == pytest.approx(opt, rel=1e-14)
    assert out["obj"][0] >= (1.0 - 1.0 / math.e) * opt
    assert out["obj"][0] <= opt + 1e-12


@pytest.mark.parametrize("cap", [[4, 4, 4], [2, 4, 6], [1, 1, 10], [6, 6]])
def test_constant_similarity_closed_form_round_robin(cap):
    n, c = 12, 0.25
    S = const_S(n, c)
    out = oracle.partition_class(S, cap, trace=True)
    # every gain ties, so sample t goes to the open block with the least f =
    # fewest members, lowest index: a round robin over the blocks still open
    cnt = [0] * len(cap)
    for t in range(n):
        k = min((k for k in range(len(cap)) if cnt[k] < cap[k]), key=lambda k: (cnt[k], k))
        assert out["tr_elem"][t] == t and out["tr_block"][t] == k
        assert out["tr_gain"][t] == (1 + (n - 1) * c if cnt[k] == 0 else 1 - c)
        cnt[k] += 1
    for k, m in enumerate(cap):
        assert out["obj"][k] == m + (n - m) * c
        assert out["fsum"][k] == m + (n - m) * c


def test_one_block_taking_everything_has_value_n():
    S = mixture_S(4, 33)
    out = oracle.partition_class(S, [33])
    assert out["obj"][0] == 33.0 and np.all(out["assign"] == 0)


def test_zero_quota_block_is_dropped_and_leftovers_stay_unassigned():
    S = mixture_S(5, 10)
    out = oracle.partition_class(S, [0, 3, 2])
    assert np.sum(out["assign"] == 0) == 0
    assert np.sum(out["assign"] == 1) == 3 and np.sum(out["assign"] == 2) == 2
    assert np.sum(out["assign"] == -1) == 5 and out["steps"] == 5
    assert out["obj"][0] == 0.0
    assert sorted(out["order"][out["order"] >= 0].tolist()) == list(range(5))


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("seed", range(4))
def test_partition_invariants_and_objective_consistency(seed):
    n = 60
    rng = np.random.default_rng(seed)
    r = rng.integers(1, 5, size=int(rng.integers(2, 7)))
    cap = oracle.quota(n, r)
    S = mixture_S(20 + seed, n)
    out = oracle.partition_class(S, cap)
    counts = np.bincount(out["assign"], minlength=len(cap))
    assert counts.tolist() == cap.tolist()                      # exact quotas, full cover
    assert sorted(out["order"].tolist()) == list(range(n))      # disjoint: one step each
    assert np.allclose(out["obj"], out["fsum"], rtol=1e-12)     # telescoped gains = definition
    assert np.all(out["obj"] >= counts - 1e-12)                 # self-coverage
    for k in range(len(cap)):
        members = np.flatnonzero(out["assign"] == k)
        ref = S[:, members].astype(np.float64).max(axis=1).sum() if len(members) else 0.0
        assert out["obj"][k] == pytest.approx(ref, rel=1e-13)


def test_permutation_equivariance_on_generic_input():
    n, cap = 40, [10, 10, 20]
    S = mixture_S(31, n)
    base = oracle.partition_class(S, cap)
    perm = np.random.default_rng(1).permutation(n)
    Sp = np.ascontiguousarray(S[np.ix_(perm, perm)])
    moved = oracle.partition_class(Sp, cap)
    assert np.array_equal(moved["assign"], base["assign"][perm])
    assert np.array_equal(moved["order"], base["order"][perm])


@pytest.mark.parametrize("n,cap", [(9, [3, 3, 3]), (10, [2, 3, 5]), (8, [4, 4]), (9, [2, 2, 2])])
def test_greedy_never_beats_exhaustive_optimum(n, cap):
    S = mixture_S(40 + n, n, d=4)
    out = oracle.partition_class(S, cap)
    best_sum, best_min, visited = oracle.bruteforce(S, cap)
    left = n - sum(cap)
    multinomial = math.factorial(n)
    for m in cap + [left]:
        multinomial //= math.factorial(m)
    assert visited == multinomial
    assert out["obj"].sum() <= best_sum + 1e-12
    assert out["obj"].min() <= best_min + 1e-12
    # the greedy is a sensible heuristic on these inputs (recorded, loose)
    assert out["obj"].min() >= 0.5 * best_min


def test_bruteforce_finds_a_known_optimum():
    # two tight pairs far apart: {0,1} close, {2,3} close.  With quotas [2,2]
    # the best min-f and the best sum put one sample of each pair in each block.
    S = np.array([[1, .9, .1, .1], [.9, 1, .1, .1], [.1, .1, 1, .9], [.1, .1, .9, 1]], dtype=np.float32)
    best_sum, best_min, visited = oracle.bruteforce(S, [2, 2])
    assert visited == 6
    mixed = 2 * (1.0 + float(np.float32(0.9)))
    assert best_min == pytest.approx(mixed, rel=1e-12)
    assert best_sum == pytest.approx(2 * mixed, rel=1e-12)
    out = oracle.partition_class(S, [2, 2])
    assert out["obj"].min() == pytest.approx(mixed, rel=1e-12)   # greedy finds it here


# ---------------------------------------------------------------- referee
def test_referee_accepts_the_oracles_own_trace_and_rejects_a_planted_swap():
    n, cap = 50, [10, 15, 25]
    S = mixture_S(50, n)
    out = oracle.partition_class(S, cap)
    ok = oracle.lockstep(S, cap, out["order"], out["assign"], rel_tol=0.0)
    assert ok["rc"] == 0 and ok["exact"] == n and ok["checked"] == n
    bad_order = out["order"].copy()
    a, b = np.flatnonzero(out["order"] == 5)[0], np.flatnonzero(out["order"] == 30)[0]
    bad_order[a], bad_order[b] = bad_order[b], bad_order[a]
    bad = oracle.lockstep(S, cap, bad_order, out["assign"], rel_tol=1e-5)
    assert bad["rc"] == 1 and bad["first_violation"] == 5
    bad_assign = out["assign"].copy()
    v = np.flatnonzero(out["order"] == 12)[0]
    bad_assign[v] = (bad_assign[v] + 1) % 3
    assert oracle.lockstep(S, cap, out["order"], bad_assign, rel_tol=1e-5)["rc"] == 1


def test_referee_near_tie_window():
    # candidates 1 and 2 differ by 2^-20 relative in their column sums
    S = np.eye(4, dtype=np.float32)
    S[0, 1] = S[1, 0] = 0.5
    S[0, 2] = S[2, 0] = np.float32(0.5 - 2.0 ** -21)
    # column sums: v0 = 2-2^-21, v1 = 1.5, v2 = 1.5-2^-21, v3 = 1.  K=1, cap=2
    cap = [2]
    out = oracle.partition_class(S, cap, trace=True)
    assert out["tr_elem"].tolist() == [0, 3]
    # a trace taking 1 then 3 instead: first choice is off by 25% -> violation
    order = np.array([-1, 0, -1, 1], dtype=np.int32)
    assign = np.array([-1, 0, -1, 0], dtype=np.int32)
    assert oracle.lockstep(S, cap, order, assign, rel_tol=1e-5)["rc"] == 1
    # K=1, cap=1 on the sub-problem without sample 0: 1 vs 2 differ by ~3e-7 relative
    sub = np.ascontiguousarray(S[1:, 1:])
    sub[0, 1] = sub[1, 0] = 0.25
    sub[0, 2] = sub[2, 0] = 0.25
    sub[1, 2] = sub[2, 1] = np.float32(0.25 + 2.0 ** -21)
    # column sums: 1.5, 1.5+2^-21, 1.5+2^-21 -> oracle takes index 1
    got = oracle.partition_class(sub, [1], trace=True)
    assert got["tr_elem"].tolist() == [1]
    order = np.array([0, -1, -1], dtype=np.int32)
    assign = np.array([0, -1, -1], dtype=np.int32)
    near = oracle.lockstep(sub, [1], order, assign, rel_tol=1e-5)
    assert near["rc"] == 0 and near["near_elem"] == 1 and near["exact"] == 0
    assert 0 < near["worst_elem_gap"] < 1e-6
    assert oracle.lockstep(sub, [1], order, assign, rel_tol=1e-8)["rc"] == 1


def test_referee_rejects_over_quota_and_malformed_traces():
    S = mixture_S(60, 12)
    cap = [4, 8]
    out = oracle.partition_class(S, cap)
    assign = out["assign"].copy()
    v = np.flatnonzero(assign == 1)[0]
    assign[v] = 0                                   # block 0 now gets 5 > 4
    assert oracle.lockstep(S, cap, out["order"], assign)["rc"] == 1
    order = out["order"].copy()
    order[0] = order[1]                             # duplicate step
    assert oracle.lockstep(S, cap, order, out["assign"])["rc"] == -1


def test_referee_sampled_steps_only():
    n, cap = 40, [20, 20]
    S = mixture_S(61, n)
    out = oracle.partition_class(S, cap)
    res = oracle.lockstep(S, cap, out["order"], out["assign"], check=[0, 7, 39])
    assert res["rc"] == 0 and res["checked"] == 3 and res["exact"] == 3


# ---------------------------------------------------------------- data set
def test_dataset_is_per_class_runs_joined():
    w = si.WORKLOADS["tiny"]
    ds = si.make_dataset(w, L=3, n_c=30, d=8)
    res = oracle.partition_dataset(ds.X, ds.labels, ds.L, ds.r, ds.sigma2)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)           # stable: ascending global index
        S = oracle.similarity(ds.X[idx], ds.sigma2)
        cap = oracle.quota(len(idx), ds.r)
        one = oracle.partition_class(S, cap)
        assert np.array_equal(res["assign"][idx], one["assign"])
        assert np.array_equal(res["order"][idx], one["order"])
        assert np.allclose(res["obj"][c], one["obj"], rtol=0, atol=0)
        assert np.bincount(res["assign"][idx], minlength=len(cap)).tolist() == cap.tolist()


def test_dataset_class_balance_is_identical_across_classes():
    w = si.WORKLOADS["hetero8"]
    ds = si.make_dataset(w, L=4, n_c=40, d=8)
    res = oracle.partition_dataset(ds.X, ds.labels, ds.L, ds.r, ds.sigma2)
    per_class = [np.bincount(res["assign"][ds.labels == c], minlength=w.K) for c in range(ds.L)]
    for row in per_class[1:]:
        assert row.tolist() == per_class[0].tolist()
    assert per_class[0].tolist() == oracle.quota(40, ds.r).tolist()


def test_dataset_handles_an_empty_class_and_bf16():
    w = si.WORKLOADS["large"]
    ds = si.make_dataset(w, L=2, n_c=24, d=16)
    res = oracle.partition_dataset(ds.X, ds.labels, 3, ds.r, ds.sigma2)   # class 2 is empty
    assert np.all(res["assign"] >= 0)
    assert np.all(res["obj"][2] == 0.0)
    assert np.all(res["obj"][:2].sum(axis=1) > 0)
