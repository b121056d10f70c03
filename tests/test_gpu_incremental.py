"""GPU parity of the incremental-gain route (RCD_MODE_INCREMENTAL through rcd_partition_class_mode): the same
Algorithm 1, with every block's gains kept current from step to step instead of rebuilt by
sweeps.  Checked like the sweep route: the oracle's lock-step referee on the same S, exact-tie
cases with a zero window, objectives from the definition, quota and cover invariants; and the
two routes against each other."""
import numpy as np
import pytest

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rcd():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU path")
    import paper_2211_00839_amd as m

    m.load_library()
    return m


def dev(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def mixture_S(seed, n, d=16):
    return oracle.similarity(si.make_class(seed=seed, n=n, d=d), float(d))


def run_class(rcd, S, cap, incremental=True):
    assign, order, obj = rcd.partition_class(S=dev(S), cap=cap,
                                             mode=rcd.MODE_INCREMENTAL if incremental else rcd.MODE_STORED)
    return assign.cpu().numpy(), order.cpu().numpy(), obj


def check_against_oracle(S, cap, assign, order, obj, exact=False):
    cap = np.asarray(cap, dtype=np.int64)
    n = S.shape[0]
    assert np.bincount(assign[assign >= 0], minlength=len(cap)).tolist() == cap.tolist()
    assert np.sum(assign < 0) == n - cap.sum()
    assert sorted(order[order >= 0].tolist()) == list(range(int(cap.sum())))
    res = oracle.lockstep(S, cap, order, assign, rel_tol=0.0 if exact else 1e-5)
    assert res["rc"] == 0, res
    assert res["checked"] == cap.sum()
    for k in range(len(cap)):
        ref = oracle.f_value(S, np.flatnonzero(assign == k))
        assert abs(obj[k] - ref) <= 1e-4 * max(ref, 1e-30), (k, obj[k], ref)
    return res


@pytest.mark.parametrize("n,r", [(1, [1]), (250, [1, 1]), (600, [1, 1, 2, 4]), (1000, [1, 1, 1, 2, 2, 3, 4, 6]),
                                 (520, [3, 1, 4, 1, 2, 2, 1, 3, 4, 4, 1, 2, 3, 3, 2, 1]), (257, [5]), (1300, [2, 1])])
def test_incremental_class_greedy_lockstep(rcd, n, r):
    print(f"incremental class greedy n={n} K={len(r)}", flush=True)
    S = mixture_S(400 + n, n)
    cap = oracle.quota(n, r)
    assign, order, obj = run_class(rcd, S, cap)
    res = check_against_oracle(S, cap, assign, order, obj)
    stats = rcd.last_stats()
    assert stats["steps"] == n
    assert stats["useful_evals"] == n * (n + 1) // 2
    # gains are carried in double: the trace is the oracle's own unless two choices tie to 1e-5
    ref = oracle.partition_class(S, cap)
    if res["near_block"] == 0 and res["near_elem"] == 0:
        assert np.array_equal(assign, ref["assign"]) and np.array_equal(order, ref["order"])
        assert np.allclose(obj, ref["obj"], rtol=1e-4)
    # far fewer similarity entries are read than one row per candidate and step
    if n > 8:
        assert stats["entries_streamed"] < n * n * (n + 1) // 2


def test_incremental_exact_ties_follow_the_lowest_index_contract(rcd):
    # constant similarity: every gain ties exactly
    n, c = 96, 0.25
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    for cap in ([32, 32, 32], [10, 30, 56], [96]):
        assign, order, obj = run_class(rcd, S, cap)
        ref = oracle.partition_class(S, cap)
        assert np.array_equal(assign, ref["assign"]) and np.array_equal(order, ref["order"])
        assert obj.tolist() == [m + (n - m) * c for m in cap]
        check_against_oracle(S, cap, assign, order, obj, exact=True)


def test_incremental_duplicate_samples_tie_exactly(rcd):
    # every sample appears twice: the copies' gains must stay equal bit for bit through all the
    # updates, so that the lower index of a pair is always the one taken first
    base = si.make_class(seed=31, n=150, d=16)
    X = np.concatenate([base, base], axis=0)
    S = oracle.similarity(X, 16.0)
    cap = oracle.quota(300, [1, 2])
    assign, order, obj = run_class(rcd, S, cap)
    check_against_oracle(S, cap, assign, order, obj, exact=False)
    ref = oracle.partition_class(S, cap)
    # whenever both copies of a sample go to the same block, the first copy goes first
    for i in range(150):
        if assign[i] == assign[i + 150]:
            assert order[i] < order[i + 150]
    assert np.allclose(obj, ref["obj"], rtol=1e-4)


def test_incremental_zero_quota_and_leftovers(rcd):
    S = mixture_S(18, 300)
    cap = [0, 40, 0, 25]
    assign, order, obj = run_class(rcd, S, cap)
    check_against_oracle(S, cap, assign, order, obj)
    assert obj[0] == 0.0 and obj[2] == 0.0
    assert np.sum(assign == -1) == 235 and np.all(order[assign == -1] == -1)
    assign, order, obj = run_class(rcd, S, [0, 0])
    assert np.all(assign == -1) and np.all(obj == 0.0)


def test_incremental_agrees_with_the_sweep_route_and_is_deterministic(rcd):
    S = mixture_S(19, 700)
    cap = oracle.quota(700, [1, 2, 3])
    a1, o1, f1 = run_class(rcd, S, cap)
    a2, o2, f2 = run_class(rcd, S, cap)
    assert np.array_equal(a1, a2) and np.array_equal(o1, o2) and np.array_equal(f1, f2)
    a3, o3, f3 = run_class(rcd, S, cap, incremental=False)
    # the two routes' contract: the same decisions except at steps whose two best gains differ by less than
    # fp32 rounding; each route's trace is a correct run of Algorithm 1 under the 1e-5 window
    print("  incremental vs sweep agreement:", np.mean(a1 == a3), flush=True)
    if not np.array_equal(a1, a3):
        first = int(min(o1[a1 != a3].min(), o3[a1 != a3].min()))
        at = oracle.lockstep(S, cap, o3, a3, rel_tol=0.0, check=[first])
        assert at["worst_elem_gap"] <= 1e-5 and at["worst_block_gap"] <= 1e-5, (first, at)
    for a, o in ((a1, o1), (a3, o3)):
        res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5)
        assert res["rc"] == 0 and res["checked"] == cap.sum(), res
    assert np.allclose(f1, f3, rtol=1e-4)


def check_dataset(rcd, ds, assign, order, obj):
    Xd = dev(ds.X)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)
        cap = oracle.quota(len(idx), ds.r)
        S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
        check_against_oracle(S, cap, assign[idx], order[idx], obj[c])
        ref = oracle.similarity(ds.X[idx], ds.sigma2)
        res = oracle.lockstep(ref, cap, order[idx], assign[idx], rel_tol=1e-4 if ds.X.dtype == np.float32 else 1e-3)
        assert res["rc"] == 0, res


@pytest.mark.parametrize("name,L,n_c,d", [("tiny", 4, 250, 64), ("cifar10", 3, 700, 96), ("hetero8", 2, 900, 64),
                                          ("cifar100", 12, 150, 48), ("large", 2, 640, 256)])
def test_incremental_dataset_scaled_workloads(rcd, name, L, n_c, d):
    print(f"incremental dataset {name} scaled L={L} n_c={n_c} d={d}", flush=True)
    ds = si.make_dataset(si.WORKLOADS[name], L=L, n_c=n_c, d=d)
    N = ds.X.shape[0]
    mn, full = rcd.dataset_workspace_bytes(N, L, n_c, len(ds.r), rcd.MODE_INCREMENTAL)
    for nbytes in (full, mn):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        assign, order, obj = rcd.partition_dataset(dev(ds.X), dev(ds.labels), L, ds.r, ds.sigma2,
                                                   rcd.MODE_INCREMENTAL, ws)
        check_dataset(rcd, ds, assign.cpu().numpy(), order.cpu().numpy(), obj)


def test_mode_auto_takes_the_incremental_route_when_s_fits_and_recomputes_when_not(rcd):
    ds = si.make_dataset(si.WORKLOADS["cifar10"], L=3, n_c=700, d=96)
    N, K = ds.X.shape[0], len(ds.r)
    Xd, yd = dev(ds.X), dev(ds.labels)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, 700, K, rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    a0, o0, f0 = rcd.partition_dataset(Xd, yd, ds.L, ds.r, ds.sigma2, rcd.MODE_AUTO, ws)
    auto_stats = rcd.last_stats()
    a1, o1, f1 = rcd.partition_dataset(Xd, yd, ds.L, ds.r, ds.sigma2, rcd.MODE_INCREMENTAL, ws)
    assert torch.equal(a0, a1) and torch.equal(o0, o1) and np.array_equal(f0, f1)
    now = rcd.last_stats()
    assert {k: v for k, v in auto_stats.items() if k != "step_ticks"} == {k: v for k, v in now.items() if k != "step_ticks"}
    check_dataset(rcd, ds, a0.cpu().numpy(), o0.cpu().numpy(), f0)
    # a workspace too small for any class's S: the same call recomputes S inside the sweeps
    mn_rc, _ = rcd.dataset_workspace_bytes(N, ds.L, 700, K, rcd.MODE_RECOMPUTE)
    mn_st, _ = rcd.dataset_workspace_bytes(N, ds.L, 700, K, rcd.MODE_STORED)
    assert mn_rc < mn_st
    small = torch.empty(mn_rc, dtype=torch.uint8, device="cuda")
    a2, o2, f2 = rcd.partition_dataset(Xd, yd, ds.L, ds.r, ds.sigma2, rcd.MODE_AUTO, small)
    check_dataset(rcd, ds, a2.cpu().numpy(), o2.cpu().numpy(), f2)
    with pytest.raises(rcd.RcdError):
        rcd.partition_dataset(Xd, yd, ds.L, ds.r, ds.sigma2, rcd.MODE_STORED, small)


def test_skewed_class_sizes_on_every_route(rcd):
    # classes of 1, 37, 0, 640 and 1300 samples in one data set (the lanes get very unequal shares, one class is
    # smaller than K, one is empty): incremental, sweep, recompute and graph-cut routes, each refereed per class
    sizes = [1, 37, 0, 640, 1300]
    L, d, r = len(sizes), 64, [1, 2, 1, 3]
    rng = np.random.default_rng(77)
    X = si.make_class(seed=78, n=sum(sizes), d=d, G=6)
    labels = np.repeat(np.arange(L), sizes).astype(np.int32)
    perm = rng.permutation(len(labels))
    X, labels = np.ascontiguousarray(X[perm]), np.ascontiguousarray(labels[perm])
    Xd, yd = dev(X), dev(labels)
    N, K = len(labels), len(r)
    _, full = rcd.dataset_workspace_bytes(N, L, max(sizes), K, rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    for label, kw in (("incremental", dict(mode=rcd.MODE_INCREMENTAL)), ("sweeps", dict(mode=rcd.MODE_STORED)),
                      ("recompute", dict(mode=rcd.MODE_RECOMPUTE)), ("graph cut", dict(graph_cut=True))):
        print(f"  skewed classes, {label}", flush=True)
        assign, order, obj = rcd.partition_dataset(Xd, yd, L, r, float(d), workspace=ws, **kw)
        assign, order = assign.cpu().numpy(), order.cpu().numpy()
        assert np.all(assign >= 0)
        for c in range(L):
            idx = np.flatnonzero(labels == c)
            if len(idx) == 0:
                assert np.all(obj[c] == 0.0)
                continue
            cap = oracle.quota(len(idx), r)
            S = rcd.similarity(Xd, float(d), row_index=dev(idx.astype(np.int32))).cpu().numpy()
            a, o = assign[idx], order[idx]
            assert np.bincount(a, minlength=K).tolist() == cap.tolist()
            objective = "gc" if label == "graph cut" else "fl"
            res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, objective=objective)
            assert res["rc"] == 0 and res["checked"] == len(idx), (label, c, res)
            for k in range(K):
                ref = oracle.f_value(S, np.flatnonzero(a == k), objective)
                assert abs(obj[c, k] - ref) <= 1e-4 * max(ref, 1e-30) + 1e-9, (label, c, k, obj[c, k], ref)
