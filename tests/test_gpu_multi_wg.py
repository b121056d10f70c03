"""GPU parity of the step loops that share a class among several workgroups (incremental-gain route and
graph-cut function, Algorithm 1's inner loop for large classes).  The library takes them from 16 384 samples
on; here the tuning switches RCD_MW_MIN_N / RCD_MW_SLICE bring them down to classes the oracle referees at
every step.  They must give the one-workgroup loops' results bit for bit, and a barrier wait that runs out
must come back as an error with every kernel finished."""
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


def run(rcd, monkeypatch, S, cap, route, shared, slice_=256):
    monkeypatch.setenv("RCD_MW_MIN_N", "1" if shared else "0")
    monkeypatch.setenv("RCD_MW_SLICE", str(slice_))
    if route == "gc":
        a, o, f = rcd.partition_class_graph_cut(dev(S), cap)
    else:
        a, o, f = rcd.partition_class(S=dev(S), cap=cap, mode=rcd.MODE_INCREMENTAL)
    return a.cpu().numpy(), o.cpu().numpy(), f


@pytest.mark.parametrize("route", ["inc", "gc"])
@pytest.mark.parametrize("n,r,slice_", [(600, [1, 1, 2, 4], 256), (1300, [2, 1], 256), (2100, [1, 1, 1, 2, 2, 3, 4, 6], 512),
                                        (1000, [3, 1, 4, 1, 2, 2, 1, 3, 4, 4, 1, 2, 3, 3, 2, 1], 256), (257, [5], 256),
                                        (3000, [1, 2, 3], 256)])
def test_shared_class_matches_one_workgroup_and_the_oracle(rcd, monkeypatch, route, n, r, slice_):
    print(f"several workgroups per class: {route} n={n} K={len(r)} slice={slice_}", flush=True)
    S = mixture_S(300 + n, n)
    cap = oracle.quota(n, r)
    a1, o1, f1 = run(rcd, monkeypatch, S, cap, route, shared=True, slice_=slice_)
    a0, o0, f0 = run(rcd, monkeypatch, S, cap, route, shared=False)
    assert np.array_equal(a1, a0) and np.array_equal(o1, o0) and np.array_equal(f1, f0)
    objective = "gc" if route == "gc" else "fl"
    res = oracle.lockstep(S, cap, o1, a1, rel_tol=1e-5, objective=objective)
    assert res["rc"] == 0 and res["checked"] == n, res
    for k in range(len(cap)):
        ref = oracle.f_value(S, np.flatnonzero(a1 == k), objective)
        assert abs(f1[k] - ref) <= 1e-4 * abs(ref) + 1e-9


@pytest.mark.parametrize("route", ["inc", "gc"])
def test_shared_class_exact_ties_zero_quotas_and_leftovers(rcd, monkeypatch, route):
    # constant similarity: every candidate ties at every step, the lowest index must win whichever workgroup owns it
    n, c = 1500, 0.25
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    cap = np.array([300, 0, 700, 200], dtype=np.int64)          # a zero quota, 300 samples left over
    a, o, f = run(rcd, monkeypatch, S, cap, route, shared=True)
    objective = "gc" if route == "gc" else "fl"
    res = oracle.lockstep(S, cap, o, a, rel_tol=0.0, objective=objective)
    assert res["rc"] == 0 and res["exact"] == cap.sum(), res
    assert np.sum(a == -1) == n - cap.sum() and np.all(o[a == -1] == -1)
    taken = np.flatnonzero(a >= 0)
    assert taken.tolist() == list(range(int(cap.sum())))        # lowest indices first
    # duplicated samples: identical columns must keep tying exactly
    X = si.make_class(seed=77, n=400, d=16)
    X = np.concatenate([X, X, X])
    S = oracle.similarity(X, 16.0)
    cap = oracle.quota(1200, [1, 2, 1])
    a, o, f = run(rcd, monkeypatch, S, cap, route, shared=True)
    res = oracle.lockstep(S, cap, o, a, rel_tol=0.0 if route == "gc" else 1e-5, objective=objective)
    assert res["rc"] == 0 and res["checked"] == 1200, res


@pytest.mark.parametrize("graph_cut", [False, True])
def test_data_set_with_shared_and_unshared_classes(rcd, monkeypatch, graph_cut):
    # classes of very different sizes in one launch: the large ones are shared, the small ones keep one workgroup
    monkeypatch.setenv("RCD_MW_MIN_N", "1")
    monkeypatch.setenv("RCD_MW_SLICE", "256")
    sizes = np.array([40, 1500, 0, 700, 3, 2300, 260])
    L, N, d, r = len(sizes), int(sizes.sum()), 64, [1, 2, 3, 1, 1]
    X = si.make_class(seed=401, n=N, d=d, G=5)
    labels = np.repeat(np.arange(L), sizes).astype(np.int32)
    perm = np.random.default_rng(5).permutation(N)
    X, labels = np.ascontiguousarray(X[perm]), np.ascontiguousarray(labels[perm])
    Xd, yd = dev(X), dev(labels)
    mode = rcd.MODE_STORED if graph_cut else rcd.MODE_INCREMENTAL
    results = []
    for which in (0, 1):
        sz = rcd.dataset_workspace_bytes(N, L, int(sizes.max()), len(r), rcd.MODE_STORED)[which]
        ws = torch.empty(sz, dtype=torch.uint8, device="cuda")
        assign, order, obj = rcd.partition_dataset(Xd, yd, L, r, float(d), mode, ws, graph_cut=graph_cut)
        results.append((assign.cpu().numpy(), order.cpu().numpy(), obj))
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    assign, order, obj = results[1]
    objective = "gc" if graph_cut else "fl"
    for c in range(L):
        idx = np.flatnonzero(labels == c)
        if len(idx) == 0:
            assert np.all(obj[c] == 0.0)
            continue
        cap = oracle.quota(len(idx), r)
        S = rcd.similarity(Xd, float(d), row_index=dev(idx.astype(np.int32))).cpu().numpy()
        res = oracle.lockstep(S, cap, order[idx], assign[idx], rel_tol=1e-5, objective=objective)
        assert res["rc"] == 0 and res["checked"] == len(idx), (c, res)
        for k in range(len(r)):
            ref = oracle.f_value(S, np.flatnonzero(assign[idx] == k), objective)
            assert abs(obj[c, k] - ref) <= 1e-4 * abs(ref) + 1e-9
    # the unshared run of the same data set gives the same bits
    monkeypatch.setenv("RCD_MW_MIN_N", "0")
    ws = torch.empty(rcd.dataset_workspace_bytes(N, L, int(sizes.max()), len(r), rcd.MODE_STORED)[1], dtype=torch.uint8,
                     device="cuda")
    a0, o0, f0 = rcd.partition_dataset(Xd, yd, L, r, float(d), mode, ws, graph_cut=graph_cut)
    assert np.array_equal(a0.cpu().numpy(), assign) and np.array_equal(o0.cpu().numpy(), order) and np.array_equal(f0, obj)


@pytest.mark.parametrize("route", ["inc", "gc"])
def test_a_barrier_wait_that_runs_out_is_reported_and_every_kernel_exits(rcd, monkeypatch, route):
    # the bound of a barrier wait set to zero from the host: the first workgroup to arrive finds the others
    # missing, raises the flag, every workgroup falls through and the call returns an error; the next call,
    # with the default bound, works
    S = mixture_S(12, 2000)
    cap = oracle.quota(2000, [1, 1])
    monkeypatch.setenv("RCD_MW_SPIN_MS", "0")
    with pytest.raises(rcd.RcdError) as e:
        run(rcd, monkeypatch, S, cap, route, shared=True)
    assert e.value.status == 6 and "grid barrier" in str(e.value)
    monkeypatch.delenv("RCD_MW_SPIN_MS")
    torch.cuda.synchronize()
    a, o, f = run(rcd, monkeypatch, S, cap, route, shared=True)
    res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, objective="gc" if route == "gc" else "fl")
    assert res["rc"] == 0 and res["checked"] == 2000, res


@pytest.mark.parametrize("route", ["inc", "gc"])
def test_thirty_two_workgroups_per_class(rcd, monkeypatch, route):
    # the most workgroups a class can have (the polling wave holds one post per lane, 32 of them here), on a class
    # of 33 slices of 256 samples; same bits as one workgroup, sampled steps refereed by the oracle
    n = 8300
    S = mixture_S(33, n)
    cap = oracle.quota(n, [1, 2, 1, 3, 1])
    monkeypatch.setenv("RCD_MW_MAX_WGS", "32")
    a1, o1, f1 = run(rcd, monkeypatch, S, cap, route, shared=True, slice_=256)
    a0, o0, f0 = run(rcd, monkeypatch, S, cap, route, shared=False)
    assert np.array_equal(a1, a0) and np.array_equal(o1, o0) and np.array_equal(f1, f0)
    objective = "gc" if route == "gc" else "fl"
    steps = [0, 1, 4, 5, 6, 100, 2000, 4150, 8000, 8298, 8299]
    res = oracle.lockstep(S, cap, o1, a1, rel_tol=1e-5, objective=objective, check=steps)
    assert res["rc"] == 0 and res["checked"] == len(steps), res
