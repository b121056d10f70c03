"""GPU parity of Algorithm 1 with the graph-cut function of Section 4 (rcd_partition_class_graph_cut,
rcd_partition_dataset_graph_cut): the oracle's lock-step referee on the same S, exact-tie cases
with a zero window, objectives from the definition, negative marginal values taken when the
quotas demand it, quota and cover invariants."""
import ctypes

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


def run_class(rcd, S, cap):
    assign, order, obj = rcd.partition_class_graph_cut(dev(S), cap)
    return assign.cpu().numpy(), order.cpu().numpy(), obj


def check_against_oracle(S, cap, assign, order, obj, rel_tol=1e-5):
    cap = np.asarray(cap, dtype=np.int64)
    n = S.shape[0]
    assert np.bincount(assign[assign >= 0], minlength=len(cap)).tolist() == cap.tolist()
    assert np.sum(assign < 0) == n - cap.sum()
    assert sorted(order[order >= 0].tolist()) == list(range(int(cap.sum())))
    res = oracle.lockstep(S, cap, order, assign, rel_tol=rel_tol, objective="gc")
    assert res["rc"] == 0, res
    assert res["checked"] == cap.sum()
    scale = max(1.0, float(S.astype(np.float64).sum()) / max(len(cap), 1))
    for k in range(len(cap)):
        ref = oracle.f_value(S, np.flatnonzero(assign == k), "gc")
        # f is a sum of marginal values of both signs: the error bound is against the mass summed
        assert abs(obj[k] - ref) <= 1e-4 * max(ref, 1e-30) + 1e-12 * scale, (k, obj[k], ref)
    return res


@pytest.mark.parametrize("n,r", [(1, [1]), (250, [1, 1]), (600, [1, 1, 2, 4]), (1000, [1, 1, 1, 2, 2, 3, 4, 6]),
                                 (520, [3, 1, 4, 1, 2, 2, 1, 3, 4, 4, 1, 2, 3, 3, 2, 1]), (257, [5]), (1300, [2, 1])])
def test_graph_cut_class_greedy_lockstep(rcd, n, r):
    print(f"graph-cut class greedy n={n} K={len(r)}", flush=True)
    S = mixture_S(700 + n, n)
    cap = oracle.quota(n, r)
    assign, order, obj = run_class(rcd, S, cap)
    res = check_against_oracle(S, cap, assign, order, obj)
    stats = rcd.last_stats()
    assert stats["steps"] == n and stats["useful_evals"] == n * (n + 1) // 2
    ref = oracle.partition_class(S, cap, trace=True, objective="gc")
    if res["near_block"] == 0 and res["near_elem"] == 0:
        assert np.array_equal(assign, ref["assign"]) and np.array_equal(order, ref["order"])
    if n > 1 and max(cap) >= 0.6 * n:
        # a block that ends up with most of the class: its late marginal values are negative and taken all the same
        assert np.min(ref["tr_gain"]) < 0.0


def test_graph_cut_exact_ties_follow_the_lowest_index_contract(rcd):
    # constant similarity: every marginal value ties exactly, and f(A) = |A| (n - |A|) c
    n, c = 96, 0.25
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    for cap in ([32, 32, 32], [10, 30, 56], [96], [5, 0, 7]):
        assign, order, obj = run_class(rcd, S, cap)
        ref = oracle.partition_class(S, cap, objective="gc")
        assert np.array_equal(assign, ref["assign"]) and np.array_equal(order, ref["order"])
        assert obj.tolist() == [m * (n - m) * c for m in cap]
        check_against_oracle(S, cap, assign, order, obj, rel_tol=0.0)


def test_graph_cut_duplicate_samples(rcd):
    base = si.make_class(seed=33, n=150, d=16)
    X = np.concatenate([base, base], axis=0)
    S = oracle.similarity(X, 16.0)
    cap = oracle.quota(300, [1, 2])
    assign, order, obj = run_class(rcd, S, cap)
    check_against_oracle(S, cap, assign, order, obj)
    # identical rows go through identical arithmetic: of two copies that land in the same block the first goes first
    for i in range(150):
        if assign[i] == assign[i + 150]:
            assert order[i] < order[i + 150]


def test_graph_cut_zero_quota_leftovers_and_determinism(rcd):
    S = mixture_S(28, 300)
    cap = [0, 40, 0, 25]
    assign, order, obj = run_class(rcd, S, cap)
    check_against_oracle(S, cap, assign, order, obj)
    assert obj[0] == 0.0 and obj[2] == 0.0
    assert np.sum(assign == -1) == 235 and np.all(order[assign == -1] == -1)
    a2, o2, f2 = run_class(rcd, S, cap)
    assert np.array_equal(assign, a2) and np.array_equal(order, o2) and np.array_equal(obj, f2)
    assign, order, obj = run_class(rcd, S, [0, 0])
    assert np.all(assign == -1) and np.all(obj == 0.0)


def test_graph_cut_pitched_input_and_bad_arguments(rcd):
    n = 333
    S = mixture_S(29, n)
    cap = oracle.quota(n, [1, 3])
    wide = torch.zeros((n, 400), dtype=torch.float32, device="cuda")
    wide[:, :n] = dev(S)
    a1, o1, f1 = rcd.partition_class_graph_cut(wide[:, :n], cap)
    a2, o2, f2 = run_class(rcd, S, cap)
    assert np.array_equal(a1.cpu().numpy(), a2) and np.array_equal(o1.cpu().numpy(), o2) and np.array_equal(f1, f2)
    lib = rcd.load_library()
    obj = np.zeros(2)
    capa = np.asarray(cap, dtype=np.int64)
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = torch.empty(rcd.class_workspace_bytes(n, 2, 1), dtype=torch.uint8, device="cuda")
    args = lambda S_ptr, ld, ws_bytes: (S_ptr, ld, n, 2, capa.ctypes.data_as(ctypes.c_void_p), out.data_ptr(), None,
                                        obj.ctypes.data_as(ctypes.c_void_p), ws.data_ptr(), ws_bytes, None)
    assert lib.rcd_partition_class_graph_cut(*args(None, n, ws.numel())) == 1         # no S
    assert lib.rcd_partition_class_graph_cut(*args(wide.data_ptr(), n - 1, ws.numel())) == 1   # ld_s < n
    assert lib.rcd_partition_class_graph_cut(*args(wide.data_ptr(), 400, ws.numel() - 256)) == 5   # workspace short
    bad = dev(S).clone()
    bad[5, 7] = 1.5
    with pytest.raises(rcd.RcdError):
        rcd.partition_class_graph_cut(bad, cap)


def check_dataset(rcd, ds, assign, order, obj):
    Xd = dev(ds.X)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)
        cap = oracle.quota(len(idx), ds.r)
        S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
        check_against_oracle(S, cap, assign[idx], order[idx], obj[c])
        ref = oracle.similarity(ds.X[idx], ds.sigma2)
        # the library's S and the oracle's agree to 1e-6 per entry, a marginal value sums n of them
        res = oracle.lockstep(ref, cap, order[idx], assign[idx], rel_tol=1e-4 if ds.X.dtype == np.float32 else 1e-3,
                              objective="gc", abs_tol=1e-6 * len(idx))
        assert res["rc"] == 0, res


@pytest.mark.parametrize("name,L,n_c,d", [("tiny", 4, 250, 64), ("cifar10", 3, 700, 96), ("hetero8", 2, 900, 64),
                                          ("cifar100", 12, 150, 48), ("large", 2, 640, 256)])
def test_graph_cut_dataset_scaled_workloads(rcd, name, L, n_c, d):
    print(f"graph-cut dataset {name} scaled L={L} n_c={n_c} d={d}", flush=True)
    ds = si.make_dataset(si.WORKLOADS[name], L=L, n_c=n_c, d=d)
    N = ds.X.shape[0]
    mn, full = rcd.dataset_workspace_bytes(N, L, n_c, len(ds.r), rcd.MODE_STORED)
    for nbytes in (full, mn):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        assign, order, obj = rcd.partition_dataset(dev(ds.X), dev(ds.labels), L, ds.r, ds.sigma2, workspace=ws,
                                                   graph_cut=True)
        check_dataset(rcd, ds, assign.cpu().numpy(), order.cpu().numpy(), obj)
