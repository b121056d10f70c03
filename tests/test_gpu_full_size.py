"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py
times (rcd_partition_dataset, stored S, all classes advanced together).  The
oracle cannot replay 50 000 steps of 5000-sample classes in test time, so it
referees SAMPLED steps: the referee replays the whole GPU trace (cheap state
updates) and, at the sampled steps, recomputes every candidate's gain from that
state and checks block and element choice.  Similarity is checked on sampled
sub-matrices; invariants and objectives are checked in full."""
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


def sampled_steps(total, rng, k):
    fixed = list(range(min(6, total))) + [total // 2, total - 2, total - 1]
    extra = rng.choice(total, size=min(k, total), replace=False).tolist()
    return sorted(set(s for s in fixed + extra if 0 <= s < total))


def run_full(rcd, ds, mode):
    N = ds.X.shape[0]
    counts = np.bincount(ds.labels, minlength=ds.L)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, int(counts.max()), len(ds.r), mode)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    Xd, yd = dev(ds.X), dev(ds.labels)
    assign, order, obj = rcd.partition_dataset(Xd, yd, ds.L, ds.r, ds.sigma2, mode, ws)
    del ws
    return Xd, assign.cpu().numpy(), order.cpu().numpy(), obj


def referee_classes(rcd, ds, Xd, assign, order, obj, rng, n_steps, sim_tol, classes):
    """check_class on several classes with the oracle's referees running side by side: the similarity
    matrices are fetched from the GPU one after the other, the (single-threaded, GIL-free) oracle calls of
    different classes run on a small thread pool.  Returns the referee's report per class."""
    from concurrent.futures import ThreadPoolExecutor

    K = len(ds.r)
    jobs = []
    for c in classes:
        idx = np.flatnonzero(ds.labels == c)
        n = len(idx)
        cap = oracle.quota(n, ds.r)
        a, o = assign[idx], order[idx]
        assert np.bincount(a, minlength=K).tolist() == cap.tolist()
        assert np.array_equal(np.sort(o), np.arange(n))
        S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
        sub = np.sort(rng.choice(n, size=min(192, n), replace=False))
        steps = sampled_steps(n, rng, n_steps)
        jobs.append((c, idx, cap, a, o, S, sub, steps))

    def one(job):
        c, idx, cap, a, o, S, sub, steps = job
        ref = oracle.similarity(ds.X[idx[sub]], ds.sigma2)
        assert np.max(np.abs(S[np.ix_(sub, sub)] - ref) / ref) <= sim_tol, c
        res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, check=steps)
        assert res["rc"] == 0 and res["checked"] == len(steps), (c, res)
        for k in range(K):
            ref_f = oracle.f_value(S, np.flatnonzero(a == k))
            assert abs(obj[c, k] - ref_f) <= 1e-4 * ref_f, (c, k)
        return c, res

    with ThreadPoolExecutor(max_workers=8) as pool:
        return dict(pool.map(one, jobs))


def check_class(rcd, ds, Xd, c, assign, order, obj, rng, n_steps, sim_tol, referee=True):
    idx = np.flatnonzero(ds.labels == c)
    n = len(idx)
    K = len(ds.r)
    cap = oracle.quota(n, ds.r)
    a, o = assign[idx], order[idx]
    # invariants: exact quotas, every sample taken exactly once, class balance
    assert np.bincount(a, minlength=K).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(n))
    if not referee:
        return None
    S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
    # similarity on a sampled sub-matrix against the oracle
    sub = np.sort(rng.choice(n, size=min(192, n), replace=False))
    ref = oracle.similarity(ds.X[idx[sub]], ds.sigma2)
    got = S[np.ix_(sub, sub)]
    assert np.max(np.abs(got - ref) / ref) <= sim_tol
    # sampled lock step on the same S
    steps = sampled_steps(n, rng, n_steps)
    res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, check=steps)
    assert res["rc"] == 0 and res["checked"] == len(steps), res
    # objectives from the definition
    for k in range(K):
        ref_f = oracle.f_value(S, np.flatnonzero(a == k))
        assert abs(obj[c, k] - ref_f) <= 1e-4 * ref_f
    return res


@pytest.mark.parametrize("name", ["cifar10", "hetero8"])
def test_full_size_stored_workloads(rcd, name):
    print(f"full size {name}", flush=True)
    ds = si.make_dataset(si.WORKLOADS[name])
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_STORED)
    stats = rcd.last_stats()
    assert stats["steps"] == ds.X.shape[0]
    rng = np.random.default_rng(11)
    # every class: invariants, similarity samples, objectives from the definition, and the referee at the
    # first, middle and last steps plus 100 steps drawn at random (about 105 of the class's 5000)
    reports = referee_classes(rcd, ds, Xd, assign, order, obj, rng, n_steps=100, sim_tol=1e-5, classes=range(ds.L))
    near = sum(r["near_block"] + r["near_elem"] for r in reports.values())
    assert len(reports) == ds.L and all(r["checked"] >= 100 for r in reports.values())
    print(f"  steps refereed: {sum(r['checked'] for r in reports.values())}, near-ties accepted: {near}; stats {stats}",
          flush=True)
    # identical class balance in every class
    per_class = [np.bincount(assign[ds.labels == c], minlength=len(ds.r)) for c in range(ds.L)]
    assert all(np.array_equal(p, per_class[0]) for p in per_class)


def test_full_size_cifar100_every_step(rcd):
    print("full size cifar100", flush=True)
    ds = si.make_dataset(si.WORKLOADS["cifar100"])
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_STORED)
    rng = np.random.default_rng(12)
    near = 0
    for c in range(ds.L):
        res = check_class(rcd, ds, Xd, c, assign, order, obj, rng, n_steps=500, sim_tol=1e-5, referee=c % 5 == 0)
        if res:
            assert res["checked"] == 500            # n_c = 500: every step is refereed
            near += res["near_block"] + res["near_elem"]
    print(f"  near-ties accepted over 20 fully refereed classes: {near}", flush=True)


def test_large_class_recompute_scaled_every_step(rcd):
    # same d, dtype, K and capacity ratios as the large-class workload, class size cut so
    # that the oracle can referee every step; S is never stored (forced recompute)
    print("large workload scaled to 2 x 2304", flush=True)
    ds = si.make_dataset(si.WORKLOADS["large"], L=2, n_c=2304)
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_RECOMPUTE)
    rng = np.random.default_rng(13)
    for c in range(ds.L):
        res = check_class(rcd, ds, Xd, c, assign, order, obj, rng, n_steps=2304, sim_tol=2e-2)
        assert res["checked"] == 2304
        print(f"  class {c}: {res}", flush=True)


def test_large_class_full_size_window_recompute_equals_stored(rcd):
    # one class of the large workload at full size (50 000 x 2048 bf16): the first 48
    # steps (quotas cut to a window, same ratios), once recomputing S inside every sweep
    # and once streaming a stored S; both must take the same decisions.
    print("large workload, one full-size class, 48-step window", flush=True)
    w = si.WORKLOADS["large"]
    X = si.make_class(seed=w.seed, n=w.n_c, d=w.d, G=w.G, dtype="bf16")
    Xd = dev(X)
    cap = np.array([2, 2, 4, 4, 6, 6, 8, 16], dtype=np.int64)
    a1, o1, f1 = rcd.partition_class(X=Xd, cap=cap, sigma2=float(w.d))
    s1 = rcd.last_stats()
    S = rcd.similarity(Xd, float(w.d))
    a2, o2, f2 = rcd.partition_class(S=S, cap=cap)
    a1, o1, a2, o2 = a1.cpu().numpy(), o1.cpu().numpy(), a2.cpu().numpy(), o2.cpu().numpy()
    assert np.bincount(a1[a1 >= 0], minlength=8).tolist() == cap.tolist()
    assert np.array_equal(a1, a2) and np.array_equal(o1, o2)
    assert np.allclose(f1, f2, rtol=1e-6)
    # sampled similarity entries against the oracle, and objective of one block from the definition
    rng = np.random.default_rng(14)
    sub = np.sort(rng.choice(w.n_c, size=96, replace=False))
    ref = oracle.similarity(X[sub], float(w.d))
    got = S[torch.from_numpy(sub).cuda()][:, torch.from_numpy(sub).cuda()].cpu().numpy()
    assert np.max(np.abs(got - ref) / ref) <= 2e-2
    members = np.flatnonzero(a1 == 0)
    cols = S[:, torch.from_numpy(members).cuda()].max(dim=1).values.double().sum().item()
    assert abs(f1[0] - cols) <= 1e-4 * cols
    print(f"  stats {s1}", flush=True)
    # the oracle referees steps of the recompute route's own trace at this size (first, middle, last of the
    # window), on the stored matrix the route never saw: 50 000 candidates x 50 000 terms per refereed step
    Sh = S.cpu().numpy()
    del S
    steps = [0, 1, 7, 8, 23, 24, 46, 47]
    res = oracle.lockstep(Sh, cap, o1, a1, rel_tol=1e-5, check=steps)
    print(f"  referee on the recompute trace: {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res


# ------------------------------------------------------------------ incremental-gain route at full size
@pytest.mark.parametrize("name", ["cifar10", "hetero8"])
def test_full_size_incremental_workloads(rcd, name):
    print(f"full size {name}, incremental gains", flush=True)
    ds = si.make_dataset(si.WORKLOADS[name])
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_INCREMENTAL)
    stats = rcd.last_stats()
    assert stats["steps"] == ds.X.shape[0]
    rng = np.random.default_rng(21)
    reports = referee_classes(rcd, ds, Xd, assign, order, obj, rng, n_steps=100, sim_tol=1e-5, classes=range(ds.L))
    assert len(reports) == ds.L and all(r["checked"] >= 100 for r in reports.values())
    print(f"  steps refereed: {sum(r['checked'] for r in reports.values())}; stats {stats}", flush=True)
    # The sweep route on the same data: the two routes' contract is the same decisions except at steps whose two
    # best gains differ by less than fp32 rounding (this route carries gains in double, the sweeps sum in fp32).
    # A class whose traces differ must differ first at such a step, as the oracle sees it.
    _, a2, o2, f2 = run_full(rcd, ds, rcd.MODE_STORED)
    print("  agreement with the sweep route:", np.mean(assign == a2), flush=True)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)
        if np.array_equal(assign[idx], a2[idx]) and np.array_equal(order[idx], o2[idx]):
            continue
        differ = (assign[idx] != a2[idx]) | (order[idx] != o2[idx])
        first = int(min(order[idx][differ].min(), o2[idx][differ].min()))
        S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
        at = oracle.lockstep(S, oracle.quota(len(idx), ds.r), o2[idx], a2[idx], rel_tol=0.0, check=[first])
        print(f"  class {c}: traces part at step {first}: {at}", flush=True)
        assert at["worst_elem_gap"] <= 1e-5 and at["worst_block_gap"] <= 1e-5, (c, first, at)
    assert np.allclose(obj, f2, rtol=1e-4)


def test_full_size_cifar100_incremental_every_step(rcd):
    print("full size cifar100, incremental gains", flush=True)
    ds = si.make_dataset(si.WORKLOADS["cifar100"])
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_INCREMENTAL)
    rng = np.random.default_rng(22)
    for c in range(ds.L):
        res = check_class(rcd, ds, Xd, c, assign, order, obj, rng, n_steps=500, sim_tol=1e-5, referee=c % 10 == 3)
        if res:
            assert res["checked"] == 500


def test_large_class_one_full_class_incremental(rcd, monkeypatch):
    # one whole class of the large workload (50 000 x 2048 bf16, K = 8, its real quotas): similarity
    # stored (10 GB), all 50 000 steps by the incremental route; the oracle referees sampled steps
    # on the same S and the objectives come from the definition
    print("large workload, one full class, all 50 000 steps, incremental gains", flush=True)
    w = si.WORKLOADS["large"]
    X = si.make_class(seed=w.seed, n=w.n_c, d=w.d, G=w.G, dtype="bf16")
    Xd = dev(X)
    S = rcd.similarity(Xd, float(w.d))
    cap = oracle.quota(w.n_c, w.r)
    assert cap.tolist() == [2083, 2083, 4166, 4166, 6251, 6250, 8334, 16667]
    a, o, f = rcd.partition_class(S=S, cap=cap, mode=rcd.MODE_INCREMENTAL)
    stats = rcd.last_stats()
    print(f"  stats {stats}", flush=True)
    a, o = a.cpu().numpy(), o.cpu().numpy()
    assert stats["steps"] == w.n_c
    assert np.bincount(a, minlength=8).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(w.n_c))
    # a class this size is shared among several workgroups: the one-workgroup loop must give the same bits
    monkeypatch.setenv("RCD_MW_MIN_N", "0")
    a1, o1, f1 = rcd.partition_class(S=S, cap=cap, mode=rcd.MODE_INCREMENTAL)
    monkeypatch.delenv("RCD_MW_MIN_N")
    print(f"  one workgroup: stats {rcd.last_stats()}", flush=True)
    assert np.array_equal(a1.cpu().numpy(), a) and np.array_equal(o1.cpu().numpy(), o) and np.array_equal(f1, f)
    # objectives from the definition, on the device (max over the block's columns, summed in double)
    for k in (0, 7):
        members = torch.from_numpy(np.flatnonzero(a == k)).cuda()
        ref = 0.0
        for lo in range(0, w.n_c, 5000):        # row chunks keep the gathered slab small
            ref += S[lo:lo + 5000][:, members].max(dim=1).values.double().sum().item()
        assert abs(f[k] - ref) <= 1e-4 * ref
    # sampled lock step by the oracle on the same S
    Sh = S.cpu().numpy()
    del S
    steps = [0, 1, 7, 8, 9, 1000, 25000, 49998, 49999]
    res = oracle.lockstep(Sh, cap, o, a, rel_tol=1e-5, check=steps)
    print(f"  referee {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res


def test_large_workload_all_classes_incremental(rcd):
    # the whole large workload: 20 classes x 50 000 samples, d = 2048 bf16, K = 8, every class's S stored
    # (202 GB of workspace), one million steps; invariants for every class, one class refereed
    print("large workload, all 20 classes, incremental gains", flush=True)
    w = si.WORKLOADS["large"]
    ds = si.make_dataset(w)
    N = ds.X.shape[0]
    _, full = rcd.dataset_workspace_bytes(N, ds.L, w.n_c, len(ds.r), rcd.MODE_INCREMENTAL)
    free, _ = torch.cuda.mem_get_info()
    if full > 0.95 * free:
        pytest.skip(f"needs {full / 1e9:.0f} GB of workspace, {free / 1e9:.0f} GB free on this device")
    Xd, assign, order, obj = run_full(rcd, ds, rcd.MODE_INCREMENTAL)
    stats = rcd.last_stats()
    print(f"  stats {stats}", flush=True)
    assert stats["steps"] == N
    cap = oracle.quota(w.n_c, ds.r)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)
        assert np.bincount(assign[idx], minlength=len(ds.r)).tolist() == cap.tolist()
        assert np.array_equal(np.sort(order[idx]), np.arange(w.n_c))
    # class 13: the library's own similarity of the class (gathered rows), sampled steps refereed on it
    idx = np.flatnonzero(ds.labels == 13)
    S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32)))
    a, o = assign[idx], order[idx]
    members = torch.from_numpy(np.flatnonzero(a == 7)).cuda()
    ref = 0.0
    for lo in range(0, w.n_c, 5000):
        ref += S[lo:lo + 5000][:, members].max(dim=1).values.double().sum().item()
    assert abs(obj[13, 7] - ref) <= 1e-4 * ref
    Sh = S.cpu().numpy()
    del S
    steps = [0, 3, 8, 500, 30000, 49999]
    res = oracle.lockstep(Sh, cap, o, a, rel_tol=1e-5, check=steps)
    print(f"  referee of class 13: {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res


def check_class_gc(rcd, ds, Xd, c, assign, order, obj, rng, n_steps):
    idx = np.flatnonzero(ds.labels == c)
    n = len(idx)
    K = len(ds.r)
    cap = oracle.quota(n, ds.r)
    a, o = assign[idx], order[idx]
    assert np.bincount(a, minlength=K).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(n))
    S = rcd.similarity(Xd, ds.sigma2, row_index=dev(idx.astype(np.int32))).cpu().numpy()
    steps = sampled_steps(n, rng, n_steps)
    res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, check=steps, objective="gc")
    assert res["rc"] == 0 and res["checked"] == len(steps), res
    mass = float(S.astype(np.float64).sum()) / K
    for k in range(K):
        ref_f = oracle.f_value(S, np.flatnonzero(a == k), "gc")
        assert abs(obj[c, k] - ref_f) <= 1e-4 * ref_f + 1e-12 * mass
    return res


@pytest.mark.parametrize("name", ["cifar10", "hetero8"])
def test_full_size_graph_cut_workloads(rcd, name):
    print(f"full size {name}, graph-cut function", flush=True)
    ds = si.make_dataset(si.WORKLOADS[name])
    N = ds.X.shape[0]
    counts = np.bincount(ds.labels, minlength=ds.L)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, int(counts.max()), len(ds.r), rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    Xd = dev(ds.X)
    assign, order, obj = rcd.partition_dataset(Xd, dev(ds.labels), ds.L, ds.r, ds.sigma2, workspace=ws, graph_cut=True)
    del ws
    stats = rcd.last_stats()
    print(f"  stats {stats}", flush=True)
    assert stats["steps"] == N
    assign, order = assign.cpu().numpy(), order.cpu().numpy()
    rng = np.random.default_rng(23)
    for c in (1, 5, 8):
        res = check_class_gc(rcd, ds, Xd, c, assign, order, obj, rng, n_steps=10)
        print(f"  class {c} referee {res}", flush=True)
    for c in range(ds.L):
        idx = np.flatnonzero(ds.labels == c)
        assert np.bincount(assign[idx], minlength=len(ds.r)).tolist() == oracle.quota(len(idx), ds.r).tolist()


def test_large_class_one_full_class_graph_cut(rcd, monkeypatch):
    # one whole class of the large workload (50 000 x 2048 bf16, K = 8, its real quotas), S stored, all
    # 50 000 steps with the graph-cut function; invariants, objectives from the definition (on the device,
    # in double), the first pick from its closed form, the oracle's referee on sampled steps
    print("large workload, one full class, all 50 000 steps, graph-cut function", flush=True)
    w = si.WORKLOADS["large"]
    X = si.make_class(seed=w.seed, n=w.n_c, d=w.d, G=w.G, dtype="bf16")
    S = rcd.similarity(dev(X), float(w.d))
    cap = oracle.quota(w.n_c, w.r)
    a, o, f = rcd.partition_class_graph_cut(S, cap)
    stats = rcd.last_stats()
    print(f"  stats {stats}", flush=True)
    a, o = a.cpu().numpy(), o.cpu().numpy()
    assert stats["steps"] == w.n_c
    assert np.bincount(a, minlength=8).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(w.n_c))
    # a class this size is shared among several workgroups: the one-workgroup loop must give the same bits
    monkeypatch.setenv("RCD_MW_MIN_N", "0")
    a1, o1, f1 = rcd.partition_class_graph_cut(S, cap)
    monkeypatch.delenv("RCD_MW_MIN_N")
    print(f"  one workgroup: stats {rcd.last_stats()}", flush=True)
    assert np.array_equal(a1.cpu().numpy(), a) and np.array_equal(o1.cpu().numpy(), o) and np.array_equal(f1, f)
    # empty blocks: the marginal value of v is its column sum without the diagonal, so the first pick is its argmax
    colsum = S.double().sum(dim=0) - S.diagonal().double()
    first = int(np.flatnonzero(o == 0)[0])
    assert colsum[first].item() >= colsum.max().item() * (1 - 1e-12)
    # f(A) = similarity mass between A and the rest of the class
    for k in (0, 7):
        inside = torch.from_numpy(a == k).cuda()
        members = torch.nonzero(inside).flatten()
        ref = 0.0
        for lo in range(0, w.n_c, 5000):
            rows = S[lo:lo + 5000]
            outside = (~inside[lo:lo + 5000]).double()
            ref += (rows[:, members].double().sum(dim=1) * outside).sum().item()
        assert abs(f[k] - ref) <= 1e-6 * ref, (k, f[k], ref)
    Sh = S.cpu().numpy()
    del S
    steps = [0, 1, 25000, 49000, 49998, 49999]
    res = oracle.lockstep(Sh, cap, o, a, rel_tol=1e-5, check=steps, objective="gc")
    print(f"  referee {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res


def test_whole_data_set_greedmax_incremental(rcd):
    # the cifar10 workload's 50 000 samples as ONE class (no class split: the whole-set greedy the paper's
    # class-wise scheme is compared with), K = 4, similarity stored (10 GB), all 50 000 steps by the
    # incremental route; invariants, objectives from the definition, sampled steps refereed on the same S
    print("whole-set GreedMax: cifar10 features as one class of 50 000", flush=True)
    ds = si.make_dataset(si.WORKLOADS["cifar10"])
    N = ds.X.shape[0]
    K = len(ds.r)
    labels = torch.zeros(N, dtype=torch.int32, device="cuda")
    Xd = dev(ds.X)
    _, full = rcd.dataset_workspace_bytes(N, 1, N, K, rcd.MODE_INCREMENTAL)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    a, o, f = rcd.partition_dataset(Xd, labels, 1, ds.r, ds.sigma2, rcd.MODE_INCREMENTAL, ws)
    stats = rcd.last_stats()
    print(f"  stats {stats}", flush=True)
    del ws
    a, o = a.cpu().numpy(), o.cpu().numpy()
    cap = oracle.quota(N, ds.r)
    assert stats["steps"] == N
    assert np.bincount(a, minlength=K).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(N))
    S = rcd.similarity(Xd, ds.sigma2)
    for k in range(K):
        members = torch.from_numpy(np.flatnonzero(a == k)).cuda()
        ref = 0.0
        for lo in range(0, N, 5000):
            ref += S[lo:lo + 5000][:, members].max(dim=1).values.double().sum().item()
        assert abs(f[0, k] - ref) <= 1e-4 * ref
    Sh = S.cpu().numpy()
    del S
    steps = [0, 1, 3, 4, 5, 1000, 25000, 49998, 49999]
    res = oracle.lockstep(Sh, cap, o, a, rel_tol=1e-5, check=steps)
    print(f"  referee {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res
    # without the class split nothing balances the labels: the shards' class counts are no longer the quotas
    per = np.stack([np.bincount(ds.labels[a == k], minlength=ds.L) for k in range(K)])
    print(f"  class counts per worker without the class split:\n{per}", flush=True)


@pytest.mark.parametrize("route", ["incremental", "sweeps", "graph_cut"])
def test_sixteen_blocks_on_a_12000_sample_class(rcd, route):
    # the largest block count on a class of 47 tiles of 256: every step taken, sampled steps refereed
    print(f"K = 16, n = 12000, {route}", flush=True)
    n, d = 12000, 128
    r = [3, 1, 4, 1, 2, 2, 1, 3, 4, 4, 1, 2, 3, 3, 2, 1]
    X = si.make_class(seed=91, n=n, d=d, G=8)
    S = rcd.similarity(dev(X), float(d))
    cap = oracle.quota(n, r)
    if route == "graph_cut":
        a, o, f = rcd.partition_class_graph_cut(S, cap)
    else:
        a, o, f = rcd.partition_class(S=S, cap=cap,
                                      mode=rcd.MODE_INCREMENTAL if route == "incremental" else rcd.MODE_STORED)
    a, o = a.cpu().numpy(), o.cpu().numpy()
    assert np.bincount(a, minlength=16).tolist() == cap.tolist()
    assert np.array_equal(np.sort(o), np.arange(n))
    Sh = S.cpu().numpy()
    objective = "gc" if route == "graph_cut" else "fl"
    steps = [0, 1, 15, 16, 17, 100, 3000, 6000, 11000, 11998, 11999]
    res = oracle.lockstep(Sh, cap, o, a, rel_tol=1e-5, check=steps, objective=objective)
    print(f"  referee {res}", flush=True)
    assert res["rc"] == 0 and res["checked"] == len(steps), res
    for k in (0, 2, 15):
        ref = oracle.f_value(Sh, np.flatnonzero(a == k), objective)
        assert abs(f[k] - ref) <= 1e-4 * ref + 1e-9
