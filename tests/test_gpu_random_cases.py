"""Seeded random cases of one class through every route of the C ABI (stored S by sweeps, stored S with
incremental gains, S recomputed in the sweeps, graph-cut function): sizes from 1 to 900, 1 to 16 blocks,
quotas that may be zero and need not cover the class, mixture features or a few distinct points
(many exact ties), each run refereed at every step by the oracle."""
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


def random_case(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 901))
    K = int(rng.integers(1, 17))
    d = int(rng.choice([8, 32, 64, 96]))
    repeated = rng.random() < 0.3
    if repeated:
        # a few distinct points, each repeated: whole groups of candidates tie exactly
        base = si.make_class(seed=seed, n=int(rng.integers(1, 6)), d=d)
        X = np.ascontiguousarray(base[rng.integers(0, len(base), size=n)])
    else:
        X = si.make_class(seed=seed, n=n, d=d, G=int(rng.integers(1, 6)))
    if rng.random() < 0.5:
        cap = oracle.quota(n, rng.integers(1, 6, size=K))
    else:
        cap = rng.multinomial(int(rng.integers(0, n + 1)), np.ones(K) / K).astype(np.int64)   # zeros, leftovers
    return X, cap, float(d), repeated


@pytest.mark.parametrize("seed", range(24))
def test_random_class_on_every_route(rcd, seed):
    X, cap, sigma2, repeated = random_case(1000 + seed)
    n, K = X.shape[0], len(cap)
    print(f"random case {seed}: n={n} K={K} d={X.shape[1]} sum of quotas {int(cap.sum())}", flush=True)
    Xd = torch.from_numpy(X).cuda()
    Sd = rcd.similarity(Xd, sigma2)
    S = Sd.cpu().numpy()
    assert np.max(np.abs(S - oracle.similarity(X, sigma2)) / np.maximum(oracle.similarity(X, sigma2), 1e-30)) <= 1e-5
    routes = [("sweeps", "fl", lambda: rcd.partition_class(S=Sd, cap=cap, mode=rcd.MODE_STORED)),
              ("incremental", "fl", lambda: rcd.partition_class(S=Sd, cap=cap, mode=rcd.MODE_INCREMENTAL)),
              ("recompute", "fl", lambda: rcd.partition_class(X=Xd, cap=cap, sigma2=sigma2, mode=rcd.MODE_RECOMPUTE)),
              ("graph cut", "gc", lambda: rcd.partition_class_graph_cut(Sd, cap))]
    for name, objective, run in routes:
        a, o, f = run()
        a, o = a.cpu().numpy(), o.cpu().numpy()
        assert np.bincount(a[a >= 0], minlength=K).tolist() == cap.tolist(), name
        assert np.sum(a < 0) == n - cap.sum() and np.all(o[a < 0] == -1), name
        # every route works on one S: the recompute route's tiles and the columns of its coverage update are
        # the bits of the stored matrix, so groups of repeated points tie exactly there as well
        res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, objective=objective)
        assert res["rc"] == 0 and res["checked"] == cap.sum(), (name, res)
        scale = max(1.0, float(S.astype(np.float64).sum()) / K)
        for k in range(K):
            ref = oracle.f_value(S, np.flatnonzero(a == k), objective)
            assert abs(f[k] - ref) <= 1e-4 * max(ref, 0.0) + 1e-12 * scale, (name, k, f[k], ref)


@pytest.mark.parametrize("seed", range(24))
def test_random_data_set(rcd, seed):
    """Random class structure through the data-set entry point: 1 to 150 classes of very unequal sizes (some
    empty), f32 or bf16 features with a row pitch, a random route and either workspace size; every class
    refereed at every step on the library's own similarity of that class."""
    rng = np.random.default_rng(5000 + seed)
    L = int(rng.choice([1, 2, 7, 40, 70, 150]))
    sizes = rng.integers(0, int(rng.choice([6, 60, 300])) + 1, size=L)
    sizes[int(rng.integers(0, L))] = int(rng.integers(1, 700))          # one class larger than the rest
    N = int(sizes.sum())
    K = int(rng.integers(1, 9))
    r = rng.integers(1, 5, size=K)
    dtype = str(rng.choice(["f32", "bf16"]))
    d = int(rng.choice([32, 64, 128]))
    X = si.make_class(seed=6000 + seed, n=N, d=d, G=5, dtype=dtype)
    labels = np.repeat(np.arange(L), sizes).astype(np.int32)
    perm = rng.permutation(N)
    X, labels = np.ascontiguousarray(X[perm]), np.ascontiguousarray(labels[perm])
    route = str(rng.choice(["sweeps", "incremental", "recompute", "graph cut", "auto"]))
    print(f"random data set {seed}: L={L} N={N} largest class {int(sizes.max())} K={K} {dtype} d={d} {route}", flush=True)
    wide = np.zeros((N, d + 16), dtype=X.dtype)
    wide[:, :d] = X
    if dtype == "bf16":
        Xd = torch.from_numpy(wide.view(np.int16)).cuda().view(torch.bfloat16)[:, :d]
    else:
        Xd = torch.from_numpy(wide).cuda()[:, :d]
    yd = torch.from_numpy(labels).cuda()
    mode = {"sweeps": rcd.MODE_STORED, "incremental": rcd.MODE_INCREMENTAL, "recompute": rcd.MODE_RECOMPUTE,
            "graph cut": rcd.MODE_STORED, "auto": rcd.MODE_AUTO}[route]
    mn, full = rcd.dataset_workspace_bytes(N, L, int(sizes.max()), K, rcd.MODE_RECOMPUTE if route == "recompute" else rcd.MODE_STORED)
    ws = torch.empty(full if rng.random() < 0.5 else mn, dtype=torch.uint8, device="cuda")
    assign, order, obj = rcd.partition_dataset(Xd, yd, L, r, float(d), mode, ws, graph_cut=route == "graph cut")
    assign, order = assign.cpu().numpy(), order.cpu().numpy()
    assert np.all(assign >= 0) and np.all(assign < K)
    objective = "gc" if route == "graph cut" else "fl"
    for c in range(L):
        idx = np.flatnonzero(labels == c)
        if len(idx) == 0:
            assert np.all(obj[c] == 0.0)
            continue
        cap = oracle.quota(len(idx), r)
        S = rcd.similarity(Xd, float(d), row_index=torch.from_numpy(idx.astype(np.int32)).cuda()).cpu().numpy()
        ref = oracle.similarity(X[idx], float(d))
        assert np.max(np.abs(S - ref) / np.maximum(ref, 1e-30)) <= (1e-5 if dtype == "f32" else 2e-2)
        a, o = assign[idx], order[idx]
        assert np.bincount(a, minlength=K).tolist() == cap.tolist()
        res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, objective=objective)
        assert res["rc"] == 0 and res["checked"] == len(idx), (c, res)
        scale = max(1.0, float(S.astype(np.float64).sum()) / K)
        for k in range(K):
            want = oracle.f_value(S, np.flatnonzero(a == k), objective)
            assert abs(obj[c, k] - want) <= 1e-4 * max(want, 0.0) + 1e-12 * scale, (c, k, obj[c, k], want)


@pytest.mark.parametrize("seed", range(30))
def test_random_similarity_and_bandwidth_shapes(rcd, monkeypatch, seed):
    """Random shapes through rcd_similarity and rcd_bandwidth: any d (whole 128-byte lines or not), rows with a
    pitch and an offset that may break the 16-byte alignment, a row gather, an output pitch that may or may not
    take 16-byte stores, the mirrored build forced on or off or left to the rule."""
    rng = np.random.default_rng(9000 + seed)
    dtype = str(rng.choice(["f32", "bf16"]))
    n_all = int(rng.integers(1, 1500))
    d = int(rng.choice([1, 7, 31, 32, 48, 64, 96, 100, 128, 200, 256, 300]))
    off = int(rng.choice([0, 0, 1, 4, 8]))
    pitch = d + off + int(rng.choice([0, 3, 8, 32]))
    X = si.make_class(seed=9100 + seed, n=n_all, d=d, G=4, dtype=dtype)
    wide = np.zeros((n_all, pitch), dtype=X.dtype)
    wide[:, off:off + d] = X
    if dtype == "bf16":
        Xd = torch.from_numpy(wide.view(np.int16)).cuda().view(torch.bfloat16)[:, off:off + d]
    else:
        Xd = torch.from_numpy(wide).cuda()[:, off:off + d]
    gather = rng.random() < 0.5
    idx = np.sort(rng.choice(n_all, size=int(rng.integers(1, n_all + 1)), replace=False)).astype(np.int32) if gather \
        else np.arange(n_all, dtype=np.int32)
    n = len(idx)
    sigma2 = float(d) * float(rng.choice([0.5, 1.0, 3.0]))
    out_pitch = n + int(rng.choice([0, 1, 4, 12]))
    mirror = str(rng.choice(["0", "1", "2"]))
    monkeypatch.setenv("RCD_SIM_MIRROR", mirror)
    print(f"random similarity {seed}: {dtype} rows {n} of {n_all} d={d} offset {off} pitch {pitch} out pitch {out_pitch} "
          f"mirror {mirror} gather {gather}", flush=True)
    out = torch.full((n, out_pitch), -7.0, dtype=torch.float32, device="cuda")
    rcd.similarity(Xd, sigma2, row_index=torch.from_numpy(idx).cuda() if gather else None, out=out[:, :n])
    got = out.cpu().numpy()
    ref = oracle.similarity(X[idx], sigma2)
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.max(np.abs(got[:, :n] - ref) / np.maximum(ref, 1e-30)) <= tol
    assert np.array_equal(got[:, :n], got[:, :n].T) and np.all(np.diag(got[:, :n]) == 1.0)
    assert np.all(got[:, n:] == -7.0)
    sigma = rcd.bandwidth(Xd, row_index=torch.from_numpy(idx).cuda() if gather else None)
    want = oracle.bandwidth(X[idx])
    # distances between near-identical rows carry the Gram identity's cancellation (absolute ~3e-4 |x| per pair)
    assert sigma == pytest.approx(want, rel=1e-5, abs=1e-5 * float(np.sqrt(d)))
