"""GPU parity of the incremental-gain route's fused update pass (Algorithm 1's inner loop with the
facility-location function of Section 4, gains kept current by differences).  While the pending update lists of
a class's blocks overlap, one pass applies them all and reads a row of S once; the library does that for
classes from 16 384 samples on.  Here the tuning switches RCD_INC_FUSE_MIN_N / RCD_INC_FUSE_PCT bring it down
to classes the oracle referees at every step: the fused pass must give the list-by-list update's results bit
for bit (same terms, same order), in the one-workgroup step loop and in the shared one."""
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
    return torch.from_numpy(a).cuda()


def mixture_S(seed, n, d=16):
    return oracle.similarity(si.make_class(seed=seed, n=n, d=d), float(d))


def run(rcd, monkeypatch, S, cap, fused, pct=50, shared=False, small_kb=None, blocks=8):
    monkeypatch.setenv("RCD_INC_FUSE_MIN_N", "1" if fused else "0")
    monkeypatch.setenv("RCD_INC_FUSE_BLOCKS", str(blocks))     # waiting blocks per workgroup of the fused pass
    monkeypatch.setenv("RCD_INC_FUSE_PCT", str(pct))
    monkeypatch.setenv("RCD_MW_MIN_N", "1" if shared else "0")
    monkeypatch.setenv("RCD_MW_SLICE", "256")
    if small_kb is not None:
        monkeypatch.setenv("RCD_INC_SMALL_KB", str(small_kb))
    a, o, f = rcd.partition_class(S=dev(S), cap=cap, mode=rcd.MODE_INCREMENTAL)
    stats = rcd.last_stats()
    return a.cpu().numpy(), o.cpu().numpy(), f, stats


@pytest.mark.parametrize("shared", [False, True])
@pytest.mark.parametrize("n,r,pct,blocks", [(1500, [1, 1, 2, 4], 50, 8), (2100, [1, 1, 1, 2, 2, 3, 4, 6], 50, 8),
                                            (2100, [1, 1, 1, 2, 2, 3, 4, 6], 1, 3), (2100, [1, 1, 1, 2, 2, 3, 4, 6], 30, 2),
                                            (1000, [3, 1, 4, 1, 2, 2, 1, 3, 4, 4, 1, 2], 1, 4), (257, [5, 5], 1, 8),
                                            (3000, [1, 2, 3], 10, 2)])
def test_fused_pass_gives_the_list_by_list_bits(rcd, monkeypatch, shared, n, r, pct, blocks):
    print(f"fused update: n={n} K={len(r)} pct={pct} blocks per workgroup={blocks} shared={shared}", flush=True)
    S = mixture_S(500 + n, n)
    cap = oracle.quota(n, r)
    # lists of more than one row go to the update launches, so that the fused pass sees sparse lists too
    a1, o1, f1, _ = run(rcd, monkeypatch, S, cap, fused=True, pct=pct, shared=shared, small_kb=1, blocks=blocks)
    a0, o0, f0, _ = run(rcd, monkeypatch, S, cap, fused=False, shared=shared, small_kb=1)
    assert np.array_equal(a1, a0) and np.array_equal(o1, o0) and np.array_equal(f1, f0)
    res = oracle.lockstep(S, cap, o1, a1, rel_tol=1e-5, objective="fl")
    assert res["rc"] == 0 and res["checked"] == n, res
    for k in range(len(cap)):
        ref = oracle.f_value(S, np.flatnonzero(a1 == k), "fl")
        assert abs(f1[k] - ref) <= 1e-4 * abs(ref) + 1e-9


def test_fused_pass_on_exact_ties_and_duplicates(rcd, monkeypatch):
    n, c = 1500, 0.25
    S = np.full((n, n), c, dtype=np.float32)
    np.fill_diagonal(S, 1.0)
    cap = np.array([300, 0, 700, 200], dtype=np.int64)
    a, o, f, _ = run(rcd, monkeypatch, S, cap, fused=True, pct=1, small_kb=1)
    res = oracle.lockstep(S, cap, o, a, rel_tol=0.0, objective="fl")
    assert res["rc"] == 0 and res["exact"] == cap.sum(), res
    assert np.flatnonzero(a >= 0).tolist() == list(range(int(cap.sum())))
    X = si.make_class(seed=78, n=400, d=16)
    X = np.concatenate([X, X, X])
    S = oracle.similarity(X, 16.0)
    cap = oracle.quota(1200, [1, 2, 1])
    a, o, f, _ = run(rcd, monkeypatch, S, cap, fused=True, pct=1, shared=True, small_kb=1)
    res = oracle.lockstep(S, cap, o, a, rel_tol=1e-5, objective="fl")
    assert res["rc"] == 0 and res["checked"] == 1200, res


def test_data_set_with_fused_and_unfused_classes(rcd, monkeypatch):
    # classes of very different sizes in one launch: every class decides by itself, launch by launch
    monkeypatch.setenv("RCD_INC_FUSE_MIN_N", "1")
    monkeypatch.setenv("RCD_INC_FUSE_PCT", "20")
    monkeypatch.setenv("RCD_INC_FUSE_BLOCKS", "3")
    monkeypatch.setenv("RCD_INC_SMALL_KB", "1")
    monkeypatch.setenv("RCD_MW_MIN_N", "1")
    monkeypatch.setenv("RCD_MW_SLICE", "512")
    sizes = np.array([40, 1500, 0, 700, 3, 2300, 260])
    L, N, d, r = len(sizes), int(sizes.sum()), 64, [1, 2, 3, 1, 1]
    X = si.make_class(seed=402, n=N, d=d, G=5)
    labels = np.repeat(np.arange(L), sizes).astype(np.int32)
    perm = np.random.default_rng(6).permutation(N)
    X, labels = np.ascontiguousarray(X[perm]), np.ascontiguousarray(labels[perm])
    Xd, yd = dev(X), dev(labels)
    sz = rcd.dataset_workspace_bytes(N, L, int(sizes.max()), len(r), rcd.MODE_STORED)[1]
    ws = torch.empty(sz, dtype=torch.uint8, device="cuda")
    assign, order, obj = rcd.partition_dataset(Xd, yd, L, r, float(d), rcd.MODE_INCREMENTAL, ws)
    assign, order = assign.cpu().numpy(), order.cpu().numpy()
    monkeypatch.setenv("RCD_INC_FUSE_MIN_N", "0")
    assign0, order0, obj0 = rcd.partition_dataset(Xd, yd, L, r, float(d), rcd.MODE_INCREMENTAL, ws)
    assert np.array_equal(assign, assign0.cpu().numpy()) and np.array_equal(order, order0.cpu().numpy())
    assert np.array_equal(obj, obj0)
    for c in range(L):
        idx = np.flatnonzero(labels == c)
        if len(idx) == 0:
            continue
        cap = oracle.quota(len(idx), r)
        S = rcd.similarity(Xd, float(d), row_index=dev(idx.astype(np.int32))).cpu().numpy()
        res = oracle.lockstep(S, cap, order[idx], assign[idx], rel_tol=1e-5, objective="fl")
        assert res["rc"] == 0 and res["checked"] == len(idx), (c, res)
