"""GPU parity of rcd_bandwidth (Section 4: sigma = mean L2 distance over all ordered pairs) against the
oracle, on both Gram paths (whole 128-byte lines straight into LDS / any shape), ragged sizes around
the 256-wide tiles, row selection, pitched input, closed forms, degenerate sets and the full-size
data set (sampled subset against the oracle, whole set against an fp64 matmul on the device)."""
import ctypes

import numpy as np
import pytest

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

REL = 1e-5      # distances come from fp32 Gram tiles: |x|^2 + |y|^2 - 2 x.y carries ~1e-7 |x|^2 of rounding


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


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("f32", 96), ("bf16", 64), ("bf16", 256),      # whole lines
                                     ("f32", 7), ("f32", 48), ("bf16", 40), ("bf16", 100)])      # general path
@pytest.mark.parametrize("n", [1, 2, 255, 256, 257, 700, 1300])
def test_bandwidth_matches_the_oracle(rcd, dtype, d, n):
    print(f"bandwidth {dtype} n={n} d={d}", flush=True)
    X = si.make_class(seed=900 + n + d, n=n, d=d, dtype=dtype)
    ref = oracle.bandwidth(X)
    got = rcd.bandwidth(dev(X))
    assert got == pytest.approx(ref, rel=REL, abs=1e-12)
    assert rcd.bandwidth(dev(X)) == got          # fixed summation order: the same bits every time


def test_bandwidth_of_a_class_through_the_row_index_and_pitched_rows(rcd):
    ds = si.make_dataset(si.WORKLOADS["cifar10"], L=3, n_c=500, d=64)
    Xd = dev(ds.X)
    for c in range(3):
        idx = np.flatnonzero(ds.labels == c)
        ref = oracle.bandwidth(ds.X[idx])
        assert rcd.bandwidth(Xd, row_index=dev(idx.astype(np.int32))) == pytest.approx(ref, rel=REL)
    assert rcd.bandwidth(Xd) == pytest.approx(oracle.bandwidth(ds.X), rel=REL)
    # rows inside a wider buffer: aligned pitch (whole lines) and an odd one (general path)
    for pitch in (96, 67):
        wide = torch.zeros((ds.X.shape[0], pitch), dtype=torch.float32, device="cuda")
        wide[:, :64] = Xd
        assert rcd.bandwidth(wide[:, :64]) == pytest.approx(oracle.bandwidth(ds.X), rel=REL)


def test_bandwidth_closed_forms_and_degenerate_sets(rcd):
    # regular simplex: every pair at a sqrt(2)
    n, a = 300, 4.0
    X = (a * np.eye(n)).astype(np.float32)[:, :]
    Xp = np.zeros((n, 320), dtype=np.float32)
    Xp[:, :n] = X
    assert rcd.bandwidth(dev(Xp)) == pytest.approx(a * np.sqrt(2.0) * (n - 1) / n, rel=1e-6)
    # unit spacing on a line through the origin: sum |i - j| / n^2 = (n^2 - 1) / (3 n); small coordinates keep the Gram exact
    n = 100
    L = np.zeros((n, 32), dtype=np.float32)
    L[:, 3] = np.arange(n) - 50
    assert rcd.bandwidth(dev(L)) == pytest.approx((n * n - 1) / (3.0 * n), rel=1e-6)
    # one sample, and n copies of one sample: sigma = 0 up to the rounding of |x|^2 + |x|^2 - 2 x.x,
    # whose root is at most ~1e-3 |x|
    one = si.make_class(seed=7, n=1, d=64)
    assert rcd.bandwidth(dev(one)) == 0.0
    same = np.repeat(one, 400, axis=0)
    assert 0.0 <= rcd.bandwidth(dev(same)) <= 1e-3 * float(np.linalg.norm(one))
    assert rcd.bandwidth(dev(np.zeros((300, 64), dtype=np.float32))) == 0.0


def test_bandwidth_argument_errors(rcd):
    lib = rcd.load_library()
    X = dev(si.make_class(seed=8, n=64, d=32))
    ws = torch.empty(rcd.load_library().rcd_bandwidth_workspace_bytes(64), dtype=torch.uint8, device="cuda")
    out = np.zeros(1)
    outp = out.ctypes.data_as(ctypes.c_void_p)
    call = lambda *a: lib.rcd_bandwidth(*a)
    assert call(X.data_ptr(), 0, 64, 32, 32, None, outp, ws.data_ptr(), ws.numel(), None) == 0 and out[0] > 0
    assert call(X.data_ptr(), 5, 64, 32, 32, None, outp, ws.data_ptr(), ws.numel(), None) == 4      # dtype
    assert call(X.data_ptr(), 0, 64, 32, 16, None, outp, ws.data_ptr(), ws.numel(), None) == 1      # ld_x < d
    assert call(X.data_ptr(), 0, 64, 32, 32, None, None, ws.data_ptr(), ws.numel(), None) == 1      # no output
    assert call(None, 0, 64, 32, 32, None, outp, ws.data_ptr(), ws.numel(), None) == 1              # no X
    assert call(X.data_ptr(), 0, 64, 32, 32, None, outp, ws.data_ptr(), 256, None) == 5             # workspace short
    assert call(X.data_ptr(), 0, 64, 32, 32, None, outp, None, 0, None) == 5
    assert call(None, 0, 0, 32, 32, None, outp, None, 0, None) == 0 and out[0] == 0.0               # empty set


def test_bandwidth_full_size_data_set(rcd):
    # the cifar10 workload's whole feature matrix (50 000 x 512): against distances from an fp64 library
    # matmul on the device, and a 1500-row sample against the oracle
    ds = si.make_dataset(si.WORKLOADS["cifar10"])
    Xd = dev(ds.X)
    got = rcd.bandwidth(Xd)
    total = 0.0
    X64 = Xd.double()
    sq = (X64 * X64).sum(dim=1)
    for lo in range(0, X64.shape[0], 2500):
        d2 = sq[lo:lo + 2500, None] + sq[None, :] - 2.0 * (X64[lo:lo + 2500] @ X64.T)
        total += d2.clamp_(min=0.0).sqrt_().sum().item()
    ref = total / float(X64.shape[0]) ** 2
    print(f"  sigma of the whole set {got}, fp64 matmul reference {ref}", flush=True)
    assert got == pytest.approx(ref, rel=REL)
    rng = np.random.default_rng(11)
    idx = np.sort(rng.choice(ds.X.shape[0], size=1500, replace=False)).astype(np.int32)
    assert rcd.bandwidth(Xd, row_index=dev(idx)) == pytest.approx(oracle.bandwidth(ds.X[idx]), rel=REL)
