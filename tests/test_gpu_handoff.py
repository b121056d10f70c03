"""GPU parity of the hand-off to Algorithm 2: rcd_worker_shards against the oracle bit for bit (ragged
sizes around the 1024-sample chunks, leftovers, empty workers, full-size assignment of a real run),
rcd_batch_sizes against the oracle (host only, checked here too so that both sit together)."""
import ctypes

import numpy as np
import pytest

import oracle
import synth_inputs as si

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


@pytest.mark.gpu
@pytest.mark.parametrize("N,K", [(1, 1), (63, 2), (1023, 3), (1024, 4), (1025, 5), (5000, 16), (70001, 8)])
def test_worker_shards_bit_exact(rcd, N, K):
    print(f"worker shards N={N} K={K}", flush=True)
    rng = np.random.default_rng(N + K)
    for low in (0, -1):                      # everyone assigned / some left over
        a = rng.integers(low, K, size=N).astype(np.int32)
        if K > 2:
            a[a == 1] = 0                    # a worker with an empty list
        index, offset = rcd.worker_shards(torch.from_numpy(a).cuda(), K)
        ref_index, ref_offset = oracle.worker_shards(a, K)
        assert offset.tolist() == ref_offset.tolist()
        assert np.array_equal(index.cpu().numpy()[: offset[K]], ref_index)


@pytest.mark.gpu
def test_worker_shards_of_a_real_partition_and_errors(rcd):
    ds = si.make_dataset(si.WORKLOADS["hetero8"], L=4, n_c=600, d=64)
    N = ds.X.shape[0]
    K = len(ds.r)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, 600, K, rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    assign, _, _ = rcd.partition_dataset(dev(ds.X), dev(ds.labels), ds.L, ds.r, ds.sigma2, rcd.MODE_STORED, ws)
    index, offset = rcd.worker_shards(assign, K)
    a = assign.cpu().numpy()
    ref_index, ref_offset = oracle.worker_shards(a, K)
    assert offset.tolist() == ref_offset.tolist() and np.array_equal(index.cpu().numpy(), ref_index)
    # every worker's shard holds its quota of every class (the point of the class-wise partition)
    idx = index.cpu().numpy()
    for k in range(K):
        shard = idx[offset[k]:offset[k + 1]]
        per_class = np.bincount(ds.labels[shard], minlength=ds.L)
        assert per_class.tolist() == [int(oracle.quota(600, ds.r)[k])] * ds.L
    lib = rcd.load_library()
    bad = assign.clone()
    bad[17] = K
    off = np.zeros(K + 1, dtype=np.int64)
    out = torch.empty(N, dtype=torch.int32, device="cuda")
    wsz = lib.rcd_worker_shards_workspace_bytes(N, K)
    w2 = torch.empty(wsz, dtype=torch.uint8, device="cuda")
    offp = off.ctypes.data_as(ctypes.c_void_p)
    assert lib.rcd_worker_shards(bad.data_ptr(), N, K, out.data_ptr(), offp, w2.data_ptr(), wsz, None) == 2
    bad[17] = -2
    assert lib.rcd_worker_shards(bad.data_ptr(), N, K, out.data_ptr(), offp, w2.data_ptr(), wsz, None) == 2
    assert lib.rcd_worker_shards(assign.data_ptr(), N, K, out.data_ptr(), offp, w2.data_ptr(), wsz - 256, None) == 5
    assert lib.rcd_worker_shards(None, N, K, out.data_ptr(), offp, w2.data_ptr(), wsz, None) == 1
    assert lib.rcd_worker_shards(assign.data_ptr(), N, 17, out.data_ptr(), offp, w2.data_ptr(), wsz, None) == 4
    assert lib.rcd_worker_shards(None, 0, K, None, offp, None, 0, None) == 0 and off.tolist() == [0] * (K + 1)


def test_batch_sizes_match_the_oracle():
    import paper_2211_00839_amd as m

    rng = np.random.default_rng(2)
    assert m.batch_sizes(64, [1, 1, 2, 4]).tolist() == [64, 64, 128, 256]
    assert m.batch_sizes(3, [2, 1]).tolist() == [3, 2]
    for _ in range(300):
        K = int(rng.integers(1, 17))
        r = rng.integers(1, 9, size=K)
        B = int(rng.integers(1, 100000))
        assert m.batch_sizes(B, r).tolist() == oracle.batch_sizes(B, r).tolist()
    with pytest.raises(m.RcdError):
        m.batch_sizes(0, [1, 2])
    with pytest.raises(m.RcdError):
        m.batch_sizes(8, [1, 0])
