"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/rcd.h declares, and its host logic (quota rule, workspace sizes,
argument validation that happens before any launch) behaves."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2211_00839_amd as rcd
from paper_2211_00839_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2211_00839_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "rcd.h")).read()
    declared = set(re.findall(r"\b(rcd_[a-z_0-9]+)\s*\(", header))
    assert declared >= {"rcd_similarity", "rcd_partition_class", "rcd_partition_dataset", "rcd_gain_sweep",
                        "rcd_quota", "rcd_strerror"}
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == declared


def test_strerror_covers_every_status(lib):
    header = open(os.path.join(ROOT, "include", "rcd.h")).read()
    codes = [int(v) for v in re.findall(r"RCD_(?:OK|ERR_[A-Z_]+)\s*=\s*(\d+)", header)]
    assert codes == list(range(len(codes)))
    texts = [rcd.strerror(c) for c in codes]
    assert len(set(texts)) == len(texts) and "unknown" not in " ".join(texts)
    assert rcd.strerror(99) == "unknown status"


def test_quota_matches_hand_worked_vectors_and_oracle(lib, golden_dir):
    with open(os.path.join(golden_dir, "quota_vectors.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            n, r, cap = line.split(";")
            got = rcd.quota(int(n), [int(x) for x in r.split()])
            assert got.tolist() == [int(x) for x in cap.split()]
    rng = np.random.default_rng(0)
    for _ in range(200):
        K = int(rng.integers(1, 17))
        r = rng.integers(1, 9, size=K)
        n = int(rng.integers(0, 100000))
        assert rcd.quota(n, r).tolist() == oracle.quota(n, r).tolist()


def test_quota_rejects_bad_capacities(lib):
    with pytest.raises(rcd.RcdError) as e:
        rcd.quota(10, [1, 0])
    assert e.value.status == 3


def test_workspace_sizes_are_aligned_and_monotone(lib):
    prev = 0
    for n in (1, 100, 256, 257, 5000):
        b = rcd.class_workspace_bytes(n, 8, rcd.MODE_STORED)
        assert b % 256 == 0 and b > prev
        assert b >= n * n * 4
        prev = b
    mn, full = rcd.dataset_workspace_bytes(50000, 10, 5000, 4, rcd.MODE_STORED)
    assert mn % 256 == 0 and full % 256 == 0 and full >= mn
    assert full >= 10 * 5000 * 5000 * 4


def test_argument_validation_happens_before_any_gpu_work(lib):
    # none of these reach a launch: they must come back with a status, not crash
    cap = np.array([1, 1], dtype=np.int64)
    obj = np.zeros(2)
    vp = ctypes.c_void_p
    call = lib.rcd_partition_class
    # K too large -> unsupported
    big = np.ones(17, dtype=np.int64)
    assert call(None, 0, None, 0, 0, 0, 1.0, 10, 17, big.ctypes.data_as(vp), None, None,
                np.zeros(17).ctypes.data_as(vp), None, 0, None) == 4
    # negative quota / quotas above n -> bad capacity
    neg = np.array([-1, 2], dtype=np.int64)
    assert call(None, 0, None, 0, 0, 0, 1.0, 10, 2, neg.ctypes.data_as(vp), None, None, obj.ctypes.data_as(vp),
                None, 0, None) == 3
    over = np.array([6, 6], dtype=np.int64)
    assert call(None, 0, None, 0, 0, 0, 1.0, 10, 2, over.ctypes.data_as(vp), None, None, obj.ctypes.data_as(vp),
                None, 0, None) == 3
    # n < 0, K < 1 -> invalid argument
    assert call(None, 0, None, 0, 0, 0, 1.0, -1, 2, cap.ctypes.data_as(vp), None, None, obj.ctypes.data_as(vp),
                None, 0, None) == 1
    assert call(None, 0, None, 0, 0, 0, 1.0, 10, 0, cap.ctypes.data_as(vp), None, None, obj.ctypes.data_as(vp),
                None, 0, None) == 1
    # empty class is legal and touches nothing
    zero = np.array([0, 0], dtype=np.int64)
    assert call(None, 0, None, 0, 0, 0, 1.0, 0, 2, zero.ctypes.data_as(vp), None, None, obj.ctypes.data_as(vp),
                None, 0, None) == 0
    # similarity: bad dtype, bad sigma
    sim = lib.rcd_similarity
    assert sim(None, 7, 4, 4, 4, None, 1.0, None, 4, None, 0, None) == 4
    assert sim(None, 0, 4, 4, 4, None, 0.0, None, 4, None, 0, None) == 1
    assert sim(None, 0, 4, 4, 2, None, 1.0, None, 4, None, 0, None) == 1
    # data set: capacity < 1, bad mode
    r = np.array([1, 0], dtype=np.int32)
    ds = lib.rcd_partition_dataset
    assert ds(None, 0, 10, 4, 4, None, 2, r.ctypes.data_as(vp), 2, 1.0, 0, None, None,
              np.zeros(4).ctypes.data_as(vp), None, 0, None) == 3
    r = np.array([1, 1], dtype=np.int32)
    assert ds(None, 0, 10, 4, 4, None, 2, r.ctypes.data_as(vp), 2, 1.0, 9, None, None,
              np.zeros(4).ctypes.data_as(vp), None, 0, None) == 4


def test_python_binding_refuses_cpu_tensors(lib):
    import torch

    with pytest.raises(rcd.RcdError):
        rcd.similarity(torch.zeros(4, 4), 1.0, workspace=torch.zeros(256, dtype=torch.uint8))


def test_argument_validation_of_the_later_entry_points(lib):
    # graph cut, bandwidth, worker shards, batch sizes: every refusal below happens before any GPU call
    vp = ctypes.c_void_p
    obj = np.zeros(2)
    objp = obj.ctypes.data_as(vp)
    cap = np.array([1, 1], dtype=np.int64)
    gc = lib.rcd_partition_class_graph_cut
    assert gc(None, 10, 10, 2, cap.ctypes.data_as(vp), None, None, objp, None, 0, None) == 1           # no S
    assert gc(None, 0, 0, 2, np.zeros(2, dtype=np.int64).ctypes.data_as(vp), None, None, objp, None, 0, None) == 0   # empty class
    assert gc(None, 10, 10, 17, np.ones(17, dtype=np.int64).ctypes.data_as(vp), None, None,
              np.zeros(17).ctypes.data_as(vp), None, 0, None) in (1, 4)                                 # no S / K too large
    over = np.array([6, 6], dtype=np.int64)
    assert gc(ctypes.c_void_p(256), 10, 10, 2, over.ctypes.data_as(vp), None, None, objp, None, 0, None) == 3   # quotas above n
    r = np.array([1, 0], dtype=np.int32)
    dsgc = lib.rcd_partition_dataset_graph_cut
    assert dsgc(None, 0, 10, 4, 4, None, 2, r.ctypes.data_as(vp), 2, 1.0, None, None,
                np.zeros(4).ctypes.data_as(vp), None, 0, None) == 3                                     # capacity < 1
    r = np.array([1, 1], dtype=np.int32)
    assert dsgc(None, 0, 10, 4, 4, None, 2, r.ctypes.data_as(vp), 2, -1.0, None, None,
                np.zeros(4).ctypes.data_as(vp), None, 0, None) == 1                                     # sigma2 <= 0

    sigma = np.zeros(1)
    sp = sigma.ctypes.data_as(vp)
    bw = lib.rcd_bandwidth
    assert bw(None, 7, 4, 4, 4, None, sp, None, 0, None) == 4             # dtype
    assert bw(None, 0, 4, 4, 2, None, sp, None, 0, None) == 1             # ld_x < d
    assert bw(None, 0, 4, 4, 4, None, None, None, 0, None) == 1           # nowhere to put sigma
    assert bw(None, 0, 4, 4, 4, None, sp, None, 0, None) == 1             # no X
    assert bw(None, 0, 0, 4, 4, None, sp, None, 0, None) == 0 and sigma[0] == 0.0     # empty set
    assert lib.rcd_bandwidth_workspace_bytes(0) == 0
    prev = 0
    for n in (1, 255, 256, 257, 5000, 50000):
        b = lib.rcd_bandwidth_workspace_bytes(n)
        assert b % 256 == 0 and b >= prev and b >= 4 * n
        prev = b

    off = np.zeros(5, dtype=np.int64)
    sh = lib.rcd_worker_shards
    assert sh(None, 10, 17, None, off.ctypes.data_as(vp), None, 0, None) == 4          # too many workers
    assert sh(None, 10, 4, None, None, None, 0, None) == 1                             # no offsets
    assert sh(None, 10, 4, None, off.ctypes.data_as(vp), None, 0, None) == 1           # no assignment
    assert sh(None, 0, 4, None, off.ctypes.data_as(vp), None, 0, None) == 0 and off.tolist() == [0] * 5
    assert lib.rcd_worker_shards_workspace_bytes(0, 4) == 0
    assert lib.rcd_worker_shards_workspace_bytes(50000, 4) % 256 == 0

    assert rcd.batch_sizes(64, [1, 1, 2, 4]).tolist() == oracle.batch_sizes(64, [1, 1, 2, 4]).tolist()
    for B, rr in ((0, [1, 2]), (8, [1, 0])):
        with pytest.raises(rcd.RcdError):
            rcd.batch_sizes(B, rr)


def test_route_argument_workspace_query_and_static_similarity_refusals(lib):
    # rcd_partition_class_mode: the route is an argument; every refusal below happens before any GPU call
    vp = ctypes.c_void_p
    cap = np.array([1, 1], dtype=np.int64)
    obj = np.zeros(2)
    objp, capp = obj.ctypes.data_as(vp), cap.ctypes.data_as(vp)
    pcm = lib.rcd_partition_class_mode
    assert pcm(None, 0, None, 0, 0, 0, 1.0, 10, 2, capp, 9, None, None, objp, None, 0, None) == 4     # unknown mode
    for mode in (rcd.MODE_STORED, rcd.MODE_INCREMENTAL):
        assert pcm(None, 0, ctypes.c_void_p(256), 0, 4, 4, 1.0, 10, 2, capp, mode, None, None, objp, None, 0, None) == 1   # no S
    assert pcm(ctypes.c_void_p(256), 10, None, 0, 0, 0, 1.0, 10, 2, capp, rcd.MODE_RECOMPUTE, None, None, objp,
               None, 0, None) == 1                                                                        # no X
    zero = np.array([0, 0], dtype=np.int64)
    for mode in (rcd.MODE_AUTO, rcd.MODE_STORED, rcd.MODE_RECOMPUTE, rcd.MODE_INCREMENTAL):
        assert pcm(None, 0, None, 0, 0, 0, 1.0, 0, 2, zero.ctypes.data_as(vp), mode, None, None, objp, None, 0, None) == 0

    # rcd_workspace_bytes: one class, or a data set of unknown class count
    for n, K, mode in ((1, 1, rcd.MODE_STORED), (5000, 8, rcd.MODE_STORED), (5000, 8, rcd.MODE_RECOMPUTE)):
        assert rcd.workspace_bytes(n, 0, 512, K, rcd.F32, mode) == rcd.class_workspace_bytes(n, K, mode)
    w = rcd.workspace_bytes(50000, 5000, 512, 4, rcd.F32, rcd.MODE_STORED)
    mn, full = rcd.dataset_workspace_bytes(50000, 10, 5000, 4, rcd.MODE_STORED)
    assert w % 256 == 0 and w >= mn and w >= 5000 * 5000 * 4
    assert rcd.workspace_bytes(50000, 5000, 512, 4, rcd.BF16, rcd.MODE_STORED) == w          # dtype and d do not enter
    assert rcd.workspace_bytes(50000, 5000, 64, 4, rcd.F32, rcd.MODE_STORED) == w
    assert rcd.workspace_bytes(10, 11, 4, 2, 0, 1) == 0 and rcd.workspace_bytes(10, 0, 4, 17, 0, 1) == 0
    assert rcd.workspace_bytes(0, 0, 4, 2, 0, 1) == 0

    # rcd_similarity_static: sizes beyond its static scratch and bad arguments are refused before any launch
    st = lib.rcd_similarity_static
    assert rcd.STATIC_MAX_N == int(re.search(r"#define RCD_STATIC_MAX_N (\d+)",
                                             open(os.path.join(ROOT, "include", "rcd.h")).read()).group(1))
    big = rcd.STATIC_MAX_N + 1
    assert st(ctypes.c_void_p(256), 0, big, 4, 4, None, 1.0, ctypes.c_void_p(256), big, None) == 4
    assert st(None, 7, 4, 4, 4, None, 1.0, None, 4, None) == 4
    assert st(None, 0, 4, 4, 4, None, 0.0, None, 4, None) == 1
    assert st(None, 0, 4, 4, 2, None, 1.0, None, 4, None) == 1
    assert st(None, 0, 4, 4, 4, None, 1.0, None, 2, None) == 1
    assert st(None, 0, 0, 4, 4, None, 1.0, None, 4, None) == 0
    # rcd_release with nothing held is a no-op
    lib.rcd_release()


def test_sweep_chunk_rule_keeps_every_variant_inside_the_workgroups_lds(lib):
    # the stored-S sweep stages one coverage chunk per slot of the compiled variant that serves nneed blocks;
    # the chunk rule (in csrc/rcd_state.h) must keep slots x chunk within RCD_SWEEP_LDS_FLOATS for every nneed
    src = open(os.path.join(ROOT, "paper_2211_00839_amd", "csrc", "rcd_state.h")).read()
    lds = int(re.search(r"#define RCD_SWEEP_LDS_FLOATS (\d+)", src).group(1))
    variants = [1, 2, 3, 4, 6, 8, 12, 16]
    kernels = open(os.path.join(ROOT, "paper_2211_00839_amd", "csrc", "greedy_kernels.hip")).read()
    assert [int(v) for v in re.findall(r"sweep_rows<(\d+)>\(st, wg\.w", kernels)] == variants
    for nneed in range(1, 17):
        slots = min(v for v in variants if v >= nneed)
        chunk = (lds // slots) // 256 * 256
        assert slots * chunk <= lds and chunk >= 256
