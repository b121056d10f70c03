"""GPU test of rcd_similarity_static, the entry point for callers that cannot allocate: through the C ABI, its
output must be the bits of rcd_similarity's on the same input, on two calls in a row (the second with a smaller
input, so that stale entries of the static scratch array are in reach of a wrong read), for both feature types,
both Gram paths, a row-index list and a pitched output."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2211_00839_amd as rcd_pkg
import synth_inputs as si
from paper_2211_00839_amd import binding

pytestmark = pytest.mark.gpu


def features(seed, n, d, dtype):
    X = si.make_class(seed=seed, n=n, d=d, G=4, dtype=dtype)
    if dtype == "bf16":
        return X, torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16)
    return X, torch.from_numpy(X).cuda()


def call_static(lib, Xd, n, sigma2, out, row_index=None):
    """Straight through the C ABI: no workspace argument exists."""
    vp = ctypes.c_void_p
    dt = 0 if Xd.dtype == torch.float32 else 1
    stream = vp(torch.cuda.current_stream().cuda_stream)
    ri = None if row_index is None else vp(row_index.data_ptr())
    return lib.rcd_similarity_static(vp(Xd.data_ptr()), dt, n, Xd.shape[1], Xd.stride(0), ri, float(sigma2),
                                     vp(out.data_ptr()), out.stride(0), stream)


@pytest.mark.parametrize("dtype,d,n1,n2", [("f32", 64, 700, 300), ("bf16", 256, 1000, 257), ("f32", 24, 515, 130),
                                           ("bf16", 40, 300, 90)])
def test_static_similarity_matches_the_workspace_entry_point_twice_in_a_row(dtype, d, n1, n2):
    lib = binding.load_library()
    assert lib.rcd_init() == 0
    for call, n in enumerate((n1, n2)):
        print(f"static similarity {dtype} d={d} call {call} n={n}", flush=True)
        X, Xd = features(40 + call, n, d, dtype)
        ref = rcd_pkg.similarity(Xd, float(d))
        out = torch.full((n, n + 8), -7.0, dtype=torch.float32, device="cuda")      # pitched output, poisoned
        before = torch.cuda.memory_allocated()
        assert call_static(lib, Xd, n, float(d), out) == 0
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(out[:, :n], ref)
        assert torch.all(out[:, n:] == -7.0)
        S_ref = oracle.similarity(X, float(d))
        err = np.max(np.abs(out[:, :n].cpu().numpy() - S_ref) / S_ref)
        assert err <= (1e-5 if dtype == "f32" else 2e-2)


def test_static_similarity_with_a_row_index_and_its_size_limit():
    lib = binding.load_library()
    X, Xd = features(7, 900, 128, "f32")
    idx = torch.from_numpy(np.random.default_rng(3).permutation(900)[:333].astype(np.int32)).cuda()
    ref = rcd_pkg.similarity(Xd, 128.0, row_index=idx)
    out = torch.empty((333, 333), dtype=torch.float32, device="cuda")
    assert call_static(lib, Xd, 333, 128.0, out, row_index=idx) == 0
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    # through the Python binding as well
    out2 = torch.empty((333, 333), dtype=torch.float32, device="cuda")
    rcd_pkg.similarity_static(Xd, 128.0, out2, row_index=idx)
    torch.cuda.synchronize()
    assert torch.equal(out2, ref)
    # beyond the static array: refused, nothing launched, the output untouched
    big = rcd_pkg.STATIC_MAX_N + 1
    canary = torch.full((4, 4), 3.0, device="cuda")
    vp = ctypes.c_void_p
    rc = lib.rcd_similarity_static(vp(Xd.data_ptr()), 0, big, 128, 128, None, 128.0, vp(canary.data_ptr()), big, None)
    assert rc == 4 and "unsupported" in rcd_pkg.strerror(rc)
    torch.cuda.synchronize()
    assert torch.all(canary == 3.0)
