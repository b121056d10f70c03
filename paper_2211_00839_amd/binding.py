"""ctypes binding of librcd.so: same names as the C entry points, argument
marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librcd.so")
_lib = None

EXPORTS = [
    "rcd_similarity", "rcd_similarity_workspace_bytes", "rcd_bandwidth", "rcd_bandwidth_workspace_bytes", "rcd_quota",
    "rcd_worker_shards", "rcd_worker_shards_workspace_bytes", "rcd_batch_sizes", "rcd_gain_sweep",
    "rcd_partition_class", "rcd_partition_dataset", "rcd_partition_class_graph_cut",
    "rcd_partition_dataset_graph_cut", "rcd_class_workspace_bytes",
    "rcd_dataset_workspace_bytes", "rcd_strerror", "rcd_last_hip_error", "rcd_last_stats",
    "rcd_profile", "rcd_profile_read", "rcd_partition_class_mode", "rcd_workspace_bytes", "rcd_init", "rcd_release",
    "rcd_similarity_static",
]


class RcdError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(what)
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load librcd.so.  torch is imported first so that the HIP runtime the
    library binds to is the one torch already brought into the process."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RcdError(-1, "librcd.so is not built: run `python -m paper_2211_00839_amd.build`")
    import torch  # noqa: F401  (loads libamdhip64 before librcd.so resolves it)

    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i64, i32, f32, sz = c.c_void_p, c.c_int64, c.c_int, c.c_float, c.c_size_t
    lib.rcd_similarity.restype = i32
    lib.rcd_similarity.argtypes = [vp, i32, i64, i64, i64, vp, f32, vp, i64, vp, sz, vp]
    lib.rcd_similarity_workspace_bytes.restype = sz
    lib.rcd_similarity_workspace_bytes.argtypes = [i64]
    lib.rcd_quota.restype = i32
    lib.rcd_bandwidth.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.rcd_bandwidth.restype = i32
    lib.rcd_bandwidth_workspace_bytes.argtypes = [i64]
    lib.rcd_bandwidth_workspace_bytes.restype = sz
    lib.rcd_worker_shards.argtypes = [vp, i64, i32, vp, vp, vp, sz, vp]
    lib.rcd_worker_shards.restype = i32
    lib.rcd_worker_shards_workspace_bytes.argtypes = [i64, i32]
    lib.rcd_worker_shards_workspace_bytes.restype = sz
    lib.rcd_batch_sizes.argtypes = [i64, vp, i32, vp]
    lib.rcd_batch_sizes.restype = i32
    lib.rcd_quota.argtypes = [i64, vp, i32, vp]
    lib.rcd_gain_sweep.restype = i32
    lib.rcd_gain_sweep.argtypes = [vp, i64, i64, i32, vp, vp, vp, sz, vp]
    lib.rcd_partition_class.restype = i32
    lib.rcd_partition_class.argtypes = [vp, i64, vp, i32, i64, i64, f32, i64, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.rcd_partition_dataset.restype = i32
    lib.rcd_partition_dataset.argtypes = [vp, i32, i64, i64, i64, vp, i32, vp, i32, f32, i32, vp, vp, vp, vp, sz, vp]
    lib.rcd_class_workspace_bytes.restype = sz
    lib.rcd_partition_class_graph_cut.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.rcd_partition_class_graph_cut.restype = i32
    lib.rcd_partition_dataset_graph_cut.argtypes = [vp, i32, i64, i64, i64, vp, i32, vp, i32, f32, vp, vp, vp, vp, sz, vp]
    lib.rcd_partition_dataset_graph_cut.restype = i32
    lib.rcd_class_workspace_bytes.argtypes = [i64, i32, i32]
    lib.rcd_dataset_workspace_bytes.restype = i32
    lib.rcd_dataset_workspace_bytes.argtypes = [i64, i32, i64, i32, i32, vp, vp]
    lib.rcd_strerror.restype = c.c_char_p
    lib.rcd_strerror.argtypes = [i32]
    lib.rcd_last_hip_error.restype = c.c_char_p
    lib.rcd_last_hip_error.argtypes = []
    lib.rcd_last_stats.restype = None
    lib.rcd_last_stats.argtypes = [vp]
    lib.rcd_profile.restype = None
    lib.rcd_profile.argtypes = [i32]
    lib.rcd_profile_read.restype = None
    lib.rcd_profile_read.argtypes = [vp]
    lib.rcd_partition_class_mode.restype = i32
    lib.rcd_partition_class_mode.argtypes = [vp, i64, vp, i32, i64, i64, f32, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.rcd_workspace_bytes.restype = sz
    lib.rcd_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, i32]
    lib.rcd_init.restype = i32
    lib.rcd_init.argtypes = []
    lib.rcd_release.restype = None
    lib.rcd_release.argtypes = []
    lib.rcd_similarity_static.restype = i32
    lib.rcd_similarity_static.argtypes = [vp, i32, i64, i64, i64, vp, f32, vp, i64, vp]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().rcd_strerror(int(status)).decode()


def _check(status: int):
    if status != 0:
        lib = load_library()
        msg = lib.rcd_strerror(status).decode()
        if status == 6:
            msg += ": " + lib.rcd_last_hip_error().decode()
        raise RcdError(status, "rcd status %d (%s)" % (status, msg))


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise RcdError(-1, "device tensor expected (there is no CPU path)")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(X) -> int:
    import torch

    if X.dtype == torch.float32:
        return 0
    if X.dtype == torch.bfloat16:
        return 1
    raise RcdError(4, "features must be float32 or bfloat16")


def _workspace(nbytes: int, device):
    import torch

    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def quota(n_l: int, r) -> np.ndarray:
    r = np.ascontiguousarray(r, dtype=np.int32)
    cap = np.zeros(len(r), dtype=np.int64)
    _check(load_library().rcd_quota(int(n_l), _np_ptr(r), len(r), _np_ptr(cap)))
    return cap


def worker_shards(assign, K: int, workspace=None):
    """Per-worker index lists of an assignment.  Returns (index int32[N] device, offset int64[K+1] numpy):
    worker k owns index[offset[k]:offset[k+1]], ascending; samples with assign == -1 are in no list."""
    import torch

    lib = load_library()
    N = assign.shape[0]
    assert assign.dtype == torch.int32 and assign.is_contiguous()
    index = torch.empty(N, dtype=torch.int32, device=assign.device)
    offset = np.zeros(K + 1, dtype=np.int64)
    if workspace is None:
        workspace = _workspace(lib.rcd_worker_shards_workspace_bytes(N, K), assign.device)
    _check(lib.rcd_worker_shards(_dev_ptr(assign), N, int(K), _dev_ptr(index), _np_ptr(offset), _dev_ptr(workspace),
                                 workspace.numel(), _stream()))
    return index, offset


def batch_sizes(B: int, r) -> np.ndarray:
    r = np.ascontiguousarray(r, dtype=np.int32)
    out = np.zeros(len(r), dtype=np.int64)
    _check(load_library().rcd_batch_sizes(int(B), _np_ptr(r), len(r), _np_ptr(out)))
    return out


def class_workspace_bytes(n: int, K: int, mode: int = 1) -> int:
    return int(load_library().rcd_class_workspace_bytes(int(n), int(K), int(mode)))


def dataset_workspace_bytes(N: int, L: int, max_class_n: int, K: int, mode: int = 1):
    mn, fl = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().rcd_dataset_workspace_bytes(int(N), int(L), int(max_class_n), int(K), int(mode),
                                                      ctypes.byref(mn), ctypes.byref(fl)))
    return int(mn.value), int(fl.value)


def workspace_bytes(N_or_n: int, max_class_n: int, d: int, K: int, dtype_code: int = 0, mode: int = 1) -> int:
    return int(load_library().rcd_workspace_bytes(int(N_or_n), int(max_class_n), int(d), int(K), int(dtype_code),
                                                  int(mode)))


def init() -> None:
    _check(load_library().rcd_init())


def release() -> None:
    load_library().rcd_release()


def similarity_static(X, sigma2: float, out, row_index=None):
    """rcd_similarity_static: `out` (n, n) float32 is the caller's; nothing is allocated, no workspace."""
    import torch

    lib = load_library()
    assert X.dim() == 2 and X.stride(1) == 1
    n = X.shape[0] if row_index is None else row_index.numel()
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape[0] >= n and out.shape[1] >= n
    _check(lib.rcd_similarity_static(_dev_ptr(X), _dtype_code(X), n, X.shape[1], X.stride(0), _dev_ptr(row_index),
                                     float(sigma2), _dev_ptr(out), out.stride(0) if n > 0 else max(n, 1), _stream()))
    return out


def similarity(X, sigma2: float, row_index=None, out=None, workspace=None):
    """X: (n, d) float32/bfloat16 device tensor (row stride = ld_x).  Returns S (n, n) float32."""
    import torch

    lib = load_library()
    assert X.dim() == 2 and X.stride(1) == 1
    n = X.shape[0] if row_index is None else row_index.numel()
    d = X.shape[1]
    if out is None:
        out = torch.empty((n, n), dtype=torch.float32, device=X.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1
    ws_bytes = int(lib.rcd_similarity_workspace_bytes(n))
    if workspace is None:
        workspace = _workspace(ws_bytes, X.device)
    _check(lib.rcd_similarity(_dev_ptr(X), _dtype_code(X), n, d, X.stride(0), _dev_ptr(row_index), float(sigma2),
                              _dev_ptr(out), out.stride(0) if n > 0 else max(n, 1), _dev_ptr(workspace),
                              workspace.numel(), _stream()))
    return out


def bandwidth(X, row_index=None, workspace=None) -> float:
    """The paper's kernel bandwidth sigma: mean L2 distance over all ordered pairs of the rows of X
    (of the rows row_index selects, if given)."""
    lib = load_library()
    n = X.shape[0] if row_index is None else row_index.shape[0]
    d = X.shape[1]
    assert X.stride(1) == 1
    if workspace is None:
        workspace = _workspace(lib.rcd_bandwidth_workspace_bytes(n), X.device)
    sigma = np.zeros(1, dtype=np.float64)
    _check(lib.rcd_bandwidth(_dev_ptr(X), _dtype_code(X), n, d, X.stride(0), _dev_ptr(row_index), _np_ptr(sigma),
                             _dev_ptr(workspace), workspace.numel(), _stream()))
    return float(sigma[0])


def gain_sweep(S, cur, workspace=None):
    """S: (n, n) float32 device, cur: (K, n) float32 device.  Returns gains (K, n)."""
    import torch

    lib = load_library()
    n = S.shape[0]
    K = cur.shape[0]
    assert S.dtype == torch.float32 and cur.dtype == torch.float32 and cur.is_contiguous() and S.stride(1) == 1
    gains = torch.empty((K, n), dtype=torch.float32, device=S.device)
    if workspace is None:
        workspace = _workspace(lib.rcd_class_workspace_bytes(n, K, 1), S.device)
    _check(lib.rcd_gain_sweep(_dev_ptr(S), S.stride(0), n, K, _dev_ptr(cur), _dev_ptr(gains), _dev_ptr(workspace),
                              workspace.numel(), _stream()))
    return gains


def partition_class(S=None, cap=None, X=None, sigma2: float = 1.0, workspace=None, want_order: bool = True,
                    mode: Optional[int] = None):
    """One class of Algorithm 1.  Give S (stored mode) or X (recompute mode).  mode=None calls
    rcd_partition_class (sweeps over a stored S, or recompute); a mode calls rcd_partition_class_mode.
    Returns (assign int32[n] device, order int32[n] device or None, obj float64[K] numpy)."""
    import torch

    lib = load_library()
    cap = np.ascontiguousarray(cap, dtype=np.int64)
    K = len(cap)
    src = S if S is not None else X
    n = src.shape[0]
    dev = src.device
    assign = torch.empty(n, dtype=torch.int32, device=dev)
    order = torch.empty(n, dtype=torch.int32, device=dev) if want_order else None
    obj = np.zeros(K, dtype=np.float64)
    if workspace is None:
        workspace = _workspace(lib.rcd_class_workspace_bytes(n, K, 1 if S is not None else 2), dev)
    if S is not None:
        assert S.dtype == torch.float32 and S.stride(1) == 1
        args = (_dev_ptr(S), S.stride(0), None, 0, 0, 0, float(sigma2))
    else:
        assert X.stride(1) == 1
        args = (None, 0, _dev_ptr(X), _dtype_code(X), X.shape[1], X.stride(0), float(sigma2))
    if mode is None:
        _check(lib.rcd_partition_class(*args, n, K, _np_ptr(cap), _dev_ptr(assign), _dev_ptr(order), _np_ptr(obj),
                                       _dev_ptr(workspace), workspace.numel(), _stream()))
    else:
        _check(lib.rcd_partition_class_mode(*args, n, K, _np_ptr(cap), int(mode), _dev_ptr(assign), _dev_ptr(order),
                                            _np_ptr(obj), _dev_ptr(workspace), workspace.numel(), _stream()))
    return assign, order, obj


def partition_class_graph_cut(S, cap, workspace=None, want_order: bool = True):
    """One class of Algorithm 1 with the graph-cut function, on a stored symmetric S.
    Returns (assign int32[n] device, order int32[n] device or None, obj float64[K] numpy)."""
    import torch

    lib = load_library()
    cap = np.ascontiguousarray(cap, dtype=np.int64)
    K = len(cap)
    n = S.shape[0]
    assert S.dtype == torch.float32 and S.stride(1) == 1
    assign = torch.empty(n, dtype=torch.int32, device=S.device)
    order = torch.empty(n, dtype=torch.int32, device=S.device) if want_order else None
    obj = np.zeros(K, dtype=np.float64)
    if workspace is None:
        workspace = _workspace(lib.rcd_class_workspace_bytes(n, K, 1), S.device)
    _check(lib.rcd_partition_class_graph_cut(_dev_ptr(S), S.stride(0), n, K, _np_ptr(cap), _dev_ptr(assign),
                                             _dev_ptr(order), _np_ptr(obj), _dev_ptr(workspace), workspace.numel(),
                                             _stream()))
    return assign, order, obj


def partition_dataset(X, labels, L: int, r, sigma2: float, mode: int = 0, workspace=None, want_order: bool = True,
                      graph_cut: bool = False):
    """Whole data set.  Returns (assign int32[N] device, order or None, obj float64[L, K] numpy).
    graph_cut=True runs Algorithm 1 with the graph-cut function (stored S; mode is not used)."""
    import torch

    lib = load_library()
    r = np.ascontiguousarray(r, dtype=np.int32)
    K = len(r)
    N, d = X.shape
    assert X.stride(1) == 1 and labels.dtype == torch.int32 and labels.is_contiguous()
    assign = torch.empty(N, dtype=torch.int32, device=X.device)
    order = torch.empty(N, dtype=torch.int32, device=X.device) if want_order else None
    obj = np.zeros((L, K), dtype=np.float64)
    if workspace is None:
        raise RcdError(5, "partition_dataset needs a workspace tensor (see dataset_workspace_bytes)")
    if graph_cut:
        _check(lib.rcd_partition_dataset_graph_cut(_dev_ptr(X), _dtype_code(X), N, d, X.stride(0), _dev_ptr(labels),
                                                   int(L), _np_ptr(r), K, float(sigma2), _dev_ptr(assign),
                                                   _dev_ptr(order), _np_ptr(obj), _dev_ptr(workspace),
                                                   workspace.numel(), _stream()))
        return assign, order, obj
    _check(lib.rcd_partition_dataset(_dev_ptr(X), _dtype_code(X), N, d, X.stride(0), _dev_ptr(labels), int(L),
                                     _np_ptr(r), K, float(sigma2), int(mode), _dev_ptr(assign), _dev_ptr(order),
                                     _np_ptr(obj), _dev_ptr(workspace), workspace.numel(), _stream()))
    return assign, order, obj


def last_stats() -> dict:
    out = np.zeros(8, dtype=np.int64)
    load_library().rcd_last_stats(_np_ptr(out))
    keys = ["steps", "sweeps", "entries_streamed", "useful_evals", "launches", "computed_evals", "step_ticks"]
    return dict(zip(keys, (int(v) for v in out)))


def profile(enable: bool) -> None:
    load_library().rcd_profile(1 if enable else 0)


def profile_read() -> dict:
    out = np.zeros(8, dtype=np.float64)
    load_library().rcd_profile_read(_np_ptr(out))
    return dict(steps_ms=out[0], sweep_ms=out[1], apply_ms=out[2], rounds=int(out[3]), similarity_ms=out[4])
