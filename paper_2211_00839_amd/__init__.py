"""MI355X (gfx950) implementation of the ratio-constrained submodular partitioner
of RCD-SGD (arXiv 2211.00839, Algorithm 1): thin Python binding over librcd.so.

Every function only marshals torch device tensors into the C ABI declared in
``include/rcd.h``; all arithmetic of the method runs in the library's HIP
kernels.  There is no CPU fallback: without the built library, or without a
GPU, calls raise.
"""
from .binding import (  # noqa: F401
    RcdError,
    bandwidth,
    batch_sizes,
    class_workspace_bytes,
    dataset_workspace_bytes,
    gain_sweep,
    init,
    last_stats,
    lib_path,
    load_library,
    partition_class,
    partition_class_graph_cut,
    partition_dataset,
    profile,
    profile_read,
    quota,
    release,
    similarity,
    similarity_static,
    strerror,
    worker_shards,
    workspace_bytes,
)

F32 = 0
BF16 = 1
MODE_AUTO = 0
MODE_STORED = 1
MODE_RECOMPUTE = 2
MODE_INCREMENTAL = 3
MAX_K = 16
STATIC_MAX_N = 65536
