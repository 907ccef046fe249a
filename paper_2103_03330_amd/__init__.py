"""MI355X-native zero-copy sparse feature gather.

GPU wavefronts read the rows named by a minibatch's node-ID list straight out
of a feature table kept in pinned, device-mapped host memory and write them as
a dense tensor in HBM (the GPU-oriented data path of the paper's Section 3).
The work is done by hand-written gfx950 kernels behind a C ABI
(``include/zcgather.h``); this package is the thin Python binding.
"""
from .binding import (  # noqa: F401
    EBUSY, ECAPACITY, ECLOSED, ETIMEDOUT,
    ALLOC_DEFAULT, ALLOC_NONCOHERENT, ALLOC_NUMA_USER, ALLOC_UNCACHED, B8, B64, F16, F32, VARIANT_ALIGNED, VARIANT_AUTO, VARIANT_HALFLINE,
    VARIANT_NAIVE, VARIANT_NAMES, VARIANT_ROWVEC, LaunchOpts, MaskedStream, Pipeline, Table, ZcgError,
    alloc_table, device_cu_count, stream_create_cu_mask, stream_destroy, table_view,
    cpu_gather_memcpy, cpu_gather_memcpy_chunked, gather, gather_ex, gather_ordered, gather_variant,
    make_order, make_order_static, order_workspace_bytes, gather_workspace_bytes, STATIC_ORDER_MAX_IDX,
    last_hip_error, load_library, pipeline_create, pinned_alloc, pinned_free, plan_gather, plan_shape,
    register_table, strerror, table_from_device, unregister_table, validate_indices, version,
)
from .unified import UnifiedTensor, to_unified  # noqa: F401,E402
