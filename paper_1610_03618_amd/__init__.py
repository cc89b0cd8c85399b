"""MI355X-native memory-bound CNN layers: layout transform, pooling, fused softmax.

The work is done by hand-written HIP kernels for gfx950 in ``libcnnmem.so``
(C ABI declared in ``include/cnnmem.h``).  This package is the thin Python
binding: it marshals torch device tensors into that ABI and nothing else.
There is no CPU fallback: without the built library, or without a GPU tensor,
calls raise.
"""
from .binding import (  # noqa: F401
    BF16, CHWN, F16, F32, LAYER_CONV, LAYER_OTHER, LAYER_POOL, NCHW, POOL_AVG, POOL_KEEPS_LAYOUT, POOL_MAX, POOL_PREFERS_CHWN,
    CnnmemError, PoolTuning, cnnmem_choose_layout, cnnmem_plan_layouts, cnnmem_pool, cnnmem_pool_out_dims, cnnmem_pool_tuned,
    cnnmem_permute, cnnmem_permute_dtype, cnnmem_pool_backward, cnnmem_pool_dtype, cnnmem_relayout, cnnmem_relayout_dtype, cnnmem_softmax, cnnmem_softmax_backward, cnnmem_softmax_dtype, cnnmem_status_string, cnnmem_transform, cnnmem_transform_dtype, cnnmem_version, library, test_hooks,
    permute, pool, pool_backward, relayout, softmax, softmax_backward, transform,
)
