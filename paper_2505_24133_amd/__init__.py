"""R-KV decode-time KV-cache compression step for AMD MI355X (gfx950).

``rkv``    ctypes binding of the HIP library (loaded on first use; no CPU fallback)
``synth``  seeded synthetic inputs with the shapes of the paper's workloads
``build``  compiles csrc/*.hip into librkv.so with hipcc
"""
from . import synth  # noqa: F401
from .rkv import (  # noqa: F401
    RKV_FLAG_GQA_SOFTMAX_THEN_MAX, RKV_FLAG_GQA_SOFTMAX_THEN_MEAN, RKV_FLAG_POOL_AFTER_MEAN, RKV_FLAG_RECENCY_TRANSPOSED, RKV_FLAG_SHARED_SELECTION, RKV_FLAG_SKIP_SATURATED, RKV_NOT_TRIGGERED, RKV_OK, RkvError, RkvParams, Shape, load_library, make_workspace,
    rkv_compact, rkv_compact_inplace, rkv_compress, rkv_compress_inplace, rkv_compress_static, rkv_score_importance, rkv_score_redundancy, rkv_select_topk,
    rkv_workspace_size, status_string,
)
