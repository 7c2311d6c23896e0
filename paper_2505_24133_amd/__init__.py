"""R-KV decode-time KV-cache compression step for AMD MI355X (gfx950).

``rkv``    ctypes binding of the HIP library (loaded on first use; no CPU fallback)
``synth``  seeded synthetic inputs with the shapes of the paper's workloads
``build``  compiles csrc/*.hip into librkv.so with hipcc

The binding's names are also reachable from the package itself (``paper_2505_24133_amd.rkv_compress``);
they are resolved on first use, so that importing ``synth`` alone (as the input-drawing worker processes
do) does not pull in torch.
"""
from . import synth  # noqa: F401

_BINDING_NAMES = (
    "RKV_FLAG_GQA_SOFTMAX_THEN_MAX", "RKV_FLAG_GQA_SOFTMAX_THEN_MEAN", "RKV_FLAG_POOL_AFTER_MEAN",
    "RKV_FLAG_RECENCY_TRANSPOSED", "RKV_FLAG_SHARED_SELECTION", "RKV_FLAG_TRIANGULAR_SCAN", "RKV_FLAG_SKIP_SATURATED", "RKV_NOT_TRIGGERED",
    "RKV_OK", "RKV_STATIC_SCRATCH_BYTES", "RkvError", "RkvParams", "Shape", "load_library", "make_workspace",
    "rkv_compact", "rkv_compact_inplace", "rkv_compress", "rkv_compress_inplace", "rkv_compress_static", "rkv_probe_mfma",
    "rkv_score_importance", "rkv_score_redundancy", "rkv_select_topk", "rkv_workspace_size", "status_string",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "rkv":
        import importlib
        mod = importlib.import_module(".rkv", __name__)
        return mod if name == "rkv" else getattr(mod, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES) + ["rkv"])
