"""MI355X-native COVAP gradient-compression hot path (arXiv 2311.04499).

``paper_2311_04499_amd.binding`` is the thin ctypes layer over the C-ABI
library ``libcovap.so`` (hand-written HIP for gfx950); it is imported on first
use so that ``paper_2311_04499_amd.workloads`` (input generators only) can be
used without the library.  There is no CPU fallback: using the binding without
a built library raises.
"""

_BINDING_NAMES = (
    "covap_plan", "covap_compress", "covap_compress_aliased", "covap_decompress", "topk_compress", "topk_workspace_bytes",
    "randk_compress", "fp16_compress", "fp16_decompress", "sparse_decompress", "sparse_decompress_sorted",
    "covap_ratio_from_ccr", "covap_ratio_from_times", "covap_ef_coeff",
    "Plan", "CovapError", "lib", "build",
)


def __getattr__(name):
    if name == "binding" or name in _BINDING_NAMES:
        import importlib
        b = importlib.import_module(__name__ + ".binding")
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
