"""MI355X-native batched verification of offloaded draft chunks (Synera, arXiv 2511.07423).

A thin ctypes binding over the C ABI in include/synera.h.  Every step of the path
runs in the HIP kernels of libsynera.so; this package only marshals arguments
(PyTorch supplies device memory and the stream).  There is no CPU fallback:
importing the binding without the built library raises.
"""
_EXPORTS = (
    "SyneraError", "Verifier", "confidence", "confidence_topk", "nucleus", "topp_count", "chunk_dispatch", "gemm_pair", "gemm_pair_static", "STATIC_GEMM_MAX_OUT", "split_pair", "LO_SITES",
    "debug_set_gemm_tile", "debug_gemm_epilogue", "debug_gemm_paired", "debug_gemm_slices", "debug_gemm_plan", "debug_gemm_plan_bk", "debug_attention_plan", "measure_hbm_copy", "measure_hbm_read", "MEASURE_READ_BLOCKS", "measure_mfma_bf16", "measure_mfma_f16",
    "validate_batch", "version", "lib_path", "Scheduler", "SCHED_IDLE", "SCHED_PREFILL", "SCHED_VERIFY",
    "OK", "EINVAL", "ERANGE", "ENOSPC", "EUNSUP", "EHIP", "ENOMEM", "PAGE_SIZE", "MAX_CHUNK", "STAGES",
)
__all__ = list(_EXPORTS)


def __getattr__(name):
    # The binding loads libsynera.so; it is imported on first use so that `paper_2511_07423_amd.build`
    # (which compiles that library) can be imported before the library exists or while it is stale.
    if name in _EXPORTS:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
