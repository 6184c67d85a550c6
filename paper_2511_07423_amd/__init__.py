"""MI355X-native batched verification of offloaded draft chunks (Synera, arXiv 2511.07423).

A thin ctypes binding over the C ABI in include/synera.h.  Every step of the path
runs in the HIP kernels of libsynera.so; this package only marshals arguments
(PyTorch supplies device memory and the stream).  There is no CPU fallback:
importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    SyneraError, Verifier, confidence, gemm_bf16, debug_set_gemm_tile, validate_batch, version, lib_path,
    OK, EINVAL, ERANGE, ENOSPC, EUNSUP, EHIP, ENOMEM, PAGE_SIZE, MAX_CHUNK, STAGES,
)
