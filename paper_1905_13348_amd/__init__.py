"""Batched per-query model-variant selection (INFaaS, arxiv 1905.13348, Section 4.1) on MI355X.

Thin Python binding over the C-ABI library ``libinfaas_sel.so`` (include/infaas_sel.h).
Every step of the selection runs in the library's HIP kernels; this package only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    ENGINE_AUTO,
    ENGINE_SCAN,
    ENGINE_INDEX,
    KERNEL_NAMES,
    InfaasSelError,
    Selector,
    library_path,
    load_library,
)
