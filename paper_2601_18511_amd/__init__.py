"""MI355X-native PCMM (plaintext-ciphertext matrix multiplication) for CKKS linear layers.

Thin Python binding over the C-ABI library libpcmm.so (see include/pcmm.h); every step of the
computation runs in the library's HIP kernels.  PyTorch is used for device memory and streams only.
"""
from .pcmm import (  # noqa: F401
    PcmmError,
    PcmmPlan,
    load_library,
    pcmm_mfma_probe,
    pcmm_plan_create,
    pcmm_plan_destroy,
    pcmm_plan_digits,
    pcmm_plan_workspace_bytes,
    pcmm_ring_compose,
    pcmm_ring_decompose,
    pcmm_run,
    pcmm_slot_rearrange,
    pcmm_run_noalloc,
    pcmm_run_profiled,
    pcmm_status_str,
    PcmvPlan,
    pcmv_plan_create,
    pcmv_plan_destroy,
    pcmv_plan_workspace_bytes,
    pcmv_run,
)
