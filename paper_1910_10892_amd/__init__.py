"""MI355X-native min-sum message passing (ISGMR, TRWP) on grid pairwise MRFs.

Thin Python binding of the C-ABI library libmrfmp (include/mrfmp.h).  PyTorch is used for
device memory and streams only; every step of the path runs in the library's HIP kernels.
"""
from .mrfmp import (  # noqa: F401
    MRF_ISGMR, MRF_TRWP, MrfError, MrfProblem, library_path, load_library, mrf_forward_window,
    mrf_isgmr_backward, mrf_isgmr_forward, mrf_scanline_count, mrf_scanline_head, mrf_set_sweep_events,
    mrf_strerror,
    mrf_last_error_detail, mrf_last_sweep_kernel, mrf_last_sweep_launch,
    mrf_energy, mrf_energy_noalloc, mrf_energy_workspace_bytes, mrf_softmin_l1, mrf_softmin_smooth_l1, mrf_softmin_l1_workspace_bytes,
    mrf_trwp_backward, mrf_trwp_forward, mrf_tune, mrf_workspace_fault, mrf_validate, mrf_version, mrf_workspace_bytes,
)
