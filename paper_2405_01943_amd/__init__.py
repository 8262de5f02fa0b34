"""MI355X-native hot path of DaSS pruning (arXiv 2405.01943) for GLU-variant MLPs.

The work is done by ``libdass.so`` (hand-written HIP for gfx950, C ABI declared
in ``include/dass.h``).  This package only marshals arguments: PyTorch supplies
device memory and streams.
"""
from .binding import (  # noqa: F401
    ACT, AXIS, DTYPE, DassError,
    calib_norms, calib_workspace_bytes,
    input_norms, input_norms_workspace_bytes,
    mlp_forward, mlp_forward_workspace_bytes, compress_24, down_proj_sparse24,
    score_mask_nm, nm_workspace_bytes,
    score_mask_nm_batched, nm_batched_workspace_bytes,
    score_mask_unstructured, score_mask_unstructured_static, unstructured_workspace_bytes,
    library_path, load_library, version,
)
