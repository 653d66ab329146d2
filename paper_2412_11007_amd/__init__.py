"""MI355X-native SpMM / SDDMM over a vector-blocked row-window sparse format.

The work happens in ``libflashsparse_hip.so`` (hand-written HIP for gfx950,
C ABI declared in ``include/flashsparse.h``).  This package is the thin Python
binding: it marshals torch device tensors into that ABI and nothing else.
"""
from .binding import (  # noqa: F401
    FsError,
    FsFormat,
    bind_sddmm,
    bind_spmm,
    fs_attention,
    fs_attention_workspace_bytes,
    fs_blk_to_csr,
    fs_convert,
    fs_copy_bytes,
    fs_csr_to_blk,
    fs_csr_transpose,
    fs_edge_softmax,
    fs_edge_softmax_backward,
    fs_edge_softmax_workspace_bytes,
    fs_format_bytes,
    fs_gather16,
    fs_gather_probe,
    fs_pack_values,
    fs_read_bytes,
    fs_sddmm,
    fs_sddmm_spmm,
    fs_spmm,
    fs_spmm_packed,
    fs_spmm_static,
    fs_spmm_workspace_bytes,
    fs_status_string,
    fs_version,
    library_path,
    load_library,
)
