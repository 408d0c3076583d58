"""MI355X-native CenteredClip aggregation and BTARD verification quantities.

Thin Python binding over the C-ABI library ``libbtard.so`` (hand-written HIP
for gfx950).  PyTorch supplies device memory and the stream, nothing else.
"""
from .binding import (  # noqa: F401
    BtardError,
    alloc_workspace,
    btard_cc_begin,
    BTARD_FLAG_GRAM,
    BTARD_FLAG_HOST_SYNC,
    btard_cc_remaining,
    cc_remaining,
    BTARD_FLAG_NONE,
    btard_cc_finish,
    btard_cc_gram,
    btard_debug_gram,
    cc_gram,
    debug_gram,
    btard_cc_iterate,
    btard_centered_clip,
    btard_debug_zhat,
    btard_split_offsets,
    btard_status_string,
    btard_verify_projections,
    btard_workspace_bytes,
    cc_begin,
    cc_finish,
    cc_iterate,
    centered_clip,
    debug_zhat,
    lib_path,
    load_library,
    make_problem,
    split_offsets,
    verify_projections,
    workspace_bytes,
)
