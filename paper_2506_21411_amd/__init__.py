"""MI355X-native forward and backward path of D-CHAG: per-channel patch tokenization + hierarchical
cross-channel cross-attention aggregation, as hand-written HIP kernels behind a C ABI.

The Python layer only marshals arguments (device pointers, sizes, the current stream) into
`libdchag.so`; every step of the path runs in the library's kernels.  There is no CPU or
PyTorch fallback: if the library is missing, importing `binding` functions raises.
"""
from .binding import (  # noqa: F401
    DCHAG_BF16, DCHAG_F32, STATIC_SCRATCH_BYTES, DchagError, LevelGrads, LevelWeights, dchag_aggregate_level,
    dchag_aggregate_level_static,
    dchag_backward, dchag_debug_reload, dchag_fold_value, dchag_forward,
    dchag_forward_folded, dchag_forward_keep, dchag_forward_pos, dchag_forward_prefolded, dchag_profile_begin,
    dchag_profile_end, dchag_tokenize, dchag_workspace_bytes, dchag_yardstick_copy, dchag_yardstick_mfma, dchag_yardstick_read, library_path,
    load_library, use_library,
)
