"""MI355X-native chunkwise linear-sequence-modeling hot path (C-ABI library + thin binding)."""
from .binding import (  # noqa: F401
    DECAY_NONE, DECAY_HEAD, DECAY_SCALAR, DECAY_VECTOR, LAYOUT_BHTD, LAYOUT_BTHD, FLAG_SAVE_STATES, FLAG_SAVE_ALWAYS,
    LsmError, library, kernel_path, keeps_states, lsm_chunk_fwd, lsm_chunk_bwd, lsm_bench_intra_chunk, lsm_step,
    lsm_chunk_fwd_workspace_bytes, lsm_chunk_bwd_workspace_bytes, make_params,
    lsm_profile_start, lsm_profile_stop, lsm_chunk_workspace, lsm_bench_intra_chunk_workspace,
    lsm_chunk_fwd_noalloc, NOALLOC_SCRATCH_BYTES, lsm_calib_copy, lsm_calib_mfma, lsm_delta_fwd, lsm_delta_bwd, lsm_delta_workspace, lsm_delta_step,
)
