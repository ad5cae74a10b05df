"""MI355X-native denoise step of block-diffusion decoding (Fast-dDrive hot path).

The compute lives in ``libfdd.so`` (hand-written HIP for gfx950, C ABI in
``include/fdd.h``).  ``binding`` holds thin wrappers with the same names that
only marshal torch tensors into that ABI.  Nothing is loaded at import time;
the first call loads the library and fails loudly if it has not been built.
"""
from .binding import (  # noqa: F401
    FddError,
    fdd_block_attn,
    fdd_block_attn_batched,
    fdd_block_attn_batched_workspace,
    fdd_block_attn_workspace,
    fdd_block_commit,
    fdd_block_kv_update,
    fdd_fork_block,
    fdd_last_error,
    fdd_prefix_pack,
    fdd_prefix_pack_bytes,
    fdd_profile_attn_events,
    fdd_traj_mean,
    fdd_unmask_step,
    fdd_unmask_workspace,
    fdd_verify_step,
    fdd_verify_workspace,
    fdd_version,
    library_path,
    load_library,
)
