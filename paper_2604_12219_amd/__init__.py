"""MI355X (gfx950) implementation of the PASA sparse self-attention forward.

The compute lives in ``libpasa_hip.so`` (hand-written HIP kernels behind the C ABI declared in
``include/pasa.h``); :mod:`paper_2604_12219_amd.pasa` is a thin ctypes binding with the same entry
points.  PyTorch is used for device memory and streams only.  There is no CPU fallback: calling any
entry point without the built library raises.
"""
from .pasa import (  # noqa: F401
    PasaError,
    Shape,
    attn_dense_ref,
    attn_workspace_bytes,
    block_score,
    check_selection,
    budget_schedule,
    forward,
    forward_single_call,
    key_prior,
    kv_stats,
    l1_distance,
    lib_path,
    load_library,
    mask_words,
    mfma_probe,
    num_blocks,
    route,
    score_workspace_bytes,
    sparse_attn_fwd,
    sparse_attn_fwd_static,
    STATIC_SCRATCH_BYTES,
    topk_count,
)
