"""MI355X-native clustering stage of ClusComp: Lloyd k-means over weight sub-vectors and the
codebook-gather decode, as hand-written gfx950 HIP kernels behind a C ABI (include/cluscomp.h).

This package is a thin binding: every step of the path runs in the HIP library. There is no CPU
fallback; calling anything without the built library (or without a GPU) raises.
"""
from .driver import CompressedLayer, compress_model  # noqa: F401
from .binding import (  # noqa: F401
    CCError,
    PROFILE_SLOTS,
    Profile,
    Stats,
    assign,
    codebook_quantize,
    decode,
    kmeans_fit,
    last_error,
    layer_codebook_grad,
    layer_codebook_grad_planned,
    layer_codebook_grad_planned_workspace_bytes,
    layer_grad_plan,
    layer_grad_plan_bytes,
    layer_grad_plan_workspace_bytes,
    layer_compress,
    layer_compress_workspace_bytes,
    layer_deficiency,
    layer_forward,
    layer_forward_q,
    layer_forward_q_workspace_bytes,
    layer_forward_workspace_bytes,
    layer_num_codes,
    layer_pack,
    layer_vectors,
    layer_weight,
    layer_weight_q,
    lib_path,
    lloyd_iter,
    load_library,
    mfma_f16_probe,
    read_stats,
    set_assign_mode,
    update,
    version,
    workspace_bytes,
)
