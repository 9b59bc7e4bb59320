"""MI355X (gfx950) hot path of ATP — attention on top principal keys.

Thin Python binding over the C ABI in ``include/atp.h``: argument marshalling
only.  Every step of the path runs in the HIP kernels of ``libatp.so``; torch is
used for device memory and streams.  There is no CPU fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    ATP_F32,
    ATP_BF16,
    ATP_W_KN,
    ATP_W_NK,
    ATP_EPI_NONE,
    ATP_EPI_SWIGLU,
    AtpError,
    lib,
    lib_path,
    version,
    set_qr_passes,
    set_overlap,
    set_factor_mode,
    set_conditioning_gram,
    principal_bases_workspace,
    principal_bases,
    alternating_bases_workspace,
    alternating_bases,
    rayleigh_ritz_workspace,
    rayleigh_ritz,
    rope,
    project_onto_bases,
    concat_factors,
    norm_factored,
    lowrank_linear_workspace,
    lowrank_linear,
    attention_workspace,
    attention,
    attention_static,
    STATIC_SCRATCH_BYTES,
    init,
    attention_linearised_workspace,
    attention_linearised,
    ATP_NORM_TAYLOR,
    ATP_NORM_ROWSUM,
    AtpLayer,
    KERNEL_CLASSES,
    profile_enable,
    profile_reset,
    profile_read,
)
