"""psattn: prefix-shared DPO attention (forward + backward) on MI355X.

Thin ctypes binding over libpsattn.so (C ABI declared in include/psattn.h).
PyTorch is used for device memory and streams only; every step of the
computation runs in the library's HIP kernels.  There is no CPU fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from .binding import (  # noqa: F401
    GRID_BWD, GRID_FWD, TILE_FULL, TILE_PARTIAL, TILE_SKIPPED, Meta, PsattnError, lib_path,
    load_library, psattn_build_meta, psattn_bwd, psattn_bwd_workspace_bytes, psattn_fwd,
    psattn_kernel_name, psattn_profile_enable, psattn_profile_read, psattn_trim_pool, BF16, F32,
    psattn_bwd_static, psattn_bwd_static_max_rows, psattn_probe_dq_atomics, psattn_pack_ffd, psattn_build_meta_multi, Rope, psattn_fwd_rope, psattn_bwd_rope,
    LogprobPlan, psattn_logprob_fwd, psattn_logprob_bwd, psattn_dpo_loss,
)
