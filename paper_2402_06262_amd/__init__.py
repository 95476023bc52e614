"""MI355X-native RoCo (arxiv 2402.06262) hot path: a C-ABI HIP library plus a thin ctypes binding.

Every step of the path runs in the HIP kernels of `libroco.so`; this package only marshals arguments.
There is no CPU fallback: if the library is not built, loading it raises.
"""
from .binding import (  # noqa: F401
    PROF_KERNELS,
    ROCO_BF16,
    ROCO_F32,
    ROCO_IMPORTANCE_AAS,
    ROCO_IMPORTANCE_MAS,
    ROCO_IMPORTANCE_OLDEST,
    ROCO_SCOPE_ALL,
    ROCO_SCOPE_STD,
    ROCO_SCOPE_WINDOW,
    RocoCache,
    RocoError,
    RocoParams,
    alloc_cache,
    block_workspace_bytes,
    decode_step_launches,
    decode_workspace_bytes,
    library_path,
    load_library,
    prefill_workspace_bytes,
    roco_decode_step,
    roco_decode_step_gqa,
    roco_encode_block,
    roco_encode_block_gqa,
    roco_prefill_compress,
    roco_probe_cache_read,
    roco_profile_kernel,
    roco_profile_read,
    roco_profile_sampling,
    roco_select_retained,
    roco_select_victims,
    roco_strerror,
    roco_version,
)
