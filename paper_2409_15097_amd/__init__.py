"""Binary Block Masking flash attention (forward and backward) for AMD MI355X: thin Python binding over libbbm.so.

The names below are those of the C ABI (include/bbm.h); the functions only marshal arguments: device memory and the
stream come from PyTorch, every computation runs in the library's HIP kernels.  There is no CPU fallback: the
binding is loaded at the first use of any of these names and raises ImportError if the library is not built (the
package itself imports without it, so that `python -m paper_2409_15097_amd.build` can build it).
"""
_NAMES = (
    "BBM_MODE_BITMAP", "BBM_MODE_RUNS", "BBM_MODE_LIST", "BBM_MODE_DENSE_BASELINE", "BBM_MODE_AUTO",
    "BBM_OK", "BBM_EINVAL", "BBM_EUNSUPPORTED", "BBM_EWORKSPACE", "BBM_EHIP",
    "BbmError", "BlockIndex", "lib", "library_path",
    "bbm_last_error", "bbm_version", "bbm_build_block_mask", "bbm_build_block_mask_rect", "bbm_attn_fwd_rect",
    "bbm_attn_fwd_static", "bbm_build_runs", "bbm_build_sparse_index", "bbm_build_index", "bbm_build_col_index",
    "bbm_col_sched_bytes", "bbm_attn_bwd_workspace_bytes", "bbm_attn_bwd", "bbm_attn_fwd_workspace_bytes", "bbm_attn_fwd",
    "bbm_sched_bytes", "build_index", "bf16_from_bits", "bbm_rcm_workspace_bytes", "bbm_rcm_order", "bbm_permute_mask",
    "bbm_gather_rows", "bbm_probe_mfma_bf16", "bbm_probe_mfma_bf16_flop",
)
__all__ = list(_NAMES)


def __getattr__(name):
    if name in _NAMES:
        from . import binding          # loads libbbm.so; ImportError if it is not built
        value = getattr(binding, name)
        globals()[name] = value
        return value
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_NAMES))
