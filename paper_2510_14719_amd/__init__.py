"""MI355X-native fused attention forward (gfx950 HIP kernels behind a C ABI).

``attn_fwd`` and friends live in :mod:`paper_2510_14719_amd.binding`; they are
imported lazily so that the input generators can be used on a machine that has
no built library.
"""

__all__ = ["attn_fwd", "attn_fwd_f16", "attn_fwd_bf16", "attn_fwd_fp8", "AttnFwdError", "load_library"]


def __getattr__(name):
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
