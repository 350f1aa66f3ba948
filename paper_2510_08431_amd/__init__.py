"""MI355X-native fused attention forward + Jacobian-vector product (paper App. C.1, Alg. 2).

`attn_jvp_fwd` and friends are thin ctypes bindings over the C-ABI library built from
`csrc/`; they are imported lazily so that `workloads` can be used without the library.
"""

__all__ = ["attn_jvp_fwd", "attn_jvp_fwd_ex", "attn_jvp_fwd_static", "attn_jvp_static_scratch_bytes", "attn_jvp_rmsnorm_fwd", "attn_jvp_mfma_rate_probe", "attn_jvp_strerror", "attn_jvp_version",
           "attn_jvp_workspace_bytes", "load_library"]


def __getattr__(name):
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
