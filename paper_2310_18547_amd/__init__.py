"""libsgmv for MI355X: Python binding of the C ABI (argument marshalling only).

Every step of the operator runs in the HIP kernels of ``libsgmv.so``; there is
no Python or CPU implementation behind these names.  The binding is loaded on
first use of any of its names and raises ``ImportError`` if the library has not
been built (``python -m paper_2310_18547_amd.build``).
"""
_BINDING_NAMES = (
    "F16", "BF16", "PATH_AUTO", "PATH_VECTOR", "PATH_MATRIX", "PATH_FUSED", "PATH_WHOLE", "PATH_ROWS", "SgmvError", "SgmvProblem", "lib",
    "SgmvPlan", "KERNEL_NONE", "KERNEL_FUSED", "KERNEL_TILE", "KERNEL_MULTI_SIDE", "KERNEL_MULTI_PIPELINED",
    "KERNEL_VECTOR", "KERNEL_MATRIX", "KERNEL_WHOLE", "KERNEL_NAMES", "sgmv_add_lora_multi", "sgmv_add_lora_static", "sgmv_plan_add_lora", "sgmv_plan_shrink", "sgmv_plan_expand", "sgmv_workspace_bytes_multi",
    "library_path", "make_problem", "sgmv_add_lora", "sgmv_expand", "sgmv_shrink",
    "sgmv_status_string", "sgmv_validate_segments", "sgmv_workspace_bytes", "sgmv_workspace_init",
    "sgmv_workspace_check", "sgmv_probe", "PROBE_EMPTY", "PROBE_READ", "PROBE_COPY", "PROBE_HANDOFF",
    "STATIC_SCRATCH_BYTES", "STATIC_MAX_WORKSPACE_BYTES",
)
__all__ = list(_BINDING_NAMES)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
