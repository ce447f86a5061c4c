"""MI355X-native VeLoRA hot path: thin Python binding over libvelora's C ABI.

The functions here only marshal arguments (device pointers, sizes, the current
HIP stream) into the ``velora_*`` entry points declared in ``include/velora.h``;
every step of the path runs in the library's gfx950 kernels.  There is no CPU
or PyTorch fallback: if the shared library has not been built, the first use of
any of these names raises ImportError.

The shared library is loaded on first use rather than at package import, so
that ``python -m paper_2405_17991_amd.build`` can (re)build it.
"""
_NAMES = (
    "VeloraError", "lib_path", "velora_compress", "velora_init_v", "velora_reconstruct",
    "velora_status_string", "velora_version", "velora_weight_grad", "velora_weight_grad_static",
    "STATIC_SCRATCH_BYTES", "velora_bandwidth_probe", "velora_weight_grad_factor",
    "velora_expand_factor", "velora_update_v", "velora_compress_update", "velora_adamw_step_factor", "velora_swiglu_compress", "velora_rmsnorm_compress", "velora_linear_compress", "velora_grad_input",
    "velora_workspace_bytes", "OP_COMPRESS", "OP_INIT_V", "OP_RECONSTRUCT",
    "OP_WEIGHT_GRAD", "OP_WEIGHT_GRAD_FACTOR", "F32", "BF16", "STATUS",
)


def __getattr__(name):
    if name in _NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_NAMES))
