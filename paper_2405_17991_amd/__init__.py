"""MI355X-native VeLoRA hot path: thin Python binding over libvelora's C ABI.

The functions here only marshal arguments (device pointers, sizes, the current
HIP stream) into the ``velora_*`` entry points declared in ``include/velora.h``;
every step of the path runs in the library's gfx950 kernels.  There is no CPU
or PyTorch fallback: if the shared library has not been built the import of
:mod:`paper_2405_17991_amd.binding` raises.
"""
from .binding import (  # noqa: F401
    VeloraError,
    lib_path,
    velora_compress,
    velora_init_v,
    velora_reconstruct,
    velora_status_string,
    velora_version,
    velora_weight_grad,
    velora_workspace_bytes,
    OP_COMPRESS,
    OP_INIT_V,
    OP_RECONSTRUCT,
    OP_WEIGHT_GRAD,
    F32,
    BF16,
    STATUS,
)
