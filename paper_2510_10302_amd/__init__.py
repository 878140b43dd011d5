"""MI355X-native SP-MoE hot path: thin Python binding over the C-ABI library ``libspmoe.so``.

The binding only marshals arguments (torch tensors -> raw device pointers, numpy arrays -> host
pointers); every step of the path runs inside the library's HIP kernels and host runtime.
There is no CPU fallback: importing :mod:`paper_2510_10302_amd.binding` raises if the library has
not been built (``python -m paper_2510_10302_amd.build`` or ``__graft_entry__.build()``).
"""
from .binding import (  # noqa: F401
    SpmoeError, Config, Context, Stats, ProfileRecord, expert_blob_bytes, pack_expert, lib_path, load_library, suggest_cutoff, gemm_plan,
    moe_layer_resident_static,
    F32, BF16, DECLARED_SYMBOLS,
)
