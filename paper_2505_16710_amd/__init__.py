"""MI355X-native chunk-wise attention for SeCO / SpaCO (thin binding over libseco_hip.so).

The package holds the HIP sources (csrc/), the build script and a ctypes binding whose
functions carry the names of the C ABI in include/seco.h.  Every step of the path runs in
the HIP kernels; PyTorch is used only for device memory and streams.  There is no CPU or
PyTorch fallback: if the library has not been built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    SecoError,
    kv_append,
    kvgrad_accumulate,
    kvgrad_readout,
    kvgrad_zero,
    library_path,
    load_library,
    rope_rotate,
    seco_chunk_attn_bwd,
    seco_chunk_attn_bwd_gather,
    seco_chunk_attn_bwd_noalloc,
    seco_chunk_attn_fwd,
    seco_device_info,
    seco_launch_plan,
    seco_profile_enable,
    seco_profile_read,
    seco_profile_set,
    seco_strerror,
    seco_workspace_bytes,
    spaco_chunk_attn_bwd,
    spaco_chunk_weights,
    spaco_compensation_factor,
    spaco_gather_row_weights,
    spaco_percall_weights,
    spaco_select_bernoulli,
    spaco_select_chunks,
)
