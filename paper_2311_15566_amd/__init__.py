"""MI355X-native decode shard + KV-cache re-partition (after SpotServe, arXiv 2311.15566).

Thin Python binding over the C-ABI library `libspotshard.so` (hand-written HIP kernels for
gfx950).  PyTorch is used for device memory and streams only; every step of the path runs in
the library's kernels.  There is no CPU fallback: importing `binding` without the built
library raises.
"""
from .binding import (  # noqa: F401
    LIB_PATH,
    Shard,
    SpotShardError,
    committed_len,
    decode_step,
    decode_step_static,
    device_kv_bytes,
    force_gemm_shape,
    force_prefill_block,
    kv_export,
    kv_import,
    kv_repack,
    lib,
    matrix_core_probe,
    prefill,
    stage_decode_step,
    stage_prefill,
    static_scratch_bytes,
    version,
)
