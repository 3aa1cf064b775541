"""MI355X-native LSH-MoE token compression path (hash -> compress -> decompress).

The work is done by hand-written gfx950 HIP kernels in ``lib/liblshmoe.so``
(built from ``csrc/`` by ``python -m paper_2411_08446_amd.build``); this package
is the thin ctypes binding over the library's C ABI (``include/lshmoe.h``).
"""
from .binding import (  # noqa: F401
    LIB_PATH, LshmoeError, CompressOutputs, load_library,
    lshmoe_hash, lshmoe_hash_sphere, lshmoe_hash_gate, lshmoe_compress, lshmoe_compress_static, lshmoe_decompress, lshmoe_decompress_combine, lshmoe_workspace_bytes,
    lshmoe_backward_workspace_bytes, lshmoe_decompress_backward, lshmoe_compress_backward,
    lshmoe_decompress_combine_backward,
    LSHMOE_OK, LSHMOE_ERR_NULL, LSHMOE_ERR_SHAPE, LSHMOE_ERR_UNSUPPORTED, LSHMOE_ERR_WORKSPACE, LSHMOE_ERR_HIP,
    LSHMOE_F32, LSHMOE_BF16, LSHMOE_FLAG_NO_RESIDUAL,
)
