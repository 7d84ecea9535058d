"""zc: fZ-light error-bounded compression and the compressed-Allreduce local step on MI355X.

`binding` holds thin ctypes wrappers with the names of the C ABI (include/zc.h); every step
of the path runs in the HIP kernels of libzc.so.  `synth` makes seeded synthetic inputs.
"""
from . import binding, synth  # noqa: F401
from .binding import (  # noqa: F401
    ZcError, zc_compress, zc_compress_bound, zc_compress_noalloc, zc_compress_part, zc_debug_block_offsets, zc_debug_quantize, zc_debug_stream, zc_decompress, zc_decompress_average, zc_decompress_many, zc_decompress_range,
    zc_finish, zc_peek_header, zc_profile_collect, zc_profile_enable, zc_quality, zc_reduce_compressed, zc_reduce_compressed_op, zc_reduce_compressed_part, zc_reduce_step, zc_reduce_step_part, zc_reduce_step_op,
    zc_strerror,
    zc_workspace_bytes,
)
