"""MI355X-native byte-level BPE batch encoder (BlockBPE's hot path).

Thin Python binding over the C ABI in ``include/bpe.h`` (``libbpe_hip.so``, hand-written HIP for gfx950).
PyTorch is used for device memory and streams only; every step of the encode runs in the library's kernels.
There is no CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from ._binding import (BpeError, Table, build_table, build_table_vocab, encode_batch, encode_batch_static, encode_strings, read_profile, lib_path, load_library,
                       set_profiling, table_image, workspace_bytes, MAX_STRING_BYTES)

__all__ = ["BpeError", "Table", "build_table", "build_table_vocab", "encode_batch", "encode_batch_static", "encode_strings", "read_profile", "lib_path",
           "load_library", "set_profiling", "table_image", "workspace_bytes", "MAX_STRING_BYTES"]
