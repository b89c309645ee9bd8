"""MI355X-native hot path of C2T token-tree construction: thin Python binding of the C ABI
(include/c2t.h).  All computation happens in the HIP kernels of the shared library;
PyTorch is used for device memory and streams only."""
from .binding import (C2TConfig, C2TContext, C2TError, build, lib_path, load_library, stream_read, stream_read_rows)  # noqa: F401
