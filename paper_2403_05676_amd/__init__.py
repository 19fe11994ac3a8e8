"""MI355X-native IVF-PQ retrieval (the retrieval step of PipeRAG, Section 3.2 S3 of the paper).

Thin ctypes binding of `libpiperag.so` (C ABI in include/piperag.h).  It only marshals arguments:
torch tensors provide device memory and the current HIP stream; every step of the search and
encode paths runs in the library's HIP kernels.  There is no CPU fallback: importing works
anywhere, but any call fails loudly if the shared library has not been built.
"""
from .binding import (  # noqa: F401
    Index,
    kmeans,
    max_nprobe,
    project_latency,
    stream_create_cu_slice,
    stream_destroy,
    PiperagError,
    lib_path,
    load_library,
    NSTAGES,
    STAGE_NAMES,
)
