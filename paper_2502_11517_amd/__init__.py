"""MI355X-native multi-stream decode attention for PASTA's asynchronous decoding
(arxiv 2502.11517, Section 3 "Efficiency"): a thin ctypes binding over the C-ABI library
built from csrc/ (hand-written gfx950 HIP kernels) and the seeded workload generators."""
from . import workloads  # noqa: F401
from .binding import (  # noqa: F401
    PastaAttn,
    PastaError,
    build_library,
    library_path,
    load_library,
)
