"""MI355X-native chunked block-diffusion attention (Optimus elastic decoding hot path).

The package is a thin binding over a C-ABI shared library of hand-written
gfx950 HIP kernels (``csrc/``).  Importing the package does not load the
library; the first call does, and fails loudly if it has not been built.
"""
from .binding import (  # noqa: F401
    AttnParams,
    Plan,
    HostBatch,
    DeviceBuffers,
    OptimusError,
    library_path,
    load_library,
    status_string,
    static_scratch_bytes,
    commit_params,
    kv_write,
    commit_forward,
    reorg_forward,
    LatencyModel,
    latency_fit,
    latency_eval,
    select_chunk,
)
