"""MI355X-native chunked causal power attention (arXiv 2507.04239, Sec. 4 and App. E).

``power_attn_fwd`` / ``power_attn_bwd`` marshal torch device tensors into the C-ABI
library built from ``csrc/``; every step of the computation runs in its HIP kernels.
The library is loaded on first use and a missing library is an error, never a fallback.
"""
from .binding import (  # noqa: F401
    PowerAttnError,
    library_path,
    load_library,
    power_attn_bwd,
    power_attn_fwd,
    power_attn_workspace_bytes,
)
