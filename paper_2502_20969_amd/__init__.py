"""MI355X-native IVF-Flat search with lookahead prefetch (the retrieval hot path of TeleRAG,
arxiv 2502.20969): hand-written HIP kernels behind a C-ABI library, and this thin binding."""
from .binding import (  # noqa: F401
    IVF_BF16, IVF_F16, IVF_F32, IVF_IP, IVF_L2, IVF_MAX_K, IVF_PLACE_DEVICE, IVF_PLACE_HOST,
    IVF_PREFETCH_RESET, EXPORTS, Index, IvfError, ivf_adopt_layout, ivf_build_layout, ivf_cache_plan, ivf_host_scan, ivf_prefetch_amount, ivf_prefetch_plan, load,
)
