"""BitLinear W1.58A8 hot path for AMD MI355X: hand-written HIP kernels behind a
small C-ABI (include/bitlinear.h), with a thin ctypes binding.

    from paper_2504_12285_amd import binding as bl
    packed, beta = bl.bl_pack_ternary(W)            # offline
    q, scale, rowsum = bl.bl_quant_act_int8(X)      # per token absmax int8
    acc, y = bl.bl_gemv_w158a8(packed, beta, bl.BL_LAYOUT_K16, q, scale, rowsum, N)

The library is loaded on first use and there is no fallback if it is missing.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
