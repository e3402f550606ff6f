"""MI355X-native binary-coding GEMV (inference path of GPTQT, arXiv 2407.02891).

Thin Python binding over the C ABI in include/bcq.h; see `binding`.
"""
from .binding import (  # noqa: F401
    BcqError, Desc, PackedLayer, from_linear, from_linear_rows, gemm_skinny, gemv, gemv_noalloc, lib, pack, pack_rows, packed_bytes, quant_factor, quant_factor_workspace_bytes, quant_gptq, quant_hessian, quant_search, quant_workspace_bytes,
    read_probe, set_option, status_string, unpack, workspace_bytes, workspace_init,
)
