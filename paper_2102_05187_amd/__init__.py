"""MI355X (gfx950) implementation of the sparse x dense contractions of the COMET paper.

The product is the C-ABI library `libcomet_hip.so` (see include/comet.h); this package is its
thin Python binding.  `from paper_2102_05187_amd import comet_spmv, ...` loads the library on
first use and raises if it has not been built.
"""
from .binding import (  # noqa: F401
    COMET_BORROW, COMET_CN, COMET_COPY, COMET_CU, COMET_D, COMET_LEAN, COMET_S, COMET_VALIDATE, CometError, EXPORTS, LIB_PATH,
    Tensor, comet_calibrate_gather, comet_calibrate_read, comet_mttkrp, comet_mttkrp_axpby, comet_spmm_axpby, comet_spmv_axpby, comet_spmm, comet_spmv, comet_spmv_static, comet_tensor_create, comet_tensor_destroy, comet_tensor_convert, comet_tensor_reorder,
    comet_ttm, comet_ttv,
    from_levels,
)
