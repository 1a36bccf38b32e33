"""MI355X-native SBP matmul + boxing: thin Python binding over libsbp_mi355x.so.

Everything here is argument marshalling for the C ABI declared in include/sbp.h; all
computation runs in the HIP library.  PyTorch is used by callers for device memory and
streams only.  Importing the package does not need a GPU; loading the library does need
the built .so (python -m paper_2110_15032_amd.build) and fails loudly without it.
"""
from .binding import (  # noqa: F401
    S, B, P_SUM, P_MAX, AUTO, F32, BF16, I32, EPI_NONE, EPI_GELU, KNOB_GEMM_VARIANT, KNOB_TILE_ORDER, KNOB_BOX_REDUCE,
    SbpError, SbpTensor, lib, lib_path,
    sbp_infer_matmul, sbp_local_shape, sbp_matmul, sbp_matmul_ex, sbp_matmul_rowmax, sbp_boxing, sbp_boxing_across, sbp_boxing_cast,
    sbp_infer_matmul_2d, sbp_local_shape_2d, sbp_matmul_2d, sbp_boxing_2d,
    sbp_row_max, sbp_row_sumexp, sbp_xent_loss, sbp_xent_grad, sbp_set_knob, sbp_probe_mfma, sbp_probe_mfma_static, sbp_strerror, EXPORTS,
)
