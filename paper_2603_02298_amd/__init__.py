"""MI355X-native layout algebra and layout-driven tensor copy (COPY of the CuTe layout method).

The work is done by liblayoutcopy.so (C++ host algebra and planner, HIP kernels for gfx950) behind
the C ABI of include/layoutcopy.h; this package only marshals arguments.
"""
from .binding import (GemmPlan, gemm_tensor, lc_gemm, lc_mfma_fragment_layout, DTYPES, DTYPE_BYTES, Layout, LayoutCopyError, Plan, copy_tensor, lc_coalesce,  # noqa: F401
                      lc_coalesce_bymode, lc_complement, lc_composition, lc_composition_bymode, lc_copy,
                      lc_admissible, lc_blocked_product, lc_layout_slice, lc_left_inverse, lc_logical_divide, lc_logical_divide_bymode, lc_logical_product,
                      lc_max_common_vector, lc_raked_product, lc_right_inverse, SLayout, lc_slayout_coalesce,
                      lc_slayout_composition, lc_slayout_right_inverse, lc_slayout_xor_right_inverse,
                      lc_zipped_divide, lib)
