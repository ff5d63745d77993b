"""MI355X-native CSR SpMM / SDDMM (libspdl) and its Python binding."""
from .binding import (  # noqa: F401
    SpdlError, spdl_spmm, spdl_sddmm, spdl_spmm_f16, spdl_sddmm_f16, spdl_build_row_order,
    spdl_validate_csr_host, spdl_select_spmm, spdl_select_sddmm, spdl_force_variant,
    spdl_variant_name, spdl_status_string, spdl_version, spdl_spmm_bias_relu, spdl_spmm_bias_relu_f16,
    spdl_csr_softmax, spdl_sddmm_scaled, spdl_sddmm_scaled_f16,
    spdl_sddmm_nt, spdl_sddmm_nt_f16, spdl_spmm_f16_i16, spdl_sddmm_ordered, spdl_spmm_banded, spdl_sddmm_banded, spdl_spmm_skewed, spdl_sddmm_skewed, spdl_build_transpose_host, spdl_permute_values, lib, LIB_PATH, EXPORTS,
)
