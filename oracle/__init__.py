"""CPU oracle (test infrastructure only; the product path never imports this package)."""
from .oracle import (  # noqa: F401
    build, num_threads, set_num_threads, spmm, sddmm, row_order, csr_softmax, spmm_bias_relu,
    transpose_topology, sddmm_scaled, sddmm_nt,
)
