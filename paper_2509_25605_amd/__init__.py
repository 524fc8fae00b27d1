"""MI355X-native CSR SpMV / SpMM (the sparse kernel of Section 6.2 of the LAPIS
paper) behind a C ABI; this package is the thin Python binding plus the build
step.  All computation runs in the HIP kernels of csrc/."""
from .binding import (  # noqa: F401
    LAPIS_ERR_ALLOC, LAPIS_ERR_DEVICE, LAPIS_ERR_INVALID_ARG, LAPIS_ERR_UNSUPPORTED, LAPIS_F32,
    LAPIS_F64, LAPIS_OK, LapisError, lapis_csr_copy_partition, lapis_csr_create, lapis_csr_destroy,
    lapis_csr_partition_sizes, lapis_csr_half_bandwidth, lapis_csr_split_sizes, lapis_csr_copy_split, lapis_last_error, lapis_partition_constants, lapis_spmm, lapis_spmv,
    lapis_spmv_paper_shape, lapis_paper_vector_length, load, DualView, lapis_spmv_dualview, lapis_spmv_transpose, lapis_csr_create_transpose, lapis_csr_shape, lapis_csr_copy_arrays, lapis_csr_copy_index16,
    lapis_csr_copy_patterns, lapis_batched_gemm, lapis_spmv_static_scratch, lapis_spmv_scratch_bytes,
)
from .matrix import CsrMatrix  # noqa: F401
