"""MI355X (gfx950) RSR++ vector x binary/ternary-matrix product.

Thin Python binding over the C ABI declared in ``include/rsr.h``; the functions have the same
names and do argument marshalling only.  Every step of the product runs in the HIP kernels of
``csrc/``; there is no CPU fallback: a missing ``librsr.so`` raises ``ImportError``-like
``RuntimeError`` on first use (build it with ``python -m paper_2411_06360_amd.build``).
"""
from .binding import (  # noqa: F401
    RsrError,
    RsrInfo,
    lib_path,
    load,
    rsr_destroy,
    rsr_export_block,
    rsr_host_export_block,
    rsr_host_free,
    rsr_host_info,
    rsr_host_pack,
    rsr_host_streams,
    rsr_info,
    rsr_last_error,
    rsr_matvec,
    rsr_matvec_i8,
    rsr_matvec_acc,
    rsr_matvec_acc_i8,
    rsr_qbit_preprocess,
    rsr_qbit_matvec,
    rsr_qbit_matvec_i8,
    rsr_qbit_planes,
    rsr_qbit_table_bytes,
    rsr_qbit_destroy,
    rsr_matvec_multi,
    rsr_matvec_multi_i8,
    make_jobs,
    rsr_dense_preprocess,
    rsr_dense_matvec,
    rsr_dense_matvec_i8,
    rsr_dense_matvec_static,
    rsr_dense_table_bytes,
    rsr_dense_destroy,
    rsr_model_k,
    rsr_autotune_k,
    rsr_set_step2,
    RSR_STEP2_FOLD,
    RSR_STEP2_PLAIN,
    rsr_preprocess,
    rsr_preprocess_device,
)
