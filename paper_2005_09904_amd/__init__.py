"""BiQGEMM lookup-table matrix multiply for AMD MI355X (gfx950).

The product is libbiq.so (HIP kernels behind the C ABI of include/biq.h); this package is the
thin ctypes binding plus the synthetic workload generator.
"""
from .binding import (  # noqa: F401
    BIQ_EHIP, BIQ_EINVAL, BIQ_EUNSUPPORTED, BIQ_EWORKSPACE, BIQ_OK, BiqError, BiqPlan, BiqProblem, PreparedGemm, PreparedGroup, PreparedLstmCell, biq_gemm_grouped, biq_lstm_cell,
    biq_build_lut, biq_gemm, biq_gemm_ex, biq_gemm_noalloc, biq_init, biq_noalloc_scratch_bytes, biq_kernel_name, biq_key_row_stride, biq_lut_bytes,
    biq_num_chunks, biq_pack, biq_packed_bytes, biq_plan_check, biq_plan_get, biq_plan_get_lut, biq_plan_get_mfma, biq_plan_workspace_bytes, biq_quantize, biq_query,
    biq_unpack_keys, biq_unpack_keys16, biq_workspace_bytes, load_library, status_str,
)
