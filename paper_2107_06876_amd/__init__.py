"""MI355X-native LCN-Sinkhorn (hand-written HIP for gfx950 behind a C ABI).

The Python layer only marshals arguments: torch supplies device memory and
streams, every step of the method runs in the HIP library.  Importing this
package does not load the library; the first call does, and fails loudly if it
has not been built (python -m paper_2107_06876_amd.build).
"""
from .binding import (  # noqa: F401
    COST_COSINE, COST_EUCLID, COST_SQEUCLID, HASH_CROSSPOLYTOPE, HASH_KMEANS, INIT_GIVEN, INIT_KMEANSPP, INIT_SAMPLE,
    MODE_DENSE, MODE_LCN, MODE_NYSTROM,
    MODE_SPARSE, LcnError, LcnHandle, library_path, load_library, lcn_build, lcn_destroy, lcn_get_buckets,
    lcn_get_csr, lcn_get_factors, lcn_get_info, lcn_get_landmarks, lcn_get_scalings, lcn_last_run_timing,
    lcn_set_scalings, lcn_status_string, lcn_workspace_bytes, plan_marginals, sinkhorn_run, transport_cost,
    LcnBatchHandle, lcn_batched_get, lcn_batched_results, lcn_build_batched, lcn_backward,
    lcn_backward_scratch_bytes, lcn_plan_rows, lcn_deletion_costs, lcn_head_lambdas, lcn_last_error_counts, lcn_backward_static,
    lcn_calibrate, CAL_COPY_GBS, CAL_READ_GBS, CAL_MFMA_BF16_TFLOPS, CAL_MFMA_F64_TFLOPS, CAL_LAUNCH_US)
