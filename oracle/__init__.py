"""CPU oracle for the hybrid SpMM hot path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product (the HIP library and its Python binding) never does, and
this package never imports the product.
"""
from .numeric import (  # noqa: F401
    build_oracle_lib,
    spmm,
    spmm_rows,
    gemm,
    gcn_layer,
    gcn_layer_rows,
    aggregate_update,
    aggregate_update_rows,
    layer_backward,
    round_to_16bit,
    num_threads,
    set_num_threads,
    DT_F32, DT_BF16, DT_F16, DT_F64,
)
from .plan import (  # noqa: F401
    window_features,
    sparsity,
    computing_intensity,
    select_route,
    launch_guard,
    derive_plan,
    derive_plan_vectorised,
    derive_window,
    derive_runs,
)
