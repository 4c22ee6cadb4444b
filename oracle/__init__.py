"""CPU oracle for tensor-network linear layers. TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: only tests/, the smoke
check and the benchmark's cpu_baseline leg use it. It shares no code with the
HIP library and never imports it.
"""
from .tn_oracle import (  # noqa: F401
    tt_dense,
    tr_dense,
    tr_dense_rows,
    tucker_dense,
    dense_weight,
    apply_linear,
    forward,
    brute_force_weight,
    tt_svd,
    rel_max_err,
    param_gradients,
    mxfp4_quantize,
    mxfp4_dequantized,
)
