"""MI355X-native forward pass of tensor-network linear layers.

The work is done by hand-written HIP kernels behind a C-ABI shared library
(include/tn_linear.h); this package is the thin ctypes binding over it. PyTorch
is used only for device memory and streams. There is no CPU fallback: if the
library is missing or no GPU is present, calls raise.
"""
from .binding import (  # noqa: F401
    TNLinear,
    TNLinearError,
    library_path,
    load_library,
    plan_query,
    tn_linear_create,
    tn_linear_destroy,
    tn_linear_forward,
    tn_linear_forward_scratch,
    tn_linear_forward2,
    tn_linear_param_gradients,
    tn_linear_quantized_tensor,
    forward2,
    tn_linear_plan_query,
    tn_linear_profile,
    tn_linear_profile_read,
    tn_linear_query,
    tn_linear_strerror,
    tn_linear_version,
    EXPORTED_SYMBOLS,
    TN_FORMAT_DENSE, TN_FORMAT_TT, TN_FORMAT_TR, TN_FORMAT_TUCKER,
    TN_DTYPE_F32, TN_DTYPE_BF16,
    TN_FLAG_SCALAR_KERNELS, TN_FLAG_NO_MERGE, TN_FLAG_NO_SPLIT_K, TN_FLAG_MERGE_GROW,
    TN_FLAG_NO_PAIR_CHAIN, TN_FLAG_NO_CHAIN2, TN_FLAG_TRANSPOSE, TN_FLAG_NO_SMALL_CHAIN, TN_FLAG_VARIANT_SHIFT, TN_FLAG_NO_LAZY_MERGE, TN_FLAG_MERGE_HALVES, TN_FLAG_SCALAR_GENERATE, TN_FLAG_NO_DECODE_FUSION, TN_FLAG_TRAINABLE, TN_FLAG_QUANT_MXFP4, TN_FLAG_NO_Q4_STREAM, TN_FLAG_NO_SKINNY, TN_QUERY_QUANT_BYTES, TN_QUERY_QUANT_STREAM_BYTES, TN_QUERY_BACKWARD_CHUNK_TOKENS, TN_QUERY_BACKWARD_WORKSPACE_BYTES, TN_QUERY_PAIR_CHAINABLE, TN_QUERY_KRON_CHAINABLE,
    TN_QUERY_LAZY_MIN_TOKENS, TN_QUERY_LAZY_FLOPS_PER_TOKEN,
    TN_QUERY_PARAM_COUNT, TN_QUERY_PACKED_BYTES, TN_QUERY_FLOPS_PER_TOKEN, TN_QUERY_WORKSPACE_BYTES,
    TN_QUERY_NUM_STEPS, TN_QUERY_CHUNK_TOKENS, TN_QUERY_MAX_INTERMEDIATE, TN_QUERY_OUT_FEATURES,
    TN_QUERY_IN_FEATURES, TN_QUERY_NUM_MERGES, TN_QUERY_STEP_BASE,
)
