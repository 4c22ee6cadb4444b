"""ctypes binding of libtn_linear.so: argument marshalling only.

Function names mirror the C ABI (include/tn_linear.h). Tensors are torch CUDA
(ROCm) tensors; the binding passes their data pointers and the current HIP
stream. Nothing here computes.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libtn_linear.so"

TN_FORMAT_DENSE, TN_FORMAT_TT, TN_FORMAT_TR, TN_FORMAT_TUCKER = 0, 1, 2, 3
TN_DTYPE_F32, TN_DTYPE_BF16 = 0, 1
TN_FLAG_SCALAR_KERNELS = 1
TN_FLAG_NO_MERGE = 2
TN_FLAG_NO_SPLIT_K = 4
TN_FLAG_MERGE_GROW = 16
TN_FLAG_NO_PAIR_CHAIN = 32
TN_FLAG_NO_CHAIN2 = 64
TN_FLAG_TRANSPOSE = 128
TN_FLAG_NO_SMALL_CHAIN = 1 << 20
TN_FLAG_VARIANT_SHIFT = 8
TN_FLAG_NO_LAZY_MERGE = 1 << 21
TN_FLAG_MERGE_HALVES = 1 << 22
TN_FLAG_SCALAR_GENERATE = 1 << 23
TN_FLAG_NO_DECODE_FUSION = 1 << 24
TN_FLAG_TRAINABLE = 1 << 25
TN_FLAG_QUANT_MXFP4 = 1 << 26
TN_FLAG_NO_Q4_STREAM = 1 << 27
TN_FLAG_NO_SKINNY = 1 << 28
TN_QUERY_PARAM_COUNT = 0
TN_QUERY_PACKED_BYTES = 1
TN_QUERY_FLOPS_PER_TOKEN = 2
TN_QUERY_WORKSPACE_BYTES = 3
TN_QUERY_NUM_STEPS = 4
TN_QUERY_CHUNK_TOKENS = 5
TN_QUERY_MAX_INTERMEDIATE = 6
TN_QUERY_OUT_FEATURES = 7
TN_QUERY_IN_FEATURES = 8
TN_QUERY_NUM_MERGES = 9
TN_QUERY_PAIR_CHAINABLE = 10
TN_QUERY_KRON_CHAINABLE = 11
TN_QUERY_LAZY_MIN_TOKENS = 12
TN_QUERY_LAZY_FLOPS_PER_TOKEN = 13
TN_QUERY_BACKWARD_CHUNK_TOKENS = 14
TN_QUERY_BACKWARD_WORKSPACE_BYTES = 15
TN_QUERY_QUANT_BYTES = 16
TN_QUERY_QUANT_STREAM_BYTES = 17
TN_QUERY_STEP_BASE = 100

EXPORTED_SYMBOLS = (
    "tn_linear_create",
    "tn_linear_forward",
    "tn_linear_forward_scratch",
    "tn_linear_forward2",
    "tn_linear_param_gradients",
    "tn_linear_quantized_tensor",
    "tn_linear_destroy",
    "tn_linear_query",
    "tn_linear_plan_query",
    "tn_linear_profile",
    "tn_linear_profile_read",
    "tn_linear_strerror",
    "tn_linear_version",
)


class TNLinearError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tn_linear_strerror(status)} (status {status})")


class _Desc(ctypes.Structure):
    _fields_ = [
        ("format", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("n_out_modes", ctypes.c_int32),
        ("out_modes", ctypes.POINTER(ctypes.c_int32)),
        ("n_in_modes", ctypes.c_int32),
        ("in_modes", ctypes.POINTER(ctypes.c_int32)),
        ("n_ranks", ctypes.c_int32),
        ("ranks", ctypes.POINTER(ctypes.c_int32)),
        ("n_tensors", ctypes.c_int32),
        ("tensors", ctypes.POINTER(ctypes.c_void_p)),
        ("max_tokens", ctypes.c_int64),
        ("workspace_limit_bytes", ctypes.c_int64),
        ("flags", ctypes.c_int32),
        ("stream", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_int64),
    ]


_lib = None


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2602_01613_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    lib.tn_linear_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(_Desc)]
    lib.tn_linear_create.restype = ctypes.c_int
    lib.tn_linear_forward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p]
    lib.tn_linear_forward.restype = ctypes.c_int
    lib.tn_linear_forward_scratch.argtypes = lib.tn_linear_forward.argtypes
    lib.tn_linear_forward_scratch.restype = ctypes.c_int
    lib.tn_linear_forward2.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int64, ctypes.c_void_p]
    lib.tn_linear_forward2.restype = ctypes.c_int
    lib.tn_linear_param_gradients.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64, ctypes.c_void_p]
    lib.tn_linear_param_gradients.restype = ctypes.c_int
    lib.tn_linear_quantized_tensor.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p]
    lib.tn_linear_quantized_tensor.restype = ctypes.c_int
    lib.tn_linear_destroy.argtypes = [ctypes.c_void_p]
    lib.tn_linear_destroy.restype = ctypes.c_int
    lib.tn_linear_query.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)]
    lib.tn_linear_query.restype = ctypes.c_int
    lib.tn_linear_plan_query.argtypes = [ctypes.POINTER(_Desc), ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)]
    lib.tn_linear_plan_query.restype = ctypes.c_int
    lib.tn_linear_profile.argtypes = [ctypes.c_void_p, ctypes.c_int32]
    lib.tn_linear_profile.restype = ctypes.c_int
    lib.tn_linear_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int64)]
    lib.tn_linear_profile_read.restype = ctypes.c_int
    lib.tn_linear_strerror.argtypes = [ctypes.c_int]
    lib.tn_linear_strerror.restype = ctypes.c_char_p
    lib.tn_linear_version.argtypes = []
    lib.tn_linear_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _int_array(values: Sequence[int]):
    arr = (ctypes.c_int32 * max(1, len(values)))(*[int(v) for v in values])
    return arr


def _make_desc(fmt, dtype, out_modes, in_modes, ranks, tensor_ptrs, max_tokens, workspace_limit_bytes, flags,
               stream, workspace_ptr=None, workspace_bytes=0):
    keep = []
    d = _Desc()
    d.format, d.dtype = int(fmt), int(dtype)
    om, im, rk = _int_array(out_modes), _int_array(in_modes), _int_array(ranks)
    keep += [om, im, rk]
    d.n_out_modes, d.out_modes = len(out_modes), om
    d.n_in_modes, d.in_modes = len(in_modes), im
    d.n_ranks, d.ranks = len(ranks), rk
    if tensor_ptrs is not None:
        tp = (ctypes.c_void_p * max(1, len(tensor_ptrs)))(*tensor_ptrs)
        keep.append(tp)
        d.n_tensors, d.tensors = len(tensor_ptrs), tp
    else:
        d.n_tensors, d.tensors = 0, None
    d.max_tokens = int(max_tokens)
    d.workspace_limit_bytes = int(workspace_limit_bytes)
    d.flags = int(flags)
    d.stream = stream
    d.workspace = workspace_ptr
    d.workspace_bytes = int(workspace_bytes)
    return d, keep


def tn_linear_version() -> int:
    return int(load_library().tn_linear_version())


def tn_linear_strerror(status: int) -> str:
    return load_library().tn_linear_strerror(int(status)).decode()


def tn_linear_plan_query(fmt, dtype, out_modes, in_modes, ranks, what, max_tokens=1, flags=0) -> int:
    """Host-only plan property; needs no GPU."""
    d, keep = _make_desc(fmt, dtype, out_modes, in_modes, ranks, None, max_tokens, 0, flags, None)
    val = ctypes.c_int64(0)
    rc = load_library().tn_linear_plan_query(ctypes.byref(d), int(what), ctypes.byref(val))
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_plan_query")
    return int(val.value)


plan_query = tn_linear_plan_query


def tn_linear_create(fmt, dtype, out_modes, in_modes, ranks, tensor_ptrs, max_tokens,
                     workspace_limit_bytes=0, flags=0, stream=None, workspace_ptr=None, workspace_bytes=0) -> int:
    """Returns the opaque handle (an integer address)."""
    d, keep = _make_desc(fmt, dtype, out_modes, in_modes, ranks, tensor_ptrs, max_tokens,
                         workspace_limit_bytes, flags, stream, workspace_ptr, workspace_bytes)
    h = ctypes.c_void_p(0)
    rc = load_library().tn_linear_create(ctypes.byref(h), ctypes.byref(d))
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_create")
    return int(h.value)


def tn_linear_forward(handle: int, x_ptr: int, y_ptr: int, tokens: int, stream) -> None:
    rc = load_library().tn_linear_forward(handle, x_ptr, y_ptr, int(tokens), stream)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_forward")


def tn_linear_forward_scratch(handle: int, x_ptr: int, y_ptr: int, tokens: int, stream) -> None:
    rc = load_library().tn_linear_forward_scratch(handle, x_ptr, y_ptr, int(tokens), stream)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_forward_scratch")


def tn_linear_forward2(handle_a: int, handle_b: int, x_ptr: int, ya_ptr: int, yb_ptr: int, tokens: int, stream) -> None:
    rc = load_library().tn_linear_forward2(handle_a, handle_b, x_ptr, ya_ptr, yb_ptr, int(tokens), stream)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_forward2")


def forward2(layer_a: "TNLinear", layer_b: "TNLinear", x: torch.Tensor, out_a: Optional[torch.Tensor] = None,
             out_b: Optional[torch.Tensor] = None):
    """Both layers applied to x through tn_linear_forward2; returns (ya, yb)."""
    if not (x.is_cuda and x.is_contiguous() and x.dtype == layer_a.torch_dtype and x.dim() == 2
            and x.shape[1] == layer_a.N == layer_b.N):
        raise ValueError("x must be a contiguous CUDA [tokens, N] tensor of the layers' dtype")
    tokens = x.shape[0]
    outs = []
    for layer, out in ((layer_a, out_a), (layer_b, out_b)):
        if out is None:
            out = torch.empty((tokens, layer.M), dtype=layer.torch_dtype, device=x.device)
        elif not (out.is_cuda and out.is_contiguous() and tuple(out.shape) == (tokens, layer.M)):
            raise ValueError("out has the wrong shape or layout")
        outs.append(out)
    tn_linear_forward2(layer_a._handle, layer_b._handle, x.data_ptr(), outs[0].data_ptr(), outs[1].data_ptr(), tokens,
                       torch.cuda.current_stream().cuda_stream)
    return outs[0], outs[1]


def tn_linear_param_gradients(handle: int, x_ptr: int, dy_ptr: int, grad_ptrs: Sequence[Optional[int]], tokens: int,
                              stream) -> None:
    arr = (ctypes.c_void_p * max(1, len(grad_ptrs)))(*grad_ptrs)
    rc = load_library().tn_linear_param_gradients(handle, x_ptr, dy_ptr, arr, int(tokens), stream)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_param_gradients")


def tn_linear_quantized_tensor(handle: int, slot: int, codes_ptr, exps_ptr, stream) -> None:
    rc = load_library().tn_linear_quantized_tensor(handle, int(slot), codes_ptr, exps_ptr, stream)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_quantized_tensor")


def tn_linear_destroy(handle: Optional[int]) -> None:
    rc = load_library().tn_linear_destroy(handle)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_destroy")


def tn_linear_query(handle: int, what: int) -> int:
    val = ctypes.c_int64(0)
    rc = load_library().tn_linear_query(handle, int(what), ctypes.byref(val))
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_query")
    return int(val.value)


def tn_linear_profile(handle: int, enable: bool) -> None:
    rc = load_library().tn_linear_profile(handle, 1 if enable else 0)
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_profile")


def tn_linear_profile_read(handle: int, step: int):
    """(total milliseconds, launches) recorded for one contraction step."""
    ms = ctypes.c_double(0)
    n = ctypes.c_int64(0)
    rc = load_library().tn_linear_profile_read(handle, int(step), ctypes.byref(ms), ctypes.byref(n))
    if rc != 0:
        raise TNLinearError(rc, "tn_linear_profile_read")
    return float(ms.value), int(n.value)


_TORCH_DTYPE = {TN_DTYPE_F32: torch.float32, TN_DTYPE_BF16: torch.bfloat16}


class TNLinear:
    """One tensor-network linear layer living on the current GPU."""

    def __init__(self, fmt: int, dtype: int, out_modes: Sequence[int], in_modes: Sequence[int],
                 ranks: Sequence[int], tensors: List[torch.Tensor], max_tokens: int,
                 workspace_limit_bytes: int = 0, flags: int = 0, workspace: Optional[torch.Tensor] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("TNLinear needs a GPU: there is no CPU path")
        self.dtype = int(dtype)
        self.torch_dtype = _TORCH_DTYPE[self.dtype]
        for t in tensors:
            if not (t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype):
                raise ValueError("tensors must be contiguous CUDA tensors of the layer dtype")
        stream = torch.cuda.current_stream().cuda_stream
        self._workspace = workspace          # keep the caller's block alive as long as the handle
        ws_ptr, ws_bytes = None, 0
        if workspace is not None:
            if not (workspace.is_cuda and workspace.is_contiguous()):
                raise ValueError("workspace must be a contiguous CUDA tensor")
            ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        self._tensor_shapes = [tuple(t.shape) for t in tensors]
        self._handle = tn_linear_create(fmt, dtype, out_modes, in_modes, ranks,
                                        [t.data_ptr() for t in tensors], max_tokens,
                                        workspace_limit_bytes, flags, stream, ws_ptr, ws_bytes)
        self.M = tn_linear_query(self._handle, TN_QUERY_OUT_FEATURES)
        self.N = tn_linear_query(self._handle, TN_QUERY_IN_FEATURES)

    def forward(self, x: torch.Tensor, out: Optional[torch.Tensor] = None, scratch: bool = False) -> torch.Tensor:
        """scratch=True calls tn_linear_forward_scratch (intermediates in the library's static array); out is
        then required, since that entry point is for callers that do not allocate."""
        if self._handle is None:
            raise RuntimeError("layer was closed")
        if not (x.is_cuda and x.is_contiguous() and x.dtype == self.torch_dtype and x.dim() == 2
                and x.shape[1] == self.N):
            raise ValueError(f"x must be a contiguous CUDA [tokens, {self.N}] tensor of the layer dtype")
        tokens = x.shape[0]
        if out is None:
            out = torch.empty((tokens, self.M), dtype=self.torch_dtype, device=x.device)
        elif not (out.is_cuda and out.is_contiguous() and out.dtype == self.torch_dtype
                  and tuple(out.shape) == (tokens, self.M)):
            raise ValueError("out has the wrong shape, dtype or layout")
        call = tn_linear_forward_scratch if scratch else tn_linear_forward
        call(self._handle, x.data_ptr(), out.data_ptr(), tokens, torch.cuda.current_stream().cuda_stream)
        return out

    __call__ = forward

    def param_gradients(self, x: torch.Tensor, dy: torch.Tensor, out: Optional[List[torch.Tensor]] = None):
        """fp32 gradients of sum(dy * forward(x)) with respect to every parameter tensor (the layer must have been
        created with TN_FLAG_TRAINABLE); returns one tensor per parameter tensor, in the caller's shapes."""
        if self._handle is None:
            raise RuntimeError("layer was closed")
        tokens = x.shape[0]
        if not (x.is_cuda and x.is_contiguous() and x.dtype == self.torch_dtype and tuple(x.shape) == (tokens, self.N)
                and dy.is_cuda and dy.is_contiguous() and dy.dtype == self.torch_dtype
                and tuple(dy.shape) == (tokens, self.M)):
            raise ValueError("x [tokens, N] and dy [tokens, M] must be contiguous CUDA tensors of the layer dtype")
        if out is None:
            out = [torch.empty(shp, dtype=torch.float32, device=x.device) for shp in self._tensor_shapes]
        tn_linear_param_gradients(self._handle, x.data_ptr(), dy.data_ptr(), [g.data_ptr() for g in out], tokens,
                                  torch.cuda.current_stream().cuda_stream)
        return out

    def quantized_tensor(self, slot: int):
        """(codes uint8 [ceil(n/2)], exponents int8 [ceil(n/32)]) of tensor `slot` of a TN_FLAG_QUANT_MXFP4 layer."""
        n = 1
        for e in self._tensor_shapes[slot]:
            n *= e
        codes = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
        exps = torch.empty((n + 31) // 32, dtype=torch.int8, device="cuda")
        tn_linear_quantized_tensor(self._handle, slot, codes.data_ptr(), exps.data_ptr(),
                                   torch.cuda.current_stream().cuda_stream)
        return codes, exps

    def query(self, what: int) -> int:
        return tn_linear_query(self._handle, what)

    def profile(self, enable: bool) -> None:
        tn_linear_profile(self._handle, enable)

    def profile_read(self, step: int):
        return tn_linear_profile_read(self._handle, step)

    def close(self) -> None:
        if self._handle is not None:
            tn_linear_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
