"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch

import paper_2602_01613_amd as tn

TOL = {"bf16": 2e-2, "f32": 1e-5}     # max|y - y_ref| / max|y_ref|


def dtype_code(name):
    return tn.TN_DTYPE_BF16 if name == "bf16" else tn.TN_DTYPE_F32


def to_dev(a64, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a64)).to(torch.float32)
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda().contiguous()


def to_host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def make_layer(spec, tensors64, max_tokens, workspace_limit_bytes=0, flags=0):
    dev = [to_dev(t, spec.dtype) for t in tensors64]
    layer = tn.TNLinear(spec.format, dtype_code(spec.dtype), spec.out_modes, spec.in_modes, spec.ranks,
                        dev, max_tokens, workspace_limit_bytes, flags)
    torch.cuda.synchronize()
    return layer


def run_layer(spec, tensors64, x64, workspace_limit_bytes=0, flags=0, max_tokens=None):
    layer = make_layer(spec, tensors64, max_tokens or max(1, x64.shape[0]), workspace_limit_bytes, flags)
    y = layer(to_dev(x64, spec.dtype))
    torch.cuda.synchronize()
    out = to_host(y)
    layer.close()
    return out
