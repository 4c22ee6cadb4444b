"""tn_linear_forward_scratch (the entry point that allocates nothing: intermediates and partial sums in the
library's static device array) against tn_linear_forward, through the C ABI, on two calls in a row, the second
with a smaller input; and the refusal of calls beyond the array's size."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as wl
import paper_2602_01613_amd as tn
from gpu_util import TOL, make_layer, to_dev, to_host

pytestmark = pytest.mark.gpu


def _spec(fmt, om, im, rk):
    return wl.TNSpec(fmt, "bf16", tuple(om), tuple(im), tuple(rk))


CASES = [
    # (spec, flags, token counts of the two calls): several steps with intermediates in memory and split-K sums
    (wl.baseline_spec(2)[0], 0, (48, 5)),                                                      # Tucker: 5 steps, 2 chained pairs
    (wl.baseline_spec(1)[0], 0, (20, 3)),                                                      # merged train: two launches
    (wl.baseline_spec(1)[0], tn.TN_FLAG_NO_MERGE, (12, 1)),                                    # four-core chain
    (_spec(tn.TN_FORMAT_TUCKER, (160, 96, 16), (64,), (48, 32, 1, 16)), 0, (64, 7)),           # chained pair mid-chain
    (wl.stack_spec(wl.FORMAT_DENSE, 5120, 8192, 0), 0, (64, 2)),                               # split-K with partial sums only
    (wl.baseline_spec(3)[0], tn.TN_FLAG_MERGE_GROW, (9, 2)),                                   # Kronecker-sum kernel, bond split
    (_spec(tn.TN_FORMAT_TT, (8, 4, 8, 8), (8, 2, 8, 8), (1, 64, 64, 64, 1)), 0, (300, 256)),   # chained pair kernel: partial sums only
    (wl.baseline_spec(1)[0], tn.TN_FLAG_NO_PAIR_CHAIN, (20, 3)),                               # the same train as two launches
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_forward_scratch_matches_forward(case):
    spec, flags, token_counts = CASES[case]
    ts = wl.make_tensors(spec, 70 + case)
    layer = make_layer(spec, ts, max(token_counts), flags=flags)
    w = O.dense_weight(spec.format, ts, len(spec.out_modes))
    poison = torch.full((max(token_counts), spec.M), float("nan"), dtype=torch.bfloat16, device="cuda")
    for tokens in token_counts:
        x = wl.make_x(spec, tokens, 70 + case)
        xd = to_dev(x, "bf16")
        y_ref = layer.forward(xd)
        y = poison[:tokens].clone()
        layer.forward(xd, out=y, scratch=True)
        torch.cuda.synchronize()
        if spec.format == wl.FORMAT_TR:
            # the bond may be split differently (the static array bounds the partial sums): summation order only
            assert O.rel_max_err(to_host(y), to_host(y_ref)) <= 1e-2, (case, tokens)
        else:
            assert torch.equal(y, y_ref), (case, tokens)                  # same kernels, same order: same bits
        assert O.rel_max_err(to_host(y), O.apply_linear(w, x)) <= TOL["bf16"], (case, tokens)
    layer.close()


def test_forward_scratch_refuses_what_does_not_fit():
    spec = wl.baseline_spec(1)[0]
    ts = wl.make_tensors(spec, 1)
    layer = make_layer(spec, ts, 64, flags=tn.TN_FLAG_NO_PAIR_CHAIN)     # two launches with the intermediate in memory
    x = to_dev(wl.make_x(spec, 64, 1), "bf16")
    y = torch.empty((64, spec.M), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(tn.TNLinearError) as e:                            # 64 tokens x 2 x 655 KB > 32 MiB
        layer.forward(x, out=y, scratch=True)
    assert e.value.status == -5
    layer.forward(x[:8].contiguous(), out=y[:8], scratch=True)            # and the handle still works
    torch.cuda.synchronize()
    assert torch.equal(y[:8], layer.forward(x[:8].contiguous()))
    layer.profile(True)
    with pytest.raises(tn.TNLinearError) as e:
        layer.forward(x[:8].contiguous(), out=y[:8], scratch=True)
    assert e.value.status == -1
    layer.close()
