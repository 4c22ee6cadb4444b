"""Randomly drawn layers (seeded): formats, mode factorisations, ranks, flags and token counts nobody picked by hand,
every one against the fp64 oracle. The extents are drawn from the values that switch kernels (multiples and
non-multiples of 8, 32 and 64), the token counts around the decode-size kernel switches."""
import numpy as np
import pytest

import oracle as O
import workloads as wl
import paper_2602_01613_amd as tn
from gpu_util import TOL, make_layer, to_dev, to_host

pytestmark = pytest.mark.gpu

MODES = [2, 3, 4, 5, 6, 8, 10, 12, 16, 20, 24, 32, 40, 64]
RANKS = [1, 2, 3, 4, 8, 12, 16, 24, 32, 48, 64]
FLAGS = [0, 0, tn.TN_FLAG_NO_MERGE, tn.TN_FLAG_QUANT_MXFP4, tn.TN_FLAG_QUANT_MXFP4 | tn.TN_FLAG_NO_MERGE, tn.TN_FLAG_MERGE_HALVES,
         tn.TN_FLAG_NO_DECODE_FUSION, tn.TN_FLAG_NO_SKINNY]


def _draw(rng):
    """A layer of at most 6144 x 6144 (the oracle rebuilds the dense matrix) with at most 3 modes a side."""
    fmt = [tn.TN_FORMAT_TT, tn.TN_FORMAT_TR, tn.TN_FORMAT_TUCKER, tn.TN_FORMAT_DENSE][int(rng.integers(0, 4))]
    while True:
        if fmt == tn.TN_FORMAT_DENSE:
            om, im, rk = (int(rng.integers(1, 3000)),), (int(rng.integers(1, 6000)),), ()
        elif fmt in (tn.TN_FORMAT_TT, tn.TN_FORMAT_TR):
            d = int(rng.integers(1, 4))
            om = tuple(int(rng.choice(MODES)) for _ in range(d))
            im = tuple(int(rng.choice(MODES)) for _ in range(d))
            inner = [int(rng.choice(RANKS)) for _ in range(d - 1)]
            r0 = int(rng.choice(RANKS[1:])) if fmt == tn.TN_FORMAT_TR else 1
            rk = tuple([r0] + inner + [r0])
        else:
            p, q = int(rng.integers(1, 4)), int(rng.integers(1, 3))
            om = tuple(int(rng.choice(MODES)) for _ in range(p))
            im = tuple(int(rng.choice(MODES)) for _ in range(q))
            rk = tuple(min(int(rng.choice(RANKS)), m) for m in om + im)
        spec = wl.TNSpec(fmt, "bf16", om, im, rk)
        if spec.M <= 6144 and spec.N <= 6144 and spec.M * spec.N <= 16_000_000 and spec.n_params <= 8_000_000:
            return spec


@pytest.mark.parametrize("seed", range(160))
def test_random_layer_against_the_oracle(seed):
    rng = np.random.default_rng(77000 + seed)
    spec = _draw(rng)
    flags = int(FLAGS[int(rng.integers(0, len(FLAGS)))])
    ts = [wl.round_to_dtype(rng.standard_normal(shp) / np.sqrt(max(1.0, 0.5 * (shp[0] + shp[-1]))), "bf16")
          for shp in spec.tensor_shapes()]
    print(f"seed {seed}: format {spec.format} out {spec.out_modes} in {spec.in_modes} ranks {spec.ranks} flags {flags}", flush=True)
    used = O.mxfp4_dequantized(ts) if flags & tn.TN_FLAG_QUANT_MXFP4 else ts
    w = O.dense_weight(spec.format, used, len(spec.out_modes))
    scale = np.abs(w).max()
    if scale == 0.0:
        pytest.skip("the drawn layer is the zero matrix")
    layer = make_layer(spec, ts, 130, flags=flags)
    # one batch of 130 tokens; smaller calls take its first rows, and every call is measured against the largest
    # reference value of the whole batch (a one-token output of two values can be small by cancellation, which would
    # turn the rounding of the bf16 intermediates into a large relative figure)
    x = wl.round_to_dtype(rng.standard_normal((130, spec.N)), "bf16")
    ref = O.apply_linear(w, x)
    top = np.abs(ref).max()
    for tokens in (1, 2, 4, 5, 8, 31, 33, 64, 65, 130):
        y = to_host(layer(to_dev(x[:tokens], "bf16")))
        err = np.abs(y - ref[:tokens]).max() / top
        assert err <= TOL["bf16"], (seed, tokens, err)
    layer.close()


@pytest.mark.parametrize("seed", range(40))
def test_random_layer_large_calls(seed):
    """The same draw at token counts that run the tiled, chained and Kronecker-sum kernels over several tiles with
    ragged ends."""
    rng = np.random.default_rng(88000 + seed)
    spec = _draw(rng)
    flags = int(FLAGS[int(rng.integers(0, len(FLAGS)))])
    ts = [wl.round_to_dtype(rng.standard_normal(shp) / np.sqrt(max(1.0, 0.5 * (shp[0] + shp[-1]))), "bf16")
          for shp in spec.tensor_shapes()]
    print(f"seed {seed}: format {spec.format} out {spec.out_modes} in {spec.in_modes} ranks {spec.ranks} flags {flags}", flush=True)
    used = O.mxfp4_dequantized(ts) if flags & tn.TN_FLAG_QUANT_MXFP4 else ts
    w = O.dense_weight(spec.format, used, len(spec.out_modes))
    if np.abs(w).max() == 0.0:
        pytest.skip("the drawn layer is the zero matrix")
    layer = make_layer(spec, ts, 1100, flags=flags)
    x = wl.round_to_dtype(rng.standard_normal((1100, spec.N)), "bf16")
    ref = O.apply_linear(w, x)
    top = np.abs(ref).max()
    for tokens in (257, 1100):
        y = to_host(layer(to_dev(x[:tokens], "bf16")))
        err = np.abs(y - ref[:tokens]).max() / top
        assert err <= TOL["bf16"], (seed, tokens, err)
    layer.close()
