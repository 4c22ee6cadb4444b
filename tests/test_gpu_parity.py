"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle
on the same seeded inputs. Tolerance: max|y - y_ref| / max|y_ref| <= 2e-2 (bf16)
or 1e-5 (fp32) over the whole output."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as wl
import paper_2602_01613_amd as tn
from gpu_util import TOL, make_layer, run_layer, to_dev, to_host

pytestmark = pytest.mark.gpu


def _spec(fmt, dtype, om, im, rk):
    return wl.TNSpec(fmt, dtype, tuple(om), tuple(im), tuple(rk))


def _rand_layer(spec, seed):
    rng = np.random.default_rng(seed)
    ts = []
    for shp in spec.tensor_shapes():
        ts.append(wl.round_to_dtype(rng.standard_normal(shp) / np.sqrt(max(1, shp[-1])), spec.dtype))
    return ts


SMALL = [
    (tn.TN_FORMAT_TT, (2, 3, 2, 2), (2, 2, 3, 2), (1, 4, 2, 4, 1)),      # end cores merge at create time
    (tn.TN_FORMAT_TT, (8, 16, 8), (8, 10, 8), (1, 64, 64, 1)),           # both merges, MFMA-sized
    (tn.TN_FORMAT_TT, (4, 8, 8), (4, 8, 8), (1, 8, 8, 1)),
    (tn.TN_FORMAT_TT, (3, 4, 2), (2, 5, 3), (1, 3, 4, 1)),               # odd extents, K not multiple of 8
    (tn.TN_FORMAT_TT, (2, 3, 2, 2), (5, 2, 3, 2), (1, 2, 5, 3, 1)),      # first step gathers from x
    (tn.TN_FORMAT_TT, (8, 16, 8), (8, 10, 8), (1, 32, 16, 1)),
    (tn.TN_FORMAT_TT, (1, 3, 1), (2, 1, 3), (1, 1, 2, 1)),
    (tn.TN_FORMAT_TR, (2, 3, 2), (3, 2, 2), (3, 2, 4, 3)),
    (tn.TN_FORMAT_TR, (4, 6, 4), (6, 4, 8), (8, 16, 8, 8)),
    (tn.TN_FORMAT_TR, (5,), (7,), (3, 3)),
    (tn.TN_FORMAT_TUCKER, (4, 5), (3, 6), (2, 3, 2, 4)),
    (tn.TN_FORMAT_TUCKER, (16, 24), (8, 40), (8, 16, 8, 16)),
    (tn.TN_FORMAT_TUCKER, (3, 2, 4), (5,), (2, 2, 3, 4)),
    (tn.TN_FORMAT_DENSE, (200,), (136,), ()),
    (tn.TN_FORMAT_DENSE, (9,), (11,), ()),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("flags", [0, tn.TN_FLAG_SCALAR_KERNELS])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_shapes(case, flags, dtype):
    fmt, om, im, rk = SMALL[case]
    spec = _spec(fmt, dtype, om, im, rk)
    ts = _rand_layer(spec, 100 + case)
    for tokens in (1, 17, 130):
        x = wl.round_to_dtype(np.random.default_rng(case * 7 + tokens).standard_normal((tokens, spec.N)), dtype)
        y = run_layer(spec, ts, x, flags=flags)
        ref = O.forward(fmt, ts, x, n_out_modes=len(om))
        err = O.rel_max_err(y, ref)
        assert err <= TOL[dtype], (case, tokens, err)


def test_config0_fp32():
    spec, toks = wl.baseline_spec(0)
    ts = wl.make_tensors(spec, 0)
    x = wl.make_x(spec, toks[0], 0)
    y = run_layer(spec, ts, x)
    assert O.rel_max_err(y, O.forward(spec.format, ts, x)) <= 1e-5


@pytest.fixture(scope="module")
def dense_w():
    cache = {}

    def get(i):
        if i not in cache:
            spec, toks = wl.baseline_spec(i)
            ts = wl.make_tensors(spec, i)
            print(f"[oracle] rebuilding dense W for workload {i}", flush=True)
            cache[i] = (spec, ts, O.dense_weight(spec.format, ts, len(spec.out_modes)))
        return cache[i]

    return get


# workload 1 is run both ways: with its end cores merged at create time (the default) and as
# the four-core chain exactly as given
CONFIG_RUNS = [(1, 0), (1, tn.TN_FLAG_NO_MERGE), (2, 0), (3, 0), (3, tn.TN_FLAG_MERGE_GROW)]


def full_rel_err(yd, w, x, block=1024):
    """max|y - y_ref| / max|y_ref| over EVERY row of a device result, the oracle product taken block by block."""
    num, den = 0.0, 0.0
    for r0 in range(0, x.shape[0], block):
        ref = O.apply_linear(w, x[r0:r0 + block])
        y = to_host(yd[r0:r0 + block])
        num = max(num, float(np.max(np.abs(y - ref))))
        den = max(den, float(np.max(np.abs(ref))))
    return num / den


@pytest.mark.parametrize("i,flags", CONFIG_RUNS)
def test_baseline_configs_decode_sizes(i, flags, dense_w):
    spec, ts, w = dense_w(i)
    layer = make_layer(spec, ts, 64, flags=flags)
    assert layer.query(tn.TN_QUERY_NUM_STEPS) == {(1, 0): 2, (1, 2): 4, (2, 0): 5, (3, 0): 4, (3, 16): 2}[(i, flags)]
    for tokens in (1, 64):
        x = wl.make_x(spec, tokens, i)
        y = to_host(layer(to_dev(x, spec.dtype)))
        err = O.rel_max_err(y, O.apply_linear(w, x))
        print(f"workload {i} T={tokens} rel err {err:.3e}", flush=True)
        assert err <= TOL[spec.dtype]
    layer.close()


@pytest.mark.parametrize("i,flags", CONFIG_RUNS)
def test_baseline_configs_prefill_8192(i, flags, dense_w):
    """Full size, in the launch configuration the benchmark times: every one of the 8192 x M outputs is
    compared with the oracle's fp64 product."""
    spec, ts, w = dense_w(i)
    tokens = 8192
    print(f"[gen] x for workload {i}", flush=True)
    x = wl.make_x(spec, tokens, i)
    layer = make_layer(spec, ts, tokens, flags=flags)
    xd = to_dev(x, spec.dtype)
    yd = layer(xd)
    torch.cuda.synchronize()
    print(f"[oracle] workload {i}: fp64 product of all {tokens} rows", flush=True)
    err = full_rel_err(yd, w, x)
    print(f"workload {i} T=8192 rel err over all rows {err:.3e}", flush=True)
    assert err <= TOL[spec.dtype]
    # determinism: a second call gives the same bits
    yd2 = layer(xd)
    torch.cuda.synchronize()
    assert torch.equal(yd, yd2)
    # token independence on the GPU path: rows computed alone agree with the batch up to the summation order
    # (a 3-token call runs other kernels than the 8192-token one)
    sub = layer(xd[:3].contiguous())
    torch.cuda.synchronize()
    assert O.rel_max_err(to_host(sub), to_host(yd[:3])) <= 1e-2
    layer.close()


@pytest.mark.parametrize("tokens", [0, 1, 2, 15, 16, 17, 63, 64, 65, 255, 257])
def test_token_count_boundaries(tokens, dense_w):
    spec, ts, w = dense_w(1)
    x = wl.make_x(spec, max(tokens, 1), 1)[:tokens]
    y = run_layer(spec, ts, x, max_tokens=300)
    assert y.shape == (tokens, spec.M)
    if tokens:
        assert O.rel_max_err(y, O.apply_linear(w, x)) <= TOL["bf16"]


def test_chunked_passes_match_single_pass(dense_w):
    spec, ts, w = dense_w(1)
    x = wl.make_x(spec, 75, 1)
    # the per-step path (the chained pair kernel keeps no intermediates): 16 MiB of workspace, two buffers of the
    # largest intermediate (bf16) per token
    two = tn.TN_FLAG_NO_PAIR_CHAIN
    layer = make_layer(spec, ts, 75, workspace_limit_bytes=16 << 20, flags=two)
    per_token = 2 * 2 * layer.query(tn.TN_QUERY_MAX_INTERMEDIATE)
    assert layer.query(tn.TN_QUERY_CHUNK_TOKENS) == (16 << 20) // per_token < 75
    y_small = layer(to_dev(x, "bf16"))
    torch.cuda.synchronize()
    layer.close()
    layer = make_layer(spec, ts, 75, flags=two)
    assert layer.query(tn.TN_QUERY_CHUNK_TOKENS) == 75
    y_big = layer(to_dev(x, "bf16"))
    torch.cuda.synchronize()
    layer.close()
    # pass size changes which kernel (tiled or split-K) and which split a launch gets, hence the
    # summation order: the two agree to rounding, not bit for bit
    ref = O.apply_linear(w, x)
    assert O.rel_max_err(to_host(y_small), ref) <= TOL["bf16"]
    assert O.rel_max_err(to_host(y_big), ref) <= TOL["bf16"]
    assert O.rel_max_err(to_host(y_small), to_host(y_big)) <= 1e-2
    # more tokens than max_tokens: processed in several passes
    layer = make_layer(spec, ts, 10, flags=two)
    y_cap = layer(to_dev(x, "bf16"))
    torch.cuda.synchronize()
    layer.close()
    assert O.rel_max_err(to_host(y_cap), ref) <= TOL["bf16"]


def test_linearity_on_gpu(dense_w):
    spec, ts, w = dense_w(1)
    layer = make_layer(spec, ts, 8)
    rng = np.random.default_rng(5)
    x1 = wl.round_to_dtype(rng.standard_normal((8, spec.N)), "bf16")
    x2 = wl.round_to_dtype(rng.standard_normal((8, spec.N)), "bf16")
    xs = wl.round_to_dtype(2.0 * x1 - 0.5 * x2, "bf16")
    y1, y2, ysum = (to_host(layer(to_dev(v, "bf16"))) for v in (x1, x2, xs))
    ref = O.apply_linear(w, xs)
    assert O.rel_max_err(ysum, ref) <= TOL["bf16"]
    # 2 y1 - 0.5 y2 differs from f(xs) only by the rounding of xs and of the outputs
    assert O.rel_max_err(2.0 * y1 - 0.5 * y2, ref) <= 3 * TOL["bf16"]
    layer.close()


def test_errors_through_the_abi():
    with pytest.raises(tn.TNLinearError):
        tn.tn_linear_create(tn.TN_FORMAT_TT, 1, (4, 4), (4, 4), (1, 2, 1), [0, 0], 4)      # NULL tensors
    t = torch.zeros(16, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(tn.TNLinearError):
        tn.tn_linear_create(tn.TN_FORMAT_TT, 1, (4, 4), (4, 4), (1, 2, 1), [t.data_ptr()], 4)  # too few tensors
    with pytest.raises(tn.TNLinearError):
        tn.tn_linear_forward(None, t.data_ptr(), t.data_ptr(), 1, None)
    tn.tn_linear_destroy(None)
    # activations that are not 16-byte aligned are refused before anything is launched
    spec = _spec(tn.TN_FORMAT_TT, "bf16", (4, 4), (4, 4), (1, 2, 1))
    layer = make_layer(spec, _rand_layer(spec, 5), 2)
    buf = torch.zeros(2 * 16 + 8, device="cuda", dtype=torch.bfloat16)
    y = torch.zeros(2 * 16, device="cuda", dtype=torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream
    y.fill_(7.0)
    tn.tn_linear_forward(layer._handle, buf.data_ptr(), y.data_ptr(), 0, stream)          # no tokens: nothing is launched
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    tn.tn_linear_forward(layer._handle, buf.data_ptr(), y.data_ptr(), 2, stream)
    for xp, yp in ((buf.data_ptr() + 2, y.data_ptr()), (buf.data_ptr(), y.data_ptr() + 6)):
        with pytest.raises(tn.TNLinearError):
            tn.tn_linear_forward(layer._handle, xp, yp, 2, stream)
    torch.cuda.synchronize()
    layer.close()


def _stack_classes():
    """Every distinct (format, modes, ranks) the 448-matrix stack draws, in a fixed order."""
    seen = {}
    for s in wl.qwen3_32b_stack(64):
        seen.setdefault((s.format, s.out_modes, s.in_modes, s.ranks), s)
    return [seen[k] for k in sorted(seen)]


STACK_CLASSES = _stack_classes()
N_SAMPLED_W_ROWS = 24


def _class_reference(spec, ts, instance):
    """Rows of W the comparison uses and those rows of the oracle's W: all of them, except for rings, whose
    full rebuild costs 2 M N r^2 (minutes at rank 96); there a seeded sample of output features is rebuilt."""
    if spec.format != wl.FORMAT_TR:
        return None, O.dense_weight(spec.format, ts, len(spec.out_modes))
    rng = np.random.default_rng(1000 + instance)
    rows = np.unique(np.concatenate([rng.choice(spec.M, size=N_SAMPLED_W_ROWS - 2, replace=False), [0, spec.M - 1]]))
    return rows, O.tr_dense_rows(ts, rows)


@pytest.mark.parametrize("n", range(len(STACK_CLASSES)))
def test_every_stack_class(n):
    """One matrix of EVERY (format, shape, rank) class the 64-layer stack draws, at 3 tokens (decode-size
    kernels) and at 64 tokens (rings: the rebuilt half-ring plan with the bond split over workgroups), against the
    oracle: the whole output, or for rings a seeded sample of output features over all tokens."""
    spec = STACK_CLASSES[n]
    ts = wl.make_tensors(spec, 4, instance=100 + n)
    print(f"[stack class {n}] {wl.FORMAT_NAMES[spec.format]} {spec.N}->{spec.M} ranks {spec.ranks}: oracle", flush=True)
    rows, w = _class_reference(spec, ts, n)
    layer = make_layer(spec, ts, 64)
    for tokens in (3, 64):
        x = wl.make_x(spec, tokens, 4, instance=100 + n)
        y = to_host(layer(to_dev(x, spec.dtype)))
        if rows is not None:
            y = y[:, rows]
        err = O.rel_max_err(y, O.apply_linear(w, x))
        print(f"[stack class {n}] T={tokens} rel err {err:.3e}", flush=True)
        assert err <= TOL["bf16"], (n, tokens, err)
    layer.close()


@pytest.mark.parametrize("n_in,n_out,r", [(25600, 5120, 96), (5120, 25600, 64), (8192, 5120, 96), (5120, 8192, 64)])
def test_stack_rings_prefill_8192(n_in, n_out, r):
    """The rings that carry the stack's prefill time (ranks 64 and 96 on the wide projections: bonds of 4096 and
    9216 values through the Kronecker-sum kernel on slices rebuilt per call) at 8192 tokens as the stack
    benchmark launches them: a seeded sample of output features over all 8192 tokens."""
    tokens = 8192
    spec = wl.stack_spec(wl.FORMAT_TR, n_in, n_out, r)
    ts = wl.make_tensors(spec, 4, instance=9)
    print(f"[ring 8192] {n_in}->{n_out} r={r}: oracle rows", flush=True)
    rows, w = _class_reference(spec, ts, n_in + r)
    print(f"[ring 8192] x", flush=True)
    x = wl.make_x(spec, tokens, 4, instance=9)
    layer = make_layer(spec, ts, tokens)
    assert layer.query(tn.TN_QUERY_LAZY_MIN_TOKENS) == 1
    yd = layer(to_dev(x, spec.dtype))
    torch.cuda.synchronize()
    y = to_host(yd[:, torch.from_numpy(rows).cuda()])
    layer.close()
    err = O.rel_max_err(y, O.apply_linear(w, x))
    print(f"[ring 8192] rel err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("fmt,n_in,n_out,r", [
    (wl.FORMAT_DENSE, 5120, 1024, 0), (wl.FORMAT_DENSE, 25600, 5120, 0), (wl.FORMAT_DENSE, 5120, 25600, 0),
    (wl.FORMAT_TUCKER, 25600, 5120, 80), (wl.FORMAT_TT, 5120, 25600, 96), (wl.FORMAT_TR, 5120, 1024, 32),
])
def test_stack_shapes_prefill_8192(fmt, n_in, n_out, r):
    """Matrices of the 64-layer stack at 8192 tokens, in the launch configuration the stack benchmark times
    (dense: 128 tiles run as half-width tiles, 640 tiles = two rounds and a half, 3200 tiles; a Tucker layer,
    a merged train and a ring on its rebuilt half-ring plan): a seeded sample of token rows in full."""
    tokens = 8192
    spec = wl.stack_spec(fmt, n_in, n_out, r)
    ts = wl.make_tensors(spec, 4, instance=7)
    print(f"[stack 8192] {wl.FORMAT_NAMES[fmt]} {n_in}->{n_out} r={r}: x", flush=True)
    x = wl.make_x(spec, tokens, 4, instance=7)
    layer = make_layer(spec, ts, tokens)
    yd = layer(to_dev(x, spec.dtype))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.random.default_rng(n_in + n_out).choice(tokens, size=12, replace=False),
                                     [0, 255, 256, tokens - 1]]))
    y = to_host(yd[torch.from_numpy(rows).cuda()])
    layer.close()
    ref = O.forward(fmt, ts, x[rows], n_out_modes=len(spec.out_modes))
    err = O.rel_max_err(y, ref)
    print(f"[stack 8192] rel err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("n_out,n_in", [(9216, 64), (8448, 96), (1024, 160), (4352, 64)])
def test_partly_filled_last_round(n_out, n_in):
    """The 256x256 kernel at 2048 rows (8 row tiles, one per XCD): 36 and 33 column tiles leave a last
    round of 4 and 1 tiles per XCD, which runs as half-width tiles in a second launch; 4 column tiles run
    as half-width tiles altogether; 17 stay as they are. Whole output against the oracle."""
    spec = _spec(tn.TN_FORMAT_DENSE, "bf16", (n_out,), (n_in,), ())
    ts = _rand_layer(spec, 900 + n_out)
    x = wl.round_to_dtype(np.random.default_rng(n_out).standard_normal((2048, spec.N)), "bf16")
    y = run_layer(spec, ts, x, flags=(12 << 8) | tn.TN_FLAG_NO_SPLIT_K)
    err = O.rel_max_err(y, O.forward(spec.format, ts, x, n_out_modes=1))
    print(f"dense {n_in}->{n_out} rel err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]


@pytest.mark.parametrize("variant", [3, 8, 9, 12])
def test_wide_step_kernel_variants(variant):
    """Every tile variant of the wide bf16 steps (tuning override) on shapes with ragged row
    and column tiles, a K that is not a multiple of the K tile, and a gathered first step."""
    cases = [
        _spec(tn.TN_FORMAT_TT, "bf16", (8, 16, 8), (8, 10, 8), (1, 32, 24, 1)),
        _spec(tn.TN_FORMAT_TT, "bf16", (2, 3, 2, 2), (5, 2, 3, 2), (1, 2, 5, 3, 1)),
        _spec(tn.TN_FORMAT_TR, "bf16", (4, 6, 4), (6, 4, 8), (8, 16, 8, 8)),
        _spec(tn.TN_FORMAT_DENSE, "bf16", (200,), (136,), ()),
        _spec(tn.TN_FORMAT_TUCKER, "bf16", (16, 24), (8, 40), (8, 16, 8, 16)),
        _spec(tn.TN_FORMAT_TT, "bf16", (8, 16, 8), (8, 12, 8), (1, 32, 16, 1)),     # K = 96, 128, 384: 32-wide tiles
        _spec(tn.TN_FORMAT_DENSE, "bf16", (328,), (1056,), ()),
    ]
    for n, spec in enumerate(cases):
        ts = _rand_layer(spec, 300 + n)
        for tokens in (3, 67, 300):
            x = wl.round_to_dtype(np.random.default_rng(n + tokens).standard_normal((tokens, spec.N)), "bf16")
            # the tiled kernels themselves: no split-K, no create-time merging
            flags = (variant << 8) | tn.TN_FLAG_NO_SPLIT_K | tn.TN_FLAG_NO_MERGE
            y = run_layer(spec, ts, x, flags=flags)
            err = O.rel_max_err(y, O.forward(spec.format, ts, x, n_out_modes=len(spec.out_modes)))
            assert err <= TOL["bf16"], (variant, n, tokens, err)


@pytest.mark.parametrize("tokens", [1, 3, 33, 64, 100])
def test_split_k_small_launches(tokens):
    """Launches too small to fill the chip run on the split-K kernel (decode regime): long-K
    dense, Tucker and merged-TT shapes, odd extents, gathered first step; checked against the
    oracle and against the tiled kernels."""
    cases = [
        _spec(tn.TN_FORMAT_DENSE, "bf16", (200,), (1000,), ()),
        _spec(tn.TN_FORMAT_DENSE, "bf16", (1024,), (2048,), ()),
        _spec(tn.TN_FORMAT_TUCKER, "bf16", (40, 48), (32, 40), (24, 32, 16, 24)),
        _spec(tn.TN_FORMAT_TT, "bf16", (8, 16, 8), (8, 10, 8), (1, 64, 64, 1)),
        _spec(tn.TN_FORMAT_TT, "bf16", (4, 6, 5), (6, 20, 4), (1, 8, 16, 1)),
        _spec(tn.TN_FORMAT_TR, "bf16", (4, 6, 4), (6, 4, 8), (8, 16, 8, 8)),
    ]
    for n, spec in enumerate(cases):
        ts = _rand_layer(spec, 500 + n)
        x = wl.round_to_dtype(np.random.default_rng(n + tokens).standard_normal((tokens, spec.N)), "bf16")
        ref = O.forward(spec.format, ts, x, n_out_modes=len(spec.out_modes))
        y = run_layer(spec, ts, x)
        y_tiled = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_SPLIT_K)
        assert O.rel_max_err(y, ref) <= TOL["bf16"], (n, tokens)
        assert O.rel_max_err(y_tiled, ref) <= TOL["bf16"], (n, tokens)
        # a second run of the split path gives the same bits (fixed-order reduction, no atomics)
        assert np.array_equal(y, run_layer(spec, ts, x))


@pytest.mark.parametrize("case", range(6))
def test_decode_size_kernel_family(case):
    """Launches of one row tile (1 to 64 rows) choose between the split-K kernel of one column block with A gathered
    from memory, the same with the rows of A in LDS (up to 4 rows), and the kernel that gives a workgroup 256
    columns (5 to 64 rows, chosen by rows x K): every row count around the switches, on shapes with ragged column
    tiles, a K with a half piece of 64 at the end, few and many splits; against the oracle and against the layer with
    the 256-column kernel switched off."""
    cases = [
        _spec(tn.TN_FORMAT_DENSE, "bf16", (1000,), (5120,), ()),           # 32 column blocks (the last ragged), 80 pieces
        _spec(tn.TN_FORMAT_DENSE, "bf16", (300,), (2464,), ()),            # 10 column blocks, K = 38.5 pieces
        _spec(tn.TN_FORMAT_DENSE, "bf16", (256,), (25600,), ()),           # one column tile, long K: many splits
        _spec(tn.TN_FORMAT_DENSE, "bf16", (4096,), (544,), ()),            # short K: one or two splits
        _spec(tn.TN_FORMAT_TUCKER, "bf16", (40, 48), (32, 40), (24, 32, 16, 24)),      # core 768 x 384 inside a chain
        _spec(tn.TN_FORMAT_TUCKER, "bf16", (160, 160), (64, 80), (48, 48, 24, 24)),
    ]
    spec = cases[case]
    ts = _rand_layer(spec, 900 + case)
    layer = make_layer(spec, ts, 64)
    plain = make_layer(spec, ts, 64, flags=tn.TN_FLAG_NO_SKINNY)
    w = O.dense_weight(spec.format, ts, len(spec.out_modes))
    for tokens in (1, 2, 4, 5, 7, 8, 9, 16, 23, 24, 31, 32, 33, 47, 64):
        x = wl.round_to_dtype(np.random.default_rng(case * 100 + tokens).standard_normal((tokens, spec.N)), "bf16")
        xd = to_dev(x, "bf16")
        y = to_host(layer(xd))
        err = O.rel_max_err(y, O.apply_linear(w, x))
        assert err <= TOL["bf16"], (case, tokens, err)
        assert O.rel_max_err(y, to_host(plain(xd))) <= 1e-2, (case, tokens)
        assert np.array_equal(y, to_host(layer(xd))), (case, tokens)        # fixed-order sums: the same bits again
    layer.close()
    plain.close()


def test_shared_caller_workspace(dense_w):
    """Several handles keep their intermediates in one caller-owned block (run one after the
    other on one stream); results equal those of handles with their own workspace."""
    spec1, ts1, w1 = dense_w(1)
    spec2, ts2, w2 = dense_w(2)
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    layers = []
    for spec, ts in ((spec1, ts1), (spec2, ts2), (spec1, ts1)):
        dev = [to_dev(t, spec.dtype) for t in ts]
        layers.append(tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks,
                                  dev, 200, workspace=ws))
        assert layers[-1].query(tn.TN_QUERY_WORKSPACE_BYTES) == 0        # nothing allocated by the library
    for tokens in (1, 150):
        x = wl.make_x(spec1, tokens, 1)
        xd = to_dev(x, "bf16")
        y1 = to_host(layers[0](xd))
        y2 = to_host(layers[1](xd))
        y3 = to_host(layers[2](xd))
        assert O.rel_max_err(y1, O.apply_linear(w1, x)) <= TOL["bf16"]
        assert O.rel_max_err(y2, O.apply_linear(w2, x)) <= TOL["bf16"]
        assert np.array_equal(y1, y3)
    for layer in layers:
        layer.close()
    # a block that cannot hold one token's intermediates is refused
    tiny = torch.empty(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(tn.TNLinearError) as e:
        tn.TNLinear(spec2.format, tn.TN_DTYPE_BF16, spec2.out_modes, spec2.in_modes, spec2.ranks,
                    [to_dev(t, "bf16") for t in ts2], 8, workspace=tiny)
    assert e.value.status == -1


PAIR_CASES = [
    # (out modes, in modes, ranks): trains whose end bonds have full rank, so the four cores become two
    # tensors at create time and the plan is a short-K step feeding a long-K step over a bond of 64
    ((6, 8, 8, 8), (8, 2, 8, 8), (1, 48, 64, 64, 1)),       # A = 16, 48 output columns per j (ragged c tile)
    ((8, 4, 8, 8), (8, 2, 8, 8), (1, 64, 64, 64, 1)),       # A = 16, 32 columns
    ((8, 16, 4, 4), (3, 5, 8, 8), (1, 24, 64, 32, 1)),      # A = 15, 128 columns, 16 j (two j sets)
]


@pytest.mark.parametrize("case", range(len(PAIR_CASES)))
def test_chained_pair_kernel_small(case):
    """The chained pair kernel (both steps of a two-tensor train in one launch, intermediate in
    registers) against the oracle and against the two separate launches, at token counts with
    ragged 32-token tiles."""
    om, im, rk = PAIR_CASES[case]
    spec = _spec(tn.TN_FORMAT_TT, "bf16", om, im, rk)
    ts = _rand_layer(spec, 700 + case)
    assert tn.plan_query(spec.format, tn.TN_DTYPE_BF16, om, im, rk, tn.TN_QUERY_PAIR_CHAINABLE) == 1
    w = O.dense_weight(spec.format, ts, len(om))
    for tokens in (1, 5, 33, 256, 257, 1000):          # up to 8 token tiles the range of a is split over workgroups
        x = wl.round_to_dtype(np.random.default_rng(case + tokens).standard_normal((tokens, spec.N)), "bf16")
        ref = O.apply_linear(w, x)
        layer = make_layer(spec, ts, tokens)
        assert layer.query(tn.TN_QUERY_STEP_BASE + 6) == 2
        yd = layer(to_dev(x, "bf16"))
        torch.cuda.synchronize()
        assert torch.equal(yd, layer(to_dev(x, "bf16")))          # same bits on a second call
        layer.close()
        y = to_host(yd)
        y_two = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_PAIR_CHAIN)
        assert O.rel_max_err(y, ref) <= TOL["bf16"], (case, tokens, O.rel_max_err(y, ref))
        assert O.rel_max_err(y_two, ref) <= TOL["bf16"], (case, tokens)
        # both round the intermediate to bf16 once: they differ by summation order only
        assert O.rel_max_err(y, y_two) <= 1e-2, (case, tokens)


@pytest.mark.parametrize("tokens", [1, 8, 31, 64, 100, 256, 300, 2049])
def test_chained_pair_kernel_q_proj(tokens, dense_w):
    spec, ts, w = dense_w(1)
    x = wl.make_x(spec, tokens, 1)
    layer = make_layer(spec, ts, tokens)
    assert layer.query(tn.TN_QUERY_PAIR_CHAINABLE) == 1
    y = to_host(layer(to_dev(x, "bf16")))
    layer.close()
    assert O.rel_max_err(y, O.apply_linear(w, x)) <= TOL["bf16"]
    y_two = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_PAIR_CHAIN)
    assert O.rel_max_err(y, y_two) <= 1e-2


KRON_FORCE = 20 << tn.TN_FLAG_VARIANT_SHIFT
KRON_CASES = [
    # (format, out modes, in modes, ranks, flags, instantiation): two-step plans over a shared bond
    (tn.TN_FORMAT_TT, (40, 36), (10, 64), (1, 40, 1), KRON_FORCE, 3),          # plain x, K0 = 64, one chunk of o1
    (tn.TN_FORMAT_TT, (70, 150), (4, 32), (1, 40, 1), KRON_FORCE, 7),          # 150 values of o1: five chunks of one tile, ragged
    (tn.TN_FORMAT_TT, (70, 120), (4, 32), (1, 40, 1), KRON_FORCE, 3),          # 120 values of o1: two chunks of two tiles, ragged
    (tn.TN_FORMAT_TT, (12, 8), (120, 64), (1, 24, 1), KRON_FORCE, 2),          # A = 120: four tiles of a, ragged
    (tn.TN_FORMAT_TR, (4, 6, 5, 8), (2, 5, 7, 8), (3, 4, 2, 5, 3),             # a ring as two half rings, x gathered
     KRON_FORCE | tn.TN_FLAG_MERGE_GROW | tn.TN_FLAG_NO_SMALL_CHAIN, 5),       # in 16-byte pieces, K0 = 56
    (tn.TN_FORMAT_TR, (8, 16, 8, 8), (8, 10, 8, 8), (16,) * 5, tn.TN_FLAG_MERGE_GROW, 6),   # taken without forcing
    (tn.TN_FORMAT_TR, (8, 10, 8, 8), (8, 16, 8, 8), (16,) * 5, tn.TN_FLAG_MERGE_GROW, 4),   # x gathered element-wise, 3 tiles of o1
    (tn.TN_FORMAT_TR, (10, 16, 10, 16), (8, 10, 8, 8), (12,) * 5, tn.TN_FLAG_MERGE_GROW, 7),  # o1 = 160: five chunks, two tokens per wave
]


@pytest.mark.parametrize("case", range(len(KRON_CASES)))
def test_kronecker_sum_kernel(case):
    """Both steps of a two-tensor plan in one launch (intermediate in MFMA registers, the shared bond
    streamed through LDS) against the oracle and against the two separate launches: one token (the bond
    split over workgroups, partial sums reduced), a ragged group of four, and enough tokens that nothing
    is split."""
    fmt, om, im, rk, flags, cfg = KRON_CASES[case]
    spec = _spec(fmt, "bf16", om, im, rk)
    ts = _rand_layer(spec, 900 + case)
    assert tn.plan_query(fmt, tn.TN_DTYPE_BF16, om, im, rk, tn.TN_QUERY_KRON_CHAINABLE, flags=flags) == 1 + cfg
    w = O.dense_weight(fmt, ts, len(om))
    unfused = (flags & (tn.TN_FLAG_MERGE_GROW | tn.TN_FLAG_NO_SMALL_CHAIN)) | tn.TN_FLAG_NO_PAIR_CHAIN
    for tokens in (1, 3, 6, 1100):
        print(f"kron case {case} tokens {tokens}", flush=True)
        x = wl.round_to_dtype(np.random.default_rng(case + tokens).standard_normal((tokens, spec.N)), "bf16")
        ref = O.apply_linear(w, x)
        layer = make_layer(spec, ts, tokens, flags=flags)
        assert layer.query(tn.TN_QUERY_NUM_STEPS) == 2 and layer.query(tn.TN_QUERY_STEP_BASE + 6) == 4
        yd = layer(to_dev(x, "bf16"))
        torch.cuda.synchronize()
        assert torch.equal(yd, layer(to_dev(x, "bf16")))          # same bits on a second call
        layer.close()
        y = to_host(yd)
        y_two = run_layer(spec, ts, x, flags=unfused)
        assert O.rel_max_err(y, ref) <= TOL["bf16"], (case, tokens, O.rel_max_err(y, ref))
        assert O.rel_max_err(y_two, ref) <= TOL["bf16"], (case, tokens)
        # both round the intermediate to bf16 once: they differ by summation order only
        assert O.rel_max_err(y, y_two) <= 1e-2, (case, tokens)


def test_kronecker_sum_kernel_caller_workspace(dense_w):
    """The ring workload as two half rings with a caller-owned workspace: the partial sums of small calls
    live in the caller's block, and a block too small for many splits only lowers their number."""
    spec, ts, w = dense_w(3)
    for ws_bytes in (1 << 20, 64 << 20):
        block = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        layer = tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks,
                            [to_dev(t, "bf16") for t in ts], 8, flags=tn.TN_FLAG_MERGE_GROW, workspace=block)
        assert layer.query(tn.TN_QUERY_STEP_BASE + 6) == 4
        for tokens in (1, 5):
            x = wl.make_x(spec, tokens, 3)
            y = to_host(layer(to_dev(x, "bf16")))
            assert O.rel_max_err(y, O.apply_linear(w, x)) <= TOL["bf16"], (ws_bytes, tokens)
        layer.close()


LAZY_CASES = [
    # rings of four cores whose large calls run on the two-half-ring plan rebuilt in the workspace
    ((8, 10, 8, 8), (10, 16, 10, 16), (32,) * 5),       # the down_proj workload
    ((10, 16, 10, 16), (8, 10, 8, 8), (32,) * 5),       # five chunks of o1, x gathered element-wise
    ((8, 16, 8, 8), (8, 10, 8, 8), (48,) * 5),          # 2304 values of the shared bond: over a quarter of dense
    ((4, 8, 4, 8), (8, 10, 8, 8), (32,) * 5),           # 32 x 32 outputs per term: the smallest instantiation
]


@pytest.mark.parametrize("case", range(len(LAZY_CASES)))
def test_lazily_merged_ring(case):
    """A default ring layer stores its compact cores; every call rebuilds the half-ring slices in the workspace and
    runs the Kronecker-sum kernel (one-token calls with the four waves of a workgroup sharing the token). Against
    the oracle, against the compact steps and against a layer that keeps the merged tensors, and again after a
    small call has used the same workspace."""
    om, im, rk = LAZY_CASES[case]
    spec = _spec(tn.TN_FORMAT_TR, "bf16", om, im, rk)
    ts = wl.make_tensors(spec, 40 + case)
    w = O.dense_weight(spec.format, ts, len(om))
    layer = make_layer(spec, ts, 64)
    assert layer.query(tn.TN_QUERY_NUM_STEPS) == 4 and layer.query(tn.TN_QUERY_LAZY_MIN_TOKENS) == 1
    assert 0 < layer.query(tn.TN_QUERY_LAZY_FLOPS_PER_TOKEN) < layer.query(tn.TN_QUERY_FLOPS_PER_TOKEN)
    compact = make_layer(spec, ts, 64, flags=tn.TN_FLAG_NO_LAZY_MERGE)
    assert compact.query(tn.TN_QUERY_LAZY_MIN_TOKENS) == 0
    stored = make_layer(spec, ts, 64, flags=tn.TN_FLAG_MERGE_HALVES)
    assert stored.query(tn.TN_QUERY_NUM_STEPS) == 2 and stored.query(tn.TN_QUERY_STEP_BASE + 6) == 4
    scalar_gen = make_layer(spec, ts, 64, flags=tn.TN_FLAG_SCALAR_GENERATE)      # slices rebuilt without MFMA
    first = None
    for tokens in (40, 1, 2, 15, 40):
        print(f"lazy case {case} tokens {tokens}", flush=True)
        x = wl.make_x(spec, tokens, 40 + case)
        xd = to_dev(x, "bf16")
        yd = layer(xd)
        torch.cuda.synchronize()
        y = to_host(yd)
        ref = O.apply_linear(w, x)
        assert O.rel_max_err(y, ref) <= TOL["bf16"], (case, tokens, O.rel_max_err(y, ref))
        yc = to_host(compact(xd))
        assert O.rel_max_err(yc, ref) <= TOL["bf16"], (case, tokens)
        assert O.rel_max_err(y, yc) <= 1e-2
        assert O.rel_max_err(y, to_host(stored(xd))) <= 1e-2         # rebuilt vs stored slices
        assert O.rel_max_err(y, to_host(scalar_gen(xd))) <= 1e-2      # the two rebuild kernels: summation order only
        if tokens == 40:
            if first is None:
                first = yd.clone()
            else:
                assert torch.equal(first, yd)                 # the workspace was reused in between
    for l in (layer, compact, stored, scalar_gen):
        l.close()


def test_lazily_merged_ring_workspace_limits(dense_w):
    """The slices of a lazily merged plan live in the workspace: in a caller's block they share the space of
    the two intermediate buffers; a workspace limit too small for them switches the lazy plan off and every
    call runs the compact steps."""
    spec, ts, w = dense_w(3)
    dev = [to_dev(t, "bf16") for t in ts]
    x = wl.make_x(spec, 20, 3)
    ref = O.apply_linear(w, x)
    for ws_bytes, lazy in ((256 << 20, True),):
        block = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        layer = tn.TNLinear(spec.format, tn.TN_DTYPE_BF16, spec.out_modes, spec.in_modes, spec.ranks, dev, 20,
                            workspace=block)
        assert (layer.query(tn.TN_QUERY_LAZY_MIN_TOKENS) > 0) == lazy
        for tokens in (20, 1, 20):
            y = to_host(layer(to_dev(x[:tokens], "bf16")))
            assert O.rel_max_err(y, ref[:tokens]) <= TOL["bf16"], (ws_bytes, tokens)
        layer.close()
    small = make_layer(spec, ts, 20, workspace_limit_bytes=32 << 20)
    assert small.query(tn.TN_QUERY_LAZY_MIN_TOKENS) == 0
    assert O.rel_max_err(to_host(small(to_dev(x, "bf16"))), ref) <= TOL["bf16"]
    small.close()


CHAIN2_CASES = [
    # Tucker layers whose factor products run as chained launches (out modes, in modes, ranks)
    ((160, 160), (64, 80), (96, 96, 48, 48)),     # the up_proj workload: 64x80 -> 48x48, 96x96 -> 160x160
    ((80, 96), (64, 128), (64, 64, 32, 32)),      # K1 = 128 (the 8-k-step instantiation), ragged c1 tiles
    ((48, 40), (64, 80), (32, 32, 16, 16)),       # one row tile, two k-steps
    ((40, 72), (24, 40), (24, 40, 16, 24)),       # nothing a multiple of 32; the in-factor order makes the
                                                  # first step gather from x, so only the out-factors chain
]
CHAIN2_FUSED = [[1, 0, 0, 1, 0], [1, 0, 0, 1, 0], [1, 0, 0, 1, 0], [0, 0, 0, 1, 0]]


@pytest.mark.parametrize("tokens", [1, 7, 130, 1100])
@pytest.mark.parametrize("case", range(len(CHAIN2_CASES)))
def test_chained_factor_products(case, tokens):
    """Pairs of transposing small steps (Tucker in-factor and out-factor products) as one launch
    with the intermediate in registers: against the oracle and against one launch per step, with a
    wave per (token, column tile) (few tokens) and a wave per token (many)."""
    om, im, rk = CHAIN2_CASES[case]
    spec = _spec(tn.TN_FORMAT_TUCKER, "bf16", om, im, rk)
    ts = _rand_layer(spec, 900 + case)
    x = wl.round_to_dtype(np.random.default_rng(case * 31 + tokens).standard_normal((tokens, spec.N)), "bf16")
    layer = make_layer(spec, ts, tokens)
    n_steps = layer.query(tn.TN_QUERY_NUM_STEPS)
    fused = [layer.query(tn.TN_QUERY_STEP_BASE + 10 * s + 6) for s in range(n_steps)]
    assert n_steps == 5 and fused == CHAIN2_FUSED[case], fused
    xd = to_dev(x, "bf16")
    yd = layer(xd)
    torch.cuda.synchronize()
    assert torch.equal(yd, layer(xd))
    layer.close()
    y = to_host(yd)
    ref = O.forward(spec.format, ts, x, n_out_modes=len(om))
    y_sep = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_CHAIN2)
    assert O.rel_max_err(y, ref) <= TOL["bf16"], (case, tokens, O.rel_max_err(y, ref))
    assert O.rel_max_err(y_sep, ref) <= TOL["bf16"], (case, tokens)
    assert O.rel_max_err(y, y_sep) <= 1e-2, (case, tokens)


DECODE_FUSION_CASES = [
    # Tucker layers whose in-factor pair and core run as one launch at a few tokens (out modes, in modes, ranks)
    ((160, 160), (64, 80), (96, 96, 48, 48)),     # the up_proj workload: 2304 core inputs, 18 k-steps per wave
    ((64, 128), (64, 128), (64, 64, 32, 32)),     # K1 = 128: the 8-k-step instantiation, 1024 core inputs
    ((32, 40), (64, 72), (24, 40, 40, 24)),       # ragged tiles everywhere (C1 = 40: two c1 tiles, one of them of 8)
]


@pytest.mark.parametrize("case", range(len(DECODE_FUSION_CASES)))
def test_factor_pair_and_core_in_one_launch(case):
    """Calls of one or two tokens of a Tucker layer run the in-factor pair and the core step as one launch (the
    pair's result recomputed per workgroup into LDS), and every chained pair with its operands requested up front:
    against the oracle and against the separate launches; three tokens and more take the separate launches."""
    om, im, rk = DECODE_FUSION_CASES[case]
    spec = _spec(tn.TN_FORMAT_TUCKER, "bf16", om, im, rk)
    ts = _rand_layer(spec, 1700 + case)
    w = O.dense_weight(spec.format, ts, 2)
    layer = make_layer(spec, ts, 8)
    plain = make_layer(spec, ts, 8, flags=tn.TN_FLAG_NO_DECODE_FUSION)
    for tokens in (1, 2, 3, 8):
        x = wl.round_to_dtype(np.random.default_rng(case * 13 + tokens).standard_normal((tokens, spec.N)), "bf16")
        xd = to_dev(x, "bf16")
        yd = layer(xd)
        torch.cuda.synchronize()
        assert torch.equal(yd, layer(xd))
        ref = O.apply_linear(w, x)
        assert O.rel_max_err(to_host(yd), ref) <= TOL["bf16"], (case, tokens, O.rel_max_err(to_host(yd), ref))
        yp = to_host(plain(xd))
        assert O.rel_max_err(yp, ref) <= TOL["bf16"], (case, tokens)
        assert O.rel_max_err(to_host(yd), yp) <= 1e-2, (case, tokens)
    layer.close()
    plain.close()


@pytest.mark.parametrize("tokens", [1, 40, 1100])
def test_chained_pair_in_the_middle_of_a_chain(tokens):
    """A Tucker layer with three out-modes and an axis of extent 1: its five steps hold a chained pair that is
    neither first nor last, so the launch reads one workspace buffer and must write the other."""
    spec = _spec(tn.TN_FORMAT_TUCKER, "bf16", (160, 96, 16), (64,), (48, 32, 1, 16))
    ts = _rand_layer(spec, 1500)
    x = wl.round_to_dtype(np.random.default_rng(1500 + tokens).standard_normal((tokens, spec.N)), "bf16")
    layer = make_layer(spec, ts, tokens)
    n_steps = layer.query(tn.TN_QUERY_NUM_STEPS)
    fused = [layer.query(tn.TN_QUERY_STEP_BASE + 10 * s + 6) for s in range(n_steps)]
    assert any(fused[1:n_steps - 2]), fused
    y = to_host(layer(to_dev(x, "bf16")))
    layer.close()
    ref = O.forward(spec.format, ts, x, n_out_modes=3)
    assert O.rel_max_err(y, ref) <= TOL["bf16"], (tokens, O.rel_max_err(y, ref))
    y_sep = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_CHAIN2)
    assert O.rel_max_err(y_sep, ref) <= TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_transposed_small_shapes(case, dtype):
    """TN_FLAG_TRANSPOSE (Y = X W, the gradient of the forward with respect to its input) on the
    small shapes, against the oracle's dense W."""
    fmt, om, im, rk = SMALL[case]
    spec = _spec(fmt, dtype, om, im, rk)
    ts = _rand_layer(spec, 1100 + case)
    w = O.dense_weight(fmt, ts, len(om))
    for tokens in (1, 17, 130):
        x = wl.round_to_dtype(np.random.default_rng(case * 5 + tokens).standard_normal((tokens, spec.M)), dtype)
        y = run_layer(spec, ts, x, flags=tn.TN_FLAG_TRANSPOSE)
        assert y.shape == (tokens, spec.N)
        err = O.rel_max_err(y, O.apply_linear(w.T, x))
        assert err <= TOL[dtype], (case, tokens, err)


@pytest.mark.parametrize("i", [1, 2, 3])
def test_transposed_baseline_configs(i, dense_w):
    """The three bf16 workloads applied transposed, at decode size in full and at 2048 tokens on a
    sample of rows."""
    spec, ts, w = dense_w(i)
    rng = np.random.default_rng(40 + i)
    layer = make_layer(spec, ts, 2048, flags=tn.TN_FLAG_TRANSPOSE)
    assert (layer.N, layer.M) == (spec.M, spec.N)
    for tokens in (1, 64, 2048):
        x = wl.round_to_dtype(rng.standard_normal((tokens, spec.M)), "bf16")
        yd = layer(to_dev(x, "bf16"))
        torch.cuda.synchronize()
        rows = np.unique(np.concatenate([rng.choice(tokens, size=min(tokens, 16), replace=False), [0, tokens - 1]]))
        err = O.rel_max_err(to_host(yd[torch.from_numpy(rows).cuda()]), O.apply_linear(w.T, x[rows]))
        print(f"workload {i} transposed T={tokens} rel err {err:.3e}", flush=True)
        assert err <= TOL["bf16"]
    layer.close()


@pytest.mark.parametrize("i", [1, 2, 3])
def test_forward_under_stream_capture(i, dense_w):
    """tn_linear_forward neither allocates nor synchronises: the very first call of a fresh handle may be
    recorded into a HIP graph. Replays (with eager work and synchronisations in between) must give the
    eager result bit for bit, at a decode size and at a size that runs the chained kernels (for the ring:
    the rebuild of the half-ring slices, the Kronecker-sum launch and the reduction of its partial sums)."""
    spec, ts, w = dense_w(i)
    for tokens in (1, 300):
        x = to_dev(wl.make_x(spec, tokens, i), "bf16")
        layer = make_layer(spec, ts, tokens)
        y_graph = torch.empty((tokens, spec.M), dtype=torch.bfloat16, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x, out=y_graph)
        y_eager = layer(x)
        torch.cuda.synchronize()
        for _ in range(3):
            y_graph.fill_(0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y_graph, y_eager)
            assert torch.equal(layer(x), y_eager)
        assert O.rel_max_err(to_host(y_graph), O.apply_linear(w, wl.make_x(spec, tokens, i))) <= TOL["bf16"]
        del graph
        layer.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_layers_in_one_launch(case, dtype):
    """Layers whose tensors and intermediates fit in LDS run all their steps as one launch (fp32 at any
    token count, bf16 up to 32 tokens): against the oracle and against one launch per step."""
    fmt, om, im, rk = SMALL[case]
    spec = _spec(fmt, dtype, om, im, rk)
    ts = _rand_layer(spec, 1300 + case)
    for tokens in (1, 17, 32, 700):
        x = wl.round_to_dtype(np.random.default_rng(case * 3 + tokens).standard_normal((tokens, spec.N)), dtype)
        ref = O.forward(fmt, ts, x, n_out_modes=len(om))
        layer = make_layer(spec, ts, tokens)
        n_steps = layer.query(tn.TN_QUERY_NUM_STEPS)
        one_launch = n_steps > 1 and layer.query(tn.TN_QUERY_STEP_BASE + 6) == 3
        y = to_host(layer(to_dev(x, dtype)))
        layer.close()
        y_steps = run_layer(spec, ts, x, flags=tn.TN_FLAG_NO_SMALL_CHAIN)
        assert O.rel_max_err(y, ref) <= TOL[dtype], (case, tokens, one_launch)
        assert O.rel_max_err(y_steps, ref) <= TOL[dtype], (case, tokens)
    if case in (1, 5):       # the two MFMA-sized trains do not fit
        assert not one_launch
    if case == 2:            # the small fp32 train of the baseline configs
        assert one_launch


def test_config0_one_launch():
    spec, toks = wl.baseline_spec(0)
    ts = wl.make_tensors(spec, 0)
    layer = make_layer(spec, ts, toks[0])
    assert [layer.query(tn.TN_QUERY_STEP_BASE + 10 * s + 6) for s in range(3)] == [3, 3, 0]
    x = wl.make_x(spec, toks[0], 0)
    y = to_host(layer(to_dev(x, "f32")))
    layer.close()
    assert O.rel_max_err(y, O.forward(spec.format, ts, x)) <= 1e-5


FORWARD2_CASES = [
    # (spec of layer a, spec of layer b): same input width
    (wl.baseline_spec(2)[0], wl.baseline_spec(2)[0]),                                                   # gate / up as Tucker layers
    (wl.stack_spec(wl.FORMAT_TUCKER, 8192, 5120, 64), wl.stack_spec(wl.FORMAT_TUCKER, 8192, 5120, 64)),   # K1 = 128 instantiation
    (wl.baseline_spec(2)[0], wl.stack_spec(wl.FORMAT_TUCKER, 5120, 25600, 64)),                         # different ranks: other core widths
    (wl.baseline_spec(2)[0], wl.stack_spec(wl.FORMAT_DENSE, 5120, 8192, 0)),                            # different formats: back to back
    (wl.baseline_spec(1)[0], wl.baseline_spec(1)[0]),                                                   # trains: back to back
]


@pytest.mark.parametrize("case", range(len(FORWARD2_CASES)))
def test_two_layers_in_one_call(case):
    """tn_linear_forward2 (two layers on the same activations, e.g. gate and up projections): both results against
    two separate oracle forwards and against tn_linear_forward on each handle, at token counts that take the shared
    decode-size launches (1, 2), the per-step path (5, 40) and the large-call kernels (300)."""
    sa, sb = FORWARD2_CASES[case]
    ta, tb = wl.make_tensors(sa, 80 + case, instance=0), wl.make_tensors(sb, 80 + case, instance=1)
    wa, wb = O.dense_weight(sa.format, ta, len(sa.out_modes)), O.dense_weight(sb.format, tb, len(sb.out_modes))
    la, lb = make_layer(sa, ta, 300), make_layer(sb, tb, 300)
    for tokens in (1, 2, 5, 40, 300):
        x = wl.make_x(sa, tokens, 80 + case)
        xd = to_dev(x, "bf16")
        ya, yb = tn.forward2(la, lb, xd)
        torch.cuda.synchronize()
        for y, w, layer in ((ya, wa, la), (yb, wb, lb)):
            err = O.rel_max_err(to_host(y), O.apply_linear(w, x))
            assert err <= TOL["bf16"], (case, tokens, err)
            assert torch.equal(y, layer(xd)), (case, tokens)             # the same kernels on the same data
    # under stream capture: both layers in one graph, replayed
    xd = to_dev(wl.make_x(sa, 1, 80 + case), "bf16")
    ga = torch.empty((1, sa.M), dtype=torch.bfloat16, device="cuda")
    gb = torch.empty((1, sb.M), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        tn.forward2(la, lb, xd, ga, gb)
    ea, eb = tn.forward2(la, lb, xd)
    torch.cuda.synchronize()
    for _ in range(2):
        ga.fill_(0)
        gb.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ga, ea) and torch.equal(gb, eb)
    del graph
    la.close()
    lb.close()
    with pytest.raises(tn.TNLinearError):                                  # different input widths
        l1 = make_layer(wl.baseline_spec(2)[0], wl.make_tensors(wl.baseline_spec(2)[0], 2), 4)
        l3 = make_layer(wl.stack_spec(wl.FORMAT_DENSE, 8192, 5120, 0), wl.make_tensors(wl.stack_spec(wl.FORMAT_DENSE, 8192, 5120, 0), 4), 4)
        try:
            tn.tn_linear_forward2(l1._handle, l3._handle, xd.data_ptr(), ga.data_ptr(), gb.data_ptr(), 1, None)
        finally:
            l1.close()
            l3.close()
