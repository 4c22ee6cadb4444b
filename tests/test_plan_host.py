"""Host logic of the library: planner order, FLOP totals, layouts, scatter
tables and packing recipes, executed on the CPU in double precision by a
test-only C++ walker of the plan and compared with the oracle."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

import oracle as O
import workloads as wl
import paper_2602_01613_amd as tn
from paper_2602_01613_amd.binding import _Desc, _make_desc

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def host_exec():
    out = os.path.join(tempfile.mkdtemp(prefix="tn_plan_host_"), "libplan_host_exec.so")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC",
                           os.path.join(HERE, "plan_host_exec.cpp"), "-o", out])
    lib = ctypes.CDLL(out)
    lib.plan_host_forward.restype = ctypes.c_int
    lib.plan_host_forward.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(ctypes.c_void_p),
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
    lib.plan_host_launch_buffers.restype = ctypes.c_int
    lib.plan_host_launch_buffers.argtypes = [ctypes.POINTER(_Desc), ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                             ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.plan_host_step_hint.restype = ctypes.c_int
    lib.plan_host_step_hint.argtypes = [ctypes.POINTER(_Desc), ctypes.c_int, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_int64)]
    return lib


def _run(lib, fmt, out_modes, in_modes, ranks, tensors, x, flags=0):
    d, keep = _make_desc(fmt, tn.TN_DTYPE_F32, out_modes, in_modes, ranks, None, 1, 0, flags, None)
    ts = [np.ascontiguousarray(t, dtype=np.float64) for t in tensors]
    ptrs = (ctypes.c_void_p * len(ts))(*[t.ctypes.data for t in ts])
    x = np.ascontiguousarray(x, dtype=np.float64)
    m = int(np.prod(out_modes))
    y = np.zeros((x.shape[0], m))
    rc = lib.plan_host_forward(ctypes.byref(d), ptrs, x.ctypes.data, y.ctypes.data, x.shape[0])
    assert rc == 0, f"plan_host_forward failed with {rc}"
    return y


def _rand_tensors(rng, fmt, out_modes, in_modes, ranks):
    spec = wl.TNSpec(fmt, "f32", tuple(out_modes), tuple(in_modes), tuple(ranks))
    return [rng.standard_normal(s) for s in spec.tensor_shapes()]


CASES = [
    (tn.TN_FORMAT_TT, (4, 8, 8), (4, 8, 8), (1, 8, 8, 1)),
    (tn.TN_FORMAT_TT, (3, 4, 2), (2, 5, 3), (1, 3, 4, 1)),
    (tn.TN_FORMAT_TT, (2, 3, 2, 2), (5, 2, 3, 2), (1, 2, 5, 3, 1)),       # best order is not right-to-left
    (tn.TN_FORMAT_TT, (7,), (5,), (1, 1)),
    (tn.TN_FORMAT_TT, (1, 3, 1), (2, 1, 3), (1, 1, 2, 1)),                 # size-1 modes and bonds
    (tn.TN_FORMAT_TR, (2, 3, 2), (3, 2, 2), (3, 2, 4, 3)),
    (tn.TN_FORMAT_TR, (2, 3, 2, 2), (3, 2, 2, 3), (2, 3, 2, 3, 2)),
    (tn.TN_FORMAT_TR, (4, 3), (3, 5), (2, 3, 2)),
    (tn.TN_FORMAT_TR, (5,), (7,), (3, 3)),                                  # ring of one core: partial trace
    (tn.TN_FORMAT_TR, (3, 2), (2, 4), (1, 3, 1)),
    (tn.TN_FORMAT_TUCKER, (4, 5), (3, 6), (2, 3, 2, 4)),
    (tn.TN_FORMAT_TUCKER, (6,), (5,), (3, 4)),
    (tn.TN_FORMAT_TUCKER, (3, 2, 4), (5,), (2, 2, 3, 4)),
    (tn.TN_FORMAT_TUCKER, (4,), (2, 3, 2), (3, 2, 2, 2)),
    (tn.TN_FORMAT_DENSE, (9,), (11,), ()),
    (tn.TN_FORMAT_DENSE, (3, 3), (2, 5), ()),
    # boundary bonds at full rank: the end cores are contracted into their neighbours at create time
    (tn.TN_FORMAT_TT, (2, 3, 2, 2), (2, 2, 3, 2), (1, 4, 2, 4, 1)),
    (tn.TN_FORMAT_TT, (2, 3, 2), (2, 2, 2), (1, 4, 4, 1)),
    (tn.TN_FORMAT_TT, (2, 4, 2), (3, 4, 2), (1, 6, 5, 1)),
    # with TN_FLAG_MERGE_GROW these rings become two half-rings
    (tn.TN_FORMAT_TR, (4, 4, 4, 4), (4, 4, 4, 4), (2, 2, 2, 2, 2)),
    (tn.TN_FORMAT_TR, (4, 3, 4, 2), (2, 4, 3, 4), (2, 3, 2, 3, 2)),
]


@pytest.mark.parametrize("flags", [0, tn.TN_FLAG_NO_MERGE, tn.TN_FLAG_MERGE_GROW, tn.TN_FLAG_MERGE_HALVES,
                                   # layers with 4-bit tensors order the contracted indices of a step differently
                                   # (the planner only: this executor multiplies the tensors as given)
                                   tn.TN_FLAG_QUANT_MXFP4, tn.TN_FLAG_QUANT_MXFP4 | tn.TN_FLAG_NO_MERGE])
@pytest.mark.parametrize("fmt,om,im,rk", CASES)
def test_plan_executes_to_oracle(host_exec, fmt, om, im, rk, flags):
    rng = np.random.default_rng(hash((fmt, om, im, rk)) % (2 ** 32))
    if fmt == tn.TN_FORMAT_DENSE:
        tensors = [rng.standard_normal((int(np.prod(om)), int(np.prod(im))))]
    else:
        tensors = _rand_tensors(rng, fmt, om, im, rk)
    x = rng.standard_normal((3, int(np.prod(im))))
    y = _run(host_exec, fmt, om, im, rk, tensors, x, flags)
    ref = O.forward(fmt, tensors, x, n_out_modes=len(om))
    assert O.rel_max_err(y, ref) < 1e-12


@pytest.mark.parametrize("fmt,om,im,rk", CASES)
def test_transposed_plan_executes_to_oracle(host_exec, fmt, om, im, rk):
    """TN_FLAG_TRANSPOSE: the same tensors applied as W^T (activations carry the out-modes), walked on
    the host in double precision and compared with X W for the oracle's dense W."""
    rng = np.random.default_rng(sum(om) * 17 + sum(im))
    ts = _rand_tensors(rng, fmt, om, im, rk)
    w = O.dense_weight(fmt, ts, len(om))
    x = rng.standard_normal((3, w.shape[0]))
    for flags in (tn.TN_FLAG_TRANSPOSE, tn.TN_FLAG_TRANSPOSE | tn.TN_FLAG_NO_MERGE):
        d, keep = _make_desc(fmt, tn.TN_DTYPE_F32, om, im, rk, None, 1, 0, flags, None)
        t64 = [np.ascontiguousarray(t, dtype=np.float64) for t in ts]
        ptrs = (ctypes.c_void_p * len(t64))(*[t.ctypes.data for t in t64])
        y = np.zeros((3, w.shape[1]))
        xc = np.ascontiguousarray(x)
        assert host_exec.plan_host_forward(ctypes.byref(d), ptrs, xc.ctypes.data, y.ctypes.data, 3) == 0
        assert O.rel_max_err(y, O.apply_linear(w.T, x)) <= 1e-12
    assert tn.plan_query(fmt, tn.TN_DTYPE_F32, om, im, rk, tn.TN_QUERY_IN_FEATURES, flags=tn.TN_FLAG_TRANSPOSE) == w.shape[0]
    assert tn.plan_query(fmt, tn.TN_DTYPE_F32, om, im, rk, tn.TN_QUERY_OUT_FEATURES, flags=tn.TN_FLAG_TRANSPOSE) == w.shape[1]


def test_plan_small_baseline_config(host_exec):
    spec, toks = wl.baseline_spec(0)
    tensors = wl.make_tensors(spec, 0)
    x = wl.make_x(spec, toks[0], 0)
    y = _run(host_exec, spec.format, spec.out_modes, spec.in_modes, spec.ranks, tensors, x)
    assert O.rel_max_err(y, O.forward(spec.format, tensors, x)) < 1e-12


def _q(spec, what, flags=tn.TN_FLAG_NO_MERGE):
    dt = tn.TN_DTYPE_BF16 if spec.dtype == "bf16" else tn.TN_DTYPE_F32
    return tn.plan_query(spec.format, dt, spec.out_modes, spec.in_modes, spec.ranks, what, flags=flags)


def test_flop_totals_and_orders():
    # fewest-FLOP orders of the four single-layer workloads (2 * multiply-adds per token)
    expect = {0: 311296, 1: 1020264448, 2: 51118080, 3: 12666798080}
    for i, f in expect.items():
        spec, _ = wl.baseline_spec(i)
        assert _q(spec, tn.TN_QUERY_FLOPS_PER_TOKEN) == f
        assert _q(spec, tn.TN_QUERY_PARAM_COUNT) == spec.n_params
        assert _q(spec, tn.TN_QUERY_OUT_FEATURES) == spec.M
        assert _q(spec, tn.TN_QUERY_IN_FEATURES) == spec.N
    # TT q_proj: right-to-left, steps (rows, K, cols)
    spec, _ = wl.baseline_spec(1)
    steps = [[_q(spec, 100 + 10 * s + f) for f in range(5)] for s in range(4)]
    assert [s[4] for s in steps] == [3, 2, 1, 0]
    assert [tuple(s[:3]) for s in steps] == [(640, 8, 512), (640, 512, 512), (512, 640, 1024), (1024, 512, 8)]
    # TR down_proj: core 4, then across the ring bond to core 1, then 3, and core 2 closes two bonds
    spec, _ = wl.baseline_spec(3)
    steps = [[_q(spec, 100 + 10 * s + f) for f in range(5)] for s in range(4)]
    assert [s[4] for s in steps] == [3, 0, 2, 1]
    assert tuple(steps[3][:3]) == (512, 16384, 10)
    # Tucker up_proj: in-factors, core, out-factors
    spec, _ = wl.baseline_spec(2)
    assert _q(spec, tn.TN_QUERY_NUM_STEPS) == 5
    assert [_q(spec, 100 + 10 * s + 4) for s in range(3)] == [4, 3, 0]
    assert tuple(_q(spec, 120 + f) for f in range(3)) == (1, 2304, 9216)


def test_create_time_merging():
    # TT q_proj: r_1 = m_1 n_1 = 64 and r_3 = m_4 n_4 = 64, so both end cores merge into their
    # neighbours without adding parameters; two steps remain:
    #   rows n_1 n_2 = 80, K = n_3 n_4 = 64, cols m_3 m_4 r_2 = 4096   (41 943 040 FLOP)
    #   rows m_3 m_4 = 64, K = n_1 n_2 r_2 = 5120, cols m_1 m_2 = 128   (83 886 080 FLOP)
    spec, _ = wl.baseline_spec(1)
    assert _q(spec, tn.TN_QUERY_NUM_MERGES, 0) == 2
    assert _q(spec, tn.TN_QUERY_NUM_STEPS, 0) == 2
    assert _q(spec, tn.TN_QUERY_FLOPS_PER_TOKEN, 0) == 41943040 + 83886080
    steps = [tuple(_q(spec, 100 + 10 * s + f, 0) for f in range(3)) for s in range(2)]
    assert steps == [(80, 64, 4096), (64, 5120, 128)]
    assert _q(spec, tn.TN_QUERY_PARAM_COUNT, 0) == spec.n_params
    # nothing to merge where a merge would add parameters
    for i in (0, 2, 3):
        spec, _ = wl.baseline_spec(i)
        assert _q(spec, tn.TN_QUERY_NUM_MERGES, 0) == 0
        assert _q(spec, tn.TN_QUERY_FLOPS_PER_TOKEN, 0) == _q(spec, tn.TN_QUERY_FLOPS_PER_TOKEN)
    # the flag keeps the chain as given
    spec, _ = wl.baseline_spec(1)
    assert _q(spec, tn.TN_QUERY_NUM_MERGES) == 0 and _q(spec, tn.TN_QUERY_NUM_STEPS) == 4
    # rank above what the end cores can carry (96 > 8*8): merging shrinks the parameters
    big = wl.stack_spec(wl.FORMAT_TT, 5120, 8192, 96)
    assert _q(big, tn.TN_QUERY_NUM_MERGES, 0) == 2
    small = wl.stack_spec(wl.FORMAT_TT, 5120, 8192, 32)
    assert _q(small, tn.TN_QUERY_NUM_MERGES, 0) == 0


def test_pair_chainable_plans():
    """Which plans qualify for the chained pair kernel: two-tensor trains over a bond of 64 with a
    64-long first contraction, and nothing else."""
    q = lambda fmt, om, im, rk, flags=0: tn.plan_query(fmt, tn.TN_DTYPE_BF16, om, im, rk,
                                                        tn.TN_QUERY_PAIR_CHAINABLE, flags=flags)
    spec, _ = wl.baseline_spec(1)
    assert q(spec.format, spec.out_modes, spec.in_modes, spec.ranks) == 1
    assert q(spec.format, spec.out_modes, spec.in_modes, spec.ranks, tn.TN_FLAG_NO_MERGE) == 0     # four steps
    assert tn.plan_query(spec.format, tn.TN_DTYPE_F32, spec.out_modes, spec.in_modes, spec.ranks,
                         tn.TN_QUERY_PAIR_CHAINABLE) == 0                                        # bf16 only
    assert q(tn.TN_FORMAT_TT, (6, 8, 8, 8), (8, 2, 8, 8), (1, 48, 64, 64, 1)) == 1
    assert q(tn.TN_FORMAT_TT, (8, 16, 4, 4), (3, 5, 8, 8), (1, 24, 64, 32, 1)) == 1
    assert q(tn.TN_FORMAT_TT, (8, 16, 8, 8), (8, 10, 8, 8), (1, 64, 32, 64, 1)) == 0              # bond of 32
    assert q(tn.TN_FORMAT_TT, (8, 16, 4, 8), (8, 10, 4, 8), (1, 64, 64, 64, 1)) == 0              # K0 = 32
    assert q(tn.TN_FORMAT_TT, (8, 10, 8, 8), (8, 16, 8, 8), (1, 64, 64, 64, 1)) == 0              # other order wins
    for i in (2, 3):
        s, _ = wl.baseline_spec(i)
        assert q(s.format, s.out_modes, s.in_modes, s.ranks) == 0


def test_kronecker_sum_plans():
    """Which plans run on the Kronecker-sum kernel: two steps over a shared bond whose intermediate is
    large (a ring contracted into two half rings), in the instantiation with the least padding; small
    shapes only when forced; never the plans of the chained pair kernel, fp32, or with chaining off."""
    q = lambda fmt, om, im, rk, flags=0, dt=tn.TN_DTYPE_BF16: tn.plan_query(fmt, dt, om, im, rk,
                                                                             tn.TN_QUERY_KRON_CHAINABLE, flags=flags)
    ring, _ = wl.baseline_spec(3)
    grow, force = tn.TN_FLAG_MERGE_GROW, 20 << tn.TN_FLAG_VARIANT_SHIFT
    assert q(ring.format, ring.out_modes, ring.in_modes, ring.ranks) == 0                  # four steps
    assert q(ring.format, ring.out_modes, ring.in_modes, ring.ranks, grow) == 1            # <5, 10, 3, 2>
    assert q(ring.format, ring.out_modes, ring.in_modes, ring.ranks, grow | tn.TN_FLAG_NO_PAIR_CHAIN) == 0
    assert q(ring.format, ring.out_modes, ring.in_modes, ring.ranks, grow, tn.TN_DTYPE_F32) == 0
    assert q(ring.format, ring.in_modes[:0] + (10, 16, 10, 16), (8, 10, 8, 8), (32,) * 5, grow) == 8    # <2, 5, 5, 1>: o1 = 160 is five tiles
    assert q(tn.TN_FORMAT_TR, (8, 16, 8, 8), (8, 10, 8, 8), (16,) * 5, grow) == 7          # <3, 4, 4, 2>
    assert q(tn.TN_FORMAT_TR, (8, 10, 8, 8), (8, 16, 8, 8), (16,) * 5, grow) == 5          # <2, 8, 2, 3>
    train, _ = wl.baseline_spec(1)
    assert q(train.format, train.out_modes, train.in_modes, train.ranks) == 0             # the pair kernel's plan
    small = (tn.TN_FORMAT_TT, (40, 36), (10, 64), (1, 40, 1))
    assert q(*small) == 0 and q(*small, force) == 4                                        # <2, 5, 5, 2>
    assert q(tn.TN_FORMAT_TT, (12, 8), (120, 64), (1, 24, 1), force) == 3                  # <4, 4, 3, 2>
    assert q(tn.TN_FORMAT_TT, (8, 12), (16, 8), (1, 24, 1), force) == 6                    # <2, 5, 1, 1>; x gathered element-wise
    # the plan large calls of a default ring layer run on: two half rings whatever their size
    halves = tn.TN_FLAG_MERGE_HALVES
    assert q(ring.format, ring.out_modes, ring.in_modes, (96,) * 5, grow) == 0             # over a quarter of dense
    assert q(ring.format, ring.out_modes, ring.in_modes, (96,) * 5, halves) == 1
    assert q(tn.TN_FORMAT_TR, (4, 8, 4, 8), (8, 10, 8, 8), (32,) * 5, halves) == 6
    assert q(tn.TN_FORMAT_TT, (20, 6), (24, 10), (1, 40, 1), force) == 0                   # K0 = 10: not 8-aligned


def test_chain2_shapes():
    """Which step pairs qualify for the transposing chain kernel: the factor products of Tucker layers
    whose first step reads a plain matrix, in the smaller instantiation where it fits."""
    def shapes(fmt, om, im, rk, flags=0):
        n = tn.plan_query(fmt, tn.TN_DTYPE_BF16, om, im, rk, tn.TN_QUERY_NUM_STEPS, flags=flags)
        return [tn.plan_query(fmt, tn.TN_DTYPE_BF16, om, im, rk, tn.TN_QUERY_STEP_BASE + 10 * s + 7, flags=flags)
                for s in range(n)]
    s2, _ = wl.baseline_spec(2)
    # in-factors 64x80 -> 48x48 fit the small instantiation (2), out-factors 96x96 -> 160x160 the large one (1)
    assert shapes(s2.format, s2.out_modes, s2.in_modes, s2.ranks) == [2, 0, 0, 1, 0]
    assert shapes(tn.TN_FORMAT_TUCKER, (40, 72), (24, 40), (24, 40, 16, 24)) == [0, 0, 0, 2, 0]   # first step gathers
    assert shapes(tn.TN_FORMAT_TUCKER, (160, 160), (160, 160), (96, 96, 48, 48))[0] == 0          # 160 input rows
    for i in (1, 3):
        s, _ = wl.baseline_spec(i)
        assert not any(shapes(s.format, s.out_modes, s.in_modes, s.ranks))
        assert not any(shapes(s.format, s.out_modes, s.in_modes, s.ranks, tn.TN_FLAG_NO_MERGE))
    assert tn.plan_query(s2.format, tn.TN_DTYPE_F32, s2.out_modes, s2.in_modes, s2.ranks, tn.TN_QUERY_STEP_BASE + 7) == 0


def _launch_buffers(lib, fmt, om, im, rk, flags=0):
    d, keep = _make_desc(fmt, tn.TN_DTYPE_BF16, om, im, rk, None, 1, 0, flags, None)
    cap = 32
    a, b, c = (ctypes.c_int * cap)(), (ctypes.c_int * cap)(), (ctypes.c_int * cap)()
    n = lib.plan_host_launch_buffers(ctypes.byref(d), cap, a, b, c)
    assert n > 0, n
    return [(a[i], b[i], c[i]) for i in range(n)]


def test_no_launch_writes_the_buffer_it_reads(host_exec):
    """Buffers alternate per launch, not per step: a chained pair in the middle of a chain (a Tucker layer
    with three modes on one side and an axis of extent 1) must not get the same workspace buffer as input
    and output. Also over random descriptions with small extents (1 included)."""
    sched = _launch_buffers(host_exec, tn.TN_FORMAT_TUCKER, (160, 96, 16), (64,), (48, 32, 1, 16))
    assert any(steps == 2 and first_in >= 0 and out >= 0 for first_in, out, steps in sched), sched
    rng = np.random.default_rng(77)
    seen_mid_pair = 0
    for trial in range(3000):
        p, q = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        om = tuple(int(v) for v in rng.choice([1, 8, 16, 32, 48, 64, 96, 160], p))
        im = tuple(int(v) for v in rng.choice([1, 8, 16, 32, 48, 64, 96, 160], q))
        rk = tuple(int(min(m, v)) for m, v in zip(om + im, rng.choice([1, 8, 16, 32, 48, 64, 96], p + q)))
        sched = _launch_buffers(host_exec, tn.TN_FORMAT_TUCKER, om, im, rk)
        assert sched[0][0] == -1 and sched[-1][1] == -2
        for n, (src, dst, steps) in enumerate(sched):
            assert src != dst, (om, im, rk, sched)
            if n:
                assert src == sched[n - 1][1]
            if steps == 2 and 0 < n < len(sched) - 1:
                seen_mid_pair += 1
    assert seen_mid_pair > 0


def test_growing_merges_half_ring():
    # TR down_proj with TN_FLAG_MERGE_GROW: cores (4,1) and (2,3) are contracted at create time
    # (23.6 M parameters, under a quarter of the dense 131 M) and the chain is two steps,
    # 5 033 164 800 FLOP per token instead of 12 666 798 080
    spec, _ = wl.baseline_spec(3)
    g = tn.TN_FLAG_MERGE_GROW
    assert _q(spec, tn.TN_QUERY_NUM_MERGES, g) == 2
    assert _q(spec, tn.TN_QUERY_NUM_STEPS, g) == 2
    assert _q(spec, tn.TN_QUERY_FLOPS_PER_TOKEN, g) == 5033164800
    # rank 96: every merge would exceed the budget, the plan is unchanged
    big = wl.stack_spec(wl.FORMAT_TR, 25600, 5120, 96)
    assert _q(big, tn.TN_QUERY_NUM_MERGES, g) == 0
    # TN_FLAG_MERGE_HALVES (the plan large calls of a default ring layer run on, rebuilt per call): two half
    # rings whatever the size. Per token 2*A*O1*P*(K0 + C1) with A = K0 = 160, O1 = 64, C1 = 80, P = r*r.
    hv = tn.TN_FLAG_MERGE_HALVES
    for spec_r, r in ((spec, 32), (big, 96)):
        assert _q(spec_r, tn.TN_QUERY_NUM_MERGES, hv) == 2 and _q(spec_r, tn.TN_QUERY_NUM_STEPS, hv) == 2
        assert _q(spec_r, tn.TN_QUERY_FLOPS_PER_TOKEN, hv) == 2 * 160 * 64 * r * r * (160 + 80)
    assert _q(big, tn.TN_QUERY_FLOPS_PER_TOKEN, 0) == 331433902080           # its compact four steps


def test_planned_flops_equal_brute_force_minimum():
    # exhaustive search over all absorption orders of a TT and a TR, in Python
    from itertools import permutations

    def cost(order, ms, ns, rs, ring):
        d = len(ms)
        live = {("n", k): ns[k] for k in range(d)}
        total = 0
        for k in order:
            bonds = [("b", k % d if ring else k), ("b", (k + 1) % d if ring else k + 1)]
            ext = {bonds[0]: rs[k], bonds[1]: rs[k + 1]}
            if not ring:
                ext = {b: e for b, e in ext.items() if b[1] not in (0, d)}
            size = int(np.prod(list(live.values()))) if live else 1
            new = ms[k]
            for b, e in ext.items():
                if b not in live:
                    new *= e
            total += 2 * size * new
            del live[("n", k)]
            live[("m", k)] = ms[k]
            for b, e in ext.items():
                if b in live:
                    del live[b]
                else:
                    live[b] = e
        return total

    for fmt, ms, ns, rs in [(tn.TN_FORMAT_TT, (8, 16, 8, 8), (8, 10, 8, 8), (1, 64, 64, 64, 1)),
                            (tn.TN_FORMAT_TR, (8, 10, 8, 8), (10, 16, 10, 16), (32,) * 5),
                            (tn.TN_FORMAT_TT, (2, 3, 2, 2), (5, 2, 3, 2), (1, 2, 5, 3, 1)),
                            (tn.TN_FORMAT_TR, (2, 3, 2), (3, 2, 2), (3, 2, 4, 3))]:
        best = min(cost(o, ms, ns, rs, fmt == tn.TN_FORMAT_TR) for o in permutations(range(len(ms))))
        assert tn.plan_query(fmt, 1, ms, ns, rs, tn.TN_QUERY_FLOPS_PER_TOKEN, flags=tn.TN_FLAG_NO_MERGE) == best


def test_vector_store_hints(host_exec):
    # TT q_proj: intermediate steps store runs of 64 contiguous bond entries, the last step
    # stores contiguous rows; every step after the first reads a plain matrix.
    spec, _ = wl.baseline_spec(1)
    d, keep = _make_desc(spec.format, 1, spec.out_modes, spec.in_modes, spec.ranks, None, 1, 0,
                         tn.TN_FLAG_NO_MERGE, None)
    v = ctypes.c_int64(0)
    hints = []
    for s in range(4):
        row = []
        for f in range(3):
            assert host_exec.plan_host_step_hint(ctypes.byref(d), s, f, ctypes.byref(v)) == 0
            row.append(v.value)
        hints.append(row)
    assert [h[2] for h in hints] == [1, 1, 1, 1]
    assert [h[0] for h in hints[:3]] == [8, 8, 8]
    assert hints[3][1] == 8


def test_invalid_descriptions_are_rejected():
    bad = [
        (tn.TN_FORMAT_TT, (4, 4), (4,), (1, 2, 1)),          # mode count mismatch
        (tn.TN_FORMAT_TT, (4, 4), (4, 4), (2, 2, 1)),        # r_0 != 1
        (tn.TN_FORMAT_TR, (4, 4), (4, 4), (2, 2, 3)),        # ring bond mismatch
        (tn.TN_FORMAT_TT, (4, 0), (4, 4), (1, 2, 1)),        # zero extent
        (tn.TN_FORMAT_TUCKER, (4, 4), (4, 4), (2, 2, 2)),    # wrong number of ranks
        (7, (4,), (4,), ()),                                  # unknown format
    ]
    for fmt, om, im, rk in bad:
        with pytest.raises(tn.TNLinearError) as e:
            tn.plan_query(fmt, 1, om, im, rk, tn.TN_QUERY_FLOPS_PER_TOKEN)
        assert e.value.status == -1
    with pytest.raises(tn.TNLinearError):
        tn.plan_query(tn.TN_FORMAT_TT, 5, (4,), (4,), (1, 1), tn.TN_QUERY_FLOPS_PER_TOKEN)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """There is no CPU or fallback path: without the built library the binding raises."""
    import paper_2602_01613_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "library_path", lambda: str(tmp_path / "libtn_linear.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        b.load_library()


def test_library_exports_every_declared_symbol():
    import re
    hdr = open(os.path.join(os.path.dirname(HERE), "include", "tn_linear.h")).read()
    declared = set(re.findall(r"\b(tn_linear_[a-z_0-9]+)\s*\(", hdr))
    declared -= {"tn_linear_s"}
    assert declared == set(tn.EXPORTED_SYMBOLS)
    lib = tn.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert tn.tn_linear_version() == 6
    assert tn.tn_linear_strerror(0) == "success"
    assert "invalid" in tn.tn_linear_strerror(-1)
