"""Pins of the fp64 oracle against what the definitions and mathematics fix.

None of these re-type the oracle's own formula: they use Kronecker products,
SVD round trips, per-entry matrix products and traces from numpy, nested-loop
summation, gauge and rotation invariances, and closed-form statistics.
"""
from math import prod

import numpy as np
import pytest

import oracle
from oracle import tn_oracle as O
import workloads as wl

TT, TR, TUCKER, DENSE = O.FORMAT_TT, O.FORMAT_TR, O.FORMAT_TUCKER, O.FORMAT_DENSE


def _cores(rng, ms, ns, rs):
    return [rng.standard_normal((rs[k], ms[k], ns[k], rs[k + 1])) for k in range(len(ms))]


# ---- 1. rank-1 TT is the Kronecker product of its cores (pins C-order digits,
#         the [r, m, n, r] axis order and the [out, in] orientation) ------------
def test_rank1_tt_is_kronecker():
    rng = np.random.default_rng(1)
    ms, ns = (3, 4, 2), (2, 5, 3)        # non-square modes: a transposed core cannot pass
    cores = _cores(rng, ms, ns, (1, 1, 1, 1))
    w = O.tt_dense(cores)
    k = cores[0][0, :, :, 0]
    for g in cores[1:]:
        k = np.kron(k, g[0, :, :, 0])
    assert w.shape == (24, 30)
    np.testing.assert_allclose(w, k, rtol=0, atol=1e-13)


def test_rank1_tr_is_kronecker():
    rng = np.random.default_rng(2)
    cores = _cores(rng, (2, 3), (3, 2), (1, 1, 1))
    k = np.kron(cores[0][0, :, :, 0], cores[1][0, :, :, 0])
    np.testing.assert_allclose(O.tr_dense(cores), k, atol=1e-13)


# ---- 2. TR with boundary rank 1 is TT (pins the trace closure) ---------------
@pytest.mark.parametrize("d", [2, 3, 4, 5])
def test_tr_boundary_rank1_equals_tt(d):
    rng = np.random.default_rng(10 + d)
    ms = [2, 3, 2, 2, 3][:d]
    ns = [3, 2, 2, 3, 2][:d]
    rs = [1] + [3, 2, 4, 3][: d - 1] + [1]
    cores = _cores(rng, ms, ns, rs)
    np.testing.assert_allclose(O.tr_dense(cores), O.tt_dense(cores), atol=1e-13)


# ---- 2b. TR entry = trace of the product of core slices, entry by entry ------
def test_tr_entries_are_traces_of_matrix_products():
    rng = np.random.default_rng(3)
    ms, ns, rs = (2, 3, 2), (3, 2, 2), (3, 2, 4, 3)
    cores = _cores(rng, ms, ns, rs)
    w = O.tr_dense(cores)
    for i in [(0, 0, 0), (1, 2, 1), (0, 1, 1), (1, 0, 0)]:
        for j in [(0, 0, 0), (2, 1, 1), (1, 0, 1)]:
            mat = np.eye(rs[0])
            for k in range(3):
                mat = mat @ cores[k][:, i[k], j[k], :]
            fi = np.ravel_multi_index(i, ms)
            fj = np.ravel_multi_index(j, ns)
            assert abs(w[fi, fj] - np.trace(mat)) < 1e-12


def test_tt_entries_are_matrix_products():
    rng = np.random.default_rng(4)
    ms, ns, rs = (2, 3, 2, 2), (3, 2, 2, 3), (1, 3, 2, 4, 1)
    cores = _cores(rng, ms, ns, rs)
    w = O.tt_dense(cores)
    for i in [(0, 0, 0, 0), (1, 2, 1, 1), (0, 1, 1, 0)]:
        for j in [(0, 0, 0, 0), (2, 1, 1, 2), (1, 0, 1, 1)]:
            mat = np.eye(1)
            for k in range(4):
                mat = mat @ cores[k][:, i[k], j[k], :]
            assert abs(w[np.ravel_multi_index(i, ms), np.ravel_multi_index(j, ns)] - mat[0, 0]) < 1e-12


def test_tr_single_core_is_partial_trace():
    rng = np.random.default_rng(5)
    g = rng.standard_normal((3, 4, 5, 3))
    w = O.tr_dense([g])
    ref = sum(g[a, :, :, a] for a in range(3))
    np.testing.assert_allclose(w, ref, atol=1e-14)


# ---- 3. Tucker special cases ---------------------------------------------------
def test_tucker_identity_factors_return_core():
    rng = np.random.default_rng(6)
    core = rng.standard_normal((3, 4, 2, 5))
    us = [np.eye(3), np.eye(4)]
    vs = [np.eye(2), np.eye(5)]
    w = O.tucker_dense(core, us, vs)
    np.testing.assert_array_equal(w, core.reshape(12, 10))


def test_tucker_one_mode_per_side_is_u_c_vt():
    rng = np.random.default_rng(7)
    c = rng.standard_normal((3, 4))
    u = rng.standard_normal((6, 3))
    v = rng.standard_normal((5, 4))
    np.testing.assert_allclose(O.tucker_dense(c, [u], [v]), u @ c @ v.T, atol=1e-13)


def test_tucker_is_kron_factor_sandwich():
    # W = (U1 kron U2) C_mat (V1 kron V2)^T for C-order flattening
    rng = np.random.default_rng(8)
    core = rng.standard_normal((2, 3, 2, 2))
    u1, u2 = rng.standard_normal((4, 2)), rng.standard_normal((3, 3))
    v1, v2 = rng.standard_normal((3, 2)), rng.standard_normal((5, 2))
    ref = np.kron(u1, u2) @ core.reshape(6, 4) @ np.kron(v1, v2).T
    np.testing.assert_allclose(O.tucker_dense(core, [u1, u2], [v1, v2]), ref, atol=1e-12)


def test_tucker_orthonormal_factors_preserve_frobenius_norm():
    rng = np.random.default_rng(9)
    core = rng.standard_normal((3, 2, 2, 3))
    fs = [np.linalg.qr(rng.standard_normal(s))[0] for s in [(5, 3), (4, 2), (3, 2), (6, 3)]]
    w = O.tucker_dense(core, fs[:2], fs[2:])
    assert abs(np.linalg.norm(w) - np.linalg.norm(core)) < 1e-12


# ---- 4. untruncated TT-SVD round trip ------------------------------------------
@pytest.mark.parametrize("ms,ns", [((2, 3, 2), (3, 2, 2)), ((4, 2), (3, 5)), ((2, 2, 3, 2), (3, 2, 2, 2))])
def test_tt_svd_round_trip(ms, ns):
    rng = np.random.default_rng(11)
    w = rng.standard_normal((prod(ms), prod(ns)))
    cores = O.tt_svd(w, ms, ns)
    for k, g in enumerate(cores):
        assert g.shape[1] == ms[k] and g.shape[2] == ns[k]
    assert cores[0].shape[0] == 1 and cores[-1].shape[3] == 1
    assert np.max(np.abs(O.tt_dense(cores) - w)) < 1e-12


# ---- 5. nested-loop summation on tiny shapes ------------------------------------
def test_brute_force_tt():
    rng = np.random.default_rng(12)
    cores = _cores(rng, (2, 3, 2), (3, 2, 2), (1, 2, 3, 1))
    np.testing.assert_allclose(O.tt_dense(cores), O.brute_force_weight(TT, cores), atol=1e-13)


def test_brute_force_tr():
    rng = np.random.default_rng(13)
    cores = _cores(rng, (2, 3, 2), (3, 2, 2), (2, 2, 3, 2))
    np.testing.assert_allclose(O.tr_dense(cores), O.brute_force_weight(TR, cores), atol=1e-13)
    cores4 = _cores(rng, (2, 2, 2, 2), (2, 3, 2, 2), (2, 2, 2, 3, 2))
    np.testing.assert_allclose(O.tr_dense(cores4), O.brute_force_weight(TR, cores4), atol=1e-13)


def test_brute_force_tucker():
    rng = np.random.default_rng(14)
    core = rng.standard_normal((2, 3, 2, 2))
    ts = [core, rng.standard_normal((3, 2)), rng.standard_normal((4, 3)),
          rng.standard_normal((3, 2)), rng.standard_normal((2, 2))]
    np.testing.assert_allclose(O.dense_weight(TUCKER, ts, 2), O.brute_force_weight(TUCKER, ts, 2), atol=1e-13)
    # three out modes, one in mode (the paper's "3-way reshaping" flavour)
    core = rng.standard_normal((2, 2, 2, 3))
    ts = [core, rng.standard_normal((3, 2)), rng.standard_normal((2, 2)), rng.standard_normal((2, 2)),
          rng.standard_normal((4, 3))]
    np.testing.assert_allclose(O.dense_weight(TUCKER, ts, 3), O.brute_force_weight(TUCKER, ts, 3), atol=1e-13)


# ---- 6. gauge invariance on every bond, ring bond included ------------------------
@pytest.mark.parametrize("fmt", [TT, TR])
def test_gauge_invariance(fmt):
    rng = np.random.default_rng(15)
    rs = (1, 3, 2, 1) if fmt == TT else (3, 3, 2, 3)
    cores = _cores(rng, (2, 3, 2), (3, 2, 2), rs)
    w0 = O.dense_weight(fmt, cores)
    d = len(cores)
    bonds = range(1, d) if fmt == TT else range(0, d)
    for b in bonds:
        r = rs[b]
        a = rng.standard_normal((r, r)) + 3 * np.eye(r)
        ainv = np.linalg.inv(a)
        mod = [g.copy() for g in cores]
        left = (b - 1) % d
        right = b % d
        mod[left] = np.einsum("amnb,bc->amnc", mod[left], a)
        mod[right] = np.einsum("ab,bmnc->amnc", ainv, mod[right])
        np.testing.assert_allclose(O.dense_weight(fmt, mod), w0, atol=1e-10)


# ---- 6b. rotating a ring by one core permutes the digits of W accordingly ------
def test_tr_cyclic_rotation():
    rng = np.random.default_rng(16)
    ms, ns, rs = (2, 3, 2), (3, 2, 2), (2, 3, 2, 2)
    cores = _cores(rng, ms, ns, rs)
    w = O.tr_dense(cores).reshape(*ms, *ns)
    rot = cores[1:] + cores[:1]
    w_rot = O.tr_dense(rot).reshape(ms[1], ms[2], ms[0], ns[1], ns[2], ns[0])
    np.testing.assert_allclose(w_rot, w.transpose(1, 2, 0, 4, 5, 3), atol=1e-12)


# ---- 7. closed-form statistics of the synthetic workloads ---------------------------
def test_tt_qproj_statistics():
    spec, _ = wl.baseline_spec(1)
    cores = wl.make_tensors(spec, 1)
    w = O.dense_weight(spec.format, cores)
    assert w.shape == (8192, 5120)
    # Var(W_ij) = prod_{k<d} r_k * prod_k sigma_k^2 = 1/N, so ||W||_F^2 ~ M
    assert abs(np.sum(w * w) / spec.M - 1.0) < 0.1
    x = wl.make_x(spec, 8, 1)
    y = O.apply_linear(w, x)
    assert abs(y.var() - 1.0) < 0.1


def test_tucker_upproj_statistics():
    spec, _ = wl.baseline_spec(2)
    ts = wl.make_tensors(spec, 2)
    for f in ts[1:]:
        assert np.max(np.abs(f.T @ f - np.eye(f.shape[1]))) < 2e-2      # bf16-rounded orthonormal
    w = O.dense_weight(spec.format, ts, 2)
    assert w.shape == (25600, 5120)
    # orthonormal factors keep ||W||_F = ||C||_F and every core row has unit norm
    assert abs(np.sum(w * w) / (96 * 96) - 1.0) < 2e-2


def test_tr_downproj_statistics():
    spec, _ = wl.baseline_spec(3)
    cores = wl.make_tensors(spec, 3)
    w = O.dense_weight(spec.format, cores)
    assert w.shape == (5120, 25600)
    assert abs(np.sum(w * w) / spec.M - 1.0) < 0.1
    x = wl.make_x(spec, 4, 3)
    assert abs(O.apply_linear(w, x).var() - 1.0) < 0.15


# ---- 8. contracting the activations core by core equals rebuild-then-multiply ------
def _tt_chain_left_to_right(cores, x):
    """z[t, out digits so far, bond, remaining in digits] absorbed one core at a time."""
    t = x.shape[0]
    ns = [g.shape[2] for g in cores]
    z = x.reshape(t, 1, 1, *ns)                       # [t, I, a, n_1..n_d]
    for g in cores:
        # contract bond a and the leading remaining in-digit
        z = np.tensordot(z, g, axes=([2, 3], [0, 2]))  # [t, I, rest..., m_k, b]
        nd = z.ndim
        z = np.moveaxis(z, [nd - 2, nd - 1], [2, 3])   # [t, I, m_k, b, rest...]
        z = z.reshape(t, z.shape[1] * z.shape[2], z.shape[3], *z.shape[4:])
    return z.reshape(t, -1)


def _tt_chain_right_to_left(cores, x):
    t = x.shape[0]
    ns = [g.shape[2] for g in cores]
    z = x.reshape(t, *ns, 1, 1)                        # [t, n_1..n_k, b, Itail]
    for g in reversed(cores):
        k = z.ndim - 3                                  # axis of the last remaining in-digit
        z = np.tensordot(z, g, axes=([k, k + 1], [2, 3]))   # [t, rest..., Itail, a, m_k]
        nd = z.ndim
        z = np.moveaxis(z, [nd - 2, nd - 1], [nd - 3, nd - 2])   # [t, rest..., a, m_k, Itail]
        z = z.reshape(*z.shape[: nd - 2], z.shape[nd - 2] * z.shape[nd - 1])
    return z.reshape(t, -1)


def test_chain_equals_rebuild():
    rng = np.random.default_rng(17)
    ms, ns, rs = (2, 3, 2, 3), (3, 2, 4, 2), (1, 3, 4, 2, 1)
    cores = _cores(rng, ms, ns, rs)
    x = rng.standard_normal((5, prod(ns)))
    y = O.forward(TT, cores, x)
    np.testing.assert_allclose(_tt_chain_left_to_right(cores, x), y, atol=1e-12)
    np.testing.assert_allclose(_tt_chain_right_to_left(cores, x), y, atol=1e-12)


# ---- 9. d = 1 TT is a dense layer; linearity; token independence --------------------
def test_single_core_tt_is_dense():
    rng = np.random.default_rng(18)
    w = rng.standard_normal((7, 5))
    x = rng.standard_normal((3, 5))
    np.testing.assert_allclose(O.forward(TT, [w.reshape(1, 7, 5, 1)], x), x @ w.T, atol=1e-14)
    np.testing.assert_allclose(O.forward(DENSE, [w], x), x @ w.T, atol=1e-14)


def test_token_independence():
    spec, _ = wl.baseline_spec(0)
    cores = wl.make_tensors(spec, 0)
    x = wl.make_x(spec, 16, 0)
    y = O.forward(spec.format, cores, x)
    y3 = O.forward(spec.format, cores, x[3:4])
    np.testing.assert_allclose(y[3:4], y3, atol=1e-13)


# ---- 10. parameter counts of the four single-layer workloads ----------------------
def test_parameter_counts():
    expect = {0: 4736, 1: 925696, 2: 21271296, 3: 458752}
    for i, n in expect.items():
        spec, _ = wl.baseline_spec(i)
        assert spec.n_params == n


# ---- a planted mistake must be caught: little-endian digits fail the Kronecker pin ---
def test_planted_digit_order_mistake_is_detected():
    rng = np.random.default_rng(19)
    ms, ns = (3, 4), (2, 5)
    cores = _cores(rng, ms, ns, (1, 1, 1))
    wrong = O.tt_dense(cores[::-1])          # digits in the wrong significance order
    k = np.kron(cores[0][0, :, :, 0], cores[1][0, :, :, 0])
    assert np.max(np.abs(wrong - k)) > 1e-3


def test_rel_max_err():
    a = np.array([[1.0, -2.0], [0.5, 4.0]])
    b = a + np.array([[0.0, 0.0], [0.0, 0.04]])
    assert abs(O.rel_max_err(b, a) - 0.01) < 1e-15
    assert O.rel_max_err(np.zeros((0, 3)), np.zeros((0, 3))) == 0.0


# ---- row-sampled ring rebuild: per-entry traces, brute force, ring of one core, boundary rank 1 ----
def test_tr_rows_entries_are_traces_of_matrix_products():
    rng = np.random.default_rng(21)
    ms, ns, rs = (2, 3, 2, 3), (3, 2, 4, 2), (3, 2, 4, 2, 3)      # non-square modes, unequal bonds
    cores = _cores(rng, ms, ns, rs)
    rows = [0, 7, 17, 35, 20]
    w = O.tr_dense_rows(cores, rows)
    assert w.shape == (5, prod(ns))
    for n, fi in enumerate(rows):
        i = np.unravel_index(fi, ms)
        for fj in (0, 5, 13, 47, 30):
            j = np.unravel_index(fj, ns)
            mat = np.eye(rs[0])
            for k in range(4):
                mat = mat @ cores[k][:, i[k], j[k], :]
            assert abs(w[n, fj] - np.trace(mat)) < 1e-12


@pytest.mark.parametrize("d", [1, 2, 3, 5])
def test_tr_rows_brute_force_and_train(d):
    rng = np.random.default_rng(30 + d)
    ms = [2, 3, 2, 2, 2][:d]
    ns = [3, 2, 2, 3, 2][:d]
    rs = ([2] + [3, 2, 2, 3][: d - 1] + [2]) if d > 1 else [3, 3]
    cores = _cores(rng, ms, ns, rs)
    rows = list(range(prod(ms)))[::-1]                              # every row, in reverse order
    brute = O.brute_force_weight(TR, cores)
    np.testing.assert_allclose(O.tr_dense_rows(cores, rows), brute[rows], atol=1e-12)
    # boundary rank 1: the ring is a train, whose rows the Kronecker-pinned tt_dense gives
    rs1 = [1] + rs[1:-1] + [1]
    train = _cores(rng, ms, ns, rs1)
    np.testing.assert_allclose(O.tr_dense_rows(train, rows[:3]), O.tt_dense(train)[rows[:3]], atol=1e-12)


def test_planted_row_digit_mistake_is_detected():
    """A little-endian reading of the sampled row's digits must not pass the trace pin."""
    rng = np.random.default_rng(33)
    ms, ns, rs = (2, 3), (3, 2), (2, 3, 2)
    cores = _cores(rng, ms, ns, rs)
    fi = 1                                                          # digits (0, 1); little-endian would read (1, 0)
    wrong = np.trace(cores[0][:, 1, 0, :] @ cores[1][:, 0, 0, :])
    assert abs(O.tr_dense_rows(cores, [fi])[0, 0] - wrong) > 1e-6


# ---- a dense matrix handed over as a single core [1, M, N, 1] --------------------------------
def test_dense_weight_accepts_a_single_core():
    rng = np.random.default_rng(34)
    w = rng.standard_normal((5, 7))                                 # non-square: a transposed reshape fails
    np.testing.assert_array_equal(O.dense_weight(DENSE, [w.reshape(1, 5, 7, 1)]), w)
    np.testing.assert_array_equal(O.dense_weight(DENSE, [w.reshape(1, 5, 7, 1)]), O.tt_dense([w.reshape(1, 5, 7, 1)]))
    x = rng.standard_normal((3, 7))
    np.testing.assert_allclose(O.forward(DENSE, [w.reshape(1, 5, 7, 1)], x), x @ w.T, atol=1e-13)


# ---- parameter gradients: the loss is linear in each tensor alone, so an entry of the gradient is the loss with
#      that tensor replaced by the unit tensor of the entry; plus central differences and the dense closed form ----
GRAD_CASES = [
    (TT, (2, 3, 2), (3, 2, 2), (1, 2, 3, 1), None),
    (TT, (3,), (4,), (1, 1), None),
    (TR, (2, 3, 2), (3, 2, 2), (2, 3, 2, 2), None),
    (TR, (2, 2), (3, 2), (3, 2, 3), None),
    (TR, (3,), (4,), (2, 2), None),                       # a ring of one core: the bond is traced inside the tensor
    (TUCKER, (3, 2), (2, 4), (2, 2, 2, 3), 2),
    (TUCKER, (3, 2, 2), (5,), (2, 2, 1, 3), 3),
    (DENSE, (5,), (7,), (), None),
]


def _loss(fmt, ts, x, dy, p):
    return float(np.sum(dy * O.forward(fmt, ts, x, n_out_modes=p)))


@pytest.mark.parametrize("fmt,ms,ns,rs,p", GRAD_CASES)
def test_param_gradients_equal_the_loss_on_unit_tensors(fmt, ms, ns, rs, p):
    rng = np.random.default_rng(50 + len(ms) + 7 * fmt)
    spec = wl.TNSpec(fmt, "f32", tuple(ms), tuple(ns), tuple(rs))
    ts = [rng.standard_normal(s) for s in spec.tensor_shapes()]
    x = rng.standard_normal((4, spec.N))
    dy = rng.standard_normal((4, spec.M))
    grads = O.param_gradients(fmt, ts, x, dy, n_out_modes=p)
    assert [g.shape for g in grads] == [t.shape for t in ts]
    for k, t in enumerate(ts):
        for e in range(t.size):
            unit = np.zeros(t.size)
            unit[e] = 1.0
            probe = list(ts)
            probe[k] = unit.reshape(t.shape)
            assert abs(grads[k].reshape(-1)[e] - _loss(fmt, probe, x, dy, p)) < 1e-10, (k, e)


@pytest.mark.parametrize("fmt,ms,ns,rs,p", GRAD_CASES[:6])
def test_param_gradients_match_central_differences(fmt, ms, ns, rs, p):
    rng = np.random.default_rng(60 + len(ms) + 7 * fmt)
    spec = wl.TNSpec(fmt, "f32", tuple(ms), tuple(ns), tuple(rs))
    ts = [rng.standard_normal(s) for s in spec.tensor_shapes()]
    x = rng.standard_normal((3, spec.N))
    dy = rng.standard_normal((3, spec.M))
    grads = O.param_gradients(fmt, ts, x, dy, n_out_modes=p)
    h = 1e-5
    for k, t in enumerate(ts):
        for e in rng.choice(t.size, size=min(t.size, 6), replace=False):
            up, dn = [a.copy() for a in ts], [a.copy() for a in ts]
            up[k].reshape(-1)[e] += h
            dn[k].reshape(-1)[e] -= h
            fd = (_loss(fmt, up, x, dy, p) - _loss(fmt, dn, x, dy, p)) / (2 * h)
            assert abs(fd - grads[k].reshape(-1)[e]) < 1e-6 * max(1.0, abs(fd))


def test_param_gradient_of_a_dense_layer_is_dyT_x():
    rng = np.random.default_rng(70)
    w, x, dy = rng.standard_normal((5, 7)), rng.standard_normal((4, 7)), rng.standard_normal((4, 5))
    np.testing.assert_allclose(O.param_gradients(DENSE, [w], x, dy)[0], dy.T @ x, atol=1e-13)
    # and the gradients are linear in dY and additive over tokens
    ts = _cores(rng, (2, 3), (3, 2), (1, 2, 1))
    x, dy = rng.standard_normal((6, 6)), rng.standard_normal((6, 6))
    whole = O.param_gradients(TT, ts, x, dy)
    parts = [O.param_gradients(TT, ts, x[a:b], dy[a:b]) for a, b in ((0, 2), (2, 6))]
    for k in range(2):
        np.testing.assert_allclose(whole[k], parts[0][k] + parts[1][k], atol=1e-12)


# ---- MXFP4 quantiser: against the format's bit-field definition by brute force, plus invariants ------------------
def _e2m1_values():
    """The 16 values of a 4-bit E2M1 code from its fields: sign, 2 exponent bits (bias 1), 1 mantissa bit."""
    vals = []
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        mag = (m / 2.0) if e == 0 else (1.0 + m / 2.0) * 2.0 ** (e - 1)
        vals.append(-mag if s else mag)
    return np.array(vals)


def test_mxfp4_codes_are_nearest_e2m1_values_ties_to_even():
    rng = np.random.default_rng(80)
    vals = _e2m1_values()
    # one block whose maximum is exactly 4 * 2^e pins the scale to 2^e... use 7.5 (scale 1: floor(log2 7.5) - 2 = 0)
    probes = np.concatenate([rng.uniform(-7.4, 7.4, 1000), [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -2.5, -5.0, 0.0,
                                                            6.0, 6.9, -6.9, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0]])
    for start in range(0, probes.size, 31):
        chunk = np.concatenate([probes[start:start + 31], [7.5]])          # amax 7.5 -> X = 1
        codes, e, deq = O.mxfp4_quantize(chunk)
        assert e.tolist() == [0]
        for v, c, d in zip(chunk, codes, deq):
            mags = np.abs(vals[:8])
            dist = np.abs(abs(v) - mags)
            best = np.flatnonzero(dist == dist.min())
            want = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]     # tie: even mantissa bit
            assert (c & 7) == want, (v, c)
            assert d == (np.sign(v) if want else 1.0) * mags[want] or (want == 0 and d == 0)
            assert (c >> 3) == (1 if (v < 0 and want) else 0)


def test_mxfp4_scale_and_invariants():
    rng = np.random.default_rng(81)
    t = rng.standard_normal((7, 45)) * np.exp2(rng.integers(-20, 20, size=(7, 1)))      # 315 elements: a short last block
    codes, e, deq = O.mxfp4_quantize(t)
    assert codes.shape == (315,) and e.shape == (10,) and deq.shape == t.shape
    flat = np.abs(t).reshape(-1)
    for b in range(10):
        amax = flat[32 * b:32 * b + 32].max()
        x = 2.0 ** int(e[b])
        assert amax / 8 < x <= amax / 4                                    # amax / X in [4, 8)
        assert np.all(np.abs(deq.reshape(-1)[32 * b:32 * b + 32]) <= 6 * x)
        assert np.max(np.abs(deq.reshape(-1)[32 * b:32 * b + 32] - t.reshape(-1)[32 * b:32 * b + 32])) <= 2 * x
    # quantising what was dequantised changes nothing
    c2, e2, d2 = O.mxfp4_quantize(deq)
    np.testing.assert_array_equal(d2, deq)
    # zero blocks and the dequantised values are exact in bf16 (three significant bits)
    cz, ez, dz = O.mxfp4_quantize(np.zeros(40))
    assert not cz.any() and ez.tolist() == [-127, -127] and not dz.any()
    np.testing.assert_array_equal(wl.round_to_dtype(deq, "bf16"), deq)
    assert [a.shape for a in O.mxfp4_dequantized([t, t[:2]])] == [(7, 45), (2, 45)]
