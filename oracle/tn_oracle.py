"""Plain fp64 oracle for y = W x with W held as tensor-network factors.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product path, and it imports nothing
from the HIP library.

What is computed. The paper's Stage 2 (Section 3.3) stores weight matrices as
Tucker, tensor-train (TT) or tensor-ring (TR) factors and Stage 4 (Section 3.5)
applies them to activations; the paper names the three formats without writing
their formulas, so the standard definitions are used (every such reading is
listed in the design notes). The factorised forward is a re-association of one
exact sum, so the oracle is that sum written out: rebuild the dense W from the
factors by full contraction, then one matrix product Y = X W^T.

Conventions (all arrays float64, row-major):
  * W is [M, N] = [out, in]; X is [T, N]; Y is [T, M]; no bias.
  * flat index <-> mode multi-index is C order, first mode most significant:
    i = ((i_1 m_2 + i_2) m_3 + i_3)..., the same as ndarray.reshape.
  * TT / TR core k is G_k[r_{k-1}, m_k, n_k, r_k].
      TT: r_0 = r_d = 1, W[i, j] = G_1[:, i_1, j_1, :] ... G_d[:, i_d, j_d, :]
      TR: r_0 = r_d = r, W[i, j] = trace of the same matrix product
  * Tucker: core C[R_1..R_p, S_1..S_q], out factors U_a[m_a, R_a], in factors
    V_b[n_b, S_b],
      W[(i_1..i_p), (j_1..j_q)] = sum_{a, c} C[a, c] prod_a U_a[i_a, a_a] prod_b V_b[j_b, c_b]
  * dense: W given directly.

Pins (tests/test_oracle_pins.py): rank-1 TT equals the Kronecker product of its
cores; TR with boundary rank 1 equals TT; Tucker with identity factors returns
the core and with one mode per side equals U C V^T; untruncated TT-SVD of a
random matrix rebuilds it to 1e-12; the nested-loop evaluator below agrees on
tiny shapes; gauge invariance on every bond including the ring bond; cyclic
rotation of a ring; closed-form output variance and Frobenius norms; a stepwise
chain contraction of the activations agrees with rebuild-then-multiply; the
row-sampled ring rebuild (tr_dense_rows) agrees entry by entry with traces of
matrix products taken with numpy and with the nested-loop evaluator; a dense
weight handed over as a [1, M, N, 1] core equals the plain matrix; the parameter
gradients (param_gradients) equal, entry by entry, the loss evaluated with that
tensor replaced by a unit tensor (the loss is linear in each tensor alone), and
central finite differences of the loss; the MXFP4 quantiser (mxfp4_quantize)
agrees with a brute-force nearest-value search over the code table built from the
E2M1 bit fields, is idempotent, and keeps the block scale within (amax/8, amax/4].
"""
from __future__ import annotations

from itertools import product as _iproduct
from math import prod
from typing import List, Sequence

import numpy as np

FORMAT_DENSE, FORMAT_TT, FORMAT_TR, FORMAT_TUCKER = 0, 1, 2, 3


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def tt_dense(cores: Sequence[np.ndarray]) -> np.ndarray:
    """Dense [M, N] matrix of a TT-matrix (Section 3.3, tensor-train item).

    P_1 = G_1[0] as [m_1, n_1, r_1]; absorbing core k appends i_k and j_k as the
    least significant out and in digits:
    P_k[(i,i_k), (j,j_k), b] = sum_a P_{k-1}[i, j, a] G_k[a, i_k, j_k, b].
    """
    cores = [_f64(g) for g in cores]
    if cores[0].shape[0] != 1 or cores[-1].shape[3] != 1:
        raise ValueError("TT needs r_0 = r_d = 1")
    p = cores[0][0]                                    # [m1, n1, r1]
    for g in cores[1:]:
        if g.shape[0] != p.shape[2]:
            raise ValueError("bond mismatch")
        q = np.einsum("ija,akbs->ikjbs", p, g)          # [I, m_k, J, n_k, r_k]
        p = q.reshape(p.shape[0] * g.shape[1], p.shape[1] * g.shape[2], g.shape[3])
    return p[:, :, 0]


def _open_chain(cores: Sequence[np.ndarray]) -> np.ndarray:
    """Product of consecutive cores with both end bonds kept open:
    P[a, (i_1..i_h), (j_1..j_h), b], built by the TT recursion."""
    p = cores[0]
    for g in cores[1:]:
        if g.shape[0] != p.shape[3]:
            raise ValueError("bond mismatch")
        q = np.einsum("zija,akbs->zikjbs", p, g)
        p = q.reshape(p.shape[0], p.shape[1] * g.shape[1], p.shape[2] * g.shape[2], g.shape[3])
    return p


def tr_dense(cores: Sequence[np.ndarray]) -> np.ndarray:
    """Dense [M, N] matrix of a tensor ring (Section 3.3, tensor-ring item).

    W[i, j] = Tr(G_1[i_1, j_1] ... G_d[i_d, j_d]). The matrix product is split
    once, Tr(L R) with L the product of the first ceil(d/2) cores and R of the
    rest (each with both end bonds open), so that the largest temporary is W
    itself and not W times r^2; the trace is the sum over both shared bonds.
    """
    cores = [_f64(g) for g in cores]
    if cores[0].shape[0] != cores[-1].shape[3]:
        raise ValueError("TR needs r_0 = r_d")
    d = len(cores)
    if d == 1:
        return np.einsum("zijz->ij", cores[0])
    h = (d + 1) // 2
    left = _open_chain(cores[:h])                      # [z, I1, J1, b]
    right = _open_chain(cores[h:])                     # [b, I2, J2, z]
    z, i1, j1, b = left.shape
    _, i2, j2, _ = right.shape
    lm = left.transpose(1, 2, 0, 3).reshape(i1 * j1, z * b)           # [(I1 J1), (z b)]
    rm = right.transpose(3, 0, 1, 2).reshape(z * b, i2 * j2)          # [(z b), (I2 J2)]
    w4 = (lm @ rm).reshape(i1, j1, i2, j2)
    return np.ascontiguousarray(w4.transpose(0, 2, 1, 3)).reshape(i1 * i2, j1 * j2)


def tr_dense_rows(cores: Sequence[np.ndarray], rows: Sequence[int]) -> np.ndarray:
    """Rows W[rows, :] of a tensor ring (Section 3.3, tensor-ring item) without building all of W.

    For one flat out index i = (i_1..i_d) (C order) the cores are cut at their out digit,
    A_k = G_k[:, i_k, :, :] of shape [r_{k-1}, n_k, r_k], and W[i, j] = Tr(A_1[:, j_1, :] ... A_d[:, j_d, :]).
    The trace is taken as in tr_dense: the product is split once into the first ceil(d/2) and the remaining
    matrices, each half built over all of its in digits with both end bonds open, and the two shared
    bonds are summed. Cost per row 2 N r^2 instead of 2 M N r^2 for the whole matrix, which is what makes
    rank-96 rings of the 25600-wide projections checkable in seconds.
    """
    cores = [_f64(g) for g in cores]
    if cores[0].shape[0] != cores[-1].shape[3]:
        raise ValueError("TR needs r_0 = r_d")
    d = len(cores)
    ms = [g.shape[1] for g in cores]
    n_total = prod(g.shape[2] for g in cores)
    out = np.empty((len(rows), n_total))
    h = (d + 1) // 2
    for n, i in enumerate(rows):
        digits = np.unravel_index(int(i), ms)
        cut = [cores[k][:, digits[k], :, :] for k in range(d)]          # [r_{k-1}, n_k, r_k]
        if d == 1:
            out[n] = np.einsum("zjz->j", cut[0])
            continue

        def half(mats):
            p = mats[0]                                                  # [a, J, b]
            for g in mats[1:]:
                if g.shape[0] != p.shape[2]:
                    raise ValueError("bond mismatch")
                p = np.einsum("zja,aks->zjks", p, g).reshape(p.shape[0], p.shape[1] * g.shape[1], g.shape[2])
            return p

        left, right = half(cut[:h]), half(cut[h:])                       # [z, J1, b], [b, J2, z]
        z, j1, b = left.shape
        lm = left.transpose(1, 0, 2).reshape(j1, z * b)                  # [J1, (z b)]
        rm = right.transpose(2, 0, 1).reshape(z * b, right.shape[1])     # [(z b), J2]
        out[n] = (lm @ rm).reshape(-1)
    return out


def tucker_dense(core: np.ndarray, out_factors: Sequence[np.ndarray],
                 in_factors: Sequence[np.ndarray]) -> np.ndarray:
    """Dense [M, N] matrix of a Tucker-factorised weight (Section 3.3, Tucker item).

    Every core axis is multiplied by its factor matrix (mode product), out modes
    first; the result [m_1..m_p, n_1..n_q] is flattened to [M, N] in C order.
    """
    w = _f64(core)
    factors = [_f64(f) for f in list(out_factors) + list(in_factors)]
    if w.ndim != len(factors):
        raise ValueError("one factor per core axis")
    for axis, f in enumerate(factors):
        if f.shape[1] != w.shape[axis]:
            raise ValueError("factor/core rank mismatch")
        w = np.moveaxis(np.tensordot(f, w, axes=([1], [axis])), 0, axis)
    p = len(out_factors)
    return w.reshape(prod(w.shape[:p]), prod(w.shape[p:]))


def dense_weight(fmt: int, tensors: Sequence[np.ndarray], n_out_modes: int | None = None) -> np.ndarray:
    """Dense W for any format from tensors in canonical ABI order."""
    if fmt == FORMAT_DENSE:
        w = _f64(tensors[0])
        return w.reshape(w.shape[-3], w.shape[-2]) if w.ndim == 4 else w
    if fmt == FORMAT_TT:
        return tt_dense(tensors)
    if fmt == FORMAT_TR:
        return tr_dense(tensors)
    if fmt == FORMAT_TUCKER:
        if n_out_modes is None:
            raise ValueError("Tucker needs the number of out modes")
        p = n_out_modes
        return tucker_dense(tensors[0], tensors[1:1 + p], tensors[1 + p:])
    raise ValueError("unknown format")


def apply_linear(w: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Y[t, i] = sum_j W[i, j] X[t, j] in float64."""
    return _f64(x) @ _f64(w).T


def forward(fmt: int, tensors: Sequence[np.ndarray], x: np.ndarray,
            n_out_modes: int | None = None) -> np.ndarray:
    """Rebuild W, then multiply: the reference result for one layer."""
    return apply_linear(dense_weight(fmt, tensors, n_out_modes), x)


def _network_labels(fmt: int, tensors: Sequence[np.ndarray], n_out_modes: int | None):
    """The layer as a labelled tensor network: (labels of every tensor, out-mode labels, in-mode labels), integer
    labels, such that W[out..., in...] = sum over every other label of the product of the tensors."""
    if fmt == FORMAT_DENSE:
        return [[0, 1]], [0], [1]
    if fmt in (FORMAT_TT, FORMAT_TR):
        d = len(tensors)
        out = list(range(d))
        inn = list(range(d, 2 * d))
        bond = list(range(2 * d, 3 * d + 1))
        bond[d] = bond[0]                            # the ring bond: one label, two owners (a train is a ring of boundary rank 1)
        return [[bond[k], out[k], inn[k], bond[k + 1]] for k in range(d)], out, inn
    if fmt == FORMAT_TUCKER:
        p = n_out_modes
        q = len(tensors) - 1 - p
        out = list(range(p))
        inn = list(range(p, p + q))
        ranks = list(range(p + q, 2 * (p + q)))
        labels = [ranks]
        labels += [[out[a], ranks[a]] for a in range(p)]
        labels += [[inn[b], ranks[p + b]] for b in range(q)]
        return labels, out, inn
    raise ValueError("unknown format")


def param_gradients(fmt: int, tensors: Sequence[np.ndarray], x: np.ndarray, dy: np.ndarray,
                    n_out_modes: int | None = None) -> List[np.ndarray]:
    """Gradients of L = sum_{t,i} dY[t,i] Y[t,i], Y = X W^T, with respect to every parameter tensor (what the
    fine-tuning of the factors, Section 3.4, back-propagates), each in its tensor's own shape.

    dL/dW = D = dY^T X. W is linear in each tensor taken alone, so dL/dtheta_k is the network of W with theta_k
    taken out and D put in over the out- and in-mode labels: one einsum per tensor, written from the definitions
    of the formats (Section 3.3) and not from the chain the GPU walks. A ring of one core carries its bond label
    twice: its gradient is D on the diagonal of the two bond axes.
    """
    ts = [_f64(t) for t in tensors]
    d_w = _f64(dy).T @ _f64(x)                                            # [M, N]
    if fmt == FORMAT_DENSE:
        return [d_w.reshape(ts[0].shape)]
    labels, out, inn = _network_labels(fmt, ts, n_out_modes)
    if fmt in (FORMAT_TT, FORMAT_TR) and len(ts) == 1:
        r, m, n, _ = ts[0].shape
        g = np.zeros_like(ts[0])
        for a in range(r):
            g[a, :, :, a] = d_w
        return [g]
    if fmt in (FORMAT_TT, FORMAT_TR):
        ms = [t.shape[1] for t in ts]
        ns = [t.shape[2] for t in ts]
    else:
        p = n_out_modes
        ms = [u.shape[0] for u in ts[1:1 + p]]
        ns = [v.shape[0] for v in ts[1 + p:]]
    d_t = d_w.reshape(*ms, *ns)
    grads = []
    for k in range(len(ts)):
        operands = [d_t, out + inn]
        for l in range(len(ts)):
            if l != k:
                operands += [ts[l], labels[l]]
        g = np.einsum(*operands, labels[k], optimize="greedy")
        grads.append(np.ascontiguousarray(g))
    return grads


# ---- 4-bit quantisation of the parameter tensors (Section 6 names 4-bit quantisation of the cores as the next
#      step and gives no scheme; the reading taken is the OCP microscaling format MXFP4, weight-only) -------------
MX_BLOCK = 32
# the eight magnitudes an E2M1 code (2 exponent bits with bias 1, 1 mantissa bit) can take, in code order
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def mxfp4_quantize(t: np.ndarray):
    """MXFP4 quantisation of one tensor: (codes, scale exponents, dequantised tensor).

    The tensor is cut into blocks of 32 consecutive elements of its row-major flattening (the last block may be
    shorter). A block shares the scale X = 2^(floor(log2(max|v|)) - 2), clamped to the E8M0 range 2^-127 .. 2^127
    (an all-zero block takes 2^-127); an element is v / X rounded to the nearest E2M1 value, ties to the value with
    an even mantissa bit, saturating at +-6. codes: uint8, bit 3 = sign, bits 0..2 = index into E2M1_GRID;
    exponents: int16, one per block; dequantised = sign * grid[code] * X, in the tensor's shape (float64, exact).
    """
    v = _f64(t).reshape(-1)
    n = v.size
    nb = (n + MX_BLOCK - 1) // MX_BLOCK
    pad = np.zeros(nb * MX_BLOCK)
    pad[:n] = v
    blocks = pad.reshape(nb, MX_BLOCK)
    amax = np.max(np.abs(blocks), axis=1)
    _, ex = np.frexp(amax)                              # amax = m * 2^ex, m in [0.5, 1): floor(log2 amax) = ex - 1
    e = np.where(amax > 0, ex - 1 - 2, -127)
    e = np.clip(e, -127, 127).astype(np.int16)
    q = np.abs(blocks) / np.exp2(e.astype(np.float64))[:, None]
    # nearest grid value; at a midpoint the neighbour whose mantissa bit is 0 (codes 0, 2, 4, 6)
    code = ((q > 0.25).astype(np.uint8) + (q >= 0.75) + (q > 1.25) + (q >= 1.75) + (q > 2.5) + (q >= 3.5) + (q > 5.0))
    code = code.astype(np.uint8)
    sign = (blocks < 0) & (code > 0)
    deq = np.where(sign, -1.0, 1.0) * E2M1_GRID[code] * np.exp2(e.astype(np.float64))[:, None]
    codes = (code | (sign.astype(np.uint8) << 3)).reshape(-1)[:n]
    return codes, e, deq.reshape(-1)[:n].reshape(np.shape(t))


def mxfp4_dequantized(tensors: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Every tensor replaced by its MXFP4 quantisation, dequantised: what a layer with 4-bit tensors applies."""
    return [mxfp4_quantize(t)[2] for t in tensors]


def brute_force_weight(fmt: int, tensors: Sequence[np.ndarray], n_out_modes: int | None = None) -> np.ndarray:
    """Second, independent evaluator: explicit loops over every index of the
    defining sum. Tiny shapes only (cost grows with the product of all extents)."""
    ts = [_f64(t) for t in tensors]
    if fmt in (FORMAT_TT, FORMAT_TR):
        d = len(ts)
        ms = [g.shape[1] for g in ts]
        ns = [g.shape[2] for g in ts]
        rs = [ts[0].shape[0]] + [g.shape[3] for g in ts]
        w = np.zeros((prod(ms), prod(ns)))
        for iflat, imulti in enumerate(_iproduct(*[range(m) for m in ms])):
            for jflat, jmulti in enumerate(_iproduct(*[range(n) for n in ns])):
                total = 0.0
                for bonds in _iproduct(*[range(r) for r in rs[:-1]]):
                    # bonds = (b_0 .. b_{d-1}); b_d equals b_0 (ring) or 0 (train)
                    last = bonds[0] if fmt == FORMAT_TR else 0
                    if fmt == FORMAT_TT and bonds[0] != 0:
                        continue
                    chain = list(bonds) + [last]
                    term = 1.0
                    for k in range(d):
                        term *= ts[k][chain[k], imulti[k], jmulti[k], chain[k + 1]]
                    total += term
                w[iflat, jflat] = total
        return w
    if fmt == FORMAT_TUCKER:
        p = n_out_modes
        core, us, vs = ts[0], ts[1:1 + p], ts[1 + p:]
        ms = [u.shape[0] for u in us]
        ns = [v.shape[0] for v in vs]
        w = np.zeros((prod(ms), prod(ns)))
        for iflat, imulti in enumerate(_iproduct(*[range(m) for m in ms])):
            for jflat, jmulti in enumerate(_iproduct(*[range(n) for n in ns])):
                total = 0.0
                for idx in _iproduct(*[range(r) for r in core.shape]):
                    term = core[idx]
                    for a in range(p):
                        term *= us[a][imulti[a], idx[a]]
                    for b in range(len(vs)):
                        term *= vs[b][jmulti[b], idx[p + b]]
                    total += term
                w[iflat, jflat] = total
        return w
    if fmt == FORMAT_DENSE:
        return _f64(ts[0]).copy()
    raise ValueError("unknown format")


def tt_svd(w: np.ndarray, out_modes: Sequence[int], in_modes: Sequence[int]) -> List[np.ndarray]:
    """Untruncated TT-SVD of a matrix into cores [r_{k-1}, m_k, n_k, r_k].

    Used only to pin tt_dense: W[M, N] -> [m_1..m_d, n_1..n_d] -> pair the modes
    as [(m_1 n_1), .., (m_d n_d)] -> sequential full-rank SVDs.
    """
    w = _f64(w)
    d = len(out_modes)
    t = w.reshape(*out_modes, *in_modes)
    perm = [ax for k in range(d) for ax in (k, d + k)]
    t = t.transpose(perm)
    cores = []
    r_prev = 1
    rest = t.reshape(1, -1)
    for k in range(d - 1):
        mk, nk = out_modes[k], in_modes[k]
        mat = rest.reshape(r_prev * mk * nk, -1)
        u, s, vt = np.linalg.svd(mat, full_matrices=False)
        r = u.shape[1]
        cores.append(u.reshape(r_prev, mk, nk, r))
        rest = s[:, None] * vt
        r_prev = r
    cores.append(rest.reshape(r_prev, out_modes[-1], in_modes[-1], 1))
    return cores


def rel_max_err(y: np.ndarray, y_ref: np.ndarray) -> float:
    """max|y - y_ref| / max|y_ref| over the whole output (the parity metric)."""
    y_ref = _f64(y_ref)
    denom = float(np.max(np.abs(y_ref))) if y_ref.size else 0.0
    if y_ref.size == 0:
        return 0.0
    num = float(np.max(np.abs(_f64(y) - y_ref)))
    return num / denom if denom > 0 else num
