"""Shapes, seeds and value distributions of the synthetic workloads.

The layers stand in for the projections of a 32B-parameter decoder (hidden
5120, query width 8192, key/value width 1024, MLP width 25600, 64 layers), the
model the paper's Table 1 is quoted on; the paper discloses no ranks, mode
factorisations or weights, so every value here is drawn from a seeded
generator.

Canonical tensor layouts (row-major), the ones the C ABI takes:
  * dense          one tensor  [M, N]
  * TT / TR        d cores     [r_{k-1}, m_k, n_k, r_k]
  * Tucker         core [R_1..R_p, S_1..S_q], then U_a [m_a, R_a] (a = 1..p),
                   then V_b [n_b, S_b] (b = 1..q)

Everything returned is a float64 numpy array whose values are exactly
representable in the spec's storage type (fp32 or bf16), so that the oracle and
the GPU receive identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import prod, sqrt
from typing import List, Sequence, Tuple

import numpy as np

FORMAT_DENSE = 0
FORMAT_TT = 1
FORMAT_TR = 2
FORMAT_TUCKER = 3
FORMAT_NAMES = {0: "dense", 1: "tt", 2: "tr", 3: "tucker"}

SEED_BASE = 260201613


@dataclass(frozen=True)
class TNSpec:
    """Structure of one tensor-network linear layer (no values)."""

    format: int
    dtype: str                      # "f32" or "bf16"
    out_modes: Tuple[int, ...]
    in_modes: Tuple[int, ...]
    ranks: Tuple[int, ...]          # TT/TR: r_0..r_d; Tucker: R_1..R_p,S_1..S_q; dense: ()
    name: str = ""

    @property
    def M(self) -> int:
        return prod(self.out_modes)

    @property
    def N(self) -> int:
        return prod(self.in_modes)

    def tensor_shapes(self) -> List[Tuple[int, ...]]:
        if self.format == FORMAT_DENSE:
            return [(self.M, self.N)]
        if self.format in (FORMAT_TT, FORMAT_TR):
            d = len(self.out_modes)
            return [(self.ranks[k], self.out_modes[k], self.in_modes[k], self.ranks[k + 1])
                    for k in range(d)]
        p, q = len(self.out_modes), len(self.in_modes)
        shapes = [tuple(self.ranks)]
        shapes += [(self.out_modes[a], self.ranks[a]) for a in range(p)]
        shapes += [(self.in_modes[b], self.ranks[p + b]) for b in range(q)]
        return shapes

    @property
    def n_params(self) -> int:
        return sum(prod(s) for s in self.tensor_shapes())


def bf16_bits(a32: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to fp32 or bf16 and return them as float64 again."""
    a32 = np.asarray(a, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return a32.astype(np.float64)
    if dtype == "bf16":
        bits = bf16_bits(a32).astype(np.uint32) << 16
        return bits.view(np.float32).reshape(a32.shape).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def _rng(config_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([SEED_BASE, int(config_id), int(tensor_id)]))


def _orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """Q of the reduced QR of a rows x cols Gaussian, signs fixed so diag(R) > 0."""
    if cols > rows:
        raise ValueError("an orthonormal factor needs rank <= mode size")
    g = rng.standard_normal((rows, cols))
    q, r = np.linalg.qr(g)
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return q * s[None, :]


def make_tensors(spec: TNSpec, config_id: int, instance: int = 0) -> List[np.ndarray]:
    """Draw the parameter tensors of one layer in canonical layout.

    TT/TR cores are N(0, sigma_k) with standard deviation
    sigma_k = (r_{k-1} n_k)^(-1/2); dense weights use sigma = N^(-1/2); Tucker
    factors are orthonormal and every [a_1..a_p, :, ...] slice of the core has
    unit Frobenius norm.
    """
    shapes = spec.tensor_shapes()
    base = 1000 * instance
    out = []
    if spec.format == FORMAT_DENSE:
        g = _rng(config_id, base).standard_normal(shapes[0]) / sqrt(spec.N)
        out.append(g)
    elif spec.format in (FORMAT_TT, FORMAT_TR):
        for k, shp in enumerate(shapes):
            sigma = 1.0 / sqrt(shp[0] * shp[2])
            out.append(_rng(config_id, base + k).standard_normal(shp) * sigma)
    elif spec.format == FORMAT_TUCKER:
        p = len(spec.out_modes)
        core = _rng(config_id, base).standard_normal(shapes[0])
        rows = prod(shapes[0][:p])
        flat = core.reshape(rows, -1)
        flat = flat / np.linalg.norm(flat, axis=1, keepdims=True)
        out.append(flat.reshape(shapes[0]))
        for i, shp in enumerate(shapes[1:]):
            out.append(_orthonormal(_rng(config_id, base + 1 + i), shp[0], shp[1]))
    else:
        raise ValueError("unknown format")
    return [round_to_dtype(t, spec.dtype) for t in out]


def make_x(spec: TNSpec, tokens: int, config_id: int, instance: int = 0) -> np.ndarray:
    """Activations [tokens, N], N(0,1), rounded to the spec's storage type."""
    g = _rng(config_id, 900 + 1000 * instance).standard_normal((tokens, spec.N))
    return round_to_dtype(g, spec.dtype)


def baseline_spec(i: int) -> Tuple[TNSpec, Tuple[int, ...]]:
    """The four single-layer workloads and the token counts each is run at."""
    if i == 0:
        return TNSpec(FORMAT_TT, "f32", (4, 8, 8), (4, 8, 8), (1, 8, 8, 1), "tt_small_f32"), (16,)
    if i == 1:
        return (TNSpec(FORMAT_TT, "bf16", (8, 16, 8, 8), (8, 10, 8, 8), (1, 64, 64, 64, 1), "tt_q_proj"),
                (1, 64, 8192))
    if i == 2:
        return (TNSpec(FORMAT_TUCKER, "bf16", (160, 160), (64, 80), (96, 96, 48, 48), "tucker_up_proj"),
                (1, 64, 8192))
    if i == 3:
        return (TNSpec(FORMAT_TR, "bf16", (8, 10, 8, 8), (10, 16, 10, 16), (32, 32, 32, 32, 32), "tr_down_proj"),
                (1, 64, 8192))
    raise ValueError("single-layer workloads are numbered 0..3")


# Mode factorisations used for the 64-layer stack.
_TT_MODES = {5120: (8, 10, 8, 8), 8192: (8, 16, 8, 8), 25600: (10, 16, 10, 16), 1024: (4, 8, 4, 8)}
_TUCKER_MODES = {5120: (64, 80), 25600: (160, 160), 8192: (64, 128), 1024: (32, 32)}
_STACK_PROJECTIONS = (
    ("q", 5120, 8192), ("k", 5120, 1024), ("v", 5120, 1024), ("o", 8192, 5120),
    ("gate", 5120, 25600), ("up", 5120, 25600), ("down", 25600, 5120),
)


def stack_spec(fmt: int, n_in: int, n_out: int, r: int, name: str = "") -> TNSpec:
    """One projection of the stack in the given format with drawn rank r."""
    if fmt == FORMAT_DENSE:
        return TNSpec(FORMAT_DENSE, "bf16", (n_out,), (n_in,), (), name)
    if fmt == FORMAT_TT:
        return TNSpec(FORMAT_TT, "bf16", _TT_MODES[n_out], _TT_MODES[n_in], (1, r, r, r, 1), name)
    if fmt == FORMAT_TR:
        return TNSpec(FORMAT_TR, "bf16", _TT_MODES[n_out], _TT_MODES[n_in], (r,) * 5, name)
    om, im = _TUCKER_MODES[n_out], _TUCKER_MODES[n_in]
    ranks = (min(r, om[0]), min(r, om[1]), min(r // 2, im[0]), min(r // 2, im[1]))
    return TNSpec(FORMAT_TUCKER, "bf16", om, im, ranks, name)


def qwen3_32b_stack(layers: int = 64) -> List[TNSpec]:
    """64 layers x 7 projections; format drawn i.i.d. from {dense 40 %, TT, TR,
    Tucker 20 % each} and rank from {32, 64, 96}, in (layer, q, k, v, o, gate,
    up, down) order from one seeded generator."""
    rng = _rng(4, 0)
    specs = []
    for layer in range(layers):
        for pname, n_in, n_out in _STACK_PROJECTIONS:
            u = rng.random()
            fmt = FORMAT_DENSE if u < 0.4 else FORMAT_TT if u < 0.6 else FORMAT_TR if u < 0.8 else FORMAT_TUCKER
            r = int(rng.choice([32, 64, 96]))
            specs.append(stack_spec(fmt, n_in, n_out, r, f"L{layer}.{pname}"))
    return specs
