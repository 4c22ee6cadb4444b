"""The seeded generators: rounding, shapes, determinism, the stack draw."""
import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -1e-40])])
    got = wl.round_to_dtype(a, "bf16")
    ref = torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(got, ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert wl.round_to_dtype(np.array([1.00390625]), "bf16")[0] == 1.0
    assert wl.round_to_dtype(np.array([1.01171875]), "bf16")[0] == 1.015625


def test_f32_rounding():
    a = np.array([0.1, 1.0 + 2.0 ** -30])
    np.testing.assert_array_equal(wl.round_to_dtype(a, "f32"), a.astype(np.float32).astype(np.float64))


def test_baseline_shapes_and_determinism():
    spec, toks = wl.baseline_spec(1)
    assert (spec.M, spec.N) == (8192, 5120) and toks == (1, 64, 8192)
    assert spec.tensor_shapes() == [(1, 8, 8, 64), (64, 16, 10, 64), (64, 8, 8, 64), (64, 8, 8, 1)]
    spec0, _ = wl.baseline_spec(0)
    a = wl.make_tensors(spec0, 0)
    b = wl.make_tensors(spec0, 0)
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)
    c = wl.make_tensors(spec0, 0, instance=1)
    assert not np.array_equal(a[1], c[1])
    # sigma_k = (r_{k-1} n_k)^(-1/2)
    assert abs(a[1].std() - 0.125) < 0.01
    spec2, _ = wl.baseline_spec(2)
    assert spec2.tensor_shapes() == [(96, 96, 48, 48), (160, 96), (160, 96), (64, 48), (80, 48)]
    spec3, _ = wl.baseline_spec(3)
    assert spec3.tensor_shapes()[1] == (32, 10, 16, 32)


def test_stack_draw():
    s1 = wl.qwen3_32b_stack()
    s2 = wl.qwen3_32b_stack()
    assert len(s1) == 448 and s1 == s2
    fmts = np.array([s.format for s in s1])
    frac_dense = (fmts == wl.FORMAT_DENSE).mean()
    assert 0.3 < frac_dense < 0.5
    for s in s1:
        assert s.N in (5120, 8192, 25600) and s.M in (8192, 1024, 5120, 25600)
        if s.format == wl.FORMAT_TUCKER:
            p = len(s.out_modes)
            for a in range(p):
                assert s.ranks[a] <= s.out_modes[a]
            for b in range(len(s.in_modes)):
                assert s.ranks[p + b] <= s.in_modes[b]
