"""Pins for the oracle's RoPE (Eq. 3) and its storage rounding, against things the
paper and the mathematics fix: closed forms, group properties, the complex-number
form of the rotation, and library conversions."""
import math

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(7)


def test_theta_closed_form():
    # text after Eq. 3: theta_m = 10000^(-2m/d); theta_0 = 1
    for base, d in [(1e4, 64), (1e6, 128), (5e5, 128), (1e4, 8)]:
        th = oracle.theta(base, d)
        assert th.shape == (d // 2,)
        assert th[0] == 1.0
        for m in range(d // 2):
            assert th[m] == pytest.approx(base ** (-2.0 * m / d), rel=1e-15)
        assert np.all(np.diff(th) < 0)
    assert np.allclose(oracle.theta(1e4, 8), [1.0, 0.1, 0.01, 0.001], rtol=1e-14)


def test_pair_zero_turns_by_exactly_p_radians():
    # theta_0 = 1, so the vector (1, 0) in pair 0 becomes (cos p, sin p); (0, 1) becomes (-sin p, cos p)
    d = 8
    for p in [0, 1, 2, 17, 1000, 32768]:
        x = np.zeros((1, 1, d)); x[0, 0, 0] = 1.0
        y = oracle.rope(x, [p], 1e4)
        assert y[0, 0, 0] == pytest.approx(math.cos(p), abs=1e-15)
        assert y[0, 0, 1] == pytest.approx(math.sin(p), abs=1e-15)
        x = np.zeros((1, 1, d)); x[0, 0, 1] = 1.0
        y = oracle.rope(x, [p], 1e4)
        assert y[0, 0, 0] == pytest.approx(-math.sin(p), abs=1e-15)
        assert y[0, 0, 1] == pytest.approx(math.cos(p), abs=1e-15)


def test_literal_eq3_two_term_form():
    # Eq. 3 as printed: q' = q (*) [cos t th_0, cos t th_0, ...] + [-q1, q0, -q3, q2, ...] (*) [sin ..]
    d, base = 16, 1e4
    x = RNG.standard_normal((5, 3, d))
    pos = np.array([0, 1, 5, 77, 4095])
    th = np.array([base ** (-2.0 * m / d) for m in range(d // 2)])
    swapped = np.empty_like(x)
    swapped[..., 0::2] = -x[..., 1::2]
    swapped[..., 1::2] = x[..., 0::2]
    ang = pos[:, None] * th[None, :]
    cos2 = np.repeat(np.cos(ang), 2, axis=1)[:, None, :]
    sin2 = np.repeat(np.sin(ang), 2, axis=1)[:, None, :]
    want = x * cos2 + swapped * sin2
    assert np.allclose(oracle.rope(x, pos, base), want, rtol=0, atol=1e-14)


def test_complex_multiplication_form():
    # interleaved RoPE == multiplying (x_2m + i x_2m+1) by exp(i p theta_m)
    d, base = 64, 1e6
    x = RNG.standard_normal((9, 2, d))
    pos = RNG.integers(0, 40000, 9)
    z = x[..., 0::2] + 1j * x[..., 1::2]
    th = base ** (-2.0 * np.arange(d // 2) / d)
    w = z * np.exp(1j * pos[:, None, None] * th[None, None, :])
    y = oracle.rope(x, pos, base)
    assert np.allclose(y[..., 0::2], w.real, atol=1e-12)
    assert np.allclose(y[..., 1::2], w.imag, atol=1e-12)


def test_group_properties():
    d, base = 32, 5e5
    x = RNG.standard_normal((6, 4, d))
    zero = np.zeros(6, np.int64)
    assert np.array_equal(oracle.rope(x, zero, base), x)                       # R(0) = I
    a = RNG.integers(0, 5000, 6); b = RNG.integers(0, 5000, 6)
    ya = oracle.rope(x, a, base)
    assert np.allclose(np.linalg.norm(ya, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)   # isometry
    assert np.allclose(oracle.rope(ya, b, base), oracle.rope(x, a + b, base), atol=1e-11)     # R(b)R(a) = R(a+b)
    assert np.allclose(oracle.rope(ya, -a, base), x, atol=1e-11)                                # R(p)^-1 = R(-p)


def test_relative_position_property():
    # Sec. 3.1: the product of the two position embeddings depends only on the position difference
    d, base = 128, 1e6
    q = RNG.standard_normal((20, 1, d)); k = RNG.standard_normal((20, 1, d))
    a = RNG.integers(0, 30000, 20); b = RNG.integers(0, 30000, 20)
    lhs = np.einsum("nhd,nhd->n", oracle.rope(q, a, base), oracle.rope(k, b, base))
    rhs = np.einsum("nhd,nhd->n", q, oracle.rope(k, b - a, base))
    assert np.allclose(lhs, rhs, atol=1e-9)
    shift = 12345
    lhs2 = np.einsum("nhd,nhd->n", oracle.rope(q, a + shift, base), oracle.rope(k, b + shift, base))
    assert np.allclose(lhs, lhs2, atol=1e-9)


def test_half_split_layout_is_a_channel_permutation_of_interleaved():
    d, base = 16, 1e4
    x = RNG.standard_normal((4, 2, d)); pos = np.array([3, 10, 200, 9999])
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])   # half[j] = inter[perm[j]]
    y_inter = oracle.rope(x, pos, base, oracle.ROPE_INTERLEAVED)
    y_half = oracle.rope(x[..., perm], pos, base, oracle.ROPE_HALF)
    assert np.allclose(y_half, y_inter[..., perm], atol=1e-14)


def test_rope_reads_storage_dtypes_exactly():
    d = 8
    xf = RNG.standard_normal((3, 2, d)).astype(np.float32)
    assert np.array_equal(oracle.rope(xf, [0, 0, 0], 1e4), xf.astype(np.float64))
    xb = torch.from_numpy(xf).to(torch.bfloat16)
    bits = xb.view(torch.uint16).numpy()
    assert np.array_equal(oracle.rope(bits, [0, 0, 0], 1e4), xb.to(torch.float64).numpy())
    assert np.array_equal(oracle.widen(bits), xb.to(torch.float64).numpy())


def test_bf16_rounding_matches_library_and_nearest_search():
    # (a) library routine: torch's float32 -> bfloat16 conversion on float32-representable inputs
    x32 = np.concatenate([RNG.standard_normal(20000).astype(np.float32) * 3,
                          np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-39])])
    want = torch.from_numpy(x32).to(torch.bfloat16).view(torch.uint16).numpy()
    got = oracle.round_to(x32.astype(np.float64), oracle.BF16)
    assert np.array_equal(got, want)
    # (b) ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 2 + 2.0 ** -7])
    got = oracle.widen(oracle.round_to(ties, oracle.BF16))
    assert np.array_equal(got, [1.0, 1 + 2.0 ** -6, -1.0, 2.0])
    # (c) brute force: the result is the closest bf16 among its neighbours, for doubles that are not float32s
    xs = RNG.standard_normal(300) * 2 + RNG.standard_normal(300) * 1e-9
    got = oracle.widen(oracle.round_to(xs, oracle.BF16))
    for x, g in zip(xs, got):
        bits = np.array([g], np.float32).view(np.uint32)[0] >> 16
        for nb in (bits - 1, bits + 1):
            cand = np.array([np.uint32(nb) << 16], np.uint32).view(np.float32)[0]
            assert abs(x - g) <= abs(x - float(cand))
    # (d) float32 target is the C cast
    assert np.array_equal(oracle.round_to(xs, oracle.F32), xs.astype(np.float32))
