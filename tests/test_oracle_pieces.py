"""Pins for the oracle's fp16 conversion, linear layer and element-wise pieces.

Each check compares the oracle with something it does not share code with: a
library routine (numpy float16, fp64 matmul), a closed form, or an invariant.
"""
import math

import numpy as np
import pytest

from paper_2505_23219_amd import workloads as wl


# ------------------------------------------------------------------ fp16 --
def test_half_to_float_all_bit_patterns(orc32):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([orc32.half_to_float(int(b)) for b in bits], dtype=np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(np.signbit(got), np.signbit(ref))


def test_float_to_half_rounds_to_nearest_even(orc32):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(5000) * 1e-5).astype(np.float32),       # subnormal range
        (rng.standard_normal(5000) * 3e4).astype(np.float32),        # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                  1.5 * 2.0 ** -25, 2.0 ** -14, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11],
                 dtype=np.float32),
    ])
    # ties: midpoints between adjacent fp16 values must go to the even mantissa
    h = np.arange(0x0001, 0x7bff, 37, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals = np.concatenate([vals, ((lo + hi) / 2).astype(np.float32)])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([orc32.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- linear --
@pytest.mark.parametrize("M,N,K", [(1, 7, 5), (3, 16, 33), (16, 64, 256), (64, 130, 688)])
def test_linear_matches_fp64_matmul(orc32, orc64, M, N, K):
    x = wl.activations(M, K, 11).numpy().astype(np.float32)
    W = wl.activations(N, K, 12, tag="w", std=0.02).numpy()
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    y64 = orc64.linear(x, W)
    y32 = orc32.linear(x, W)
    np.testing.assert_allclose(y64, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(y32, ref, rtol=0, atol=2e-5)


def test_linear_is_not_transposed_and_picks_rows(orc32):
    # one-hot weight rows copy single input columns: catches a swapped operand
    M, N, K = 4, 6, 9
    x = np.arange(M * K, dtype=np.float32).reshape(M, K)
    W = np.zeros((N, K), dtype=np.float16)
    cols = [3, 0, 8, 8, 1, 5]
    for n, c in enumerate(cols):
        W[n, c] = 1.0
    y = orc32.linear(x, W)
    assert np.array_equal(y, x[:, cols])


def test_linear_row_is_a_dot_product(orc32):
    x = wl.activations(1, 300, 5).numpy().astype(np.float32)
    W = wl.activations(1, 300, 6, tag="w").numpy()
    y = orc32.linear(x, W)
    ref = math.fsum(float(a) * float(b) for a, b in zip(x[0], W[0].astype(np.float32)))
    assert abs(float(y[0, 0]) - ref) < 1e-4


# --------------------------------------------------------------- rmsnorm --
def test_rmsnorm_unit_gain_gives_unit_rms(orc64):
    x = wl.activations(5, 256, 3).numpy().astype(np.float64) * 3.0
    g = np.ones(256, dtype=np.float16)
    out = orc64.rmsnorm(x, g, 0.0)
    np.testing.assert_allclose(np.sqrt((out ** 2).mean(axis=1)), 1.0, atol=1e-12)
    # direction unchanged
    np.testing.assert_allclose(out / np.linalg.norm(out, axis=1, keepdims=True),
                               x / np.linalg.norm(x, axis=1, keepdims=True), atol=1e-12)


def test_rmsnorm_gain_eps_and_scale(orc32, orc64):
    x = wl.activations(3, 64, 4).numpy().astype(np.float64)
    g = (1.0 + 0.25 * wl.activations(1, 64, 5, tag="g").numpy()[0]).astype(np.float16)
    # constant row c with gain g: out = g * c / sqrt(c^2 + eps)
    c = np.full((1, 64), 0.5)
    out = orc64.rmsnorm(c, g, 0.75)
    np.testing.assert_allclose(out[0], g.astype(np.float64) * 0.5 / math.sqrt(0.25 + 0.75),
                               atol=1e-12)
    # scaling the input by a power of two leaves the output unchanged when eps = 0
    np.testing.assert_allclose(orc64.rmsnorm(x * 4.0, g, 0.0), orc64.rmsnorm(x, g, 0.0), atol=1e-12)
    # and the fp32 build agrees with the fp64 one
    np.testing.assert_allclose(orc32.rmsnorm(x, g, 1e-6), orc64.rmsnorm(x, g, 1e-6), atol=2e-6)


# ------------------------------------------------------------------ rope --
def test_rope_position_zero_is_identity(orc64):
    t = wl.activations(4, 2 * 64, 8).numpy().astype(np.float64).reshape(4, 2, 64)
    out = orc64.rope(t, [0, 0, 0, 0], 10000.0)
    assert np.array_equal(out, t)


def test_rope_closed_form_on_basis_vectors(orc64):
    d, base = 8, 10000.0
    for j in range(d // 2):
        for pos in (1, 5, 1000):
            t = np.zeros((1, 1, d))
            t[0, 0, j] = 1.0
            out = orc64.rope(t, [pos], base)[0, 0]
            ang = pos * base ** (-2.0 * j / d)
            want = np.zeros(d)
            want[j], want[j + d // 2] = math.cos(ang), math.sin(ang)
            np.testing.assert_allclose(out, want, atol=1e-13)
            t = np.zeros((1, 1, d))
            t[0, 0, j + d // 2] = 1.0
            out = orc64.rope(t, [pos], base)[0, 0]
            want = np.zeros(d)
            want[j], want[j + d // 2] = -math.sin(ang), math.cos(ang)
            np.testing.assert_allclose(out, want, atol=1e-13)


def test_rope_preserves_pair_norms_and_relative_position(orc64):
    d = 64
    q = wl.activations(1, d, 1).numpy().astype(np.float64).reshape(1, 1, d)
    k = wl.activations(1, d, 2).numpy().astype(np.float64).reshape(1, 1, d)
    rq = orc64.rope(q, [17], 10000.0)
    pair = lambda v: v[0, 0, :d // 2] ** 2 + v[0, 0, d // 2:] ** 2
    np.testing.assert_allclose(pair(rq), pair(q), atol=1e-12)
    dots = []
    for m, n in ((9, 4), (105, 100), (2053, 2048)):
        dots.append(float((orc64.rope(q, [m], 10000.0) * orc64.rope(k, [n], 10000.0)).sum()))
    np.testing.assert_allclose(dots, dots[0], atol=1e-9)
    # heads rotate alike, rows use their own position
    t = np.concatenate([q, k], axis=1)          # [1, 2, d]
    out = orc64.rope(np.concatenate([t, t]), [3, 11], 10000.0)
    np.testing.assert_allclose(out[0, 0], orc64.rope(q, [3], 10000.0)[0, 0], atol=0)
    np.testing.assert_allclose(out[1, 1], orc64.rope(k, [11], 10000.0)[0, 0], atol=0)


# ---------------------------------------------------------------- swiglu --
def test_swiglu_closed_forms(orc64):
    F = 5
    gate = np.array([[0.0, 40.0, -40.0, 1.0, -1.0]])
    up = np.array([[3.0, 2.0, 2.0, -1.5, 4.0]])
    a = orc64.swiglu(np.concatenate([gate, up], axis=1))[0]
    assert a[0] == 0.0                                   # silu(0) = 0
    np.testing.assert_allclose(a[1], 80.0, rtol=1e-12)   # silu(z) -> z
    assert abs(a[2]) < 1e-15                             # silu(-z) -> 0
    np.testing.assert_allclose(a[3], -1.5 / (1 + math.exp(-1.0)), rtol=1e-14)
    np.testing.assert_allclose(a[4], -4.0 / (1 + math.exp(1.0)), rtol=1e-14)
    # gate is the first half, up the second: swapping them changes the result
    b = orc64.swiglu(np.concatenate([up, gate], axis=1))[0]
    assert not np.allclose(a, b)
