"""Pins of the paper's own integer noise (App. "Adding EGGROLL Perturbations": int8 values round(16 z) from a
pre-generated table indexed at random) as the oracle defines it: the table against scipy's normal quantile, its
symmetry and moments, the indexing of the stream, and the exact-integer identity of the perturbed matmul."""
import numpy as np
from scipy.stats import norm

import oracle

T16 = oracle.BOUND_NORMAL16


def test_table_is_the_rounded_normal_quantile():
    t = oracle.normal_int_table().astype(np.int64)
    z16 = 16.0 * norm.ppf((np.arange(65536) + 0.5) / 65536.0)
    want = np.where(z16 >= 0, np.floor(z16 + 0.5), -np.floor(-z16 + 0.5)).astype(np.int64)
    # no quantile sits within 1e-7 of a rounding boundary, so two independent inverse CDFs must agree everywhere
    assert np.abs(np.abs(z16 - np.floor(z16)) - 0.5).min() > 1e-7   # (the closest is 4e-7)
    assert np.array_equal(t, want)


def test_table_symmetry_monotonicity_and_moments():
    t = oracle.normal_int_table().astype(np.int64)
    assert np.array_equal(t[::-1], -t)                  # exactly symmetric: zero mean, all odd moments zero
    assert (np.diff(t) >= 0).all() and t.max() == 69 and t.min() == -69
    assert t.sum() == 0
    std = np.sqrt((t.astype(np.float64) ** 2).mean())
    assert abs(std - 16.0) < 0.02                       # "round(16 N(0,1))": standard deviation 16
    kurt = (t.astype(np.float64) ** 4).mean() / std ** 4
    assert abs(kurt - 3.0) < 0.01


def test_stream_indexing_low_half_first():
    t = oracle.normal_int_table()
    for which, member, first, n in ((0, 3, 0, 64), (1, 2 ** 32 - 2, 5, 37), (0, 77, 1, 9)):
        got = oracle.noise_int(9, 4, 11, which, member, first, n, T16)
        idx = np.arange(first, first + n)
        words = oracle.raw_words(9, 4, 11, which, member, 0, (first + n + 1) // 2 + 1)
        half = (words[idx >> 1] >> (16 * (idx & 1)).astype(np.uint32)) & np.uint32(0xFFFF)
        assert np.array_equal(got, t[half])
    # random access equals a slice of the whole vector
    whole = oracle.noise_int(9, 4, 11, 0, 5, 0, 100, T16)
    assert np.array_equal(oracle.noise_int(9, 4, 11, 0, 5, 33, 20, T16), whole[33:53])


def test_matmul_with_table_noise_is_the_exact_integer_matrix():
    """corr_shift = 0: h (theta + A B^T)^T exactly, then the output shift and the clamp (the identity that pins
    the uniform noise, now with the table noise, whose products reach 69^2)."""
    rng = np.random.default_rng(5)
    d_out, d_in, N = 48, 64, 7
    W = rng.integers(-127, 128, (d_out, d_in)).astype(np.int8)
    H = rng.integers(-127, 128, (N, d_in)).astype(np.int8)
    got = oracle.matmul_i8(2, 1, 6, 10, N, d_out, d_in, T16, 0, 9, W, H)
    for m in range(N):
        A = oracle.noise_int(2, 1, 6, 0, 10 + m, 0, d_out, T16).astype(np.int64)
        B = oracle.noise_int(2, 1, 6, 1, 10 + m, 0, d_in, T16).astype(np.int64)
        Wi = W.astype(np.int64) + np.outer(A, B)
        want = np.clip((Wi @ H[m].astype(np.int64)) >> 9, -127, 127)
        assert np.array_equal(got[m].astype(np.int64), want)
    # the paper's setting: the correction is shifted by 4 + sigma_hat before it is added
    got8 = oracle.matmul_i8(2, 1, 6, 10, N, d_out, d_in, T16, 8, 9, W, H)
    A = oracle.noise_int(2, 1, 6, 0, 10, 0, d_out, T16).astype(np.int64)
    B = oracle.noise_int(2, 1, 6, 1, 10, 0, d_in, T16).astype(np.int64)
    h = H[0].astype(np.int64)
    want = np.clip(((W.astype(np.int64) @ h) + (((B @ h) * A) >> 8)) >> 9, -127, 127)
    assert np.array_equal(got8[0].astype(np.int64), want)
