"""Pins for the oracle's integer parameter update and antithetic pairs (CPU only).

Integer update (App. "Parameter Update" of the integer pretraining section): E = (diag(F)A)^T B in
int32, one-bin moves where |E| reaches the threshold, clamp to [-127, 127]; the threshold formula
I32(16 Phi^-1(.)) * 16 sqrt(N).  Antithetic pairs (App. "Fitness Shaping"): the two members of a
pair evaluate M + sigma E and M - sigma E.  Each test holds the oracle against something other
than itself: numpy einsum over separately drawn factors, hand-built cases, scipy's normal
quantile, the already pinned non-antithetic functions, closed-form symmetries.
"""
import numpy as np
import pytest
import scipy.stats

import oracle

SEED, STEP, LAYER = 777, 2, 5


def int_factors(member, d_out, d_in, bound):
    A = oracle.noise_int(SEED, STEP, LAYER, oracle.WHICH_A, member, 0, d_out, bound)
    B = oracle.noise_int(SEED, STEP, LAYER, oracle.WHICH_B, member, 0, d_in, bound)
    return A.astype(np.int64), B.astype(np.int64)


@pytest.mark.parametrize("d_out,d_in,N,bound,mb", [(7, 9, 5, 8, 0), (16, 12, 33, 3, 10), (5, 5, 64, 127, 1)])
def test_E_is_the_sum_of_signed_outer_products(d_out, d_in, N, bound, mb):
    rng = np.random.default_rng(0)
    F = rng.integers(-1, 2, N).astype(np.int8)
    theta = rng.integers(-127, 128, (d_out, d_in)).astype(np.int8)
    A = np.stack([int_factors(mb + m, d_out, d_in, bound)[0] for m in range(N)])
    B = np.stack([int_factors(mb + m, d_out, d_in, bound)[1] for m in range(N)])
    E_ref = np.einsum("i,ij,ik->jk", F.astype(np.int64), A, B)          # (diag(F)A)^T B
    tau = int(np.median(np.abs(E_ref))) + 1
    out, E = oracle.update_i8(SEED, STEP, LAYER, mb, N, d_out, d_in, bound, F, tau, theta)
    assert (E == E_ref).all()
    step = np.sign(E_ref) * (np.abs(E_ref) >= tau)
    assert (out == np.clip(theta.astype(np.int64) + step, -127, 127)).all()
    assert 0 < (step != 0).sum() < step.size  # the case exercises both branches


def test_single_member_fitness_reads_back_its_outer_product_and_sign():
    d_out, d_in, N, bound = 6, 8, 9, 8
    theta = np.zeros((d_out, d_in), np.int8)
    for i, f in ((0, 1), (4, -1), (8, 1)):
        F = np.zeros(N, np.int8)
        F[i] = f
        out, E = oracle.update_i8(SEED, STEP, LAYER, 20, N, d_out, d_in, bound, F, 1, theta)
        A, B = int_factors(20 + i, d_out, d_in, bound)
        assert (E == f * np.outer(A, B)).all()
        assert (out == np.sign(f * np.outer(A, B))).all()  # threshold 1: every non-zero entry moves one bin


def test_zero_fitness_and_threshold_edges():
    d_out, d_in, N, bound = 4, 4, 6, 8
    rng = np.random.default_rng(3)
    theta = rng.integers(-127, 128, (d_out, d_in)).astype(np.int8)
    out, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, np.zeros(N, np.int8), 0, theta)
    assert (E == 0).all() and (out == theta).all()          # E = 0 never moves, even at threshold 0
    F = np.ones(N, np.int8)
    _, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, 0, theta)
    j, k = np.unravel_index(np.abs(E).argmax(), E.shape)
    big = int(abs(E[j, k]))
    at, _ = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, big, theta)      # |E| == threshold moves
    above, _ = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, big + 1, theta)
    assert (above == theta).all()
    moved = np.argwhere(at != theta)
    assert all(abs(E[a, b]) == big for a, b in moved) and (theta[j, k] in (-127, 127) or at[j, k] != theta[j, k])


def test_moves_saturate_at_plus_minus_127_and_never_reach_minus_128():
    d_out, d_in, N, bound = 8, 8, 5, 8
    F = np.ones(N, np.int8)
    for fill in (127, -127):
        theta = np.full((d_out, d_in), fill, np.int8)
        out, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, 1, theta)
        want = np.clip(fill + np.sign(E), -127, 127)
        assert (out == want).all() and out.min() >= -127 and (np.sign(E) != 0).any()


def test_update_is_additive_over_member_chunks_and_odd_in_F():
    d_out, d_in, N, bound = 10, 6, 24, 8
    rng = np.random.default_rng(5)
    F = rng.integers(-1, 2, N).astype(np.int8)
    theta = np.zeros((d_out, d_in), np.int8)
    _, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, 1, theta)
    _, E1 = oracle.update_i8(SEED, STEP, LAYER, 0, 10, d_out, d_in, bound, F[:10], 1, theta)
    _, E2 = oracle.update_i8(SEED, STEP, LAYER, 10, 14, d_out, d_in, bound, F[10:], 1, theta)
    _, En = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, -F, 1, theta)
    assert (E == E1 + E2).all() and (En == -E).all()


@pytest.mark.parametrize("alpha", [0.9, 0.5, 0.3173, 0.1, 0.05, 0.01, 1e-4])
def test_threshold_matches_the_normal_quantile(alpha):
    # two-sided alpha-quantile: P(|Z| >= z) = alpha, z = Phi^-1(1 - alpha/2) from scipy
    z = scipy.stats.norm.ppf(1.0 - alpha / 2.0)
    for n, std in ((4096, 16.0), (1024, 16.0), (8192, np.sqrt(24.0))):
        want = int(std * z) * int(round(std * np.sqrt(n)))
        assert oracle.int_threshold(alpha, n, std) == want
    # the paper's printed form, noise std 16 and N a power of 4: I32(16 z) * 16 sqrt(N)
    assert oracle.int_threshold(alpha, 4 ** 6, 16.0) == int(16 * z) * 16 * 64


def test_threshold_limits_and_monotonicity():
    assert oracle.int_threshold(1.0, 4096, 16.0) == 0
    ts = [oracle.int_threshold(a, 4096, 16.0) for a in (0.99, 0.5, 0.2, 0.05, 0.001)]
    assert ts == sorted(ts) and ts[0] == 0 and ts[-1] > ts[1]
    assert oracle.int_threshold(0.0, 4096, 16.0) > 2 ** 40   # alpha -> 0: nothing moves


def test_fraction_moved_is_about_alpha():
    # "alpha approximately equals the fraction of parameters that are updated": E over N members of
    # uniform {-8..8} noise is close to normal with std (b(b+1)/3) sqrt(N) = 24 sqrt(N)
    d, N, bound = 48, 1024, 8
    rng = np.random.default_rng(11)
    F = rng.choice(np.array([-1, 1], np.int8), N)
    std = np.sqrt(bound * (bound + 1) / 3.0)
    theta = np.zeros((d, d), np.int8)
    for alpha in (0.5, 0.1):
        tau = oracle.int_threshold(alpha, N, std)
        out, _ = oracle.update_i8(SEED, STEP, LAYER, 0, N, d, d, bound, F, tau, theta)
        frac = (out != 0).mean()
        assert abs(frac - alpha) < 0.2 * alpha + 0.02, (alpha, frac)


# ---------------------------------------------------------------------------------------------------
# antithetic pairs
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d_out,d_in,pairs,S,r,nd", [(12, 10, 3, 1, 1, 0), (9, 14, 2, 3, 2, 1)])
def test_antithetic_members_are_plus_and_minus_the_pair_noise(d_out, d_in, pairs, S, r, nd):
    rng = np.random.default_rng(2)
    W = rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)
    sigma, p0 = 0.25, 4                        # first pair id 4 -> first member id 8
    Xp = rng.standard_normal((pairs * S, d_in))
    X = np.repeat(Xp.reshape(pairs, S, d_in), 2, axis=0).reshape(2 * pairs * S, d_in)   # both members see the same rows
    Y = oracle.forward(SEED, STEP, LAYER, 2 * p0, 2 * pairs, S, d_out, d_in, r, nd, sigma, 0, W, X, antithetic=True)
    plus = oracle.forward(SEED, STEP, LAYER, p0, pairs, S, d_out, d_in, r, nd, sigma, 0, W, Xp)      # pinned elsewhere
    minus = oracle.forward(SEED, STEP, LAYER, p0, pairs, S, d_out, d_in, r, nd, -sigma, 0, W, Xp)
    Y = Y.reshape(pairs, 2, S, d_out)
    np.testing.assert_array_equal(Y[:, 0].reshape(-1, d_out), plus)      # even member: noise id = pair id, +sigma
    np.testing.assert_array_equal(Y[:, 1].reshape(-1, d_out), minus)     # odd member: same factors, -sigma
    base = Xp @ W.T
    np.testing.assert_allclose(0.5 * (Y[:, 0] + Y[:, 1]).reshape(-1, d_out), base, rtol=1e-12, atol=1e-12)


def test_antithetic_with_zero_mean_weights_is_exactly_odd():
    d_out, d_in, pairs = 6, 5, 4
    X = np.random.default_rng(8).standard_normal((2 * pairs, d_in))
    X[1::2] = X[0::2]
    Y = oracle.forward(SEED, STEP, LAYER, 0, 2 * pairs, 1, d_out, d_in, 1, 1, 0.5, 0, np.zeros((d_out, d_in)), X,
                       antithetic=True)
    np.testing.assert_array_equal(Y[0::2], -Y[1::2])
    assert np.abs(Y).min() > 0


def test_antithetic_integer_step_even_is_the_pair_odd_negates_B():
    d, pairs, bound, cs, os_ = 32, 5, 8, 2, 6
    rng = np.random.default_rng(4)
    W = rng.integers(-127, 128, (d, d)).astype(np.int8)
    Hp = rng.integers(-127, 128, (pairs, d)).astype(np.int8)
    H = np.repeat(Hp, 2, axis=0)
    p0 = 3
    got = oracle.forward_i8(SEED, STEP, LAYER, 2 * p0, 2 * pairs, d, bound, cs, os_, 1, W, H, antithetic=True)
    even = oracle.forward_i8(SEED, STEP, LAYER, p0, pairs, d, bound, cs, os_, 1, W, Hp)   # pinned elsewhere
    assert (got[0::2] == even).all()
    for p in range(pairs):                       # odd member, from the printed formula with B -> -B
        A, B = int_factors(p0 + p, d, d, bound)
        h = Hp[p].astype(np.int64)
        acc = W.astype(np.int64) @ h
        corr = ((h @ (-B)) * A) >> cs            # numpy >> on int64 is arithmetic (floor)
        want = np.clip((acc + corr) >> os_, -127, 127)
        assert (got[2 * p + 1] == want).all()
    assert (got[0::2] != got[1::2]).any()


def test_antithetic_integer_recurrence_over_steps_matches_single_steps():
    d, pairs, bound = 16, 3, 8
    rng = np.random.default_rng(6)
    W = rng.integers(-127, 128, (d, d)).astype(np.int8)
    H = rng.integers(-127, 128, (2 * pairs, d)).astype(np.int8)
    three = oracle.forward_i8(SEED, STEP, LAYER, 0, 2 * pairs, d, bound, 3, 5, 3, W, H, antithetic=True)
    h = H
    for _ in range(3):
        h = oracle.forward_i8(SEED, STEP, LAYER, 0, 2 * pairs, d, bound, 3, 5, 1, W, h, antithetic=True)
    assert (three == h).all()


@pytest.mark.parametrize("d_out,d_in", [(48, 12), (12, 48), (20, 20)])
def test_rectangular_integer_matmul_follows_the_printed_formula(d_out, d_in):
    # theta in I8^{m x n}: I8((u theta^T + ((u . B) I32(A) >> s_c)) >> s_o) with A in I8^m, B in I8^n
    N, bound, cs, os_ = 7, 8, 3, 5
    rng = np.random.default_rng(d_out)
    W = rng.integers(-127, 128, (d_out, d_in)).astype(np.int8)
    H = rng.integers(-127, 128, (N, d_in)).astype(np.int8)
    got = oracle.matmul_i8(SEED, STEP, LAYER, 2, N, d_out, d_in, bound, cs, os_, W, H)
    for m in range(N):
        A, B = int_factors(2 + m, d_out, d_in, bound)
        h = H[m].astype(np.int64)
        want = np.clip((W.astype(np.int64) @ h + (((h @ B) * A) >> cs)) >> os_, -127, 127)
        assert (got[m] == want).all()
    if d_out == d_in:   # the square case is the recurrence's single step
        assert (got == oracle.forward_i8(SEED, STEP, LAYER, 2, N, d_in, bound, cs, os_, 1, W, H)).all()
