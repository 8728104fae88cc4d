"""Pins for the oracle's forward, update and integer step (CPU only).

The oracle materialises W_i = M + (sigma/sqrt r) A_i B_i^T and sums explicit outer products; these
tests hold it against what the paper and the mathematics fix: the factored identity of the
"Hardware-Efficient Implementation" section, brute-force loops on tiny shapes, special inputs with
closed-form answers, the rank statement below the EGGROLL UPDATE box, the identity covariance of
vec(E), and -- for the integer step -- the exact integer W_i = W + A_i B_i^T matmul.
"""
import numpy as np
import pytest
import scipy.special

import oracle

SEED, STEP, LAYER = 12345, 3, 7


def factors(member, d_out, d_in, r, nd):
    A = oracle.noise_matrix(SEED, STEP, LAYER, oracle.WHICH_A, member, d_out, r, nd)
    B = oracle.noise_matrix(SEED, STEP, LAYER, oracle.WHICH_B, member, d_in, r, nd)
    return A, B


def rand_inputs(d_out, d_in, rows, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((d_out, d_in)) / np.sqrt(d_in), rng.standard_normal((rows, d_in))


@pytest.mark.parametrize("d_out,d_in,N,S,r,nd", [(8, 6, 3, 1, 1, 0), (5, 7, 2, 3, 2, 1), (4, 4, 4, 2, 1, 1)])
def test_forward_brute_force_loops(d_out, d_in, N, S, r, nd):
    W, X = rand_inputs(d_out, d_in, N * S)
    sigma, mb = 0.37, 5
    Y = oracle.forward(SEED, STEP, LAYER, mb, N, S, d_out, d_in, r, nd, sigma, 0, W, X)
    for m in range(N):
        A, B = factors(mb + m, d_out, d_in, r, nd)
        for s in range(S):
            row = m * S + s
            for j in range(d_out):
                acc = 0.0
                for k in range(d_in):
                    e = sum(A[j, l] * B[k, l] for l in range(r)) / np.sqrt(r)
                    acc += (W[j, k] + sigma * e) * X[row, k]
                assert abs(Y[row, j] - acc) < 1e-12 * (1 + abs(acc))


@pytest.mark.parametrize("d_out,d_in,N,S,r,nd", [(48, 40, 6, 1, 1, 1), (33, 65, 4, 5, 4, 0), (16, 24, 3, 2, 8, 1)])
def test_explicit_equals_factored(d_out, d_in, N, S, r, nd):
    # u (M + sigma E)^T = u M^T + (sigma/sqrt r)(u B) A^T
    W, X = rand_inputs(d_out, d_in, N * S, 1)
    sigma = 0.05
    Y = oracle.forward(SEED, STEP, LAYER, 0, N, S, d_out, d_in, r, nd, sigma, 0, W, X)
    for m in range(N):
        A, B = factors(m, d_out, d_in, r, nd)
        u = X[m * S:(m + 1) * S]
        ref = u @ W.T + (sigma / np.sqrt(r)) * (u @ B) @ A.T
        np.testing.assert_allclose(Y[m * S:(m + 1) * S], ref, rtol=1e-12, atol=1e-12)


def test_forward_special_inputs():
    d_out, d_in, N, S, r = 12, 10, 4, 2, 2
    W, X = rand_inputs(d_out, d_in, N * S, 2)
    args = (SEED, STEP, LAYER, 0, N, S, d_out, d_in, r, 1)
    # sigma = 0: the unperturbed GEMM
    np.testing.assert_allclose(oracle.forward(*args, 0.0, 0, W, X), X @ W.T, rtol=1e-13, atol=1e-13)
    # linear in sigma
    y0, y1, y2 = (oracle.forward(*args, s, 0, W, X) for s in (0.0, 0.1, 0.2))
    np.testing.assert_allclose(y2 - y0, 2 * (y1 - y0), rtol=1e-10, atol=1e-12)
    # W = 0: the correction alone
    yc = oracle.forward(*args, 0.1, 0, np.zeros_like(W), X)
    np.testing.assert_allclose(yc, y1 - y0, rtol=1e-10, atol=1e-12)
    # x = e_k: column k of W_i
    k = 3
    E = np.zeros((N * S, d_in)); E[:, k] = 1.0
    ye = oracle.forward(*args, 0.1, 0, W, E)
    for m in range(N):
        A, B = factors(m, d_out, d_in, r, 1)
        col = W[:, k] + (0.1 / np.sqrt(r)) * A @ B[k]
        np.testing.assert_allclose(ye[m * S], col, rtol=1e-12, atol=1e-13)
    # different members see different perturbations; same member, same perturbation for its rows
    Xs = np.tile(X[:1], (N * S, 1))
    ys = oracle.forward(*args, 0.1, 0, W, Xs)
    assert np.allclose(ys[0], ys[1]) and not np.allclose(ys[0], ys[S])
    # member_begin shifts the global member id
    ysh = oracle.forward(SEED, STEP, LAYER, 2, 2, S, d_out, d_in, r, 1, 0.1, 0, W, Xs[:2 * S])
    np.testing.assert_array_equal(ysh, ys[2 * S:])


def test_forward_gelu_is_exact_erf_form():
    d_out, d_in, N = 9, 11, 3
    W, X = rand_inputs(d_out, d_in, N, 3)
    lin = oracle.forward(SEED, STEP, LAYER, 0, N, 1, d_out, d_in, 1, 1, 0.2, oracle.ACT_NONE, W, X * 3)
    act = oracle.forward(SEED, STEP, LAYER, 0, N, 1, d_out, d_in, 1, 1, 0.2, oracle.ACT_GELU, W, X * 3)
    np.testing.assert_allclose(act, lin * scipy.special.ndtr(lin), rtol=1e-12, atol=1e-15)
    import torch
    ref = torch.nn.functional.gelu(torch.tensor(lin, dtype=torch.float64)).numpy()
    np.testing.assert_allclose(act, ref, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("d_out,d_in,N,r,nd", [(7, 5, 9, 1, 0), (6, 8, 5, 2, 1), (10, 3, 4, 4, 1)])
def test_update_is_sum_of_outer_products(d_out, d_in, N, r, nd):
    rng = np.random.default_rng(4)
    f = rng.standard_normal(N)
    scale, mb = 0.3, 11
    G = oracle.update(SEED, STEP, LAYER, mb, N, d_out, d_in, r, nd, f, scale)
    ref = np.zeros((d_out, d_in))
    for m in range(N):
        A, B = factors(mb + m, d_out, d_in, r, nd)
        for l in range(r):
            for j in range(d_out):
                for k in range(d_in):
                    ref[j, k] += f[m] * A[j, l] * B[k, l]
    np.testing.assert_allclose(G, scale * ref, rtol=1e-12, atol=1e-13)
    # the GEMM form of the same thing: (diag(f) A)^T B with A in R^{N r x d_out}, B in R^{N r x d_in}
    As = np.stack([factors(mb + m, d_out, d_in, r, nd)[0] for m in range(N)])  # [N, d_out, r]
    Bs = np.stack([factors(mb + m, d_out, d_in, r, nd)[1] for m in range(N)])
    gemm = np.einsum("n,njl,nkl->jk", f, As, Bs)
    np.testing.assert_allclose(G, scale * gemm, rtol=1e-12, atol=1e-13)
    # single entries by random access
    for j, k in [(0, 0), (d_out - 1, d_in - 1), (2, 1)]:
        e = oracle.update_entry(SEED, STEP, LAYER, mb, N, r, nd, f, scale, j, k)
        assert abs(e - G[j, k]) < 1e-12 * (1 + abs(G[j, k]))


def test_update_special_fitness():
    d_out, d_in, N, r = 6, 5, 8, 2
    args = (SEED, STEP, LAYER, 0, N, d_out, d_in, r, 1)
    # all-equal fitness, centred -> exactly zero
    f = np.full(N, 3.25); f = f - f.mean()
    assert (oracle.update(*args, f, 1.0) == 0.0).all()
    # f = e_i reads back member i's perturbation
    for i in (0, 5):
        f = np.zeros(N); f[i] = 1.0
        A, B = factors(i, d_out, d_in, r, 1)
        np.testing.assert_allclose(oracle.update(*args, f, 0.5), 0.5 * A @ B.T, rtol=1e-13, atol=1e-15)
    # linear in f; two half-populations add up to the whole
    rng = np.random.default_rng(5)
    f = rng.standard_normal(N)
    G = oracle.update(*args, f, 1.0)
    lo = oracle.update(SEED, STEP, LAYER, 0, N // 2, d_out, d_in, r, 1, f[:N // 2], 1.0)
    hi = oracle.update(SEED, STEP, LAYER, N // 2, N // 2, d_out, d_in, r, 1, f[N // 2:], 1.0)
    np.testing.assert_allclose(G, lo + hi, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("N,r,expect", [(1, 1, 1), (2, 1, 2), (1, 2, 2), (3, 2, 5), (4, 2, 5)])
def test_update_rank_is_min_Nr_m_n(N, r, expect):
    d_out, d_in = 6, 5
    f = np.arange(1, N + 1, dtype=np.float64)
    G = oracle.update(SEED, STEP, LAYER, 0, N, d_out, d_in, r, 0, f, 1.0)
    assert np.linalg.matrix_rank(G, tol=1e-9) == expect == min(N * r, d_out, d_in)


def test_forward_and_update_reconstruct_the_same_E():
    # forward with W = 0, x = e_k gives column k of sigma E_i; update with f = e_i gives
    # scale * A_i B_i^T.  Both must describe the same matrix (catches A/B swaps, transposes,
    # which/layer/step mix-ups and inconsistent 1/sqrt r between the two).
    d_out, d_in, N, r, sigma = 5, 4, 3, 2, 0.7
    for i in range(N):
        f = np.zeros(N); f[i] = 1.0
        sigmaE_from_update = oracle.update(SEED, STEP, LAYER, 0, N, d_out, d_in, r, 1, f, sigma / np.sqrt(r))
        cols = []
        for k in range(d_in):
            X = np.zeros((N, d_in)); X[:, k] = 1.0
            cols.append(oracle.forward(SEED, STEP, LAYER, 0, N, 1, d_out, d_in, r, 1, sigma, 0,
                                       np.zeros((d_out, d_in)), X)[i])
        np.testing.assert_allclose(np.stack(cols, axis=1), sigmaE_from_update, rtol=1e-12, atol=1e-14)


def test_vecE_identity_covariance_and_outer_norm():
    # Lemma (covariance form): entries of E = A B^T / sqrt r are zero-mean with identity covariance.
    m, n, r, N = 4, 3, 2, 60000
    Es = np.empty((N, m * n))
    for i in range(N):
        A, B = factors(i, m, n, r, 0)
        Es[i] = (A @ B.T / np.sqrt(r)).reshape(-1)
    assert np.abs(Es.mean(axis=0)).max() < 5.0 / np.sqrt(N)
    cov = Es.T @ Es / N
    # fourth moments of products are larger than Gaussian ones: allow 8/sqrt(N)
    assert np.abs(cov - np.eye(m * n)).max() < 8.0 / np.sqrt(N)
    a, b = factors(0, 9, 7, 1, 0)
    assert np.isclose(np.linalg.norm(a @ b.T), np.linalg.norm(a) * np.linalg.norm(b), rtol=1e-13)


@pytest.mark.parametrize("r", [1, 2, 4, 8])
def test_entries_of_E_approach_the_gaussian_at_rate_one_over_r(r):
    # Sec. "Rank Analysis": the odd cumulants of E^r = A B^T / sqrt(r) vanish by symmetry and the fourth one
    # decays like 1/r.  Closed form for Gaussian factors: E_ij is a normalised sum of r products of independent
    # N(0,1) pairs, each with fourth moment 9, so var = 1, skewness 0, excess kurtosis = 6 / r.
    members, d = 600, 24
    e = []
    for m in range(members):
        A = oracle.noise_matrix(5, 0, 2, 0, m, d, r, oracle.NOISE_F32)
        B = oracle.noise_matrix(5, 0, 2, 1, m, d, r, oracle.NOISE_F32)
        e.append((A @ B.T / np.sqrt(r)).ravel())
    e = np.concatenate(e)
    n_eff = members * d          # entries of one member share factors: count rows, not entries, for the error bars
    assert abs(e.mean()) < 4 / np.sqrt(n_eff) and abs(e.var() - 1) < 6 / np.sqrt(n_eff)
    assert abs((e ** 3).mean()) < 30 / np.sqrt(n_eff)
    excess = (e ** 4).mean() / e.var() ** 2 - 3
    assert abs(excess - 6.0 / r) < 0.35 * 6.0 / r + 0.1, (r, excess)


def test_monte_carlo_update_recovers_linear_fitness_gradient():
    # For f(W) = <Gamma, W - M>/sigma... i.e. f_i = <Gamma, E_i>, (1/N) sum_i E_i f_i -> Gamma because
    # vec(E) has identity covariance (Eq. matrix_mc with the Gaussian score).  Statistical, loose.
    m, n, r, N = 4, 3, 1, 120000
    rng = np.random.default_rng(6)
    Gamma = rng.standard_normal((m, n))
    f = np.empty(N)
    for i in range(N):
        A, B = factors(i, m, n, r, 0)
        f[i] = np.sum(Gamma * (A @ B.T) / np.sqrt(r))
    G = oracle.update(SEED, STEP, LAYER, 0, N, m, n, r, 0, f, 1.0 / (N * np.sqrt(r)))
    assert np.linalg.norm(G - Gamma) / np.linalg.norm(Gamma) < 0.08


# ----------------------------------------------------------------------------------------------
# integer step
# ----------------------------------------------------------------------------------------------
def int_factors(member, d, bound):
    return (oracle.noise_int(SEED, STEP, LAYER, 0, member, 0, d, bound).astype(np.int64),
            oracle.noise_int(SEED, STEP, LAYER, 1, member, 0, d, bound).astype(np.int64))


def int_inputs(d, N, seed=0):
    rng = np.random.default_rng(seed)
    return (rng.integers(-127, 128, (d, d)).astype(np.int8), rng.integers(-127, 128, (N, d)).astype(np.int8))


def test_int8_corr_shift_zero_is_explicit_integer_Wi():
    d, N, bound = 32, 5, 8
    W, H = int_inputs(d, N)
    for out_shift in (0, 3, 8):
        got = oracle.forward_i8(SEED, STEP, LAYER, 2, N, d, bound, 0, out_shift, 1, W, H)
        for m in range(N):
            A, B = int_factors(2 + m, d, bound)
            Wi = W.astype(np.int64) + np.outer(A, B)
            v = (Wi @ H[m].astype(np.int64)) >> out_shift  # numpy >> on signed ints is arithmetic
            assert (got[m] == np.clip(v, -127, 127)).all()


def test_int8_zero_noise_is_plain_gemm_shift_clamp():
    d, N = 48, 4
    W, H = int_inputs(d, N, 1)
    got = oracle.forward_i8(SEED, STEP, LAYER, 0, N, d, 0, 4, 8, 1, W, H)
    ref = np.clip((H.astype(np.int64) @ W.astype(np.int64).T) >> 8, -127, 127)
    assert (got == ref).all()


def test_int8_step_by_step_formula_and_recurrence():
    d, N, bound, cs, os_ = 64, 3, 8, 4, 6
    W, H = int_inputs(d, N, 2)
    one = oracle.forward_i8(SEED, STEP, LAYER, 0, N, d, bound, cs, os_, 1, W, H)
    for m in range(N):
        A, B = int_factors(m, d, bound)
        h = H[m].astype(np.int64)
        acc = W.astype(np.int64) @ h
        corr = np.array([int(np.dot(h, B)) * int(a) for a in A]) >> cs   # floor, also for negatives
        assert (one[m] == np.clip((acc + corr) >> os_, -127, 127)).all()
    # T steps = T single steps chained with the same perturbation
    three = oracle.forward_i8(SEED, STEP, LAYER, 0, N, d, bound, cs, os_, 3, W, H)
    h = H
    for _ in range(3):
        h = oracle.forward_i8(SEED, STEP, LAYER, 0, N, d, bound, cs, os_, 1, W, h)
    assert (three == h).all()
    assert three.min() >= -127  # -128 is never produced


def test_int8_shift_floors_and_clamp_edges():
    # d = 1: h' = clamp((h*w + ((h*b)*a >> cs)) >> os): choose values by hand via bound = 0 (a = b = 0)
    for h, w, os_, expect in [(-1, 1, 8, -1), (1, 1, 8, 0), (-127, 127, 0, -127), (127, 127, 0, 127),
                              (-3, 1, 1, -2), (3, 1, 1, 1), (-127, 127, 7, -127), (-100, 100, 7, -79)]:
        got = oracle.forward_i8(0, 0, 0, 0, 1, 1, 0, 4, os_, 1, np.array([[w]], np.int8), np.array([[h]], np.int8))
        assert int(got[0, 0]) == expect, (h, w, os_, int(got[0, 0]), expect)


def test_oracle_es_steps_descend_a_quadratic():
    # Alg. 1 with the oracle's own forward and update: fitness = -sum ||y - W* x||^2 on a batch shared by all
    # members, z-scored; W += lr * G must reduce the loss.  A wrong sign, a transposed G or factors that differ
    # between forward and update would make it rise or stall.
    d, N, S, sigma, r = 8, 512, 8, 0.01, 2
    lr = 0.3 * sigma
    rng = np.random.default_rng(0)
    w_star = rng.standard_normal((d, d)) / np.sqrt(d)
    W = np.zeros((d, d), np.float32)
    losses = []
    for step in range(25):
        xb = rng.standard_normal((S, d)).astype(np.float32)
        X = np.tile(xb, (N, 1))
        target = xb @ w_star.T
        Y = oracle.forward(7, step, 0, 0, N, S, d, d, r, oracle.NOISE_F32, sigma, 0, W, X)
        f = -((Y - np.tile(target, (N, 1))) ** 2).sum(1).reshape(N, S).sum(1)
        z = (f - f.mean()) / (f.std() + 1e-8)
        G = oracle.update(7, step, 0, 0, N, d, d, r, oracle.NOISE_F32, z, 1.0 / (N * sigma * np.sqrt(r)))
        W = (W + lr * G).astype(np.float32)
        losses.append(float(((xb @ W.T - target) ** 2).sum(1).mean()))
    assert losses[0] > 4.0 and losses[-1] < 0.5 * losses[0], losses[::4]


def test_noise_gather_reads_the_same_entries_as_the_whole_matrix():
    idx = np.array([0, 1, 7, 38, 39, 5, 5], np.int64)
    for which, dt in ((0, oracle.NOISE_BF16), (1, oracle.NOISE_F32)):
        got = oracle.noise_gather(9, 2, 4, which, 100, 6, idx, dt)
        for m in range(6):
            full = oracle.noise_matrix(9, 2, 4, which, 100 + m, 10, 4, dt).reshape(-1)
            assert np.array_equal(got[m], full[idx])


def rank_convergence_closed_form(r, sigma=1.0):
    """<U, g_r> for f(W) = cos(<U, W>), U = u v^T with unit u, v, at <U, M> = pi/2 and scale 1/(sigma N):
    with X = <U, E^r> = r^{-1/2} sum_l (a_l.u)(b_l.v), E[exp(i s X)] = (1 + s^2/r)^{-r/2} (each (a.u)(b.v) is a product of
    two independent standard normals, characteristic function (1 + t^2)^{-1/2}), hence
    (1/sigma) E[cos(pi/2 + sigma X) X] = -(1/sigma) E[sin(sigma X) X] = (1/sigma) d/dsigma (1 + sigma^2/r)^{-r/2}
    = -(1 + sigma^2/r)^{-r/2-1};  the Gaussian ES limit is -exp(-sigma^2/2)."""
    return -(1.0 + sigma * sigma / r) ** (-r / 2.0 - 1.0)


def rank_convergence_problem(m=8, n=8, seed=5):
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(m); u /= np.linalg.norm(u)
    v = rng.standard_normal(n); v /= np.linalg.norm(v)
    M = (np.pi / 2.0) * np.outer(u, v)          # <U, M> = pi/2 exactly up to rounding
    return u.astype(np.float32), v.astype(np.float32), M.astype(np.float32)


def test_rank_convergence_of_the_update_is_one_over_r():
    """Sec. "Rank Analysis" (EGGROLL Rank Convergence): the expected low-rank update approaches the Gaussian ES
    gradient at rate O(1/r).  For the bounded fitness cos(<U, W>) both are known in closed form; the oracle's
    forward (fitness through the explicit W_i) and update (explicit outer products) reproduce the finite-r value
    within Monte-Carlo error, and the gap to the Gaussian limit halves with every doubling of r."""
    u, v, M = rank_convergence_problem()
    m, n, N, sigma = 8, 8, 1 << 17, 1.0
    limit = -np.exp(-0.5)
    gaps = []
    for r in (1, 2, 4, 8, 16):
        X = np.tile(v[None, :], (N, 1))
        Y = oracle.forward(7, 0, 3, 0, N, 1, m, n, r, oracle.NOISE_F32, sigma, 0, M, X)   # y_i = W_i v
        f = np.cos(Y @ u.astype(np.float64))                                             # cos(u^T W_i v)
        G = oracle.update(7, 0, 3, 0, N, m, n, r, oracle.NOISE_F32, f, 1.0 / (N * sigma * np.sqrt(r)))
        got = float(u.astype(np.float64) @ G @ v.astype(np.float64))
        want = rank_convergence_closed_form(r, sigma)
        assert abs(got - want) < 5.0 / np.sqrt(N), (r, got, want)      # Var(f X) <= E X^2 = 1
        gaps.append(abs(want - limit))
    ratios = [gaps[i] / gaps[i + 1] for i in range(4)]
    assert all(1.5 < q < 2.2 for q in ratios), ratios                  # O(1/r): the gap halves as r doubles
    assert gaps[-1] < 0.03 and gaps[0] > 0.25
