"""Pins for the oracle's integer model around the GRU cell (App. "EGG architecture": Embedding, Layer
Normalisation, MLP, Alg. "EGG forward pass"; CPU only): closed forms and invariants the paper states,
exact rational arithmetic for the divide, the lookup as one_hot(t) against an explicitly perturbed table,
agreement of the embedding's factor naming with the integer update, and the composed forward pass against
a chain of the separately pinned parts."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

SEED, STEP, LAYER = 5, 2, 100


def clip(v):
    return np.clip(v, -127, 127)


# ------------------------------------------------------------------------------------------------
# layer normalisation
# ------------------------------------------------------------------------------------------------
def test_layernorm_constant_row_returns_the_weights():
    # |u_k| = c for all k: the mean absolute value is c exactly, so out_k = sign(u_k) * ln_k
    D = 64
    rng = np.random.default_rng(0)
    ln = rng.integers(-127, 128, D).astype(np.int8)
    for c in (1, 7, 127):
        sign = rng.choice([-1, 1], D)
        U = (c * sign).astype(np.int8)[None, :]
        assert (oracle.layernorm_i8(ln, U)[0] == sign * ln.astype(np.int64)).all()


def test_layernorm_exact_rational_quotient():
    # independent arithmetic: Python Fractions, truncation toward zero, clip to I8
    D, rows = 16, 200
    rng = np.random.default_rng(1)
    ln = rng.integers(-127, 128, D).astype(np.int8)
    U = rng.integers(-127, 128, (rows, D)).astype(np.int8)
    U[:20] = rng.integers(-1, 2, (20, D))             # rows whose mean absolute value truncates to 0 or 1
    got = oracle.layernorm_i8(ln, U)
    for r in range(rows):
        mav = max(sum(abs(int(v)) for v in U[r]) // D, 1)
        for k in range(D):
            q = Fraction(int(U[r, k]) * int(ln[k]), mav)
            t = int(q) if q >= 0 else -int(-q)          # toward zero
            assert got[r, k] == max(-127, min(127, t)), (r, k)


def test_layernorm_is_odd_in_u_and_in_the_weights():
    D = 64
    rng = np.random.default_rng(2)
    ln = rng.integers(-127, 128, D).astype(np.int8)
    U = rng.integers(-127, 128, (50, D)).astype(np.int8)
    a = oracle.layernorm_i8(ln, U).astype(np.int64)
    assert (oracle.layernorm_i8(ln, -U) == -a).all()
    assert (oracle.layernorm_i8(-ln, U) == -a).all()


def test_layernorm_l1_norm_is_about_D_times_the_weight():
    # the paper's remark: after dividing by the mean absolute value the L1 norm is D (times the weight w).
    # With mav <= mean < mav + 1 and one unit lost per truncation: (w - 1) D <= sum |out| < w D (mav + 1) / mav
    D, w = 256, 16
    rng = np.random.default_rng(3)
    U = rng.integers(-40, 41, (100, D)).astype(np.int8)       # |u| w / mav stays below 127: no clipping
    out = oracle.layernorm_i8(np.full(D, w, np.int8), U).astype(np.int64)
    mav = np.abs(U.astype(np.int64)).sum(1) >> 8
    assert mav.min() >= 8 and np.abs(out).max() < 127
    l1 = np.abs(out).sum(1)
    assert (l1 >= (w - 1) * D).all() and (l1 < w * D * (mav + 1) / mav).all()


def test_layernorm_zero_row_and_tiny_rows():
    D = 16
    ln = np.full(D, 100, np.int8)
    U = np.zeros((2, D), np.int8)
    U[1, 3] = 1                                                # sum |u| = 1 < D: divisor taken as 1
    out = oracle.layernorm_i8(ln, U)
    assert (out[0] == 0).all() and out[1, 3] == 100 and np.abs(out[1]).sum() == 100


# ------------------------------------------------------------------------------------------------
# embedding
# ------------------------------------------------------------------------------------------------
def test_embedding_without_noise_is_the_lookup():
    D, N = 32, 40
    rng = np.random.default_rng(4)
    emb = rng.integers(-127, 128, (256, D)).astype(np.int8)
    tok = rng.integers(0, 256, N).astype(np.uint8)
    assert (oracle.embed_i8(SEED, STEP, LAYER, 3, N, D, 0, 4, emb, tok) == emb[tok]).all()


@pytest.mark.parametrize("anti", [False, True])
def test_embedding_is_one_hot_times_the_perturbed_table(anti):
    D, N, bound, cs, mb = 32, 12, 8, 2, 6
    rng = np.random.default_rng(5)
    emb = rng.integers(-127, 128, (256, D)).astype(np.int8)
    tok = rng.integers(0, 256, N).astype(np.uint8)
    got = oracle.embed_i8(SEED, STEP, LAYER, mb, N, D, bound, cs, emb, tok, antithetic=anti)
    for m in range(N):
        member = mb + m
        nid = member // 2 if anti else member
        sign = -1 if (anti and member & 1) else 1
        A = oracle.noise_int(SEED, STEP, LAYER, 0, nid, 0, 256, bound).astype(np.int64)
        B = oracle.noise_int(SEED, STEP, LAYER, 1, nid, 0, D, bound).astype(np.int64)
        table = clip(emb.astype(np.int64) + ((sign * np.outer(A, B)) >> cs))      # [256, D], explicit
        assert (got[m] == table[tok[m]]).all()
    assert (got != emb[tok]).any()


def test_embedding_factors_are_the_ones_the_update_contracts():
    # update with F = e_i returns A_i B_i^T in the table's layout [256, D]; a lookup with a zero table and
    # corr_shift 0 returns row t of the same matrix
    D, N, bound = 16, 6, 8
    i = 4
    F = np.zeros(N, np.int8)
    F[i] = 1
    _, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, 256, D, bound, F, 0, np.zeros((256, D), np.int8))
    tok = np.arange(N, dtype=np.uint8) * 37
    got = oracle.embed_i8(SEED, STEP, LAYER, 0, N, D, bound, 0, np.zeros((256, D), np.int8), tok)
    assert (got[i] == E[tok[i]]).all() and np.abs(E).max() <= 64


# ------------------------------------------------------------------------------------------------
# the composed forward pass
# ------------------------------------------------------------------------------------------------
def params(D, L, seed, wmax=24):
    rng = np.random.default_rng(seed)
    sh = oracle.egg_param_shapes(D, L)
    P = {k: rng.integers(-wmax, wmax + 1, sh[k]).astype(np.int8) for k in sh}
    for k in ("ln1", "ln2", "ln_out"):
        P[k] = rng.integers(8, 25, sh[k]).astype(np.int8)
    return P


def chain(P, D, L, mb, N, bound, cs, tok, S, anti):
    """Alg. "EGG forward pass" from the separately pinned parts, one token."""
    os_d = {16: 6, 64: 7, 256: 8}[D]
    mm = lambda layer, W, X, do, di, os_: oracle.matmul_i8(SEED, STEP, layer, mb, N, do, di, bound, cs, os_, W, X,
                                                          antithetic=anti)
    y = oracle.embed_i8(SEED, STEP, LAYER, mb, N, D, bound, cs, P["emb"], tok, antithetic=anti).astype(np.int64)
    S_out = np.empty_like(S)
    for i in range(L):
        base = LAYER + 1 + 6 * i
        u = oracle.layernorm_i8(P["ln1"][i], y.astype(np.int8))
        w = P["gru_w"][i]
        h = oracle.gru_step_i8(SEED, STEP, base, mb, N, D, bound, cs, os_d, w[0], w[1], w[2], w[3], P["gru_b"][i, 0],
                               P["gru_b"][i, 1], u, S[i], antithetic=anti)
        S_out[i] = h
        y = clip(h.astype(np.int64) + y)
        u = oracle.layernorm_i8(P["ln2"][i], y.astype(np.int8))
        hid = mm(base + 4, P["mlp1"][i], u, 4 * D, D, os_d)
        y = clip(mm(base + 5, P["mlp2"][i], hid, D, 4 * D, os_d + 1).astype(np.int64) + y)
    u = oracle.layernorm_i8(P["ln_out"], y.astype(np.int8))
    return mm(LAYER + 1 + 6 * L, P["head"], u, 256, D, os_d), S_out


@pytest.mark.parametrize("D,L,N,anti", [(16, 2, 6, False), (64, 3, 4, True), (16, 0, 5, False)])
def test_forward_equals_the_chain_of_its_parts(D, L, N, anti):
    P = params(D, L, D + L)
    rng = np.random.default_rng(7)
    T, mb, bound, cs = 3, 2, 8, 3
    tok = rng.integers(0, 256, (T, N)).astype(np.uint8)
    S = rng.integers(-100, 101, (L, N, D)).astype(np.int8)
    logits, S_out = oracle.egg_forward_i8(SEED, STEP, LAYER, mb, N, D, L, bound, cs, P, tok, S, antithetic=anti)
    state = S
    for t in range(T):
        want, state = chain(P, D, L, mb, N, bound, cs, tok[t], state, anti)
        assert (logits[t] == want).all(), t
    assert (S_out == state).all()
    assert logits.std() > 5 and np.abs(logits).max() <= 127


def test_zero_blocks_reduce_to_the_model_without_layers():
    # all GRU/MLP matrices, biases, noise and states zero: every block returns 0 and y stays emb[t]
    D, L, N = 16, 2, 7
    P = params(D, L, 11)
    for k in ("gru_w", "gru_b", "mlp1", "mlp2"):
        P[k][...] = 0
    P0 = {k: (v[:0] if k in ("ln1", "gru_w", "gru_b", "ln2", "mlp1", "mlp2") else v) for k, v in P.items()}
    tok = np.random.default_rng(8).integers(0, 256, (2, N)).astype(np.uint8)
    a, Sa = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 0, 4, P, tok, np.zeros((L, N, D), np.int8))
    b, _ = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, 0, 0, 4, P0, tok, np.zeros((0, N, D), np.int8))
    assert (a == b).all() and (Sa == 0).all()


def test_tokens_in_one_call_equal_calls_with_carried_state_and_member_chunks():
    D, L, N, T = 16, 2, 8, 4
    P = params(D, L, 12)
    rng = np.random.default_rng(9)
    tok = rng.integers(0, 256, (T, N)).astype(np.uint8)
    S = rng.integers(-50, 51, (L, N, D)).astype(np.int8)
    full, S_full = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 8, 3, P, tok, S, antithetic=True)
    state = S
    for t in range(T):
        lg, state = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 8, 3, P, tok[t:t + 1], state, antithetic=True)
        assert (lg[0] == full[t]).all()
    assert (state == S_full).all()
    h = N // 2
    lo, S_lo = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, h, D, L, 8, 3, P, tok[:, :h], S[:, :h], antithetic=True)
    hi, S_hi = oracle.egg_forward_i8(SEED, STEP, LAYER, h, h, D, L, 8, 3, P, tok[:, h:], S[:, h:], antithetic=True)
    assert (np.concatenate([lo, hi], 1) == full).all() and (np.concatenate([S_lo, S_hi], 1) == S_full).all()


def test_without_noise_members_with_equal_inputs_agree_and_noise_separates_them():
    D, L, N = 16, 2, 6
    P = params(D, L, 13)
    tok = np.full((3, N), 65, np.uint8)
    S = np.zeros((L, N, D), np.int8)
    quiet, _ = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 0, 3, P, tok, S)
    assert (quiet == quiet[:, :1]).all()
    noisy, _ = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 8, 1, P, tok, S)
    assert any((noisy[:, m] != noisy[:, 0]).any() for m in range(1, N))


# ------------------------------------------------------------------------------------------------
# fitness: integer log-likelihood
# ------------------------------------------------------------------------------------------------
def test_loglik_of_equal_logits_is_minus_eight_bits():
    # all 256 logits equal: every token has probability 1/256 = 8 bits = 128 sixteenths, whatever the level
    for level in (-127, -40, 0, 77, 127):
        y = np.full((3, 256), level, np.int8)
        o = oracle.loglik_i8(y, np.array([0, 100, 255], np.uint8))
        assert (np.abs(o + 128) <= 1).all(), (level, o)


def test_loglik_tracks_the_real_log_softmax_and_normalises():
    rng = np.random.default_rng(0)
    y = rng.integers(-127, 128, (200, 256)).astype(np.int8)
    y[:50] = rng.integers(-20, 21, (50, 256))                     # flat rows as well as peaked ones
    t = rng.integers(0, 256, 200).astype(np.uint8)
    o = oracle.loglik_i8(y, t)
    z = y.astype(np.float64) / 16.0                                # logits in bits
    ref = 16.0 * (z[np.arange(200), t] - np.log2(np.exp2(z).sum(1)))
    assert np.abs(o - ref).max() <= 1.5 and (o <= 1).all()        # two table roundings
    # over all 256 targets of a row the probabilities 2^(o/16) sum to about 1
    row = y[7]
    allo = oracle.loglik_i8(np.repeat(row[None], 256, 0), np.arange(256, dtype=np.uint8))
    assert abs(np.exp2(allo / 16.0).sum() - 1.0) < 0.05


def test_loglik_moves_with_the_target_logit_and_accumulates():
    y = np.zeros((2, 256), np.int8)
    y[1, 9] = 64                                                   # 4 bits above the rest
    o = oracle.loglik_i8(y, np.array([9, 9], np.uint8))
    assert o[1] > o[0] + 40
    again = oracle.loglik_i8(y, np.array([9, 9], np.uint8), out=o)
    assert (again == 2 * o).all()
