"""Pins for the oracle's integer GRU cell (App. "GRU" of the EGG architecture; CPU only): a second,
independent numpy transcription of the four printed equations on top of the separately pinned
perturbed matmul, closed-form special cases, and the range invariant of I8."""
import numpy as np
import pytest

import oracle

SEED, STEP, LAYER = 31, 1, 40


def clip(v):
    return np.clip(v, -127, 127)


def make(D, N, seed, wmax=20):
    rng = np.random.default_rng(seed)
    mats = [rng.integers(-wmax, wmax + 1, (D, D)).astype(np.int8) for _ in range(4)]
    bf, bh = rng.integers(-30, 31, D).astype(np.int8), rng.integers(-30, 31, D).astype(np.int8)
    U, S = rng.integers(-127, 128, (N, D)).astype(np.int8), rng.integers(-127, 128, (N, D)).astype(np.int8)
    return mats, bf, bh, U, S


@pytest.mark.parametrize("D,N,anti", [(16, 9, False), (32, 6, True), (48, 4, False)])
def test_cell_equals_the_four_printed_equations(D, N, anti):
    (Wf, Uf, Wh, Uh), bf, bh, U, S = make(D, N, D)
    bound, cs, os_, mb = 8, 3, 6, 4
    got = oracle.gru_step_i8(SEED, STEP, LAYER, mb, N, D, bound, cs, os_, Wf, Uf, Wh, Uh, bf, bh, U, S, antithetic=anti)
    mm = lambda layer, W, X: oracle.matmul_i8(SEED, STEP, layer, mb, N, D, D, bound, cs, os_, W, X, antithetic=anti).astype(np.int64)
    s, u = S.astype(np.int64), U
    f = clip(mm(LAYER, Wf, u) + mm(LAYER + 1, Uf, S) + bf.astype(np.int64))
    f_hat = clip(((f + 127) * s) >> 8)
    h_hat = clip(mm(LAYER + 2, Wh, u) + mm(LAYER + 3, Uh, f_hat.astype(np.int8)) + bh.astype(np.int64))
    h = clip(s + clip(((f + 127) * (h_hat - s)) >> 8))
    assert (got == h).all()
    assert np.abs(got).max() <= 127 and (got != S).any()


def test_zero_weights_closed_form():
    # all matrices, biases and noise zero: f = 0, f^ = (127 s) >> 8, h^ = 0, h = s + ((127 * (-s)) >> 8)
    D, N = 16, 5
    Z, z = np.zeros((D, D), np.int8), np.zeros(D, np.int8)
    S = np.random.default_rng(0).integers(-127, 128, (N, D)).astype(np.int8)
    U = np.random.default_rng(1).integers(-127, 128, (N, D)).astype(np.int8)
    got = oracle.gru_step_i8(SEED, STEP, LAYER, 0, N, D, 0, 4, 8, Z, Z, Z, Z, z, z, U, S)
    s = S.astype(np.int64)
    assert (got == clip(s + ((127 * (-s)) >> 8))).all()


def test_gate_extremes():
    # f = -127 (gate closed): the state is kept; f = +127 (gate open, factor 254/256): h moves to h^ almost fully
    D, N = 16, 4
    Z, z = np.zeros((D, D), np.int8), np.zeros(D, np.int8)
    S = np.random.default_rng(2).integers(-60, 61, (N, D)).astype(np.int8)   # |h^ - s| stays inside I8
    U = np.zeros((N, D), np.int8)
    closed = oracle.gru_step_i8(SEED, STEP, LAYER, 0, N, D, 0, 4, 8, Z, Z, Z, Z, np.full(D, -127, np.int8), z, U, S)
    assert (closed == S).all()
    bh = np.full(D, 50, np.int8)
    opened = oracle.gru_step_i8(SEED, STEP, LAYER, 0, N, D, 0, 4, 8, Z, Z, Z, Z, np.full(D, 127, np.int8), bh, U, S)
    s = S.astype(np.int64)
    assert (opened == clip(s + ((254 * (50 - s)) >> 8))).all()
    assert np.abs(opened.astype(np.int64) - 50).max() <= 2
