"""GPU parity: the integer GRU cell over a sequence of inputs, bit for bit against the oracle's
step-by-step transcription of the printed equations."""
import numpy as np
import pytest

import oracle
from paper_2511_16652_amd import binding as eb

pytestmark = pytest.mark.gpu

SEED, STEP, LAYER = 8, 3, 100


@pytest.fixture(scope="module")
def ctx():
    import torch
    c = eb.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def make(D, N, T, seed, wmax=14):
    rng = np.random.default_rng(seed)
    mats = [rng.integers(-wmax, wmax + 1, (D, D)).astype(np.int8) for _ in range(4)]
    bf, bh = rng.integers(-30, 31, D).astype(np.int8), rng.integers(-30, 31, D).astype(np.int8)
    U = rng.integers(-127, 128, (T, N, D)).astype(np.int8)
    S = rng.integers(-127, 128, (N, D)).astype(np.int8)
    return mats, bf, bh, U, S


def run(ctx, D, N, T, mats, bf, bh, U, S, mb, anti, bound=8, cs=4, os_=7, alias=False):
    import torch
    dev = [torch.from_numpy(m).cuda() for m in mats]
    s_in = torch.from_numpy(S.copy()).cuda()
    out = s_in if alias else torch.empty_like(s_in)
    ctx.eggroll_gru_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(mb, N, 1, D, D, 1, antithetic=anti), bound, cs, os_, T,
                       dev[0], dev[1], dev[2], dev[3], torch.from_numpy(bf).cuda(), torch.from_numpy(bh).cuda(),
                       torch.from_numpy(U).cuda(), s_in, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def ref(D, N, T, mats, bf, bh, U, S, mb, anti, bound=8, cs=4, os_=7):
    h = S
    for t in range(T):
        h = oracle.gru_step_i8(SEED, STEP, LAYER, mb, N, D, bound, cs, os_, *mats, bf, bh, U[t], h, antithetic=bool(anti))
    return h


@pytest.mark.parametrize("D,N,T,mb,anti", [(64, 33, 1, 0, 0), (256, 300, 3, 5, 0), (144, 130, 2, 6, 1), (1024, 70, 2, 0, 0),
                                            (256, 1026, 4, 2, 1),
                                            (256, 2500, 3, 0, 0), (256, 4102, 2, 4, 1)])   # row-streaming matmul kernel
def test_gru_cell_bit_exact(ctx, D, N, T, mb, anti):
    mats, bf, bh, U, S = make(D, N, T, D + N)
    got = run(ctx, D, N, T, mats, bf, bh, U, S, mb, anti)
    want = ref(D, N, T, mats, bf, bh, U, S, mb, anti)
    assert (got == want).all()
    assert np.abs(got).max() <= 127 and (got != S).mean() > 0.5
    assert (np.abs(want) == 127).mean() < 0.9   # the state is not swamped by the clamp


def test_gru_large_weights_exercise_every_clamp(ctx):
    D, N, T = 128, 200, 3
    mats, bf, bh, U, S = make(D, N, T, 17, wmax=90)
    got = run(ctx, D, N, T, mats, bf, bh, U, S, 0, 0, os_=5)
    want = ref(D, N, T, mats, bf, bh, U, S, 0, 0, os_=5)
    assert (got == want).all()
    assert (np.abs(want) == 127).mean() > 0.01


def test_gru_in_place_and_closed_forms(ctx):
    D, N = 64, 40
    mats, bf, bh, U, S = make(D, N, 1, 3)
    assert (run(ctx, D, N, 1, mats, bf, bh, U, S, 0, 0, alias=True) == ref(D, N, 1, mats, bf, bh, U, S, 0, 0)).all()
    # zero matrices and noise, gate closed (bf = -127): the state is kept exactly
    Z = [np.zeros((D, D), np.int8)] * 4
    kept = run(ctx, D, N, 1, Z, np.full(D, -127, np.int8), np.zeros(D, np.int8), U, S, 0, 0, bound=0)
    assert (kept == S).all()


def test_gru_real_shape_sampled(ctx):
    """The cell at the integer model's real width (D = 256) over a large population and 8 inputs:
    sampled members against the oracle (a member's trajectory depends on no other member)."""
    D, N, T = 256, 65536, 8
    mats, bf, bh, U, S = make(D, N, T, 99)
    got = run(ctx, D, N, T, mats, bf, bh, U, S, 0, 0)
    rng = np.random.default_rng(1)
    for m in np.sort(rng.choice(N, 32, replace=False)):
        want = ref(D, 1, T, mats, bf, bh, U[:, m:m + 1], S[m:m + 1], int(m), 0)
        assert (got[m] == want[0]).all(), int(m)
