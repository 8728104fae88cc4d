"""GPU parity: the integer parameter update (E = (diag(F)A)^T B, one-bin threshold moves), bit for
bit against the oracle's explicit outer products -- both E and the updated int8 weights."""
import numpy as np
import pytest

import oracle
from paper_2511_16652_amd import binding as eb

pytestmark = pytest.mark.gpu

SEED, STEP, LAYER = 9, 2, 6


@pytest.fixture(scope="module")
def ctx():
    import torch
    c = eb.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def run(ctx, d_out, d_in, N, bound, F, tau, theta, member_begin=0, want_E=True):
    import torch
    th = torch.from_numpy(theta.copy()).cuda()
    E = torch.full((d_out, d_in), 12345, dtype=torch.int32, device="cuda") if want_E else None
    ctx.eggroll_update_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(member_begin, N, 1, d_out, d_in, 1), bound,
                          torch.from_numpy(F).cuda(), tau, th, E)
    torch.cuda.synchronize()
    return th.cpu().numpy(), (E.cpu().numpy() if want_E else None)


def case(d_out, d_in, N, seed, zeros=0.3):
    rng = np.random.default_rng(seed)
    F = rng.choice(np.array([-1, 0, 1], np.int8), N, p=[(1 - zeros) / 2, zeros, (1 - zeros) / 2])
    theta = rng.integers(-127, 128, (d_out, d_in)).astype(np.int8)
    return F, theta


# shapes span one tile, several tiles with ragged edges, a K tail that is not a multiple of 16 members or
# of a 128-member stage, the split-K route (few tiles, many members) and the single-split route
@pytest.mark.parametrize("d_out,d_in,N,bound,mb", [
    (16, 16, 1, 8, 0), (48, 80, 37, 8, 3), (256, 128, 300, 8, 0), (144, 272, 1000, 8, 7), (128, 128, 2049, 3, 0),
    (400, 16, 130, 127, 1), (16, 400, 129, 1, 0), (1024, 1024, 500, 8, 0), (2064, 2048, 260, 8, 2),
    (4096, 3600, 70, 8, 0)])
def test_update_i8_bit_exact(ctx, d_out, d_in, N, bound, mb):
    F, theta = case(d_out, d_in, N, d_out + N)
    std = np.sqrt(bound * (bound + 1) / 3.0)
    tau = eb.eggroll_int_threshold(0.3, max(1, int((F != 0).sum())), std)
    want_t, want_E = oracle.update_i8(SEED, STEP, LAYER, mb, N, d_out, d_in, bound, F, tau, theta)
    got_t, got_E = run(ctx, d_out, d_in, N, bound, F, tau, theta, member_begin=mb)
    assert (got_E == want_E).all()
    assert (got_t == want_t).all()
    assert got_t.min() >= -127
    if N > 16 and bound > 1:
        assert 0 < (got_t != theta).sum() < theta.size  # both branches of the threshold are exercised


def test_threshold_edges_and_without_E_output(ctx):
    d_out, d_in, N, bound = 64, 96, 200, 8
    F, theta = case(d_out, d_in, N, 5, zeros=0.0)
    theta[:8] = 127
    theta[8:16] = -127
    _, E = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, 0, theta)
    for tau in (0, 1, int(np.abs(E).max()), int(np.abs(E).max()) + 1):
        want_t, _ = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, tau, theta)
        got_t, _ = run(ctx, d_out, d_in, N, bound, F, tau, theta, want_E=False)
        assert (got_t == want_t).all(), tau
    # all-zero fitness: nothing moves and E is exactly zero
    got_t, got_E = run(ctx, d_out, d_in, N, bound, np.zeros(N, np.int8), 0, theta)
    assert (got_t == theta).all() and (got_E == 0).all()


def test_repeated_calls_are_identical_and_accumulate_steps(ctx):
    d_out, d_in, N, bound = 272, 144, 3000, 8   # split-K route: the atomics must not make the result order-dependent
    F, theta = case(d_out, d_in, N, 11)
    tau = 50
    a, Ea = run(ctx, d_out, d_in, N, bound, F, tau, theta)
    b, Eb = run(ctx, d_out, d_in, N, bound, F, tau, theta)
    assert (a == b).all() and (Ea == Eb).all()
    twice, _ = run(ctx, d_out, d_in, N, bound, F, tau, a)   # second application moves the same entries again
    want, _ = oracle.update_i8(SEED, STEP, LAYER, 0, N, d_out, d_in, bound, F, tau, a)
    assert (twice == want).all()


def test_update_reads_the_factors_the_integer_forward_uses(ctx):
    # F = e_i: E = A_i B_i^T, the very factors of member i of the integer forward for the same key
    import torch
    d, N, bound, i = 64, 40, 8, 17
    F = np.zeros(N, np.int8)
    F[i] = 1
    _, E = run(ctx, d, d, N, bound, F, 1, np.zeros((d, d), np.int8))
    A = torch.empty((N, d), dtype=torch.int8, device="cuda")
    B = torch.empty((N, d), dtype=torch.int8, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(SEED, STEP, LAYER), eb.make_shape(0, N, 1, d, d, 1), eb.EGG_I8, eb.EGG_UNIFORM_INT,
                          bound, A, B)
    torch.cuda.synchronize()
    assert (E == np.outer(A[i].cpu().numpy().astype(np.int64), B[i].cpu().numpy().astype(np.int64))).all()


def test_update_i8_argument_errors(ctx):
    import torch
    th = torch.zeros((32, 32), dtype=torch.int8, device="cuda")
    F = torch.zeros(8, dtype=torch.int8, device="cuda")
    key = eb.make_key(0, 0, 0)
    for shape, bound, tau, status in ((eb.make_shape(0, 8, 1, 32, 24, 1), 8, 1, eb.EGG_EUNSUPPORTED),
                                      (eb.make_shape(0, 8, 1, 32, 32, 2), 8, 1, eb.EGG_EUNSUPPORTED),
                                      (eb.make_shape(0, 8, 1, 32, 32, 1), 8, -1, eb.EGG_EINVAL),
                                      (eb.make_shape(0, 8, 1, 32, 32, 1), 128, 1, eb.EGG_EINVAL)):
        with pytest.raises(eb.EggrollError) as e:
            ctx.eggroll_update_i8(key, shape, bound, F, tau, th)
        assert e.value.status == status
