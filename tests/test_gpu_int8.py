"""GPU parity: the integer perturbed recurrence, bit-exact against the step-by-step oracle."""
import numpy as np
import pytest

import oracle
from paper_2511_16652_amd import binding as eb
from paper_2511_16652_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    c = eb.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def run(ctx, wl, member_begin=0, alias=False):
    import torch
    W = torch.from_numpy(wl.W).cuda()
    H = torch.from_numpy(wl.H0).cuda()
    out = H if alias else torch.empty_like(H)
    ctx.eggroll_perturbed_forward_i8(eb.make_key(wl.noise_seed, wl.step, wl.layer),
                                     eb.make_shape(member_begin, wl.N, 1, wl.d, wl.d, 1), wl.bound, wl.corr_shift,
                                     wl.out_shift, wl.steps, W, H, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def ref(wl, member_begin=0):
    return oracle.forward_i8(wl.noise_seed, wl.step, wl.layer, member_begin, wl.N, wl.d, wl.bound, wl.corr_shift,
                             wl.out_shift, wl.steps, wl.W, wl.H0)


@pytest.mark.parametrize("d,N,steps,bound,cs,os_", [
    (64, 33, 1, 8, 4, 8), (144, 300, 3, 8, 4, 6), (256, 130, 5, 8, 0, 8), (1024, 70, 4, 8, 4, 8),
    (48, 9, 2, 0, 4, 5), (128, 257, 2, 127, 9, 9), (272, 40, 1, 16, 2, 0),
    (256, 2310, 3, 8, 4, 6), (256, 2048, 2, 127, 9, 9), (256, 2100, 2, 16, 6, 10), (256, 2050, 2, 8, 0, 9), (256, 2050, 1, 8, 8, 0)])   # the row-streaming kernel, with the next step's dot products
def test_int8_bit_exact(ctx, d, N, steps, bound, cs, os_):
    wl = inputs.make_int8("t", d, N, steps, 31, bound, cs, os_)
    wl.noise_seed, wl.step, wl.layer = 3, 1, 4
    assert (run(ctx, wl, member_begin=5) == ref(wl, member_begin=5)).all()


def test_int8_small_values_keep_the_state_alive(ctx):
    # with full-range inputs the state saturates quickly; small weights keep intermediate values
    # spread over the int8 range so that shifts of negative numbers and the clamp are both exercised
    wl = inputs.make_int8("s", 256, 200, 6, 32, 8, 4, 6)
    rng = np.random.default_rng(0)
    wl.W = rng.integers(-12, 13, size=wl.W.shape).astype(np.int8)
    got, want = run(ctx, wl), ref(wl)
    assert (got == want).all()
    assert 0.02 < (np.abs(want) == 127).mean() < 0.98 or np.abs(want).max() < 127


def test_int8_alias_and_big_tiles(ctx):
    wl = inputs.make_int8("a", 128, 64, 1, 33)
    assert (run(ctx, wl, alias=True) == ref(wl)).all()
    wl = inputs.make_int8("b", 1024, 12288, 2, 34)   # 4 x 48 large tiles
    got = run(ctx, wl)
    sample = np.random.default_rng(1).choice(wl.N, 48, replace=False)
    for m in sample:
        one = oracle.forward_i8(0, 0, 0, int(m), 1, wl.d, wl.bound, wl.corr_shift, wl.out_shift, wl.steps, wl.W, wl.H0[m:m + 1])
        assert (got[m] == one[0]).all()


def test_int8_errors(ctx):
    import torch
    W = torch.zeros((24, 24), dtype=torch.int8, device="cuda")
    H = torch.zeros((4, 24), dtype=torch.int8, device="cuda")
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_perturbed_forward_i8(eb.make_key(0, 0, 0), eb.make_shape(0, 4, 1, 24, 24, 1), 8, 4, 8, 1, W, H, H)
    assert e.value.status == eb.EGG_EUNSUPPORTED


@pytest.mark.parametrize("d_out,d_in,N,anti", [(1024, 256, 300, 0), (256, 1024, 130, 0), (48, 272, 70, 1), (2064, 64, 38, 1),
                                                 # d_in = 256 with at least 2048 rows: the row-streaming kernel (ragged rows, ragged and multi-slice d_out)
                                                 (256, 256, 2500, 0), (1024, 256, 2118, 1), (272, 256, 2049, 0), (48, 256, 4100, 1)])
def test_rectangular_single_step_bit_exact(ctx, d_out, d_in, N, anti):
    """One application of a d_out x d_in integer theta (the 4D x D and D x 4D matrices of the integer MLP)."""
    import torch
    rng = np.random.default_rng(d_out + d_in)
    W = rng.integers(-20, 21, (d_out, d_in)).astype(np.int8)
    H = rng.integers(-127, 128, (N, d_in)).astype(np.int8)
    out = torch.empty((N, d_out), dtype=torch.int8, device="cuda")
    ctx.eggroll_perturbed_forward_i8(eb.make_key(3, 1, 4), eb.make_shape(6, N, 1, d_out, d_in, 1, antithetic=anti), 8, 4, 7, 1,
                                     torch.from_numpy(W).cuda(), torch.from_numpy(H).cuda(), out)
    torch.cuda.synchronize()
    want = oracle.matmul_i8(3, 1, 4, 6, N, d_out, d_in, 8, 4, 7, W, H, antithetic=bool(anti))
    got = out.cpu().numpy()
    assert (got == want).all()
    assert 0.01 < (np.abs(want) == 127).mean() < 0.99 or np.abs(want).max() < 127
    if d_out == d_in:
        return
    with pytest.raises(eb.EggrollError):   # a rectangular matrix cannot be iterated
        ctx.eggroll_perturbed_forward_i8(eb.make_key(3, 1, 4), eb.make_shape(6, N, 1, d_out, d_in, 1), 8, 4, 7, 2,
                                         torch.from_numpy(W).cuda(), torch.from_numpy(H).cuda(), out)


def test_table_noise_bit_exact(ctx):
    """The paper's own integer noise (EGG_INT_NOISE_NORMAL16) through noise_gen, the perturbed matmul at the paper's
    shifts (corr_shift = 4 + sigma_hat = 8), a short recurrence, and the integer update."""
    import torch
    T16 = eb.EGG_INT_NOISE_NORMAL16
    n, d_out, d_in = 9, 130, 77
    A = torch.empty((n, d_out, 1), dtype=torch.int8, device="cuda")
    B = torch.empty((n, d_in, 1), dtype=torch.int8, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(3, 1, 4), eb.make_shape(2 ** 32 - 20, n, 1, d_out, d_in, 1), eb.EGG_I8, eb.EGG_NORMAL_INT16, 0, A, B)
    a, b = A.cpu().numpy(), B.cpu().numpy()
    for m in range(n):
        assert (a[m].reshape(-1) == oracle.noise_int(3, 1, 4, 0, 2 ** 32 - 20 + m, 0, d_out, oracle.BOUND_NORMAL16)).all()
        assert (b[m].reshape(-1) == oracle.noise_int(3, 1, 4, 1, 2 ** 32 - 20 + m, 0, d_in, oracle.BOUND_NORMAL16)).all()
    for d, N, steps, anti in ((256, 4096, 3, 0), (1024, 600, 2, 1), (96, 130, 4, 0)):
        wl = inputs.make_int8("t", d, N, steps, 9 + d)
        W, H = torch.from_numpy(wl.W).cuda(), torch.from_numpy(wl.H0).cuda()
        out = torch.empty_like(H)
        ctx.eggroll_perturbed_forward_i8(eb.make_key(0, 0, 5), eb.make_shape(0, N, 1, d, d, 1, antithetic=anti), T16, 8, 4 + int(np.log2(d)) // 2,
                                         steps, W, H, out)
        torch.cuda.synchronize()
        ref = oracle.forward_i8(0, 0, 5, 0, N, d, oracle.BOUND_NORMAL16, 8, 4 + int(np.log2(d)) // 2, steps, wl.W, wl.H0, antithetic=bool(anti))
        assert (out.cpu().numpy() == ref).all(), (d, N)
        assert (ref != oracle.forward_i8(0, 0, 5, 0, N, d, 0, 8, 4 + int(np.log2(d)) // 2, steps, wl.W, wl.H0)).mean() > 0.01   # the noise matters
    N, d = 1000, 128
    wl = inputs.make_int8("u", d, N, 1, 77)
    F = np.random.default_rng(4).choice(np.array([-1, 0, 1], np.int8), N)
    tau = eb.eggroll_int_threshold(0.3, N, 16.0)
    theta = torch.from_numpy(wl.W.copy()).cuda()
    E = torch.empty((d, d), dtype=torch.int32, device="cuda")
    ctx.eggroll_update_i8(eb.make_key(0, 0, 5), eb.make_shape(0, N, 1, d, d, 1), T16, torch.from_numpy(F).cuda(), tau, theta, E)
    torch.cuda.synchronize()
    t_ref, e_ref = oracle.update_i8(0, 0, 5, 0, N, d, d, oracle.BOUND_NORMAL16, F, tau, wl.W)
    assert (E.cpu().numpy() == e_ref).all() and (theta.cpu().numpy() == t_ref).all()
    assert 0.15 < (t_ref != wl.W).mean() < 0.45
