"""GPU parity: antithetic pairs (members 2p, 2p+1 evaluate M + sigma E_p and M - sigma E_p) in the
float forward, its caches feeding the update in the pair view, and the integer recurrence --
against the oracle's explicit definitions, same tolerances as the non-antithetic tests."""
import numpy as np
import pytest

import oracle
from helpers import assert_close, assert_close_bf16_factors, to_device, to_numpy
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


def forward(ctx, wl, member_begin, caches=False, sigma=None, y_dtype=None, W=None):
    import torch
    W = wl.W if W is None else W
    dW, dX = to_device(W, wl.dtype), to_device(wl.X, wl.dtype)
    ydt = {"f32": torch.float32, "bf16": torch.bfloat16}[y_dtype or wl.dtype]
    Y = torch.empty((wl.X.shape[0], wl.d_out), dtype=ydt, device="cuda")
    A = B = None
    if caches:
        A = torch.empty((wl.N // 2, wl.d_out, wl.rank), dtype=dW.dtype, device="cuda")
        B = torch.empty((wl.N // 2, wl.d_in, wl.rank), dtype=dW.dtype, device="cuda")
    ctx.eggroll_perturbed_forward(eb.make_key(wl.noise_seed, wl.step, wl.layer),
                                  eb.make_shape(member_begin, wl.N, wl.S, wl.d_out, wl.d_in, wl.rank, antithetic=1),
                                  wl.sigma if sigma is None else sigma, eb.EGG_ACT_NONE, dW, dX, Y, A, B)
    torch.cuda.synchronize()
    return to_numpy(Y), A, B


def ref(wl, member_begin, sigma=None, W=None):
    nd = oracle.NOISE_BF16 if wl.dtype == "bf16" else oracle.NOISE_F32
    return oracle.forward(wl.noise_seed, wl.step, wl.layer, member_begin, wl.N, wl.S, wl.d_out, wl.d_in, wl.rank, nd,
                          wl.sigma if sigma is None else sigma, 0, wl.W if W is None else W, wl.X, antithetic=True)


SHAPES = [  # dtype, d_out, d_in, members, S, rank, sigma   (every epilogue route, ragged edges)
    ("f32", 132, 100, 70, 1, 1, 0.05),     # regenerated in registers, pairs of neighbouring rows
    ("f32", 64, 36, 34, 3, 2, 0.1),        # staged slices, pair = 6 rows
    ("bf16", 388, 264, 300, 1, 1, 0.02),   # regenerated in registers
    ("bf16", 132, 520, 38, 7, 2, 0.02),    # staged slices
    ("bf16", 260, 136, 6, 16, 4, 0.02),    # pair = 32 rows: extra-MFMA correction
    ("bf16", 260, 136, 4, 64, 8, 0.02),    # extra-MFMA correction, rank 8
]


@pytest.mark.parametrize("shape", SHAPES)
def test_antithetic_forward(ctx, shape):
    dtype, d_out, d_in, N, S, r, sigma = shape
    wl = inputs.make_linear("t", dtype, d_out, d_in, N, S, r, sigma, 71)
    wl.noise_seed, wl.step, wl.layer = 5, 2, 9
    y, _, _ = forward(ctx, wl, member_begin=6)
    want = ref(wl, 6)
    assert_close(y, want, 1e-2 if dtype == "bf16" else 1e-5, str(shape))
    # the correction alone (W = 0), fp32 output: the two members of a pair are negatives of each other
    # (to fp32 rounding: the matrix cores' internal accumulation need not be exactly sign-symmetric)
    Z = np.zeros_like(wl.W)
    wl.X[S:2 * S] = wl.X[0:S]  # pair 0 sees the same rows
    y0, _, _ = forward(ctx, wl, 6, y_dtype="f32", W=Z)
    want0 = ref(wl, 6, W=Z)
    if dtype == "bf16":
        assert_close_bf16_factors(y0, want0, str(shape) + " W=0")
    else:
        assert_close(y0, want0, 1e-5, str(shape) + " W=0")
    assert np.abs(y0[0:S] + y0[S:2 * S]).max() <= 1e-6 * np.abs(y0[0:S]).max() and np.abs(y0[0:S]).min() > 0


@pytest.mark.parametrize("dtype,S,r", [("bf16", 1, 1), ("bf16", 32, 2), ("f32", 2, 1)])
def test_antithetic_caches_hold_one_entry_per_pair_and_feed_the_update(ctx, dtype, S, r):
    import torch
    d_out, d_in, N = 136, 104, 48
    wl = inputs.make_linear("c", dtype, d_out, d_in, N, S, r, 0.03, 72)
    y, A, B = forward(ctx, wl, member_begin=10, caches=True)
    assert_close(y, ref(wl, 10), 1e-2 if dtype == "bf16" else 1e-5, "with caches")
    nd = oracle.NOISE_BF16 if dtype == "bf16" else oracle.NOISE_F32
    pairs, p0 = N // 2, 5
    a_ref = np.stack([oracle.noise_matrix(wl.noise_seed, wl.step, wl.layer, 0, p0 + p, d_out, r, nd) for p in range(pairs)])
    b_ref = np.stack([oracle.noise_matrix(wl.noise_seed, wl.step, wl.layer, 1, p0 + p, d_in, r, nd) for p in range(pairs)])
    tol = 2.0 ** -5 if dtype == "bf16" else 1e-5
    assert np.abs(to_numpy(A) - a_ref).max() <= tol and np.abs(to_numpy(B) - b_ref).max() <= tol
    # the update in the pair view: member ids = pair ids, one fitness per pair
    f = np.random.default_rng(3).standard_normal(pairs).astype(np.float32)
    G = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    code = eb.EGG_BF16 if dtype == "bf16" else eb.EGG_F32
    ctx.eggroll_update(eb.make_key(wl.noise_seed, wl.step, wl.layer), eb.make_shape(p0, pairs, 1, d_out, d_in, r), code,
                       torch.from_numpy(f).cuda(), 0.25, 0, G, None, 0.0, A, B)
    torch.cuda.synchronize()
    want = oracle.update(wl.noise_seed, wl.step, wl.layer, p0, pairs, d_out, d_in, r, nd, f.astype(np.float64), 0.25)
    if dtype == "bf16":
        assert_close_bf16_factors(G.cpu().numpy(), want, "pair update")
    else:
        assert_close(G.cpu().numpy(), want, 1e-5, "pair update")


@pytest.mark.parametrize("d,N,steps,bound,cs,os_", [(64, 34, 1, 8, 4, 8), (144, 300, 3, 8, 4, 6), (1024, 70, 4, 8, 4, 8),
                                                     (128, 258, 2, 127, 9, 9)])
def test_antithetic_integer_recurrence_bit_exact(ctx, d, N, steps, bound, cs, os_):
    import torch
    wl = inputs.make_int8("t", d, N, steps, 31, bound, cs, os_)
    wl.H0[1::2] = wl.H0[0::2]    # both members of a pair start from the same state
    rng = np.random.default_rng(1)
    wl.W = rng.integers(-12, 13, size=wl.W.shape).astype(np.int8)   # keeps the state off the clamp
    W, H = torch.from_numpy(wl.W).cuda(), torch.from_numpy(wl.H0).cuda()
    out = torch.empty_like(H)
    ctx.eggroll_perturbed_forward_i8(eb.make_key(3, 1, 4), eb.make_shape(8, N, 1, d, d, 1, antithetic=1), bound, cs, os_,
                                     steps, W, H, out)
    torch.cuda.synchronize()
    want = oracle.forward_i8(3, 1, 4, 8, N, d, bound, cs, os_, steps, wl.W, wl.H0, antithetic=True)
    got = out.cpu().numpy()
    assert (got == want).all()
    assert (got[0::2] != got[1::2]).any()


def test_antithetic_argument_errors(ctx):
    import torch
    W = torch.zeros((32, 32), dtype=torch.float32, device="cuda")
    X = torch.zeros((6, 32), dtype=torch.float32, device="cuda")
    Y = torch.empty((6, 32), dtype=torch.float32, device="cuda")
    key = eb.make_key(0, 0, 0)
    for mb, n in ((1, 6), (0, 5)):
        with pytest.raises(eb.EggrollError) as e:
            ctx.eggroll_perturbed_forward(key, eb.make_shape(mb, n, 1, 32, 32, 1, antithetic=1), 0.1, eb.EGG_ACT_NONE, W, X, Y)
        assert e.value.status == eb.EGG_EINVAL
    G = torch.empty((32, 32), dtype=torch.float32, device="cuda")
    f = torch.zeros(6, dtype=torch.float32, device="cuda")
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_update(key, eb.make_shape(0, 6, 1, 32, 32, 1, antithetic=1), eb.EGG_F32, f, 1.0, 0, G)
    assert e.value.status == eb.EGG_EINVAL
