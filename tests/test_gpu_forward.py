"""GPU parity: eggroll_perturbed_forward against the explicit-W_i oracle, element by element.

Tolerance (the benchmark spec): |y - y_ref| <= rtol (|y_ref| + rms(y_ref)), rtol = 1e-5 for the fp32 path
and 1e-2 for bf16 outputs.  Because the correction is only a few percent of the output at the
configured sigma, the W = 0 cases check it on its own at the same tolerance, and the fp32-output
mode of the bf16 path checks it without the final bf16 rounding (see
helpers.assert_close_bf16_factors for the two-level bound used there).
"""
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


def run_forward(ctx, wl, sigma=None, act=eb.EGG_ACT_NONE, y_dtype=None, member_begin=0, caches=False, W=None, X=None):
    import torch
    sigma = wl.sigma if sigma is None else sigma
    W = wl.W if W is None else W
    X = wl.X if X is None else X
    dW, dX = to_device(W, wl.dtype), to_device(X, wl.dtype)
    ydt = {"f32": torch.float32, "bf16": torch.bfloat16}[y_dtype or wl.dtype]
    Y = torch.empty((X.shape[0], wl.d_out), dtype=ydt, device="cuda")
    n = X.shape[0] // wl.S
    A = B = None
    if caches:
        A = torch.empty((n, wl.d_out, wl.rank), dtype=dW.dtype, device="cuda")
        B = torch.empty((n, wl.d_in, wl.rank), dtype=dW.dtype, device="cuda")
    ctx.eggroll_perturbed_forward(eb.make_key(wl.noise_seed, wl.step, wl.layer),
                                  eb.make_shape(member_begin, n, wl.S, wl.d_out, wl.d_in, wl.rank),
                                  sigma, act, dW, dX, Y, A, B)
    torch.cuda.synchronize()
    return (to_numpy(Y), A, B)


def ref_forward(wl, sigma=None, act=0, member_begin=0, W=None, X=None):
    sigma = wl.sigma if sigma is None else sigma
    W = wl.W if W is None else W
    X = wl.X if X is None else X
    nd = oracle.NOISE_BF16 if wl.dtype == "bf16" else oracle.NOISE_F32
    return oracle.forward(wl.noise_seed, wl.step, wl.layer, member_begin, X.shape[0] // wl.S, wl.S, wl.d_out,
                          wl.d_in, wl.rank, nd, sigma, act, W, X)


RT = {"f32": 1e-5, "bf16": 1e-2}


def test_config1_fp32_full(ctx):
    wl = inputs.config1()
    y, _, _ = run_forward(ctx, wl)
    assert_close(y, ref_forward(wl), 1e-5, "cfg1")


SHAPES = [  # dtype, d_out, d_in, N, S, rank, sigma   (ragged: nothing is a multiple of a tile)
    ("f32", 132, 100, 70, 1, 1, 0.05),
    ("f32", 260, 72, 9, 5, 2, 0.05),
    ("f32", 64, 36, 33, 2, 4, 0.1),
    ("f32", 36, 40, 150, 1, 8, 0.1),
    ("bf16", 388, 264, 300, 1, 1, 0.02),
    ("bf16", 132, 520, 37, 7, 2, 0.02),
    ("bf16", 260, 136, 5, 64, 4, 0.02),
    ("bf16", 72, 72, 140, 1, 8, 0.02),
    ("f32", 40, 36, 21, 3, 16, 0.1),
    ("bf16", 136, 72, 50, 1, 16, 0.02),
    ("bf16", 96, 160, 4, 64, 16, 0.02),     # rows per member a multiple of 32: no extra-MFMA fold at this rank
    ("bf16", 64, 8192, 6, 2, 16, 0.02),     # d_in * rank beyond one LDS panel of the projection pass
]


@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes(ctx, shape):
    dtype, d_out, d_in, N, S, r, sigma = shape
    wl = inputs.make_linear("t", dtype, d_out, d_in, N, S, r, sigma, 77)
    wl.noise_seed, wl.step, wl.layer = 5, 2, 9
    y, _, _ = run_forward(ctx, wl, member_begin=3)
    assert_close(y, ref_forward(wl, member_begin=3), RT[dtype], str(shape))
    # the correction alone (W = 0), and without the final rounding of y in the bf16 path
    Z = np.zeros_like(wl.W)
    y0, _, _ = run_forward(ctx, wl, member_begin=3, W=Z, y_dtype="f32")
    if dtype == "f32":
        assert_close(y0, ref_forward(wl, member_begin=3, W=Z), 1e-5, "W=0 " + str(shape))
    else:
        assert_close_bf16_factors(y0, ref_forward(wl, member_begin=3, W=Z), "W=0 " + str(shape))


PERSISTENT = [  # d_out, d_in, N, S, rank, act, residual: >= 192 tiles of 256 x 256, bf16 in and out, 64 | S and 64 | d_in --
    # the persistent kernel with the store-only epilogue; tile edges ragged in both directions
    (1028, 128, 163, 64, 1, 0, False),
    (1028, 192, 163, 64, 4, 1, False),
    (772, 64, 131, 128, 8, 0, True),
    (1284, 128, 81, 128, 2, 1, True),
    (2052, 64, 25, 256, 1, 1, False),
]


@pytest.mark.parametrize("case", PERSISTENT)
def test_persistent_kernel_ragged_tiles(ctx, case):
    """One workgroup per compute unit walking several tiles each, last row and column tiles partial, every store-only epilogue
    variant (plain, GELU, residual, both), perturbed and unperturbed."""
    import torch
    d_out, d_in, N, S, r, act, resid = case
    wl = inputs.make_linear("p", "bf16", d_out, d_in, N, S, r, 0.05, 90 + d_out)
    wl.noise_seed, wl.step, wl.layer = 7, 3, 12
    R = N * S
    assert ((d_out + 255) // 256) * ((R + 255) // 256) >= 192 and (R % 256 or d_out % 256)
    dW, dX = to_device(wl.W, "bf16"), to_device(wl.X, "bf16")
    Rn = inputs.round_to_bf16(np.random.default_rng(d_out).standard_normal((R, d_out)).astype(np.float32)) if resid else None
    key, shape = eb.make_key(7, 3, 12), eb.make_shape(5, N, S, d_out, d_in, r)
    for sigma in (0.05, 0.0):
        Y = torch.full((R, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
        guard = torch.full((4096,), 7.0, dtype=torch.bfloat16, device="cuda")   # allocated right behind Y: stays untouched
        if resid:
            ctx.eggroll_perturbed_forward_add(key, shape, sigma, act, dW, dX, to_device(Rn, "bf16"), Y)
        else:
            ctx.eggroll_perturbed_forward(key, shape, sigma, act, dW, dX, Y)
        torch.cuda.synchronize()
        ref = oracle.forward(7, 3, 12, 5, N, S, d_out, d_in, r, oracle.NOISE_BF16, sigma, act, wl.W, wl.X)
        if resid:
            ref = ref + Rn.astype(np.float64)
        assert_close(to_numpy(Y), ref, 1e-2, "%s sigma %g" % (case, sigma))
        assert bool((guard == 7.0).all())
    # the correction on its own (W = 0): what the folded extra MFMA adds, at the tolerance of the bf16 factors
    Y0 = torch.empty((R, d_out), dtype=torch.bfloat16, device="cuda")
    ctx.eggroll_perturbed_forward(key, shape, 0.05, 0, torch.zeros_like(dW), dX, Y0)
    torch.cuda.synchronize()
    ref0 = oracle.forward(7, 3, 12, 5, N, S, d_out, d_in, r, oracle.NOISE_BF16, 0.05, 0, np.zeros_like(wl.W), wl.X)
    assert_close(to_numpy(Y0), ref0, 1e-2, "W = 0 %s" % (case,))


def test_big_tile_path_bf16(ctx):
    # enough 256x256 tiles to take the large-tile kernel; K = 136 leaves a partial K-tile
    wl = inputs.make_linear("big", "bf16", 3072, 136, 4096, 1, 1, 0.02, 78)
    y, A, B = run_forward(ctx, wl, caches=True)
    assert_close(y, ref_forward(wl), 1e-2, "big tiles")
    Z = np.zeros_like(wl.W)
    y0, _, _ = run_forward(ctx, wl, W=Z, y_dtype="f32")
    assert_close_bf16_factors(y0, ref_forward(wl, W=Z), "big tiles W=0")


def test_sigma_zero_is_plain_gemm_and_linear_in_sigma(ctx):
    wl = inputs.make_linear("s", "bf16", 260, 264, 130, 2, 2, 0.05, 79)
    y0, _, _ = run_forward(ctx, wl, sigma=0.0, y_dtype="f32")
    ref = wl.X.astype(np.float64) @ wl.W.astype(np.float64).T
    assert_close(y0, ref, 1e-5, "sigma=0")
    y1, _, _ = run_forward(ctx, wl, sigma=0.05, y_dtype="f32")
    y2, _, _ = run_forward(ctx, wl, sigma=0.1, y_dtype="f32")
    d1, d2 = (y1 - y0).astype(np.float64), (y2 - y0).astype(np.float64)
    assert np.abs(d2 - 2 * d1).max() <= 1e-5 * (np.abs(y2).max())
    # run-to-run determinism
    y1b, _, _ = run_forward(ctx, wl, sigma=0.05, y_dtype="f32")
    assert (y1 == y1b).all()


@pytest.mark.parametrize("dtype,S,r", [("bf16", 1, 1), ("bf16", 3, 2), ("f32", 1, 1), ("f32", 2, 4)])
def test_caches_equal_noise_gen_and_chunking_is_exact(ctx, dtype, S, r):
    import torch
    wl = inputs.make_linear("c", dtype, 132, 72, 40, S, r, 0.05, 80)
    y, A, B = run_forward(ctx, wl, caches=True, member_begin=10)
    A2, B2 = torch.empty_like(A), torch.empty_like(B)
    ctx.eggroll_noise_gen(eb.make_key(wl.noise_seed, wl.step, wl.layer), eb.make_shape(10, 40, 1, 132, 72, r),
                          eb.EGG_BF16 if dtype == "bf16" else eb.EGG_F32, eb.EGG_NORMAL, 0, A2, B2)
    torch.cuda.synchronize()
    assert torch.equal(A.view(torch.int16 if dtype == "bf16" else torch.int32), A2.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert torch.equal(B.view(torch.int16 if dtype == "bf16" else torch.int32), B2.view(torch.int16 if dtype == "bf16" else torch.int32))
    # two half-populations give bitwise the rows of the whole
    h = 20 * S
    ya, _, _ = run_forward(ctx, wl, member_begin=10, X=wl.X[:h])
    yb, _, _ = run_forward(ctx, wl, member_begin=30, X=wl.X[h:])
    assert (np.concatenate([ya, yb]) == y).all()


def test_gelu_epilogue(ctx):
    wl = inputs.make_linear("g", "bf16", 132, 136, 50, 2, 1, 0.05, 81)
    wl.X = inputs.round_to_bf16(wl.X * 2)
    y, _, _ = run_forward(ctx, wl, act=eb.EGG_ACT_GELU)
    assert_close(y, ref_forward(wl, act=oracle.ACT_GELU), 1e-2, "gelu")
    wl32 = inputs.make_linear("g", "f32", 64, 64, 20, 1, 1, 0.05, 81)
    y, _, _ = run_forward(ctx, wl32, act=eb.EGG_ACT_GELU)
    assert_close(y, ref_forward(wl32, act=oracle.ACT_GELU), 1e-5, "gelu f32")


def test_argument_errors(ctx):
    import torch
    W = torch.zeros((8, 12), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(eb.EggrollError) as e:  # d_in not a multiple of 8
        ctx.eggroll_perturbed_forward(eb.make_key(0, 0, 0), eb.make_shape(0, 4, 1, 8, 12, 1), 0.1, 0, W, X, Y)
    assert e.value.status == eb.EGG_EUNSUPPORTED
    with pytest.raises(eb.EggrollError) as e:  # rank
        ctx.eggroll_perturbed_forward(eb.make_key(0, 0, 0), eb.make_shape(0, 4, 1, 8, 16, 3), 0.1, 0, W, X, Y)
    assert e.value.status == eb.EGG_EINVAL
    with pytest.raises(eb.EggrollError) as e:  # negative sigma
        ctx.eggroll_perturbed_forward(eb.make_key(0, 0, 0), eb.make_shape(0, 4, 1, 8, 16, 1), -1.0, 0, W, X, Y)
    assert e.value.status == eb.EGG_EINVAL
