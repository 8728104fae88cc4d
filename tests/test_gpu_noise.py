"""GPU parity: eggroll_noise_gen against the CPU oracle (bit-exact words and integers; normals
within the float tolerance derived from the transform's arithmetic)."""
import numpy as np
import pytest

import oracle
from paper_2511_16652_amd import binding as eb

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    c = eb.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


CASES = [  # seed, step, layer, member_begin, members, d_out, d_in, rank
    (0, 0, 0, 0, 5, 64, 48, 1),
    (0xDEADBEEFCAFEF00D, 17, 96, 1000, 7, 33, 77, 1),      # odd lengths: ragged tail blocks
    (3, 2**32 - 1, 2**31 - 1, 2**32 - 9, 9, 40, 24, 4),    # extreme key words and member ids
    (12345, 3, 7, 11, 3, 130, 258, 8),
]


@pytest.mark.parametrize("case", CASES)
def test_raw_words_bit_exact(ctx, case):
    import torch
    seed, step, layer, mb, n, d_out, d_in, r = case
    A = torch.empty((n, d_out, r), dtype=torch.int32, device="cuda")
    B = torch.empty((n, d_in, r), dtype=torch.int32, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(seed, step, layer), eb.make_shape(mb, n, 1, d_out, d_in, r),
                          eb.EGG_U32, eb.EGG_RAW, 0, A, B)
    a = A.cpu().numpy().view(np.uint32)
    b = B.cpu().numpy().view(np.uint32)
    for m in range(n):
        assert (a[m].reshape(-1) == oracle.raw_words(seed, step, layer, 0, mb + m, 0, d_out * r)).all()
        assert (b[m].reshape(-1) == oracle.raw_words(seed, step, layer, 1, mb + m, 0, d_in * r)).all()


def test_raw_words_sixteen_million_bit_exact(ctx):
    """One call at configuration 2's size: 4096 members x 4096 words of each stream (1.7e7 words per stream),
    every word against the oracle."""
    import torch
    n, d = 4096, 4096
    A = torch.empty((n, d, 1), dtype=torch.int32, device="cuda")
    B = torch.empty((n, d, 1), dtype=torch.int32, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(0, 0, 0), eb.make_shape(0, n, 1, d, d, 1), eb.EGG_U32, eb.EGG_RAW, 0, A, B)
    a = A.cpu().numpy().view(np.uint32).reshape(n, d)
    b = B.cpu().numpy().view(np.uint32).reshape(n, d)
    for m in range(n):
        assert (a[m] == oracle.raw_words(0, 0, 0, 0, m, 0, d)).all(), m
        assert (b[m] == oracle.raw_words(0, 0, 0, 1, m, 0, d)).all(), m


@pytest.mark.parametrize("bound", [0, 1, 8, 127])
@pytest.mark.parametrize("case", CASES[:3])
def test_int_noise_bit_exact(ctx, case, bound):
    import torch
    seed, step, layer, mb, n, d_out, d_in, r = case
    A = torch.empty((n, d_out, r), dtype=torch.int8, device="cuda")
    B = torch.empty((n, d_in, r), dtype=torch.int8, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(seed, step, layer), eb.make_shape(mb, n, 1, d_out, d_in, r),
                          eb.EGG_I8, eb.EGG_UNIFORM_INT, bound, A, B)
    a, b = A.cpu().numpy(), B.cpu().numpy()
    for m in range(n):
        assert (a[m].reshape(-1) == oracle.noise_int(seed, step, layer, 0, mb + m, 0, d_out * r, bound)).all()
        assert (b[m].reshape(-1) == oracle.noise_int(seed, step, layer, 1, mb + m, 0, d_in * r, bound)).all()


@pytest.mark.parametrize("case", CASES)
def test_normals_fp32(ctx, case):
    # fp32 factors use library log / sincospi (<= 2 ulp each) and a correctly rounded sqrt; with the
    # final multiply that is a few fp32 ulps of |z| plus an absolute term where the cosine is near 0:
    # |z_gpu - z_ref| <= 2e-6 |z| + 5e-7.
    import torch
    seed, step, layer, mb, n, d_out, d_in, r = case
    A = torch.empty((n, d_out, r), dtype=torch.float32, device="cuda")
    B = torch.empty((n, d_in, r), dtype=torch.float32, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(seed, step, layer), eb.make_shape(mb, n, 1, d_out, d_in, r),
                          eb.EGG_F32, eb.EGG_NORMAL, 0, A, B)
    a, b = A.cpu().numpy().astype(np.float64), B.cpu().numpy().astype(np.float64)
    for m in range(n):
        for got, which, d in ((a[m], 0, d_out), (b[m], 1, d_in)):
            ref = oracle.noise_normal(seed, step, layer, which, mb + m, 0, d * r)
            err = np.abs(got.reshape(-1) - ref)
            assert (err <= 2e-6 * np.abs(ref) + 5e-7).all(), err.max()


def test_normals_bf16_large_sample(ctx):
    # bf16 factors: hardware log2 / sin / cos / sqrt, then round to nearest even.  The value must be
    # the oracle's bf16 value, except where the fp32 value sits within the approximation error of a
    # rounding boundary: then the neighbouring bf16 value is accepted.  Such flips must be rare.
    import torch
    from paper_2511_16652_amd import inputs
    n, d = 64, 8192
    A = torch.empty((n, d, 1), dtype=torch.bfloat16, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(7, 1, 2), eb.make_shape(0, n, 1, d, d, 1), eb.EGG_BF16, eb.EGG_NORMAL, 0, A, None)
    got = A.float().cpu().numpy().reshape(n, d).astype(np.float64)
    ref64 = np.stack([oracle.noise_normal(7, 1, 2, 0, m, 0, d) for m in range(n)])
    ref = inputs.round_to_bf16(ref64.astype(np.float32)).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
    diff = np.abs(got - ref)
    assert (diff <= ulp * 1.0001).all(), "bf16 normal off by more than one ulp"
    flips = (diff > 0).mean()
    assert flips < 2e-3, flips
    # and the unrounded value is close: |got - z64| <= half an ulp + hardware approximation error
    assert (np.abs(got - ref64) <= 0.5 * ulp + 4e-6 * (1 + np.abs(ref64))).all()
    z = got.reshape(-1)
    assert abs(z.mean()) < 5 / np.sqrt(z.size) and abs(z.var() - 1) < 0.01


def test_null_outputs_and_errors(ctx):
    import torch
    B = torch.empty((2, 8, 1), dtype=torch.float32, device="cuda")
    ctx.eggroll_noise_gen(eb.make_key(0, 0, 0), eb.make_shape(0, 2, 1, 8, 8, 1), eb.EGG_F32, eb.EGG_NORMAL, 0, None, B)
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_noise_gen(eb.make_key(0, 0, 0), eb.make_shape(0, 2, 1, 8, 8, 3), eb.EGG_F32, eb.EGG_NORMAL, 0, None, B)
    assert e.value.status == eb.EGG_EINVAL
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_noise_gen(eb.make_key(0, 0, 0), eb.make_shape(0, 2, 1, 8, 8, 1), eb.EGG_I8, eb.EGG_NORMAL, 0, None, B)
    assert e.value.status == eb.EGG_EUNSUPPORTED
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_noise_gen(eb.make_key(0, 0, 0), eb.make_shape(2**32 - 1, 2, 1, 8, 8, 1), eb.EGG_F32, eb.EGG_NORMAL, 0, None, B)
    assert e.value.status == eb.EGG_EINVAL
