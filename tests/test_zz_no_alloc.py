"""The no-allocation forward entry point against the ordinary one: same kernels, static projection scratch.

Two calls in a row through the C ABI, the second with a smaller input (the static array keeps the first
call's contents), each compared bit for bit with eggroll_perturbed_forward on the same inputs -- which the
other GPU tests hold to the oracle -- and within tolerance with the oracle itself."""
import numpy as np
import pytest

import oracle
from helpers import assert_close, to_device, to_numpy
from paper_2511_16652_amd import binding as eb
from paper_2511_16652_amd import inputs

pytestmark = pytest.mark.gpu


def run_pair(ctx, N, S, d_out, d_in, rank, sigma, seed):
    import torch
    wl = inputs.make_linear("t", "bf16", d_out, d_in, N, S, rank, sigma, seed)
    W, X = to_device(wl.W, "bf16"), to_device(wl.X, "bf16")
    key, shape = eb.make_key(0, 3, 5), eb.make_shape(11, N, S, d_out, d_in, rank)
    need_a = not (S == 1 and rank == 1)
    A1 = torch.empty((N, d_out, rank), dtype=torch.bfloat16, device="cuda") if need_a else None
    A2 = torch.empty_like(A1) if need_a else None
    Y1 = torch.empty((N * S, d_out), dtype=torch.bfloat16, device="cuda")
    Y2 = torch.empty_like(Y1)
    ctx.eggroll_perturbed_forward_noalloc(key, shape, sigma, eb.EGG_ACT_NONE, W, X, Y1, A1, None)
    ctx.eggroll_perturbed_forward(key, shape, sigma, eb.EGG_ACT_NONE, W, X, Y2, A2, None)
    torch.cuda.synchronize()
    assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16))
    if need_a:
        assert torch.equal(A1.view(torch.int16), A2.view(torch.int16))
    ref = oracle.forward(0, 3, 5, 11, N, S, d_out, d_in, rank, oracle.NOISE_BF16, sigma, 0, wl.W, wl.X)
    assert_close(to_numpy(Y1), ref, 1e-2, "no-allocation forward")


def test_noalloc_forward_two_calls_second_smaller():
    import torch
    ctx = eb.Context(0)
    gen = ctx.eggroll_scratch_generation()
    run_pair(ctx, 512, 1, 384, 256, 1, 0.05, 41)     # first call: 512 projections
    run_pair(ctx, 100, 1, 136, 72, 1, 0.05, 42)      # smaller: reads only what its own projection pass wrote
    run_pair(ctx, 6, 32, 128, 64, 4, 0.05, 43)       # rows per member > 1, rank 4: A_i goes to the caller's cache
    # limits are reported, not crashed on
    big = eb.make_shape(0, (1 << 20) + 1, 1, 8, 8, 1)
    t = torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(eb.EggrollError) as e:
        ctx.eggroll_perturbed_forward_noalloc(eb.make_key(0, 0, 0), big, 0.1, 0, t, t, t, None, None)
    assert e.value.status == eb.EGG_EUNSUPPORTED
    with pytest.raises(eb.EggrollError) as e:   # S > 1 without an A cache would need the growable scratch
        ctx.eggroll_perturbed_forward_noalloc(eb.make_key(0, 0, 0), eb.make_shape(0, 1, 8, 8, 8, 1), 0.1, 0, t, t, t, None, None)
    assert e.value.status == eb.EGG_EINVAL
    torch.cuda.synchronize()
    ctx.close()
