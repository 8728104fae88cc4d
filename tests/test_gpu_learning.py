"""GPU, end to end: EGGROLL steps (Alg. 1) on a small regression problem.  Parity tests hold each call against
the oracle; this one checks that the calls fit together as the method intends -- the update must move the mean
along the perturbations that the forward pass evaluated, with the sign and scale of the EGGROLL UPDATE box."""
import pytest

from paper_2511_16652_amd import binding as eb

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,rank", [("bf16", 1), ("bf16", 4), ("f32", 1)])
def test_es_steps_learn_a_linear_map(dtype, rank):
    """W* is a random 32 x 32 map; every member of a population of 2048 sees the same batch of 32 inputs (so that
    fitness differences come from the perturbations alone), fitness = -sum ||y - W* x||^2, z-scored, and the mean
    is moved by W += lr * G with G = (1 / (N sigma)) sum_i f_i E_i.  sigma ||E|| is kept small against ||W - W*||
    (the estimator is a first-order one) and lr / sigma = 0.3 is a step of 0.3 along the normalised gradient.
    The batch loss must fall from about 25 to below 1 in 40 steps."""
    import torch
    d, N, S, sigma = 32, 2048, 32, 0.002
    lr = 0.3 * sigma
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    code = eb.EGG_F32 if dtype == "f32" else eb.EGG_BF16
    g = torch.Generator(device="cuda").manual_seed(0)
    w_star = torch.randn((d, d), generator=g, device="cuda") / d ** 0.5
    W = torch.zeros((d, d), dtype=dt, device="cuda")
    ctx = eb.Context(0)
    Y = torch.empty((N * S, d), dtype=torch.float32, device="cuda")
    G = torch.empty((d, d), dtype=torch.float32, device="cuda")
    losses = []
    for step in range(40):
        xb = torch.randn((S, d), generator=g, device="cuda").to(dt)
        X = xb.repeat(N, 1).contiguous()
        target = xb.float() @ w_star.t()
        key, shape = eb.make_key(3, step, 0), eb.make_shape(0, N, S, d, d, rank)
        ctx.eggroll_perturbed_forward(key, shape, sigma, eb.EGG_ACT_NONE, W, X, Y)
        f = -((Y - target.repeat(N, 1)) ** 2).sum(1).view(N, S).sum(1)
        z = ((f - f.mean()) / (f.std() + 1e-8)).contiguous()
        ctx.eggroll_update(key, shape, code, z, eb.eggroll_default_scale(N, sigma, rank), 0, G, W, lr)
        losses.append(float(((xb.float() @ W.float().t() - target) ** 2).sum(1).mean()))
    torch.cuda.synchronize()
    ctx.close()
    assert losses[0] > 15.0 and losses[-1] < 1.0, losses[::5]
