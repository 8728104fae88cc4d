"""GPU: the library's calls can sit inside a captured HIP graph.  Scratch is allocated by an eager call of
the same shapes beforehand (allocation is the one thing a capture cannot hold); the library clears its
accumulators with fill kernels, never with memset nodes.  Each graph is replayed several times with eager
work and synchronisations in between, and every replay is compared with the eager result bit for bit."""
import numpy as np
import pytest

from paper_2511_16652_amd import binding as eb
from paper_2511_16652_amd import inputs

pytestmark = pytest.mark.gpu


def replay_and_compare(graph, outputs, eager, stream, disturb):
    import torch
    for rep in range(3):
        for o in outputs:
            o.zero_()
        disturb()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outputs, eager):
            assert torch.equal(o.view(torch.uint8), e.view(torch.uint8)), rep


def test_float_step_in_a_graph():
    import torch
    d_out, d_in, N, sigma = 512, 384, 1024, 0.01
    g = torch.Generator(device="cuda").manual_seed(0)
    W = (torch.randn((d_out, d_in), generator=g, device="cuda") / d_in ** 0.5).to(torch.bfloat16)
    X = torch.randn((N, d_in), generator=g, device="cuda").to(torch.bfloat16)
    f = torch.randn(N, generator=g, device="cuda")
    f -= f.mean()
    Y = torch.empty((N, d_out), dtype=torch.bfloat16, device="cuda")
    G = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    ctx = eb.Context(0, stream=s)
    key, shape = eb.make_key(5, 1, 2), eb.make_shape(0, N, 1, d_out, d_in, 1)
    scale = eb.eggroll_default_scale(N, sigma, 1)

    def step():
        ctx.eggroll_perturbed_forward(key, shape, sigma, eb.EGG_ACT_NONE, W, X, Y)
        ctx.eggroll_update(key, shape, eb.EGG_BF16, f, scale, 0, G)

    with torch.cuda.stream(s):
        step()                                      # eager: allocates the scratch, gives the reference
    torch.cuda.synchronize()
    eager = [Y.clone(), G.clone()]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        step()

    def disturb():                                  # the program's own eager work between replays, other shapes too
        with torch.cuda.stream(s):
            ctx.eggroll_update(eb.make_key(9, 9, 9), eb.make_shape(0, 64, 1, 128, 128, 1), eb.EGG_BF16, f[:64].contiguous(), 1.0, 0,
                               torch.empty((128, 128), dtype=torch.float32, device="cuda"))

    replay_and_compare(graph, [Y, G], eager, s, disturb)
    ctx.close()


def test_graph_survives_scratch_growth():
    """A graph bakes the scratch addresses of the calls it captured.  A later, larger eager call makes the context
    allocate bigger buffers; the outgrown ones are parked, not freed, so the graph's replays stay valid and correct.
    eggroll_scratch_generation reports the replacement."""
    import torch
    d_out, d_in, N, sigma = 256, 256, 512, 0.01
    g = torch.Generator(device="cuda").manual_seed(3)
    W = (torch.randn((d_out, d_in), generator=g, device="cuda") / d_in ** 0.5).to(torch.bfloat16)
    X = torch.randn((N, d_in), generator=g, device="cuda").to(torch.bfloat16)
    f = torch.randn(N, generator=g, device="cuda")
    Y = torch.empty((N, d_out), dtype=torch.bfloat16, device="cuda")
    G = torch.empty((d_out, d_in), dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    ctx = eb.Context(0, stream=s)
    key, shape = eb.make_key(5, 1, 2), eb.make_shape(0, N, 1, d_out, d_in, 1)

    def step():
        ctx.eggroll_perturbed_forward(key, shape, sigma, eb.EGG_ACT_NONE, W, X, Y)
        ctx.eggroll_update(key, shape, eb.EGG_BF16, f, 1.0 / N, 0, G)

    with torch.cuda.stream(s):
        step()
    torch.cuda.synchronize()
    eager = [Y.clone(), G.clone()]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        step()
    gen0 = ctx.eggroll_scratch_generation()
    # a much larger eager call on the same context: projections, packed panels and the fitness normaliser all grow
    Nb, db = 8192, 1024
    Wb = torch.zeros((db, db), dtype=torch.bfloat16, device="cuda")
    Xb = torch.zeros((Nb, db), dtype=torch.bfloat16, device="cuda")
    Yb = torch.empty((Nb, db), dtype=torch.bfloat16, device="cuda")
    Gb = torch.empty((db, db), dtype=torch.float32, device="cuda")
    fb = torch.ones(Nb, device="cuda")

    def disturb():
        with torch.cuda.stream(s):
            shb = eb.make_shape(0, Nb, 1, db, db, 1)
            ctx.eggroll_perturbed_forward(eb.make_key(1, 1, 1), shb, 0.1, eb.EGG_ACT_NONE, Wb, Xb, Yb)
            ctx.eggroll_update(eb.make_key(1, 1, 1), shb, eb.EGG_BF16, fb, 1.0, 0, Gb)

    replay_and_compare(graph, [Y, G], eager, s, disturb)
    assert ctx.eggroll_scratch_generation() > gen0
    ctx.eggroll_trim()          # no graph of this context is replayed after this point
    ctx.close()


def test_integer_step_in_a_graph():
    import torch
    wl = inputs.make_int8("g", 256, 2304, 4, 41)
    W, H = torch.from_numpy(wl.W).cuda(), torch.from_numpy(wl.H0).cuda()
    out = torch.empty_like(H)
    theta = W.clone()
    F = torch.from_numpy(np.random.default_rng(1).choice(np.array([-1, 1], np.int8), wl.N)).cuda()
    s = torch.cuda.Stream()
    ctx = eb.Context(0, stream=s)
    key, shape = eb.make_key(2, 0, 1), eb.make_shape(0, wl.N, 1, wl.d, wl.d, 1)
    thr = eb.eggroll_int_threshold(0.3, wl.N, (8 * 9 / 3.0) ** 0.5)

    def step():
        theta.copy_(W)
        ctx.eggroll_perturbed_forward_i8(key, shape, wl.bound, wl.corr_shift, wl.out_shift, wl.steps, W, H, out)
        ctx.eggroll_update_i8(key, shape, wl.bound, F, thr, theta)

    with torch.cuda.stream(s):
        step()
    torch.cuda.synchronize()
    eager = [out.clone(), theta.clone()]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        step()

    def disturb():
        with torch.cuda.stream(s):
            ctx.eggroll_perturbed_forward_i8(eb.make_key(7, 7, 7), shape, wl.bound, wl.corr_shift, wl.out_shift, 2, W, H, torch.empty_like(H))

    replay_and_compare(graph, [out, theta], eager, s, disturb)
    ctx.close()


def test_integer_model_step_in_a_graph():
    import torch
    D, L, N, T = 256, 2, 4096, 2
    P = inputs.egg_model(D, L, 5)
    model = {k: torch.from_numpy(v).cuda() for k, v in P.items()}
    saved = {k: v.clone() for k, v in model.items()}
    seq = inputs.egg_tokens(T + 1, N, 6)
    tok, tgt = torch.from_numpy(seq[:T].copy()).cuda(), torch.from_numpy(seq[1:].copy()).cuda()
    S0 = torch.zeros((L, N, D), dtype=torch.int8, device="cuda")
    S1 = torch.empty_like(S0)
    logits = torch.empty((T, N, 256), dtype=torch.int8, device="cuda")
    per = torch.empty(N * T, dtype=torch.int32, device="cuda")
    F = torch.empty(N // 2, dtype=torch.int8, device="cuda")
    s = torch.cuda.Stream()
    ctx = eb.Context(0, stream=s)
    key = eb.make_key(4, 0, 0)
    thr = eb.eggroll_int_threshold(0.3, N // 2, (8 * 9 / 3.0) ** 0.5)

    def step():
        for k in ("emb", "gru_w", "mlp1", "mlp2", "head"):
            model[k].copy_(saved[k])
        ctx.eggroll_egg_forward_i8(key, eb.make_shape(0, N, 1, D, D, 1, antithetic=1), L, 8, 4, T, model, tok, S0, S1, logits)
        ctx.eggroll_loglik_i8(N * T, logits.view(N * T, 256), tgt.view(N * T), 0, per)
        f = per.view(T, N).sum(0)
        F.copy_(torch.sign(f[0::2] - f[1::2]).to(torch.int8))
        ctx.eggroll_egg_update_i8(key, eb.make_shape(0, N // 2, 1, D, D, 1), L, 8, F, thr, model)

    with torch.cuda.stream(s):
        step()
    torch.cuda.synchronize()
    outs = [logits, S1, per, model["head"], model["mlp1"], model["emb"]]
    eager = [o.clone() for o in outs]
    assert (eager[3] != saved["head"]).any()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        step()
    replay_and_compare(graph, outs, eager, s, lambda: None)
    ctx.close()
