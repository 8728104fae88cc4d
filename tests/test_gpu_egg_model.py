"""GPU parity: the integer model around the GRU cell -- layer normalisation, perturbed embedding lookup and
the composed forward pass -- bit for bit against the oracle."""
import numpy as np
import pytest

import oracle
from paper_2511_16652_amd import binding as eb
from paper_2511_16652_amd import inputs

pytestmark = pytest.mark.gpu

SEED, STEP, LAYER = 12, 1, 7


@pytest.fixture(scope="module")
def ctx():
    import torch
    c = eb.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("D,rows", [(16, 1), (16, 1000), (64, 333), (128, 77), (256, 4099), (512, 65), (1024, 130)])
def test_layernorm_bit_exact(ctx, D, rows):
    rng = np.random.default_rng(D + rows)
    ln = rng.integers(-127, 128, D).astype(np.int8)
    U = rng.integers(-127, 128, (rows, D)).astype(np.int8)
    k = rows // 3
    U[:k] = rng.integers(-3, 4, (k, D))                     # small rows: divisor 0 -> 1, 1, 2
    out = dev(np.zeros_like(U))
    ctx.eggroll_layernorm_i8(rows, D, dev(ln), dev(U), out)
    assert (out.cpu().numpy() == oracle.layernorm_i8(ln, U)).all()


def test_layernorm_every_divisor_and_every_product(ctx):
    # row m has |u| <= 127 arranged so that its mean absolute value is m (m = 0 .. 127); weights and
    # entries sweep their whole range, so every (|product| bucket, divisor) pair of the divide occurs
    D = 256
    rng = np.random.default_rng(0)
    rows = []
    for m in range(128):
        for rep in range(8):
            mag = np.clip(m + rng.integers(-min(m, 127 - m), min(m, 127 - m) + 1, D), 0, 127)
            rows.append(mag * rng.choice([-1, 1], D))
    U = np.array(rows, np.int8)
    for w in (127, -127, 1, 64):
        ln = np.full(D, w, np.int8)
        ln[1::2] = rng.integers(-127, 128, D // 2)
        out = dev(np.zeros_like(U))
        ctx.eggroll_layernorm_i8(U.shape[0], D, dev(ln), dev(U), out)
        assert (out.cpu().numpy() == oracle.layernorm_i8(ln, U)).all()
    mav = np.abs(U.astype(np.int64)).sum(1) >> 8
    assert set(mav.tolist()) >= set(range(1, 127))


def test_layernorm_in_place(ctx):
    D, rows = 256, 513
    rng = np.random.default_rng(3)
    ln = rng.integers(-127, 128, D).astype(np.int8)
    U = rng.integers(-127, 128, (rows, D)).astype(np.int8)
    buf = dev(U)
    ctx.eggroll_layernorm_i8(rows, D, dev(ln), buf, buf)
    assert (buf.cpu().numpy() == oracle.layernorm_i8(ln, U)).all()


# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("D,N,mb,anti,cs", [(16, 50, 3, 0, 0), (64, 1026, 4, 1, 2), (256, 700, 0, 0, 4), (1024, 66, 10, 1, 3)])
def test_embedding_bit_exact(ctx, D, N, mb, anti, cs):
    rng = np.random.default_rng(D + N)
    emb = rng.integers(-127, 128, (256, D)).astype(np.int8)
    tok = rng.integers(0, 256, N).astype(np.uint8)
    out = dev(np.zeros((N, D), np.int8))
    ctx.eggroll_embed_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(mb, N, 1, D, D, 1, antithetic=anti), 8, cs, dev(emb), dev(tok), out)
    want = oracle.embed_i8(SEED, STEP, LAYER, mb, N, D, 8, cs, emb, tok, antithetic=bool(anti))
    got = out.cpu().numpy()
    assert (got == want).all() and (got != emb[tok]).any()


# ---------------------------------------------------------------------------------------------------
def run_model(ctx, P, D, L, N, T, mb, anti, tok, S, bound=8, cs=4):
    import torch
    model = {k: dev(v) for k, v in P.items()}
    S_out = torch.empty((L, N, D), dtype=torch.int8, device="cuda")
    logits = torch.empty((T, N, 256), dtype=torch.int8, device="cuda")
    ctx.eggroll_egg_forward_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(mb, N, 1, D, D, 1, antithetic=anti), L, bound, cs, T,
                               model, dev(tok), dev(S), S_out, logits)
    torch.cuda.synchronize()
    return logits.cpu().numpy(), S_out.cpu().numpy()


@pytest.mark.parametrize("D,L,N,T,mb,anti", [(64, 2, 130, 1, 0, 0), (256, 2, 300, 3, 4, 1), (16, 3, 70, 2, 1, 0),
                                              (256, 6, 258, 2, 0, 0), (64, 0, 40, 2, 0, 0), (1024, 1, 40, 2, 0, 1)])
def test_forward_bit_exact(ctx, D, L, N, T, mb, anti):
    P = inputs.egg_model(D, L, 100 + D + L)
    rng = np.random.default_rng(N)
    for k in ("ln1", "ln2", "ln_out"):
        P[k] = rng.integers(8, 25, P[k].shape).astype(np.int8)
    P["gru_b"] = rng.integers(-20, 21, P["gru_b"].shape).astype(np.int8)
    tok = inputs.egg_tokens(T, N, 5)
    S = rng.integers(-60, 61, (L, N, D)).astype(np.int8)
    logits, S_out = run_model(ctx, P, D, L, N, T, mb, anti, tok, S)
    want, S_want = oracle.egg_forward_i8(SEED, STEP, LAYER, mb, N, D, L, 8, 4, P, tok, S, antithetic=bool(anti))
    assert (S_out == S_want).all()
    assert (logits == want).all()
    assert want.std() > 3 and (np.abs(want) == 127).mean() < 0.5      # the logits carry information
    if L:
        assert (S_want != S).mean() > 0.5


def test_forward_65536_members_in_full(ctx):
    """One token through the whole model (D = 256, 6 layers) for 2^16 members in antithetic pairs, every logit and
    every state byte against the oracle: the row-streaming matmul kernel in all of its epilogue modes at a size
    that fills the chip many times over."""
    D, L, N, T = 256, 6, 1 << 16, 1
    P = inputs.egg_model(D, L, 4242)
    rng = np.random.default_rng(4243)
    P["gru_b"] = rng.integers(-20, 21, P["gru_b"].shape).astype(np.int8)
    tok = inputs.egg_tokens(T, N, 4244)
    S = rng.integers(-60, 61, (L, N, D)).astype(np.int8)
    logits, S_out = run_model(ctx, P, D, L, N, T, 0, 1, tok, S)
    want, S_want = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 8, 4, P, tok, S, antithetic=True)
    assert (S_out == S_want).all()
    assert (logits == want).all()


def test_forward_with_the_papers_integer_noise(ctx):
    """The integer model with the paper's own noise setting: round(16 z) factors from the table and the correction
    shifted by 4 + sigma_hat = 8 (App. "Adding EGGROLL Perturbations"), antithetic pairs, bit for bit; and its update."""
    import torch
    D, L, N, T = 256, 2, 4096, 2
    P = inputs.egg_model(D, L, 4300)
    tok = inputs.egg_tokens(T, N, 4301)
    S = np.random.default_rng(4302).integers(-60, 61, (L, N, D)).astype(np.int8)
    logits, S_out = run_model(ctx, P, D, L, N, T, 0, 1, tok, S, bound=eb.EGG_INT_NOISE_NORMAL16, cs=8)
    want, S_want = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, oracle.BOUND_NORMAL16, 8, P, tok, S, antithetic=True)
    assert (S_out == S_want).all() and (logits == want).all()
    plain, _ = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, 64, D, L, 0, 8, P, tok[:, :64], S[:, :64], antithetic=True)
    assert (want[:, :64] != plain).mean() > 0.02          # the perturbation is visible in the logits
    pairs = N // 2
    F = np.random.default_rng(4303).choice(np.array([-1, 0, 1], np.int8), pairs)
    thr = eb.eggroll_int_threshold(0.25, pairs, 16.0)
    model = {k: dev(v) for k, v in P.items()}
    ctx.eggroll_egg_update_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(0, pairs, 1, D, D, 1), L, eb.EGG_INT_NOISE_NORMAL16,
                              dev(F), thr, model)
    torch.cuda.synchronize()
    t_ref, _ = oracle.update_i8(SEED, STEP, LAYER + 1 + 4, 0, pairs, 4 * D, D, oracle.BOUND_NORMAL16, F, thr, P["mlp1"][0])
    assert (model["mlp1"][0].cpu().numpy() == t_ref).all()
    t_ref, _ = oracle.update_i8(SEED, STEP, LAYER, 0, pairs, 256, D, oracle.BOUND_NORMAL16, F, thr, P["emb"])
    assert (model["emb"].cpu().numpy() == t_ref).all()


def test_forward_noise_matters_and_pairs_mirror(ctx):
    # without noise members with the same token history agree; with antithetic noise the two members of
    # a pair differ from each other and from the unperturbed run
    D, L, N, T = 64, 2, 64, 3
    P = inputs.egg_model(D, L, 9)
    tok = np.repeat(inputs.egg_tokens(T, 1, 6), N, axis=1)
    S = np.zeros((L, N, D), np.int8)
    quiet, _ = run_model(ctx, P, D, L, N, T, 0, 0, tok, S, bound=0)
    assert (quiet == quiet[:, :1]).all()
    noisy, _ = run_model(ctx, P, D, L, N, T, 0, 1, tok, S, bound=8, cs=2)
    assert (noisy[:, 0::2] != noisy[:, 1::2]).any() and (noisy != quiet).any()
    want, _ = oracle.egg_forward_i8(SEED, STEP, LAYER, 0, N, D, L, 8, 2, P, tok, S, antithetic=True)
    assert (noisy == want).all()


def test_forward_rejects_bad_arguments(ctx):
    import torch
    D, L, N, T = 64, 1, 16, 1
    P = {k: dev(v) for k, v in inputs.egg_model(D, L, 1).items()}
    tok = dev(inputs.egg_tokens(T, N, 1))
    S = torch.zeros((L, N, D), dtype=torch.int8, device="cuda")
    lg = torch.empty((T, N, 256), dtype=torch.int8, device="cuda")
    key = eb.make_key(SEED, STEP, LAYER)
    with pytest.raises(eb.EggrollError):       # state in place
        ctx.eggroll_egg_forward_i8(key, eb.make_shape(0, N, 1, D, D, 1), L, 8, 4, T, P, tok, S, S, lg)
    with pytest.raises(eb.EggrollError):       # width not a power of 4
        ctx.eggroll_egg_forward_i8(key, eb.make_shape(0, N, 1, 128, 128, 1), L, 8, 4, T, P, tok, S, torch.empty_like(S), lg)
    with pytest.raises(eb.EggrollError):       # odd population with pairs
        ctx.eggroll_egg_forward_i8(key, eb.make_shape(0, N - 1, 1, D, D, 1, antithetic=1), L, 8, 4, T, P, tok, S, torch.empty_like(S), lg)


@pytest.mark.parametrize("N,T", [(1 << 18, 2), (1 << 20, 1)])
def test_forward_real_shape_sampled(ctx, N, T):
    """The benchmark's launch configuration (D = 256, 6 layers, 2^18 members in antithetic pairs) over 2 tokens,
    and the largest population the paper evaluates on one GPU (2^20) over one token: sampled pairs against the
    oracle (a member's trajectory depends on no other member), plus the range invariant of I8 over the whole output."""
    import torch
    D, L = 256, 6
    P = inputs.egg_model(D, L, 1006)
    tok = inputs.egg_tokens(T, N, 1007)
    model = {k: dev(v) for k, v in P.items()}
    g = torch.Generator(device="cuda").manual_seed(3)
    S = torch.randint(-40, 41, (L, N, D), generator=g, device="cuda", dtype=torch.int8)
    S_out = torch.empty_like(S)
    logits = torch.empty((T, N, 256), dtype=torch.int8, device="cuda")
    ctx.eggroll_egg_forward_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(0, N, 1, D, D, 1, antithetic=1), L, 8, 4, T,
                               model, dev(tok), S, S_out, logits)
    torch.cuda.synchronize()
    assert int(logits.min()) >= -127 and int(S_out.min()) >= -127
    rng = np.random.default_rng(2)
    for p in np.sort(rng.choice(N // 2, 12, replace=False)):
        m = 2 * int(p)
        want, S_want = oracle.egg_forward_i8(SEED, STEP, LAYER, m, 2, D, L, 8, 4, P, tok[:, m:m + 2],
                                             S[:, m:m + 2].cpu().numpy(), antithetic=True)
        assert (logits[:, m:m + 2].cpu().numpy() == want).all(), m
        assert (S_out[:, m:m + 2].cpu().numpy() == S_want).all(), m
    assert logits[:, :4096].float().std() > 3


@pytest.mark.parametrize("D,L,pairs,mb", [(64, 2, 300, 0), (256, 1, 1000, 6), (16, 0, 64, 2)])
def test_model_update_bit_exact(ctx, D, L, pairs, mb):
    """Every perturbed parameter against the oracle's integer update with that parameter's noise layer;
    normalisation weights and biases stay as they are."""
    rng = np.random.default_rng(D + pairs)
    P = inputs.egg_model(D, L, 21)
    F = rng.integers(-1, 2, pairs).astype(np.int8)
    thr = oracle.int_threshold(0.3, pairs, np.sqrt(8 * 9 / 3.0))
    model = {k: dev(v) for k, v in P.items()}
    ctx.eggroll_egg_update_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(mb, pairs, 1, D, D, 1), L, 8, dev(F), thr, model)
    got = {k: v.cpu().numpy() for k, v in model.items()}

    def want(layer, theta):
        out, _ = oracle.update_i8(SEED, STEP, layer, mb, pairs, theta.shape[0], theta.shape[1], 8, F, thr, theta)
        return out

    assert (got["emb"] == want(LAYER, P["emb"])).all()
    for i in range(L):
        base = LAYER + 1 + 6 * i
        for m in range(4):
            assert (got["gru_w"][i, m] == want(base + m, P["gru_w"][i, m])).all(), (i, m)
        assert (got["mlp1"][i] == want(base + 4, P["mlp1"][i])).all()
        assert (got["mlp2"][i] == want(base + 5, P["mlp2"][i])).all()
    assert (got["head"] == want(LAYER + 1 + 6 * L, P["head"])).all()
    for k in ("ln1", "ln2", "ln_out", "gru_b"):
        assert (got[k] == P[k]).all()
    moved = (got["head"] != P["head"]).mean()
    assert 0.1 < moved < 0.6          # about the fraction alpha = 0.3 of the entries moves by one bin


def test_forward_and_update_use_the_same_noise(ctx):
    """One member pair decides the update (F = e_p): the table row its first token selects moves toward that
    member's own perturbation of the row, the one the forward pass added."""
    D, L, N = 64, 0, 8
    P = inputs.egg_model(D, L, 5)
    P["emb"][...] = 0
    P["head"] = np.zeros_like(P["head"])
    p = 2
    tok = np.full((1, N), 65, np.uint8)
    # forward with corr_shift 0 and a zero table: y = A_p[t] * (+-B_p); recover it through the embedding entry point
    y = dev(np.zeros((N, D), np.int8))
    ctx.eggroll_embed_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(0, N, 1, D, D, 1, antithetic=1), 8, 0, dev(P["emb"]), dev(tok[0]), y)
    y = y.cpu().numpy().astype(np.int64)
    assert (y[2 * p] == -y[2 * p + 1]).all() and np.abs(y[2 * p]).max() > 0
    F = np.zeros(N // 2, np.int8)
    F[p] = 1
    model = {k: dev(v) for k, v in P.items()}
    ctx.eggroll_egg_update_i8(eb.make_key(SEED, STEP, LAYER), eb.make_shape(0, N // 2, 1, D, D, 1), L, 8, dev(F), 1, model)
    emb = model["emb"].cpu().numpy().astype(np.int64)
    assert (emb[65] == np.sign(y[2 * p])).all()


@pytest.mark.parametrize("rows", [1, 17, 4099])
def test_loglik_bit_exact(ctx, rows):
    import torch
    rng = np.random.default_rng(rows)
    y = rng.integers(-127, 128, (rows, 256)).astype(np.int8)
    k = rows // 3
    y[:k] = rng.integers(-10, 11, (k, 256))                     # flat rows
    y[k:2 * k] = -127
    y[k:2 * k, 5] = 127                                         # one-hot rows: the smallest and the largest sums
    t = rng.integers(0, 256, rows).astype(np.uint8)
    out = torch.zeros(rows, dtype=torch.int32, device="cuda")
    ctx.eggroll_loglik_i8(rows, dev(y), dev(t), 0, out)
    want = oracle.loglik_i8(y, t)
    assert (out.cpu().numpy() == want).all()
    ctx.eggroll_loglik_i8(rows, dev(y), dev(t), 1, out)         # accumulate
    assert (out.cpu().numpy() == 2 * want).all()


def test_loglik_every_level_and_every_threshold(ctx):
    # rows of equal logits at every level, and rows whose sum of exponentials sweeps the range in small steps:
    # every entry of the EXP2 table and, densely, the rounding boundaries of the inverted LOG2
    import torch
    rows = []
    for level in range(-127, 128):
        rows.append(np.full(256, level))
    rng = np.random.default_rng(1)
    for hot in range(1, 256, 3):
        for level in range(-127, 128, 7):
            r = np.full(256, -127)
            r[:hot] = level
            rows.append(r)
    y = np.array(rows, np.int8)
    t = rng.integers(0, 256, len(rows)).astype(np.uint8)
    out = torch.zeros(len(rows), dtype=torch.int32, device="cuda")
    ctx.eggroll_loglik_i8(len(rows), dev(y), dev(t), 0, out)
    assert (out.cpu().numpy() == oracle.loglik_i8(y, t)).all()


def test_integer_es_learns_a_cycle(ctx):
    """End to end on the GPU, integers only: forward pass of a small model for a population in antithetic pairs,
    log-likelihood fitness, sign(s+ - s-) shaping, integer update of all parameters.  The data is the cycle
    a b c d a b ... at a random phase per pair, so the next token follows from the current one: from about 8.5 bits
    per token (logits of a random model) the population's mean must fall below 2 bits in 30 ES steps.  Checks that
    the forward pass, the fitness and the update agree on which member carries which sign of which noise."""
    import torch
    D, L, N, T, bound, cs = 64, 1, 8192, 16, 8, 4
    model = {k: dev(v) for k, v in inputs.egg_model(D, L, 3).items()}
    rng = np.random.default_rng(0)
    sym = np.frombuffer(b"abcd", np.uint8)
    thr = eb.eggroll_int_threshold(0.3, N // 2, (bound * (bound + 1) / 3.0) ** 0.5)
    S0 = torch.zeros((L, N, D), dtype=torch.int8, device="cuda")
    S1 = torch.empty_like(S0)
    logits = torch.empty((T, N, 256), dtype=torch.int8, device="cuda")
    per = torch.empty(N * T, dtype=torch.int32, device="cuda")
    bits = []
    for step in range(30):
        phase = rng.integers(0, 4, N // 2).repeat(2)                      # both members of a pair see the same data
        seq = sym[(phase[None, :] + np.arange(T + 1)[:, None]) % 4]      # [T + 1, N]
        key = eb.make_key(1, step, 0)
        ctx.eggroll_egg_forward_i8(key, eb.make_shape(0, N, 1, D, D, 1, antithetic=1), L, bound, cs, T, model,
                                   dev(seq[:T]), S0, S1, logits)
        ctx.eggroll_loglik_i8(N * T, logits.view(N * T, 256), dev(seq[1:]).view(N * T), 0, per)
        f = per.view(T, N).sum(0)
        F = torch.sign(f[0::2] - f[1::2]).to(torch.int8).contiguous()
        ctx.eggroll_egg_update_i8(key, eb.make_shape(0, N // 2, 1, D, D, 1), L, bound, F, thr, model)
        bits.append(-float(f.float().mean()) / T / 16.0)
    torch.cuda.synchronize()
    assert bits[0] > 7.0 and bits[-1] < 2.0, bits[::5]
