"""Pins of the multi-layer oracle (oracle/models.py): MLP stack and decoder.

Each part is checked against something other than itself: torch's bf16 cast, math.erf / the normal CDF,
the plain-loop C oracle of one layer, closed forms (constant rows, zero queries, one token), causality,
torch's scaled_dot_product_attention and log_softmax on the CPU, and structural properties of the
composed models (sigma = 0 makes all members equal, a change of a later token leaves earlier positions
untouched bit for bit, noise layer ids, chunking by member)."""
import math

import numpy as np
import pytest
import torch
from scipy.special import ndtr

import oracle
from oracle import models
from paper_2511_16652_amd import inputs

EPS = 1e-5


def test_round_bf16_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -9, 3.3895e38, 1e-45])])
    want = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).double().numpy()
    got = models.round_bf16(a)
    assert np.array_equal(got, want)
    assert models.round_bf16(a.reshape(4, -1)).shape == (4, a.size // 4)


def test_gelu_is_x_times_normal_cdf():
    x = np.linspace(-9, 9, 4001)
    assert np.allclose(models.gelu(x), x * ndtr(x), rtol=1e-13, atol=2e-15)  # 1 + erf cancels for x << 0: absolute bound there
    for v in (-3.0, -0.5, 0.0, 0.7, 2.5):
        assert models.gelu(v) == pytest.approx(0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))), rel=1e-15)


@pytest.mark.parametrize("rank,S", [(1, 1), (1, 5), (4, 3)])
def test_member_linear_equals_the_plain_loop_oracle(rank, S):
    d_out, d_in, N = 24, 40, 6
    wl = inputs.make_linear("t", "bf16", d_out, d_in, N, S, rank, 0.05, 77, layer=9)
    ref = oracle.forward(3, 2, 9, 10, N, S, d_out, d_in, rank, oracle.NOISE_BF16, 0.05, 0, wl.W, wl.X)
    for i in range(N):
        got = models.member_linear(3, 2, 9, 10 + i, wl.W, wl.X[i * S:(i + 1) * S], rank, 0.05)
        assert np.allclose(got, ref[i * S:(i + 1) * S], rtol=1e-12, atol=1e-13)
    # W_i itself: entry by entry from the factors
    A = oracle.noise_matrix(3, 2, 9, 0, 12, d_out, rank, oracle.NOISE_BF16)
    B = oracle.noise_matrix(3, 2, 9, 1, 12, d_in, rank, oracle.NOISE_BF16)
    Wi = models.member_matrix(3, 2, 9, 12, wl.W, rank, 0.05)
    for j, k in ((0, 0), (5, 17), (23, 39)):
        assert Wi[j, k] == pytest.approx(wl.W[j, k] + 0.05 / math.sqrt(rank) * sum(A[j, l] * B[k, l] for l in range(rank)), rel=1e-14)
    assert models.member_matrix(3, 2, 9, 12, wl.W, rank, 0.0) is not None
    assert np.array_equal(models.member_matrix(3, 2, 9, 12, wl.W, rank, 0.0), wl.W.astype(np.float64))


def test_rmsnorm_closed_forms():
    g = np.linspace(0.5, 1.5, 16)
    # constant row c: mean square c^2  ->  c g / sqrt(c^2 + eps)
    for c in (-3.0, 0.25, 100.0):
        y = models.rmsnorm(np.full((2, 16), c), g, EPS)
        assert np.allclose(y, c * g / math.sqrt(c * c + EPS), rtol=1e-14)
    # a zero row stays zero; one-hot row of height a: mean square a^2/d
    assert not models.rmsnorm(np.zeros((1, 16)), g, EPS).any()
    x = np.zeros((1, 16)); x[0, 3] = 4.0
    y = models.rmsnorm(x, g, EPS)
    assert y[0, 3] == pytest.approx(4.0 * g[3] / math.sqrt(1.0 + EPS), rel=1e-14) and np.count_nonzero(y) == 1
    # with unit gains the output has unit mean square (up to eps), and the map is invariant to scaling x
    x = np.random.default_rng(1).standard_normal((5, 64))
    y = models.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)
    assert np.allclose(models.rmsnorm(7.5 * x, np.ones(64), 0.0), y, rtol=1e-13)
    # against torch's own rms_norm
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(np.linspace(0.5, 2, 64)), EPS).numpy()
    assert np.allclose(models.rmsnorm(x, np.linspace(0.5, 2, 64), EPS), want, rtol=1e-12)


def test_attention_closed_forms_and_causality():
    rng = np.random.default_rng(2)
    S, heads, hd = 9, 3, 4
    d = heads * hd
    q, k, v = (rng.standard_normal((S, d)) for _ in range(3))
    o = models.causal_attention(q, k, v, heads)
    # the first token sees only itself
    assert np.allclose(o[0], v[0], rtol=1e-14)
    # zero queries: uniform weights over the prefix -> running mean of v
    o0 = models.causal_attention(np.zeros_like(q), k, v, heads)
    assert np.allclose(o0, np.cumsum(v, axis=0) / np.arange(1, S + 1)[:, None], rtol=1e-13)
    # outputs are convex combinations of the prefix's values, head by head
    for h in range(heads):
        sl = slice(h * hd, (h + 1) * hd)
        for s in range(S):
            assert (o[s, sl] <= v[:s + 1, sl].max(axis=0) + 1e-12).all() and (o[s, sl] >= v[:s + 1, sl].min(axis=0) - 1e-12).all()
    # causality, bit for bit: changing tokens after position 4 leaves positions 0..4 untouched
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[5:] += 3.0; v2[5:] -= 1.0; q2[5:] *= 2.0
    assert np.array_equal(models.causal_attention(q2, k2, v2, heads)[:5], o[:5])
    # heads do not mix: changing head 1's columns leaves the other heads' outputs untouched
    k3 = k.copy(); k3[:, hd:2 * hd] += 1.0
    o3 = models.causal_attention(q, k3, v, heads)
    assert np.array_equal(o3[:, :hd], o[:, :hd]) and np.array_equal(o3[:, 2 * hd:], o[:, 2 * hd:]) and not np.array_equal(o3, o)
    # library routine (torch CPU, fp64, its own kernel)
    tq, tk, tv = (torch.from_numpy(t).reshape(S, heads, hd).transpose(0, 1) for t in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).transpose(0, 1).reshape(S, d).numpy()
    assert np.allclose(o, want, rtol=1e-12, atol=1e-14)


def test_token_loglik_against_log_softmax():
    rng = np.random.default_rng(3)
    S, V = 7, 50
    logits = rng.standard_normal((S, V)) * 4
    tok = rng.integers(0, V, S)
    ll = models.token_loglik(logits, tok)
    lsm = torch.log_softmax(torch.from_numpy(logits), dim=-1).numpy()
    assert ll[-1] == 0.0
    assert np.allclose(ll[:-1], lsm[np.arange(S - 1), tok[1:]], rtol=1e-13)
    # uniform logits: -log V whatever the target; a shift of a row changes nothing
    assert np.allclose(models.token_loglik(np.full((3, V), 2.5), [0, 1, 2])[:2], -math.log(V), rtol=1e-14)
    assert np.allclose(models.token_loglik(logits + 1000.0, tok), ll, rtol=1e-10)


def _stack(d=16, ff=48, L=3, N=5, S=4, seed=11):
    P = inputs.mlp_stack(d, ff, L, seed)
    X = [inputs.member_rows(seed + 1, m, S, d) for m in range(N)]
    return P, X


def test_mlp_stack_is_a_chain_of_the_pinned_layer():
    d, ff, L, N, S, r, sg = 16, 48, 3, 5, 4, 4, 0.05
    P, X = _stack(d, ff, L, N, S)
    Y, trace = models.mlp_stack_forward(1, 0, 100, range(N), S, r, sg, P["W1"], P["W2"], X, keep=True)
    h = np.concatenate(X).astype(np.float64)
    for l in range(L):
        u = oracle.forward(1, 0, 100 + 2 * l, 0, N, S, ff, d, r, oracle.NOISE_BF16, sg, oracle.ACT_GELU, P["W1"][l], h)
        u = models.round_bf16(u)
        assert np.array_equal(u.reshape(N, S, ff), trace[l][0])
        h = models.round_bf16(oracle.forward(1, 0, 100 + 2 * l + 1, 0, N, S, d, ff, r, oracle.NOISE_BF16, sg, 0, P["W2"][l], u))
        assert np.array_equal(h.reshape(N, S, d), trace[l][1])
    assert np.array_equal(Y, trace[-1][1])
    # member subsets and order do not matter (a member's rows depend on no other member)
    Y2 = models.mlp_stack_forward(1, 0, 100, [3, 1], S, r, sg, P["W1"], P["W2"], [X[3], X[1]])
    assert np.array_equal(Y2[0], Y[3]) and np.array_equal(Y2[1], Y[1])
    # sigma = 0: every member applies the same stack
    Y0 = models.mlp_stack_forward(1, 0, 100, [0, 4], S, r, 0.0, P["W1"], P["W2"], [X[2], X[2]])
    assert np.array_equal(Y0[0], Y0[1])
    h = X[2].astype(np.float64)
    for l in range(L):
        h = models.round_bf16(models.round_bf16(models.gelu(h @ P["W1"][l].astype(np.float64).T)) @ P["W2"][l].astype(np.float64).T)
    assert np.array_equal(Y0[0], h)


def _decoder(V=40, d=32, ff=64, L=2, heads=4, N=4, S=6, seed=21):
    P = inputs.decoder_params(V, d, ff, L, seed, norm_jitter=0.2)
    tok = inputs.decoder_tokens(N, S, V, seed + 1)
    return P, tok


def test_decoder_layer_is_a_chain_of_the_pinned_parts():
    V, d, ff, L, heads, N, S, sg = 40, 32, 64, 2, 4, 4, 6, 0.05
    P, tok = _decoder(V, d, ff, L, heads, N, S)
    logits, ll, traces = models.decoder_forward(5, 1, 30, range(N), tok, P, heads, EPS, 1, sg, keep=True)
    rb = models.round_bf16
    for i in range(N):
        x = P["emb"][tok[i]].astype(np.float64)
        for l in range(L):
            t = traces[i][l]
            assert np.array_equal(t["x_in"], x)
            lid = 30 + 6 * l
            fwd = lambda j, W, inp, act=0: oracle.forward(5, 1, lid + j, i, 1, S, W.shape[0], W.shape[1], 1, oracle.NOISE_BF16, sg, act, W, inp)  # noqa: E731
            h1 = rb(models.rmsnorm(x, P["norm1"][l], EPS))
            q, k, v = rb(fwd(0, P["wq"][l], h1)), rb(fwd(1, P["wk"][l], h1)), rb(fwd(2, P["wv"][l], h1))
            for name, val in (("h1", h1), ("q", q), ("k", k), ("v", v)):
                assert np.allclose(t[name], val, rtol=0, atol=2.0 ** -7 * np.abs(val).max()), name
                # BLAS and plain-loop sums differ in the last fp64 bits, which may flip a bf16 rounding: compare
                # exactly where no value sits near a rounding boundary
                assert (t[name] != val).mean() < 0.01, name
            o = rb(models.causal_attention(t["q"], t["k"], t["v"], heads))
            assert np.array_equal(t["o"], o)
            xm = rb(t["x_in"] + fwd(3, P["wo"][l], t["o"]))
            assert (t["x_mid"] != xm).mean() < 0.01 and np.allclose(t["x_mid"], xm, atol=2.0 ** -7 * np.abs(xm).max())
            h2 = rb(models.rmsnorm(t["x_mid"], P["norm2"][l], EPS))
            assert np.array_equal(t["h2"], h2)
            u = rb(fwd(4, P["w_up"][l], t["h2"], oracle.ACT_GELU))
            assert (t["u"] != u).mean() < 0.01 and np.allclose(t["u"], u, atol=2.0 ** -7 * np.abs(u).max())
            xo = rb(t["x_mid"] + fwd(5, P["w_down"][l], t["u"]))
            assert (t["x_out"] != xo).mean() < 0.01 and np.allclose(t["x_out"], xo, atol=2.0 ** -7 * np.abs(xo).max())
            x = t["x_out"]
        hf = rb(models.rmsnorm(x, P["norm_f"], EPS))
        assert np.array_equal(traces[i][L]["hf"], hf)
        lg = rb(oracle.forward(5, 1, 30 + 6 * L, i, 1, S, V, d, 1, oracle.NOISE_BF16, sg, 0, P["head"], hf))
        assert (logits[i] != lg).mean() < 0.01 and np.allclose(logits[i], lg, atol=2.0 ** -7 * np.abs(lg).max())
        assert np.array_equal(ll[i], models.token_loglik(logits[i], tok[i]))


def test_decoder_structure():
    V, d, ff, L, heads, N, S, sg = 40, 32, 64, 2, 4, 4, 6, 0.05
    P, tok = _decoder(V, d, ff, L, heads, N, S)
    logits, ll = models.decoder_forward(5, 1, 30, range(N), tok, P, heads, EPS, 1, sg)
    assert logits.shape == (N, S, V) and ll.shape == (N, S) and (ll[:, -1] == 0).all() and (ll[:, :-1] < 0).all()
    # sigma = 0: members with the same tokens give identical logits, whatever their ids
    same = np.repeat(tok[:1], 3, axis=0)
    l0, _ = models.decoder_forward(5, 1, 30, [0, 7, 123], same, P, heads, EPS, 1, 0.0)
    assert np.array_equal(l0[0], l0[1]) and np.array_equal(l0[0], l0[2])
    # sigma > 0: the same tokens under different member ids differ, and the perturbation is small
    l1, _ = models.decoder_forward(5, 1, 30, [0, 7], same[:2], P, heads, EPS, 1, 0.1 * sg)
    assert not np.array_equal(l1[0], l1[1])
    assert 0 < np.abs(l1[0] - l0[0]).max() < 0.25 * np.abs(l0[0]).max()
    # causality through the whole model, bit for bit: a different last token leaves every earlier position as it was
    tok2 = tok.copy(); tok2[:, -1] = (tok2[:, -1] + 1) % V
    l2, _ = models.decoder_forward(5, 1, 30, range(N), tok2, P, heads, EPS, 1, sg)
    assert np.array_equal(l2[:, :-1], logits[:, :-1]) and not np.array_equal(l2[:, -1], logits[:, -1])
    # member subsets: a member's result depends on no other member
    l3, ll3 = models.decoder_forward(5, 1, 30, [2], tok[2:3], P, heads, EPS, 1, sg)
    assert np.array_equal(l3[0], logits[2]) and np.array_equal(ll3[0], ll[2])
    # no layers: embedding -> final norm -> perturbed head, i.e. one pinned linear layer on the gathered rows
    P0 = dict(P, **{k: P[k][:0] for k in ("norm1", "norm2", "wq", "wk", "wv", "wo", "w_up", "w_down")})
    l4, _ = models.decoder_forward(5, 1, 30, [1], tok[1:2], P0, heads, EPS, 1, sg)
    hf = models.round_bf16(models.rmsnorm(P["emb"][tok[1]].astype(np.float64), P["norm_f"], EPS))
    want = oracle.forward(5, 1, 30, 1, 1, S, V, d, 1, oracle.NOISE_BF16, sg, 0, P["head"], hf)
    assert np.allclose(l4[0], want, atol=2.0 ** -8 * np.abs(want).max())
    # the noise layer id of each matrix: zeroing one matrix's perturbation source changes the result, and the
    # ids base + 6 l + j are distinct streams (q and k of one layer do not share factors)
    A_q = oracle.noise_matrix(5, 1, 30, 0, 0, d, 1, oracle.NOISE_BF16)
    A_k = oracle.noise_matrix(5, 1, 31, 0, 0, d, 1, oracle.NOISE_BF16)
    assert not np.array_equal(A_q, A_k)
