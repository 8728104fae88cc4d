"""CPU oracle of the two multi-layer float workloads (test infrastructure, not product code).

Plain numpy in fp64, written from the definitions: every perturbed linear layer MATERIALISES the member's
matrix W_i = M + (sigma / sqrt r) A_i B_i^T (Alg. 1: f_i <- f(W = M + sigma E_i); Sec. 4.1: E = A B^T / sqrt r)
and multiplies by it; the factored form of Sec. 4.2 is never used here.  ``numpy.matmul`` is the only library
step.  The factors come from the C oracle's counter stream (``oracle.noise_matrix``), so both workloads read
the same noise definition as the single-layer functions.

The paper gives no architecture for these two workloads (its own models are RWKV / Qwen / an integer GRU);
the configurations only name their sizes.  The definitions taken here:

  MLP stack:   per layer l:  h <- bf16( W2_l' * bf16( gelu( W1_l' * h ) ) ),  gelu exact (erf form), no bias,
               norm or residual; W1_l is [d_ff, d], W2_l is [d, d_ff]; noise layer ids  base + 2 l + {0, 1}.
  Decoder:     x <- emb[token]                                  (table not perturbed)
               per layer l:  h  <- bf16( rmsnorm(x; g1_l) )
                             q, k, v <- bf16( Wq' h ), bf16( Wk' h ), bf16( Wv' h )
                             o  <- bf16( causal softmax attention over the member's own S tokens, per head,
                                         scores q.k / sqrt(head_dim), no positional encoding )
                             x  <- bf16( x + Wo' o )
                             h  <- bf16( rmsnorm(x; g2_l) )
                             u  <- bf16( gelu( Wup' h ) )
                             x  <- bf16( x + Wdown' u )
               logits <- bf16( Whead' bf16( rmsnorm(x; gf) ) )
               rmsnorm(x; g)_k = x_k g_k / sqrt( mean_k x_k^2 + eps )
               noise layer ids  base + 6 l + {0..5: q, k, v, o, up, down},  base + 6 L: head.
               W' means the member's perturbed copy.  Every stored tensor is bf16; bf16(.) is
               round-to-nearest-even of the fp32 rounding of the fp64 value.
  Token log-likelihood:  ll[s] = logits[s][token[s+1]] - log sum_j exp(logits[s][j])  for s < S-1, 0 for the
               member's last token (it has no successor).

Only ``tests/``, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

from . import NOISE_BF16, noise_matrix


def round_bf16(a) -> np.ndarray:
    """fp64 array -> nearest bfloat16 (ties to even) of its fp32 rounding, returned as fp64."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32)
    finite = (bits & np.uint32(0x7F800000)) != np.uint32(0x7F800000)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    out = np.where(finite, rounded, bits).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(a))


def gelu(x) -> np.ndarray:
    """0.5 x (1 + erf(x / sqrt 2)) (the exact form, not the tanh approximation)."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + _erf(x * 0.7071067811865476))


def member_matrix(seed, step, layer, member, W, rank, sigma) -> np.ndarray:
    """W_i = M + (sigma / sqrt r) A_i B_i^T as a dense fp64 matrix (bf16 factors)."""
    W = np.asarray(W, dtype=np.float64)
    d_out, d_in = W.shape
    if sigma == 0.0:
        return W
    A = noise_matrix(seed, step, layer, 0, member, d_out, rank, NOISE_BF16)
    B = noise_matrix(seed, step, layer, 1, member, d_in, rank, NOISE_BF16)
    E = A @ B.T                                 # the explicit d_out x d_in perturbation, sum of r outer products
    E *= sigma / math.sqrt(rank)
    E += W
    return E


def member_linear(seed, step, layer, member, W, x, rank, sigma) -> np.ndarray:
    """Rows x [S, d_in] of one member through its own matrix: x W_i^T, fp64, unrounded."""
    return np.asarray(x, dtype=np.float64) @ member_matrix(seed, step, layer, member, W, rank, sigma).T


def rmsnorm(x, g, eps) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(g, dtype=np.float64) / np.sqrt(ms + eps)


def causal_attention(q, k, v, heads) -> np.ndarray:
    """One member's S tokens: q, k, v [S, d] fp64 -> [S, d]; head h owns columns h*hd .. (h+1)*hd."""
    q, k, v = (np.asarray(t, dtype=np.float64) for t in (q, k, v))
    S, d = q.shape
    hd = d // heads
    out = np.empty((S, d))
    for h in range(heads):
        sl = slice(h * hd, (h + 1) * hd)
        for s in range(S):                      # token s attends to tokens 0..s
            sc = k[: s + 1, sl] @ q[s, sl] / math.sqrt(hd)
            p = np.exp(sc - sc.max())
            p /= p.sum()
            out[s, sl] = p @ v[: s + 1, sl]
    return out


def token_loglik(logits, tokens) -> np.ndarray:
    """logits [S, V], tokens [S] of one member -> ll [S] (natural log; last entry 0)."""
    logits = np.asarray(logits, dtype=np.float64)
    S = logits.shape[0]
    ll = np.zeros(S)
    for s in range(S - 1):
        row = logits[s]
        m = row.max()
        ll[s] = row[int(tokens[s + 1])] - (m + math.log(np.exp(row - m).sum()))
    return ll


# ---------------------------------------------------------------------------------------------------
def mlp_stack_forward(seed, step, layer, members, S, rank, sigma, W1, W2, X, keep=False):
    """members: iterable of global member ids; X: dict or array giving each member's rows [S, d] in the order
    of `members`.  W1 [L, d_ff, d], W2 [L, d, d_ff].  Returns Y [len(members), S, d] (bf16 values, fp64); with
    keep=True also the list of per-layer (hidden, output) arrays."""
    members = list(members)
    L = len(W1)
    h = [round_bf16(np.asarray(X[i], dtype=np.float64)) for i in range(len(members))]
    trace = []
    for l in range(L):
        W1l, W2l = np.asarray(W1[l], dtype=np.float64), np.asarray(W2[l], dtype=np.float64)
        u = [round_bf16(gelu(member_linear(seed, step, layer + 2 * l, m, W1l, h[i], rank, sigma))) for i, m in enumerate(members)]
        h = [round_bf16(member_linear(seed, step, layer + 2 * l + 1, m, W2l, u[i], rank, sigma)) for i, m in enumerate(members)]
        if keep:
            trace.append((np.stack(u), np.stack(h)))
    Y = np.stack(h)
    return (Y, trace) if keep else Y


DECODER_MATRICES = ("wq", "wk", "wv", "wo", "w_up", "w_down")


def decoder_layer(seed, step, layer_base, l, member, P, heads, eps, rank, sigma, x, keep=None):
    """One decoder layer for one member: x [S, d] (bf16 values) -> x' [S, d].  P: dict of the weight arrays.
    keep: optional dict that receives the intermediates h1, q, k, v, o, x_mid, h2, u."""
    lid = layer_base + 6 * l
    lin = lambda j, name, inp: member_linear(seed, step, lid + j, member, P[name][l], inp, rank, sigma)  # noqa: E731
    h1 = round_bf16(rmsnorm(x, P["norm1"][l], eps))
    q, k, v = (round_bf16(lin(j, n, h1)) for j, n in enumerate(("wq", "wk", "wv")))
    o = round_bf16(causal_attention(q, k, v, heads))
    x_mid = round_bf16(x + lin(3, "wo", o))
    h2 = round_bf16(rmsnorm(x_mid, P["norm2"][l], eps))
    u = round_bf16(gelu(lin(4, "w_up", h2)))
    x_out = round_bf16(x_mid + lin(5, "w_down", u))
    if keep is not None:
        keep.update(h1=h1, q=q, k=k, v=v, o=o, x_mid=x_mid, h2=h2, u=u)
    return x_out


def decoder_forward(seed, step, layer, members, tokens, P, heads, eps, rank, sigma, keep=False):
    """members: global member ids; tokens [len(members), S] ints.  P: emb [V, d], norm1/norm2 [L, d],
    wq/wk/wv/wo [L, d, d], w_up [L, d_ff, d], w_down [L, d, d_ff], norm_f [d], head [V, d].
    Returns (logits [n, S, V], loglik [n, S]); with keep=True also a list (per member) of lists (per layer)
    of the intermediates."""
    members = list(members)
    tokens = np.asarray(tokens)
    L = len(P["wq"])
    logits, ll, traces = [], [], []
    for i, m in enumerate(members):
        x = round_bf16(np.asarray(P["emb"], dtype=np.float64)[tokens[i]])
        tr = []
        for l in range(L):
            kd = {"x_in": x} if keep else None
            x = decoder_layer(seed, step, layer, l, m, P, heads, eps, rank, sigma, x, kd)
            if keep:
                kd["x_out"] = x
                tr.append(kd)
        hf = round_bf16(rmsnorm(x, P["norm_f"], eps))
        lg = round_bf16(member_linear(seed, step, layer + 6 * L, m, P["head"], hf, rank, sigma))
        if keep:
            tr.append({"x_in": x, "hf": hf})
        logits.append(lg)
        ll.append(token_loglik(lg, tokens[i]))
        traces.append(tr)
    out = (np.stack(logits), np.stack(ll))
    return out + (traces,) if keep else out
