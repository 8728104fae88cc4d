"""Seeded synthetic inputs for the EGGROLL hot path (shared by tests, oracle runs and bench.py).

This module holds NO arithmetic of the method itself: it only draws weights, activations, targets
and raw fitness scores with the shapes and value distributions of the workloads, and rounds them
to their storage dtype so that the CPU oracle and the GPU path read identical values.
All draws come from ``numpy.random.default_rng(data_seed)``.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float array to the nearest bfloat16 (ties to even); result stays float32."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    bits = (bits + 0x7FFF + lsb) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bfloat16-representable float32 values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    return (f.view(np.uint32) >> 16).astype(np.uint16).reshape(f.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).reshape(b.shape)


@dataclass
class LinearWorkload:
    """One perturbed linear layer: the shapes of the float configurations."""
    name: str
    dtype: str            # "f32" or "bf16": storage type of W, X, Y and of the noise
    d_out: int
    d_in: int
    N: int                # population size
    S: int                # rows (tokens) per member
    rank: int
    sigma: float
    data_seed: int
    noise_seed: int = 0
    step: int = 0
    layer: int = 0
    W: np.ndarray = field(default=None, repr=False)
    X: np.ndarray = field(default=None, repr=False)
    target: np.ndarray = field(default=None, repr=False)
    raw_fitness: np.ndarray = field(default=None, repr=False)


def make_linear(name, dtype, d_out, d_in, N, S, rank, sigma, data_seed, layer=0) -> LinearWorkload:
    """W ~ N(0, 1/d_in), X ~ N(0, 1), target ~ N(0, 1), raw fitness ~ N(0, 1)."""
    rng = np.random.default_rng(data_seed)
    W = (rng.standard_normal((d_out, d_in)) / np.sqrt(d_in)).astype(np.float32)
    X = rng.standard_normal((N * S, d_in)).astype(np.float32)
    target = rng.standard_normal(d_out).astype(np.float32)
    raw = rng.standard_normal(N).astype(np.float64)
    if dtype == "bf16":
        W, X = round_to_bf16(W), round_to_bf16(X)
    return LinearWorkload(name, dtype, d_out, d_in, N, S, rank, sigma, data_seed, 0, 0, layer,
                          W, X, target, raw)


def config1() -> LinearWorkload:
    """fp32 256x256 layer, N = 64, r = 1, sigma = 0.01, one input per member."""
    return make_linear("cfg1_f32_256", "f32", 256, 256, 64, 1, 1, 0.01, 1001)


def config2(N: int = 4096, d: int = 4096) -> LinearWorkload:
    """bf16 4096x4096 layer, N = 4096, r = 1, sigma = 1e-3, one token per member."""
    return make_linear("cfg2_bf16_%d_N%d" % (d, N), "bf16", d, d, N, 1, 1, 1e-3, 1002)


def centered(f: np.ndarray) -> np.ndarray:
    """Raw scores shifted to zero mean (the caller-side shaping of the synthetic fitness)."""
    f = np.asarray(f, dtype=np.float64)
    return f - f.mean()


@dataclass
class Int8Workload:
    """The integer recurrent cell: one square int8 matrix applied `steps` times."""
    name: str
    d: int
    N: int
    bound: int
    corr_shift: int
    out_shift: int
    steps: int
    data_seed: int
    noise_seed: int = 0
    step: int = 0
    layer: int = 0
    W: np.ndarray = field(default=None, repr=False)
    H0: np.ndarray = field(default=None, repr=False)


def make_int8(name, d, N, steps, data_seed, bound=8, corr_shift=4, out_shift=8) -> Int8Workload:
    """W and h_0 uniform integers on [-127, 127]."""
    rng = np.random.default_rng(data_seed)
    W = rng.integers(-127, 128, size=(d, d), dtype=np.int64).astype(np.int8)
    H0 = rng.integers(-127, 128, size=(N, d), dtype=np.int64).astype(np.int8)
    return Int8Workload(name, d, N, bound, corr_shift, out_shift, steps, data_seed, 0, 0, 0, W, H0)


def config3(N: int = 8192, d: int = 1024, steps: int = 64) -> Int8Workload:
    return make_int8("cfg3_i8_%d_N%d_T%d" % (d, N, steps), d, N, steps, 1003)


EGG_PARAM_SHAPES = lambda D, L: {  # noqa: E731  (layouts of the integer model's parameter arrays)
    "emb": (256, D), "ln1": (L, D), "gru_w": (L, 4, D, D), "gru_b": (L, 2, D), "ln2": (L, D),
    "mlp1": (L, 4 * D, D), "mlp2": (L, D, 4 * D), "ln_out": (D,), "head": (256, D)}


def egg_model(D: int, L: int, data_seed: int, weight_std: float = 16.0, ln_weight: int = 16) -> dict:
    """Synthetic parameters of the integer model: matrices and the embedding table are 16 * N(0, 1)
    rounded to the nearest integer and clipped to [-127, 127] (the initialisation the paper's scaled
    matmul is designed around), normalisation weights a constant, biases zero."""
    rng = np.random.default_rng(data_seed)
    out = {}
    for name, shape in EGG_PARAM_SHAPES(D, L).items():
        if name in ("ln1", "ln2", "ln_out"):
            out[name] = np.full(shape, ln_weight, np.int8)
        elif name == "gru_b":
            out[name] = np.zeros(shape, np.int8)
        else:
            out[name] = np.clip(np.rint(weight_std * rng.standard_normal(shape)), -127, 127).astype(np.int8)
    return out


def egg_tokens(T: int, N: int, data_seed: int) -> np.ndarray:
    """Synthetic byte tokens [T, N] standing in for a character-level corpus: a skewed distribution over
    the printable range (frequent letters, space), independent per member and time step."""
    rng = np.random.default_rng(data_seed)
    alphabet = np.arange(32, 127)
    weights = 1.0 / (1.0 + np.arange(alphabet.size))      # Zipf-like
    return rng.choice(rng.permutation(alphabet), size=(T, N), p=weights / weights.sum()).astype(np.uint8)


def mlp_stack(d: int, d_ff: int, L: int, data_seed: int) -> dict:
    """Weights of the GELU MLP stack: W1 [L, d_ff, d] ~ N(0, 1/d), W2 [L, d, d_ff] ~ N(0, 1/d_ff), bf16 values."""
    rng = np.random.default_rng(data_seed)
    W1 = np.stack([round_to_bf16(rng.standard_normal((d_ff, d), dtype=np.float32) / np.float32(np.sqrt(d))) for _ in range(L)])
    W2 = np.stack([round_to_bf16(rng.standard_normal((d, d_ff), dtype=np.float32) / np.float32(np.sqrt(d_ff))) for _ in range(L)])
    return {"W1": W1, "W2": W2}


def member_rows(data_seed: int, member: int, S: int, d: int) -> np.ndarray:
    """Input rows x ~ N(0, 1) of one member, bf16 values, seeded per member so that any subset of a large
    population can be drawn without drawing the rest."""
    rng = np.random.default_rng([data_seed, int(member)])
    return round_to_bf16(rng.standard_normal((S, d), dtype=np.float32))


DECODER_PARAM_SHAPES = lambda V, d, d_ff, L: {  # noqa: E731  (layouts of the decoder's parameter arrays)
    "emb": (V, d), "norm1": (L, d), "wq": (L, d, d), "wk": (L, d, d), "wv": (L, d, d), "wo": (L, d, d),
    "norm2": (L, d), "w_up": (L, d_ff, d), "w_down": (L, d, d_ff), "norm_f": (d,), "head": (V, d)}


def decoder_params(V: int, d: int, d_ff: int, L: int, data_seed: int, norm_jitter: float = 0.0) -> dict:
    """Random-init decoder: linear matrices N(0, 1/fan_in), embedding N(0, 1), normalisation gains 1
    (+ norm_jitter * N(0, 1), for tests that must see the gains), all rounded to bf16."""
    rng = np.random.default_rng(data_seed)
    out = {}
    for name, shape in DECODER_PARAM_SHAPES(V, d, d_ff, L).items():
        if name.startswith("norm"):
            a = 1.0 + norm_jitter * rng.standard_normal(shape, dtype=np.float32)
        elif name == "emb":
            a = rng.standard_normal(shape, dtype=np.float32)
        else:
            a = rng.standard_normal(shape, dtype=np.float32)
            a *= np.float32(1.0 / np.sqrt(shape[-1]))
        out[name] = round_to_bf16(a)
    return out


def decoder_tokens(N: int, S: int, V: int, data_seed: int) -> np.ndarray:
    """Uniform random token ids [N, S] in [0, V)."""
    return np.random.default_rng(data_seed).integers(0, V, size=(N, S), dtype=np.int64).astype(np.int32)


def decoder_params_device(V: int, d: int, d_ff: int, L: int, data_seed: int, norm_jitter: float = 0.0) -> dict:
    """The same recipe as decoder_params, drawn on the GPU by torch's seeded generator (a billion-parameter model is
    too slow to draw on the host): dict of bf16 device tensors.  The values differ from the host recipe's; a test
    that needs them on the host copies them back."""
    import torch
    g = torch.Generator(device="cuda").manual_seed(data_seed)
    out = {}
    for name, shape in DECODER_PARAM_SHAPES(V, d, d_ff, L).items():
        if name.startswith("norm"):
            a = 1.0 + norm_jitter * torch.randn(shape, generator=g, device="cuda")
        else:
            a = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
            flat = a.view(-1, shape[-1])
            sc = 1.0 if name == "emb" else 1.0 / float(np.sqrt(shape[-1]))
            for lo in range(0, flat.shape[0], 1 << 14):      # in slabs: the fp32 draw of a whole tensor need not exist at once
                n = min(1 << 14, flat.shape[0] - lo)
                flat[lo:lo + n] = (torch.randn((n, shape[-1]), generator=g, device="cuda") * sc).to(torch.bfloat16)
        out[name] = a.to(torch.bfloat16).contiguous()
    return out


def decoder_tokens_device(N: int, S: int, V: int, data_seed: int):
    import torch
    g = torch.Generator(device="cuda").manual_seed(data_seed)
    return torch.randint(0, V, (N, S), generator=g, device="cuda", dtype=torch.int32)
