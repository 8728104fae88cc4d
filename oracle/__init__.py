"""EGGROLL CPU oracle (test infrastructure, not product code).

Thin ctypes/numpy wrapper around ``eggroll_oracle.c``.  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product (``paper_2511_16652_amd``)
never does.  Every function here cites the passage of the paper it follows in the C source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "eggroll_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

NOISE_F32 = 0
NOISE_BF16 = 1
ACT_NONE = 0
ACT_GELU = 1
WHICH_A = 0
WHICH_B = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP); returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, u32, i64, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64, ctypes.c_int
        dbl, vp = ctypes.c_double, ctypes.c_void_p
        lib.oracle_threefry2x32_20.argtypes = [vp, vp, vp]
        lib.oracle_threefry2x32_20.restype = None
        lib.oracle_stream_key.argtypes = [u64, u32, u32, i32, vp]
        lib.oracle_stream_key.restype = None
        lib.oracle_raw_words.argtypes = [u64, u32, u32, i32, i64, u64, u64, vp]
        lib.oracle_raw_words.restype = None
        lib.oracle_noise_normal.argtypes = [u64, u32, u32, i32, i64, u64, u64, vp]
        lib.oracle_noise_normal.restype = None
        lib.oracle_int_from_byte.argtypes = [ctypes.c_uint, i32]
        lib.oracle_int_from_byte.restype = i32
        lib.oracle_noise_int.argtypes = [u64, u32, u32, i32, i64, u64, u64, i32, vp]
        lib.oracle_noise_int.restype = None
        lib.oracle_normal_int_table.argtypes = [vp]
        lib.oracle_normal_int_table.restype = None
        lib.oracle_round_bf16.argtypes = [dbl]
        lib.oracle_round_bf16.restype = dbl
        lib.oracle_noise_matrix.argtypes = [u64, u32, u32, i32, i64, i64, i32, i32, vp]
        lib.oracle_noise_matrix.restype = None
        lib.oracle_noise_gather.argtypes = [u64, u32, u32, i32, i64, i64, vp, i64, i32, vp]
        lib.oracle_noise_gather.restype = None
        lib.oracle_forward.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, i32, dbl, i32,
                                       vp, vp, vp]
        lib.oracle_forward.restype = i32
        lib.oracle_update.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, vp, dbl, vp]
        lib.oracle_update.restype = i32
        lib.oracle_update_entry.argtypes = [u64, u32, u32, i64, i64, i32, i32, vp, dbl, i64, i64]
        lib.oracle_update_entry.restype = dbl
        lib.oracle_forward_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, i32,
                                          vp, vp, vp]
        lib.oracle_forward_i8.restype = None
        lib.oracle_forward_antithetic.argtypes = lib.oracle_forward.argtypes
        lib.oracle_forward_antithetic.restype = i32
        lib.oracle_forward_i8_antithetic.argtypes = lib.oracle_forward_i8.argtypes
        lib.oracle_forward_i8_antithetic.restype = None
        lib.oracle_matmul_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, i32, i32, vp, vp, vp]
        lib.oracle_matmul_i8.restype = None
        lib.oracle_gru_step_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_gru_step_i8.restype = None
        lib.oracle_update_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, vp, i64, vp, vp, vp]
        lib.oracle_update_i8.restype = i32
        lib.oracle_int_threshold.argtypes = [dbl, i64, dbl]
        lib.oracle_int_threshold.restype = i64
        lib.oracle_layernorm_i8.argtypes = [i64, i32, vp, vp, vp]
        lib.oracle_layernorm_i8.restype = None
        lib.oracle_embed_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, vp, vp, vp]
        lib.oracle_embed_i8.restype = None
        lib.oracle_egg_forward_i8.argtypes = [u64, u32, u32, i64, i64, i32, i32, i32, i32, i32, i32] + [vp] * 13
        lib.oracle_egg_forward_i8.restype = i32
        lib.oracle_loglik_i8.argtypes = [i64, vp, vp, i32, vp]
        lib.oracle_loglik_i8.restype = None
        lib.oracle_threads.argtypes = []
        lib.oracle_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def threads() -> int:
    return int(_load().oracle_threads())


def threefry2x32_20(counter, key) -> np.ndarray:
    """One Threefry-2x32-20 block: counter[2], key[2] (uint32) -> 2 uint32."""
    c = _c(counter, np.uint32)
    k = _c(key, np.uint32)
    assert c.shape == (2,) and k.shape == (2,)
    out = np.empty(2, np.uint32)
    _load().oracle_threefry2x32_20(_ptr(c), _ptr(k), _ptr(out))
    return out


def stream_key(seed, step, layer, which) -> np.ndarray:
    """The derived 64-bit key of one (seed, step, layer, which) stream, as 2 uint32."""
    out = np.empty(2, np.uint32)
    _load().oracle_stream_key(seed, step, layer, which, _ptr(out))
    return out


def raw_words(seed, step, layer, which, member, first_word, n) -> np.ndarray:
    out = np.empty(int(n), np.uint32)
    _load().oracle_raw_words(seed, step, layer, which, member, first_word, n, _ptr(out))
    return out


def noise_normal(seed, step, layer, which, member, first, n) -> np.ndarray:
    """fp64 Box-Muller normals with flat indices first..first+n-1 (before storage rounding)."""
    out = np.empty(int(n), np.float64)
    _load().oracle_noise_normal(seed, step, layer, which, member, first, n, _ptr(out))
    return out


def int_from_byte(byte: int, bound: int) -> int:
    return int(_load().oracle_int_from_byte(byte, bound))


BOUND_NORMAL16 = -16   # selects the table noise round(16 z) wherever a bound is taken


def normal_int_table() -> np.ndarray:
    """The 65536-entry int8 table T[k] = round(16 Phi^-1((k + 1/2) / 65536)) of the paper's integer noise."""
    out = np.empty(65536, np.int8)
    _load().oracle_normal_int_table(_ptr(out))
    return out


def noise_int(seed, step, layer, which, member, first, n, bound) -> np.ndarray:
    out = np.empty(int(n), np.int8)
    _load().oracle_noise_int(seed, step, layer, which, member, first, n, bound, _ptr(out))
    return out


def round_bf16(v: float) -> float:
    return float(_load().oracle_round_bf16(float(v)))


def noise_matrix(seed, step, layer, which, member, d, rank, noise_dtype) -> np.ndarray:
    """A_i (which=0) or B_i (which=1) as stored: fp64 array [d, rank] of storage-dtype values."""
    out = np.empty((int(d), int(rank)), np.float64)
    _load().oracle_noise_matrix(seed, step, layer, which, member, d, rank, noise_dtype, _ptr(out))
    return out


def noise_gather(seed, step, layer, which, member_begin, member_count, idx, noise_dtype) -> np.ndarray:
    """Entries idx (flat indices d*rank + l) of the stored factor vectors of a range of members: fp64 [count, len(idx)]."""
    idx = _c(idx, np.int64)
    out = np.empty((int(member_count), idx.size), np.float64)
    _load().oracle_noise_gather(seed, step, layer, which, member_begin, member_count, _ptr(idx), idx.size, noise_dtype, _ptr(out))
    return out


def forward(seed, step, layer, member_begin, member_count, S, d_out, d_in, rank, noise_dtype,
            sigma, act, W, X, antithetic=False) -> np.ndarray:
    """Explicit-W_i population forward; returns fp64 Y[member_count*S, d_out] (unrounded).
    antithetic: members 2p, 2p+1 evaluate M + sigma E_p and M - sigma E_p (noise id p)."""
    W = _c(W, np.float64)
    X = _c(X, np.float64)
    assert W.shape == (d_out, d_in) and X.shape == (member_count * S, d_in)
    Y = np.empty((member_count * S, d_out), np.float64)
    fn = _load().oracle_forward_antithetic if antithetic else _load().oracle_forward
    rc = fn(seed, step, layer, member_begin, member_count, S, d_out, d_in,
                                rank, noise_dtype, float(sigma), act, _ptr(W), _ptr(X), _ptr(Y))
    if rc != 0:
        raise MemoryError("oracle_forward")
    return Y


def update(seed, step, layer, member_begin, member_count, d_out, d_in, rank, noise_dtype,
           fitness, scale) -> np.ndarray:
    """G = scale * sum_i f_i A_i B_i^T as explicit outer products; fp64 [d_out, d_in]."""
    f = _c(fitness, np.float64)
    assert f.shape == (member_count,)
    G = np.empty((d_out, d_in), np.float64)
    rc = _load().oracle_update(seed, step, layer, member_begin, member_count, d_out, d_in, rank,
                               noise_dtype, _ptr(f), float(scale), _ptr(G))
    if rc != 0:
        raise MemoryError("oracle_update")
    return G


def update_entry(seed, step, layer, member_begin, member_count, rank, noise_dtype, fitness, scale,
                 j, k) -> float:
    f = _c(fitness, np.float64)
    return float(_load().oracle_update_entry(seed, step, layer, member_begin, member_count, rank,
                                             noise_dtype, _ptr(f), float(scale), j, k))


def forward_i8(seed, step, layer, member_begin, member_count, d, bound, corr_shift, out_shift,
               steps, W, H_in, antithetic=False) -> np.ndarray:
    W = _c(W, np.int8)
    H = _c(H_in, np.int8)
    assert W.shape == (d, d) and H.shape == (member_count, d)
    out = np.empty_like(H)
    fn = _load().oracle_forward_i8_antithetic if antithetic else _load().oracle_forward_i8
    fn(seed, step, layer, member_begin, member_count, d, bound, corr_shift,
                              out_shift, steps, _ptr(W), _ptr(H), _ptr(out))
    return out


def matmul_i8(seed, step, layer, member_begin, member_count, d_out, d_in, bound, corr_shift, out_shift,
              W, H_in, antithetic=False) -> np.ndarray:
    """One perturbed integer matmul with a rectangular theta [d_out, d_in]: int8 [count, d_in] -> [count, d_out]."""
    W = _c(W, np.int8)
    H = _c(H_in, np.int8)
    assert W.shape == (d_out, d_in) and H.shape == (member_count, d_in)
    out = np.empty((member_count, d_out), np.int8)
    _load().oracle_matmul_i8(seed, step, layer, member_begin, member_count, d_out, d_in, bound, corr_shift,
                             out_shift, int(bool(antithetic)), _ptr(W), _ptr(H), _ptr(out))
    return out


def gru_step_i8(seed, step, layer, member_begin, member_count, D, bound, corr_shift, out_shift,
                Wf, Uf, Wh, Uh, bf, bh, U, S, antithetic=False) -> np.ndarray:
    """One time step of the integer GRU cell for a population: returns the new state int8 [count, D].
    The four matrices use noise layers layer .. layer+3."""
    mats = [_c(m, np.int8) for m in (Wf, Uf, Wh, Uh)]
    vecs = [_c(v, np.int8) for v in (bf, bh)]
    U, S = _c(U, np.int8), _c(S, np.int8)
    assert all(m.shape == (D, D) for m in mats) and all(v.shape == (D,) for v in vecs)
    assert U.shape == (member_count, D) and S.shape == (member_count, D)
    H = np.empty_like(S)
    _load().oracle_gru_step_i8(seed, step, layer, member_begin, member_count, D, bound, corr_shift, out_shift,
                               int(bool(antithetic)), *[_ptr(m) for m in mats], *[_ptr(v) for v in vecs],
                               _ptr(U), _ptr(S), _ptr(H))
    return H


def update_i8(seed, step, layer, member_begin, member_count, d_out, d_in, bound, F, threshold, theta):
    """Integer update: returns (theta', E) with E = sum_i F_i A_i B_i^T (int32) and
    theta' = clamp(theta + sign(E) [|E| >= threshold], -127, 127)."""
    F = _c(F, np.int8)
    theta = _c(theta, np.int8)
    assert F.shape == (member_count,) and theta.shape == (d_out, d_in)
    out = np.empty_like(theta)
    E = np.empty((d_out, d_in), np.int32)
    rc = _load().oracle_update_i8(seed, step, layer, member_begin, member_count, d_out, d_in, bound, _ptr(F),
                                  int(threshold), _ptr(theta), _ptr(out), _ptr(E))
    if rc == -1:
        raise MemoryError("oracle_update_i8")
    if rc == -2:
        raise OverflowError("oracle_update_i8: |E| exceeds int32")
    return out, E


def layernorm_i8(ln, U) -> np.ndarray:
    """Mean-absolute-value layer normalisation of int8 rows [rows, D] with weight ln [D]."""
    ln, U = _c(ln, np.int8), _c(U, np.int8)
    rows, D = U.shape
    assert ln.shape == (D,) and D & (D - 1) == 0
    out = np.empty_like(U)
    _load().oracle_layernorm_i8(rows, D, _ptr(ln), _ptr(U), _ptr(out))
    return out


def embed_i8(seed, step, layer, member_begin, member_count, D, bound, corr_shift, emb, tokens,
             antithetic=False) -> np.ndarray:
    """Perturbed embedding lookup: tokens uint8 [count] -> int8 [count, D]; emb int8 [256, D]."""
    emb, tokens = _c(emb, np.int8), _c(tokens, np.uint8)
    assert emb.shape == (256, D) and tokens.shape == (member_count,)
    out = np.empty((member_count, D), np.int8)
    _load().oracle_embed_i8(seed, step, layer, member_begin, member_count, D, bound, corr_shift,
                            int(bool(antithetic)), _ptr(emb), _ptr(tokens), _ptr(out))
    return out


EGG_PARAM_NAMES = ("emb", "ln1", "gru_w", "gru_b", "ln2", "mlp1", "mlp2", "ln_out", "head")


def egg_param_shapes(D, L):
    """Shapes of the integer model's parameter arrays, in the order of EGG_PARAM_NAMES."""
    return {"emb": (256, D), "ln1": (L, D), "gru_w": (L, 4, D, D), "gru_b": (L, 2, D), "ln2": (L, D),
            "mlp1": (L, 4 * D, D), "mlp2": (L, D, 4 * D), "ln_out": (D,), "head": (256, D)}


def egg_forward_i8(seed, step, layer, member_begin, member_count, D, L, bound, corr_shift, params, tokens, S_in,
                   antithetic=False):
    """The integer model's forward pass for a population: tokens uint8 [T, count], S_in int8 [L, count, D]
    -> (logits int8 [T, count, 256], S_out int8 [L, count, D]).  params: dict of EGG_PARAM_NAMES."""
    shapes = egg_param_shapes(D, L)
    arrs = [_c(params[k], np.int8) for k in EGG_PARAM_NAMES]
    for k, a in zip(EGG_PARAM_NAMES, arrs):
        assert a.shape == shapes[k], (k, a.shape, shapes[k])
    tokens, S_in = _c(tokens, np.uint8), _c(S_in, np.int8)
    T = tokens.shape[0]
    assert tokens.shape == (T, member_count) and S_in.shape == (L, member_count, D)
    S_out = np.empty_like(S_in)
    logits = np.empty((T, member_count, 256), np.int8)
    rc = _load().oracle_egg_forward_i8(seed, step, layer, member_begin, member_count, D, L, bound, corr_shift,
                                       int(bool(antithetic)), T, *[_ptr(a) for a in arrs], _ptr(tokens),
                                       _ptr(S_in), _ptr(S_out), _ptr(logits))
    if rc != 0:
        raise MemoryError("oracle_egg_forward_i8")
    return logits, S_out


def loglik_i8(logits, targets, out=None) -> np.ndarray:
    """Log-likelihood of the target tokens in 1/16 bit: logits int8 [rows, 256], targets uint8 [rows] -> int32
    [rows]; added to `out` when given."""
    logits, targets = _c(logits, np.int8), _c(targets, np.uint8)
    rows = logits.shape[0]
    assert logits.shape == (rows, 256) and targets.shape == (rows,)
    acc = out is not None
    res = _c(out, np.int32).copy() if acc else np.empty(rows, np.int32)
    _load().oracle_loglik_i8(rows, _ptr(logits), _ptr(targets), int(acc), _ptr(res))
    return res


def int_threshold(alpha: float, n_terms: int, noise_std: float) -> int:
    """trunc(noise_std * Phi^-1(1 - alpha/2)) * round(noise_std * sqrt(n_terms))."""
    return int(_load().oracle_int_threshold(float(alpha), int(n_terms), float(noise_std)))
