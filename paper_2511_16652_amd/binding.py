"""Python binding of libeggroll (argument marshalling only; every step runs in the HIP kernels).

The functions mirror ``include/eggroll.h`` one to one and take ``torch`` CUDA(ROCm) tensors, whose
``data_ptr()`` is handed to the C ABI.  PyTorch is used for device memory and streams only.
There is no CPU fallback: if the shared library is missing, importing this module's loader raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libeggroll.so")

EGG_OK, EGG_EINVAL, EGG_EUNSUPPORTED, EGG_EHIP, EGG_ENOMEM = 0, -1, -2, -3, -4
EGG_F32, EGG_BF16, EGG_I8, EGG_U32 = 0, 1, 2, 3
EGG_NORMAL, EGG_UNIFORM_INT, EGG_RAW, EGG_NORMAL_INT16 = 0, 1, 2, 3
EGG_INT_NOISE_NORMAL16 = -16
EGG_ACT_NONE, EGG_ACT_GELU = 0, 1

EXPORTS = ["eggroll_create", "eggroll_destroy", "eggroll_strerror", "eggroll_last_error",
           "eggroll_default_scale", "eggroll_set_cache_layout", "eggroll_noise_gen", "eggroll_perturbed_forward",
           "eggroll_perturbed_forward_i8", "eggroll_gru_i8", "eggroll_layernorm_i8", "eggroll_embed_i8",
           "eggroll_egg_forward_i8", "eggroll_loglik_i8", "eggroll_egg_update_i8", "eggroll_update", "eggroll_update_i8",
           "eggroll_int_threshold", "eggroll_profile_enable", "eggroll_profile_read",
           "eggroll_scratch_generation", "eggroll_trim", "eggroll_set_conservative_waits", "eggroll_normal_int_table", "eggroll_perturbed_forward_noalloc", "eggroll_perturbed_forward_add", "eggroll_perturbed_forward_chained",
           "eggroll_embed_rows_bf16", "eggroll_rmsnorm_bf16", "eggroll_causal_attention_bf16", "eggroll_causal_attention_project_bf16", "eggroll_token_loglik_bf16",
           "eggroll_mlp_stack_forward", "eggroll_mlp_stack_update", "eggroll_decoder_forward", "eggroll_decoder_update"]


class EggKey(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("step", ctypes.c_uint32), ("layer", ctypes.c_uint32)]


EGG_CACHE_ROWS, EGG_CACHE_PANEL = 0, 1

EGG_MODEL_FIELDS = ("emb", "ln1", "gru_w", "gru_b", "ln2", "mlp1", "mlp2", "ln_out", "head")


class EggModelI8(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in EGG_MODEL_FIELDS]


class EggDecoderCfg(ctypes.Structure):
    _fields_ = [("layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("d_ff", ctypes.c_int32), ("vocab", ctypes.c_int32), ("rms_eps", ctypes.c_float)]


EGG_DECODER_FIELDS = ("emb", "norm1", "wq", "wk", "wv", "wo", "norm2", "w_up", "w_down", "norm_f", "head")


class EggDecoderWeights(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in EGG_DECODER_FIELDS]


class EggShape(ctypes.Structure):
    _fields_ = [("member_begin", ctypes.c_int64), ("member_count", ctypes.c_int64),
                ("rows_per_member", ctypes.c_int32), ("d_out", ctypes.c_int32),
                ("d_in", ctypes.c_int32), ("rank", ctypes.c_int32), ("antithetic", ctypes.c_int32)]


class EggrollError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("eggroll status %d: %s" % (status, text))
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libeggroll.so and declares the signatures.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2511_16652_amd.build` "
            "(there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float
    P = ctypes.POINTER
    lib.eggroll_create.argtypes = [P(vp), i32, vp]
    lib.eggroll_create.restype = i32
    lib.eggroll_destroy.argtypes = [vp]
    lib.eggroll_destroy.restype = i32
    lib.eggroll_strerror.argtypes = [i32]
    lib.eggroll_strerror.restype = ctypes.c_char_p
    lib.eggroll_last_error.argtypes = [vp]
    lib.eggroll_last_error.restype = ctypes.c_char_p
    lib.eggroll_default_scale.argtypes = [i64, ctypes.c_double, i32]
    lib.eggroll_default_scale.restype = ctypes.c_double
    lib.eggroll_set_cache_layout.argtypes = [vp, i32]
    lib.eggroll_set_cache_layout.restype = i32
    lib.eggroll_noise_gen.argtypes = [vp, EggKey, P(EggShape), i32, i32, i32, vp, vp]
    lib.eggroll_noise_gen.restype = i32
    lib.eggroll_perturbed_forward.argtypes = [vp, EggKey, P(EggShape), i32, i32, f32, i32, vp, vp, vp, vp, vp]
    lib.eggroll_perturbed_forward.restype = i32
    lib.eggroll_perturbed_forward_noalloc.argtypes = lib.eggroll_perturbed_forward.argtypes
    lib.eggroll_perturbed_forward_noalloc.restype = i32
    lib.eggroll_perturbed_forward_i8.argtypes = [vp, EggKey, P(EggShape), i32, i32, i32, i32, vp, vp, vp]
    lib.eggroll_perturbed_forward_i8.restype = i32
    lib.eggroll_update.argtypes = [vp, EggKey, P(EggShape), i32, vp, f32, i32, vp, vp, i32, f32, vp, vp]
    lib.eggroll_update.restype = i32
    lib.eggroll_gru_i8.argtypes = [vp, EggKey, P(EggShape), i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.eggroll_gru_i8.restype = i32
    lib.eggroll_layernorm_i8.argtypes = [vp, i64, i32, vp, vp, vp]
    lib.eggroll_layernorm_i8.restype = i32
    lib.eggroll_embed_i8.argtypes = [vp, EggKey, P(EggShape), i32, i32, vp, vp, vp]
    lib.eggroll_embed_i8.restype = i32
    lib.eggroll_egg_forward_i8.argtypes = [vp, EggKey, P(EggShape), i32, i32, i32, i32, P(EggModelI8), vp, vp, vp, vp]
    lib.eggroll_egg_forward_i8.restype = i32
    lib.eggroll_loglik_i8.argtypes = [vp, i64, vp, vp, i32, vp]
    lib.eggroll_loglik_i8.restype = i32
    lib.eggroll_egg_update_i8.argtypes = [vp, EggKey, P(EggShape), i32, i32, vp, ctypes.c_int32, P(EggModelI8)]
    lib.eggroll_egg_update_i8.restype = i32
    lib.eggroll_update_i8.argtypes = [vp, EggKey, P(EggShape), i32, vp, ctypes.c_int32, vp, vp]
    lib.eggroll_update_i8.restype = i32
    lib.eggroll_int_threshold.argtypes = [ctypes.c_double, i64, ctypes.c_double]
    lib.eggroll_int_threshold.restype = i64
    lib.eggroll_scratch_generation.argtypes = [vp]
    lib.eggroll_scratch_generation.restype = ctypes.c_uint64
    lib.eggroll_set_conservative_waits.argtypes = [vp, i32]
    lib.eggroll_set_conservative_waits.restype = i32
    lib.eggroll_normal_int_table.argtypes = [vp]
    lib.eggroll_normal_int_table.restype = None
    lib.eggroll_trim.argtypes = [vp]
    lib.eggroll_trim.restype = i32
    lib.eggroll_perturbed_forward_add.argtypes = [vp, EggKey, P(EggShape), i32, i32, f32, i32, vp, vp, vp, vp, vp, vp]
    lib.eggroll_perturbed_forward_add.restype = i32
    lib.eggroll_perturbed_forward_chained.argtypes = [vp, EggKey, P(EggShape), i32, i32, f32, i32, vp, vp, vp, vp, vp, i32, ctypes.c_uint32, vp]
    lib.eggroll_perturbed_forward_chained.restype = i32
    lib.eggroll_embed_rows_bf16.argtypes = [vp, i64, i32, i32, vp, vp, vp]
    lib.eggroll_embed_rows_bf16.restype = i32
    lib.eggroll_rmsnorm_bf16.argtypes = [vp, i64, i32, f32, vp, vp, vp]
    lib.eggroll_rmsnorm_bf16.restype = i32
    lib.eggroll_causal_attention_bf16.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.eggroll_causal_attention_bf16.restype = i32
    lib.eggroll_causal_attention_project_bf16.argtypes = [vp, EggKey, i64, i64, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.eggroll_causal_attention_project_bf16.restype = i32
    lib.eggroll_token_loglik_bf16.argtypes = [vp, i64, i32, i32, vp, vp, vp]
    lib.eggroll_token_loglik_bf16.restype = i32
    lib.eggroll_mlp_stack_forward.argtypes = [vp, EggKey, P(EggShape), i32, i32, f32, vp, vp, vp, vp, i64]
    lib.eggroll_mlp_stack_forward.restype = i32
    lib.eggroll_mlp_stack_update.argtypes = [vp, EggKey, P(EggShape), i32, i32, vp, f32, f32, vp, vp]
    lib.eggroll_mlp_stack_update.restype = i32
    lib.eggroll_decoder_forward.argtypes = [vp, EggKey, P(EggShape), P(EggDecoderCfg), P(EggDecoderWeights), f32, vp, vp, vp, i64]
    lib.eggroll_decoder_forward.restype = i32
    lib.eggroll_decoder_update.argtypes = [vp, EggKey, P(EggShape), P(EggDecoderCfg), vp, f32, f32, P(EggDecoderWeights)]
    lib.eggroll_decoder_update.restype = i32
    lib.eggroll_profile_enable.argtypes = [vp, i32]
    lib.eggroll_profile_enable.restype = i32
    lib.eggroll_profile_read.argtypes = [vp, P(ctypes.c_char_p), P(i64), P(ctypes.c_double), i32]
    lib.eggroll_profile_read.restype = i32
    _lib = lib
    return lib


def _dtype_code(t) -> int:
    import torch
    return {torch.float32: EGG_F32, torch.bfloat16: EGG_BF16, torch.int8: EGG_I8,
            torch.uint32: EGG_U32, torch.int32: EGG_U32}[t.dtype]


def make_decoder_cfg(layers, d_model, heads, d_ff, vocab, rms_eps=1e-5) -> EggDecoderCfg:
    return EggDecoderCfg(int(layers), int(d_model), int(heads), int(d_ff), int(vocab), float(rms_eps))


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous device tensors"
    return ctypes.c_void_p(t.data_ptr())


def eggroll_default_scale(population: int, sigma: float, rank: int) -> float:
    return float(load_library().eggroll_default_scale(population, sigma, rank))


def eggroll_normal_int_table():
    """The 65536-entry int8 table of the paper's integer noise, as the library computes it on the host (numpy array)."""
    import numpy as np
    out = np.empty(65536, np.int8)
    load_library().eggroll_normal_int_table(out.ctypes.data_as(ctypes.c_void_p))
    return out


def eggroll_int_threshold(alpha: float, n_terms: int, noise_std: float) -> int:
    return int(load_library().eggroll_int_threshold(float(alpha), int(n_terms), float(noise_std)))


class Context:
    """eggroll_ctx bound to a torch device and (optionally) a torch stream."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the EGGROLL library runs on MI355X only")
        self._lib = load_library()
        self._torch_stream = stream  # keep alive
        handle = ctypes.c_void_p()
        sp = ctypes.c_void_p(stream.cuda_stream) if stream is not None else ctypes.c_void_p(
            torch.cuda.current_stream(device).cuda_stream)
        st = self._lib.eggroll_create(ctypes.byref(handle), device, sp)
        if st != EGG_OK:
            raise EggrollError(st, self._lib.eggroll_strerror(st).decode())
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            self._lib.eggroll_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != EGG_OK:
            raise EggrollError(st, "%s (%s)" % (self._lib.eggroll_strerror(st).decode(),
                                                self._lib.eggroll_last_error(self._h).decode()))

    # -- entry points ------------------------------------------------------------------------
    def eggroll_noise_gen(self, key, shape, dtype, dist, int_bound, A_out, B_out):
        self._check(self._lib.eggroll_noise_gen(self._h, key, ctypes.byref(shape), dtype, dist,
                                                int_bound, _ptr(A_out), _ptr(B_out)))

    def eggroll_perturbed_forward(self, key, shape, sigma, act, W, X, Y, A_cache=None, B_cache=None):
        self._check(self._lib.eggroll_perturbed_forward(
            self._h, key, ctypes.byref(shape), _dtype_code(W), _dtype_code(Y), float(sigma), act,
            _ptr(W), _ptr(X), _ptr(Y), _ptr(A_cache), _ptr(B_cache)))

    def eggroll_perturbed_forward_noalloc(self, key, shape, sigma, act, W, X, Y, A_cache=None, B_cache=None):
        self._check(self._lib.eggroll_perturbed_forward_noalloc(
            self._h, key, ctypes.byref(shape), _dtype_code(W), _dtype_code(Y), float(sigma), act,
            _ptr(W), _ptr(X), _ptr(Y), _ptr(A_cache), _ptr(B_cache)))

    def eggroll_perturbed_forward_add(self, key, shape, sigma, act, W, X, R_in, Y, A_cache=None, B_cache=None):
        self._check(self._lib.eggroll_perturbed_forward_add(
            self._h, key, ctypes.byref(shape), _dtype_code(W), _dtype_code(Y), float(sigma), act,
            _ptr(W), _ptr(X), _ptr(R_in), _ptr(Y), _ptr(A_cache), _ptr(B_cache)))

    def eggroll_perturbed_forward_chained(self, key, shape, sigma, act, W, X, Y, R_in=None, t_in=None, next_layer=None, t_next=None):
        """next_layer given: t_next receives the next layer's rank-1 projections of Y."""
        self._check(self._lib.eggroll_perturbed_forward_chained(
            self._h, key, ctypes.byref(shape), _dtype_code(W), _dtype_code(Y), float(sigma), act, _ptr(W), _ptr(X), _ptr(R_in), _ptr(Y),
            _ptr(t_in), 0 if next_layer is None else 1, int(next_layer or 0), _ptr(t_next)))

    def eggroll_embed_rows_bf16(self, rows, d, vocab, emb, tokens, X):
        self._check(self._lib.eggroll_embed_rows_bf16(self._h, int(rows), int(d), int(vocab), _ptr(emb), _ptr(tokens), _ptr(X)))

    def eggroll_rmsnorm_bf16(self, rows, d, eps, gain, X, Y):
        self._check(self._lib.eggroll_rmsnorm_bf16(self._h, int(rows), int(d), float(eps), _ptr(gain), _ptr(X), _ptr(Y)))

    def eggroll_causal_attention_bf16(self, members, rows_per_member, heads, head_dim, Q, K, V, O):
        self._check(self._lib.eggroll_causal_attention_bf16(
            self._h, int(members), int(rows_per_member), int(heads), int(head_dim), _ptr(Q), _ptr(K), _ptr(V), _ptr(O)))

    def eggroll_causal_attention_project_bf16(self, key, member_begin, members, rows_per_member, heads, head_dim, Q, K, V, O, t_next):
        self._check(self._lib.eggroll_causal_attention_project_bf16(
            self._h, key, int(member_begin), int(members), int(rows_per_member), int(heads), int(head_dim), _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
            _ptr(t_next)))

    def eggroll_token_loglik_bf16(self, members, rows_per_member, vocab, logits, tokens, out):
        self._check(self._lib.eggroll_token_loglik_bf16(
            self._h, int(members), int(rows_per_member), int(vocab), _ptr(logits), _ptr(tokens), _ptr(out)))

    def eggroll_mlp_stack_forward(self, key, shape, layers, d_ff, sigma, W1, W2, X, Y, chunk_members=0):
        self._check(self._lib.eggroll_mlp_stack_forward(
            self._h, key, ctypes.byref(shape), int(layers), int(d_ff), float(sigma), _ptr(W1), _ptr(W2), _ptr(X), _ptr(Y),
            int(chunk_members)))

    def eggroll_mlp_stack_update(self, key, shape, layers, d_ff, fitness, scale, lr, W1, W2):
        self._check(self._lib.eggroll_mlp_stack_update(
            self._h, key, ctypes.byref(shape), int(layers), int(d_ff), _ptr(fitness), float(scale), float(lr), _ptr(W1), _ptr(W2)))

    def eggroll_decoder_forward(self, key, shape, cfg, weights, sigma, tokens, logits=None, loglik=None, chunk_members=0):
        """cfg: EggDecoderCfg; weights: mapping from the names in EGG_DECODER_FIELDS to bf16 device tensors."""
        w = EggDecoderWeights(*[_ptr(weights[name]) for name in EGG_DECODER_FIELDS])
        self._check(self._lib.eggroll_decoder_forward(
            self._h, key, ctypes.byref(shape), ctypes.byref(cfg), ctypes.byref(w), float(sigma), _ptr(tokens), _ptr(logits),
            _ptr(loglik), int(chunk_members)))

    def eggroll_decoder_update(self, key, shape, cfg, fitness, scale, lr, weights):
        """Updates the 6 layers + 1 perturbed matrices of `weights` in place."""
        w = EggDecoderWeights(*[_ptr(weights[name]) for name in EGG_DECODER_FIELDS])
        self._check(self._lib.eggroll_decoder_update(
            self._h, key, ctypes.byref(shape), ctypes.byref(cfg), _ptr(fitness), float(scale), float(lr), ctypes.byref(w)))

    def eggroll_scratch_generation(self):
        return int(self._lib.eggroll_scratch_generation(self._h))

    def eggroll_set_conservative_waits(self, on):
        self._check(self._lib.eggroll_set_conservative_waits(self._h, int(bool(on))))

    def eggroll_trim(self):
        self._check(self._lib.eggroll_trim(self._h))

    def eggroll_perturbed_forward_i8(self, key, shape, int_bound, corr_shift, out_shift, steps, W, H_in, H_out):
        self._check(self._lib.eggroll_perturbed_forward_i8(
            self._h, key, ctypes.byref(shape), int_bound, corr_shift, out_shift, steps,
            _ptr(W), _ptr(H_in), _ptr(H_out)))

    def eggroll_gru_i8(self, key, shape, int_bound, corr_shift, out_shift, steps, Wf, Uf, Wh, Uh, bf, bh, U, S_in, S_out):
        self._check(self._lib.eggroll_gru_i8(
            self._h, key, ctypes.byref(shape), int_bound, corr_shift, out_shift, steps,
            _ptr(Wf), _ptr(Uf), _ptr(Wh), _ptr(Uh), _ptr(bf), _ptr(bh), _ptr(U), _ptr(S_in), _ptr(S_out)))

    def eggroll_layernorm_i8(self, rows, D, ln, U, out):
        self._check(self._lib.eggroll_layernorm_i8(self._h, int(rows), int(D), _ptr(ln), _ptr(U), _ptr(out)))

    def eggroll_embed_i8(self, key, shape, int_bound, corr_shift, emb, tokens, Y):
        self._check(self._lib.eggroll_embed_i8(
            self._h, key, ctypes.byref(shape), int_bound, corr_shift, _ptr(emb), _ptr(tokens), _ptr(Y)))

    def eggroll_egg_forward_i8(self, key, shape, layers, int_bound, corr_shift, steps, model, tokens, S_in, S_out, logits):
        """model: mapping from the names in EGG_MODEL_FIELDS to int8 device tensors."""
        m = EggModelI8(*[_ptr(model[name]) for name in EGG_MODEL_FIELDS])
        self._check(self._lib.eggroll_egg_forward_i8(
            self._h, key, ctypes.byref(shape), int(layers), int_bound, corr_shift, int(steps), ctypes.byref(m),
            _ptr(tokens), _ptr(S_in), _ptr(S_out), _ptr(logits)))

    def eggroll_loglik_i8(self, rows, logits, targets, accumulate, out):
        self._check(self._lib.eggroll_loglik_i8(self._h, int(rows), _ptr(logits), _ptr(targets), int(accumulate), _ptr(out)))

    def eggroll_egg_update_i8(self, key, shape, layers, int_bound, fitness, threshold, model):
        """Updates model["emb"], ["gru_w"], ["mlp1"], ["mlp2"], ["head"] in place."""
        m = EggModelI8(*[_ptr(model[name]) for name in EGG_MODEL_FIELDS])
        self._check(self._lib.eggroll_egg_update_i8(
            self._h, key, ctypes.byref(shape), int(layers), int_bound, _ptr(fitness), int(threshold), ctypes.byref(m)))

    def eggroll_set_cache_layout(self, layout):
        self._check(self._lib.eggroll_set_cache_layout(self._h, int(layout)))

    def eggroll_update(self, key, shape, noise_dtype, fitness, scale, accumulate, G, W=None, lr=0.0,
                       A_cache=None, B_cache=None):
        w_dtype = _dtype_code(W) if W is not None else EGG_F32
        self._check(self._lib.eggroll_update(
            self._h, key, ctypes.byref(shape), noise_dtype, _ptr(fitness), float(scale), int(accumulate),
            _ptr(G), _ptr(W), w_dtype, float(lr), _ptr(A_cache), _ptr(B_cache)))

    def eggroll_update_i8(self, key, shape, int_bound, fitness, threshold, theta, E_out=None):
        self._check(self._lib.eggroll_update_i8(
            self._h, key, ctypes.byref(shape), int_bound, _ptr(fitness), int(threshold), _ptr(theta), _ptr(E_out)))

    # -- per-kernel timing -----------------------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(self._lib.eggroll_profile_enable(self._h, int(on)))

    def profile_read(self):
        """{kernel name: (launches, total milliseconds)} since the last read."""
        cap = 64
        names = (ctypes.c_char_p * cap)()
        launches = (ctypes.c_int64 * cap)()
        ms = (ctypes.c_double * cap)()
        n = self._lib.eggroll_profile_read(self._h, names, launches, ms, cap)
        if n < 0:
            self._check(n)
        return {names[i].decode(): (int(launches[i]), float(ms[i])) for i in range(min(n, cap))}


def make_key(seed: int, step: int, layer: int) -> EggKey:
    return EggKey(seed, step, layer)


def make_shape(member_begin, member_count, rows_per_member, d_out, d_in, rank, antithetic=0) -> EggShape:
    return EggShape(member_begin, member_count, rows_per_member, d_out, d_in, rank, int(antithetic))
