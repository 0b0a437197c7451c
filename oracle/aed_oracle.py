"""ctypes binding of the CPU oracle (oracle/aed_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product path.  Argument
marshalling only -- all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

from . import build as _build

_LAYER_FIELDS = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_cq", "b_cq", "w_ckv", "b_ckv", "w_co", "b_co",
    "ln3_g", "ln3_b", "w_ff1", "b_ff1", "w_ff2", "b_ff2",
)
_TOP_FIELDS = ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "w_out", "b_out")

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_i32p = C.POINTER(C.c_int32)


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                 "max_positions", "eos_id", "pad_id")] + \
               [("ln_eps", C.c_float), ("emb_scale", C.c_float), ("kv_fp8", C.c_int32), ("norm_type", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [(n, _f32p) for n in _LAYER_FIELDS]


class _Weights(C.Structure):
    _fields_ = [(n, _f32p) for n in _TOP_FIELDS] + [("layers", C.POINTER(_Layer))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        _lib.aedo_layernorm.argtypes = [_f64p, _f32p, _f32p, C.c_int, C.c_double, _f64p]
        _lib.aedo_layernorm.restype = None
        _lib.aedo_rmsnorm.argtypes = [_f64p, _f32p, _f32p, C.c_int, C.c_double, _f64p]
        _lib.aedo_rmsnorm.restype = None
        _lib.aedo_linear.argtypes = [_f64p, _f32p, _f32p, C.c_int, C.c_int, _f64p]
        _lib.aedo_linear.restype = None
        _lib.aedo_softmax.argtypes = [_f64p, C.c_int, _f64p]
        _lib.aedo_softmax.restype = None
        _lib.aedo_attend.argtypes = [_f64p, _f64p, _f64p, C.c_int, C.c_int, C.c_int, _f64p, _f64p]
        _lib.aedo_attend.restype = None
        _lib.aedo_argmax.argtypes = [_f64p, C.c_int]
        _lib.aedo_argmax.restype = C.c_int32
        _lib.aedo_cross_kv.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.c_int, _f32p,
                                       C.c_int, _f64p, _f64p]
        _lib.aedo_decode_forced.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), _f32p, _i32p,
                                            C.c_int, _i32p, C.c_int, _f64p]
        _lib.aedo_greedy_decode.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), _f32p, _i32p,
                                            C.c_int, _i32p, C.c_int, C.c_int, _i32p, _i32p, _i32p,
                                            _f64p]
        _lib.aedo_forward_full.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), _f32p, C.c_int,
                                           _i32p, C.c_int, _i32p, C.c_int, _i32p, _f64p]
        _lib.aedo_self_kv.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), _f32p, C.c_int, _i32p, C.c_int,
                                      C.c_int, _f64p, _f64p]
        _lib.aedo_layer_matrix_params.argtypes = [C.POINTER(_Config)]
        _lib.aedo_layer_matrix_params.restype = C.c_int64
        _lib.aedo_num_threads.restype = C.c_int
        _lib.aedo_fp8_e4m3_encode.argtypes = [C.c_float]
        _lib.aedo_fp8_e4m3_encode.restype = C.c_uint8
        _lib.aedo_fp8_e4m3_decode.argtypes = [C.c_uint8]
        _lib.aedo_fp8_e4m3_decode.restype = C.c_double
        _lib.aedo_fp8_e4m3_encode_array.argtypes = [_f32p, C.c_int64, C.POINTER(C.c_uint8)]
        _lib.aedo_fp8_e4m3_encode_array.restype = None
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p32(a):
    return None if a is None else a.ctypes.data_as(_f32p)


def _p64(a):
    return None if a is None else a.ctypes.data_as(_f64p)


def _pi(a):
    return None if a is None else a.ctypes.data_as(_i32p)


class Model:
    """Holds C views of a config + weight dict (arrays are kept alive here).

    cfg: any object with the DecoderConfig attribute names; weights: dict with
    the top-level arrays and weights['layers'] = list of per-layer dicts.  A
    bias entry may be None."""

    def __init__(self, cfg, weights: Dict):
        self.cfg = cfg
        self._keep = []
        c = _Config()
        for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                  "max_positions", "eos_id", "pad_id"):
            setattr(c, n, int(getattr(cfg, n)))
        c.ln_eps = float(cfg.ln_eps)
        c.emb_scale = float(cfg.emb_scale)
        c.kv_fp8 = int(getattr(cfg, "kv_fp8", 0))
        c.norm_type = int(getattr(cfg, "norm_type", 0))
        self.c_cfg = c
        layers = (_Layer * cfg.n_layers)()
        for i, lw in enumerate(weights["layers"]):
            for n in _LAYER_FIELDS:
                setattr(layers[i], n, self._ptr(lw.get(n)))
        self._layers = layers
        w = _Weights()
        for n in _TOP_FIELDS:
            setattr(w, n, self._ptr(weights.get(n)))
        w.layers = C.cast(layers, C.POINTER(_Layer))
        self.c_w = w

    def _ptr(self, a):
        if a is None:
            return C.cast(None, _f32p)
        a = _f32(a)
        self._keep.append(a)
        return a.ctypes.data_as(_f32p)

    # -- batch routines --------------------------------------------------
    def decode_forced(self, enc, enc_lens, tokens) -> np.ndarray:
        enc, enc_lens, tokens = _f32(enc), _i32(enc_lens), _i32(tokens)
        B, S = tokens.shape
        out = np.zeros((B, S, self.cfg.vocab), dtype=np.float64)
        rc = lib().aedo_decode_forced(C.byref(self.c_cfg), C.byref(self.c_w), _p32(enc),
                                      _pi(enc_lens), B, _pi(tokens), S, _p64(out))
        if rc != 0:
            raise ValueError(f"aedo_decode_forced: bad argument ({rc})")
        return out

    def greedy_decode(self, enc, enc_lens, prompt, max_new, max_new_per_seq=None,
                      want_logits: bool = False):
        enc, enc_lens, prompt = _f32(enc), _i32(enc_lens), _i32(prompt)
        B, P = prompt.shape
        mn = None if max_new_per_seq is None else _i32(max_new_per_seq)
        toks = np.zeros((B, max_new), dtype=np.int32)
        lens = np.zeros(B, dtype=np.int32)
        logits = np.zeros((B, max_new, self.cfg.vocab), dtype=np.float64) if want_logits else None
        rc = lib().aedo_greedy_decode(C.byref(self.c_cfg), C.byref(self.c_w), _p32(enc),
                                      _pi(enc_lens), B, _pi(prompt), P, int(max_new), _pi(mn),
                                      _pi(toks), _pi(lens), _p64(logits))
        if rc != 0:
            raise ValueError(f"aedo_greedy_decode: bad argument ({rc})")
        return (toks, lens, logits) if want_logits else (toks, lens)

    def forward_full(self, enc_padded, enc_lens, tokens, tok_lens) -> np.ndarray:
        enc_padded, enc_lens = _f32(enc_padded), _i32(enc_lens)
        tokens, tok_lens = _i32(tokens), _i32(tok_lens)
        B, T_max, _ = enc_padded.shape
        S_max = tokens.shape[1]
        out = np.zeros((B, S_max, self.cfg.vocab), dtype=np.float64)
        rc = lib().aedo_forward_full(C.byref(self.c_cfg), C.byref(self.c_w), _p32(enc_padded),
                                     T_max, _pi(enc_lens), B, _pi(tokens), S_max, _pi(tok_lens),
                                     _p64(out))
        if rc != 0:
            raise ValueError(f"aedo_forward_full: bad argument ({rc})")
        return out

    def cross_kv(self, layer: int, enc):
        enc = _f32(enc)
        T, d = enc.shape
        K = np.zeros((T, d), dtype=np.float64)
        V = np.zeros((T, d), dtype=np.float64)
        rc = lib().aedo_cross_kv(C.byref(self.c_cfg), C.byref(self.c_w), int(layer), _p32(enc), T,
                                 _p64(K), _p64(V))
        if rc != 0:
            raise ValueError(f"aedo_cross_kv: bad argument ({rc})")
        return K, V

    def self_kv(self, layer: int, enc, tokens):
        """Self-attention keys and values [S, d] of `layer` after one sequence was fed tokens [S]."""
        enc, tokens = _f32(enc), _i32(tokens)
        S, d = tokens.shape[0], self.cfg.d_model
        K = np.zeros((S, d), dtype=np.float64)
        V = np.zeros((S, d), dtype=np.float64)
        rc = lib().aedo_self_kv(C.byref(self.c_cfg), C.byref(self.c_w), _p32(enc), enc.shape[0], _pi(tokens), S,
                                int(layer), _p64(K), _p64(V))
        if rc != 0:
            raise ValueError(f"aedo_self_kv: bad argument ({rc})")
        return K, V

    def layer_matrix_params(self) -> int:
        return int(lib().aedo_layer_matrix_params(C.byref(self.c_cfg)))


# -- primitives -----------------------------------------------------------
def layernorm(z, g, b, eps):
    z, g, b = _f64(z), _f32(g), _f32(b)
    y = np.zeros_like(z)
    lib().aedo_layernorm(_p64(z), _p32(g), _p32(b), z.size, float(eps), _p64(y))
    return y


def rmsnorm(z, g, b, eps):
    z, g = _f64(z), _f32(g)
    b = None if b is None else _f32(b)
    y = np.zeros_like(z)
    lib().aedo_rmsnorm(_p64(z), _p32(g), _p32(b), z.size, float(eps), _p64(y))
    return y


def linear(x, W, bias=None):
    x, W = _f64(x), _f32(W)
    bias = None if bias is None else _f32(bias)
    n_out, n_in = W.shape
    y = np.zeros(n_out, dtype=np.float64)
    lib().aedo_linear(_p64(x), _p32(W), _p32(bias), n_in, n_out, _p64(y))
    return y


def softmax(a):
    a = _f64(a)
    p = np.zeros_like(a)
    lib().aedo_softmax(_p64(a), a.size, _p64(p))
    return p


def attend(q, K, V, want_probs: bool = False):
    """q [dh]; K, V [n, dh] (contiguous)."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    n, dh = K.shape
    out = np.zeros(dh, dtype=np.float64)
    probs = np.zeros(n, dtype=np.float64) if want_probs else None
    lib().aedo_attend(_p64(q), _p64(K), _p64(V), n, dh, dh, _p64(out), _p64(probs))
    return (out, probs) if want_probs else out


def argmax(a) -> int:
    a = _f64(a)
    return int(lib().aedo_argmax(_p64(a), a.size))


def fp8_e4m3_encode(x) -> np.ndarray:
    """E4M3 codes (uint8) of an array of float32 values."""
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().aedo_fp8_e4m3_encode_array(_p32(x), x.size, out.ctypes.data_as(C.POINTER(C.c_uint8)))
    return out


def fp8_e4m3_decode(codes) -> np.ndarray:
    """Values (float64) of an array of E4M3 codes."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    f = lib().aedo_fp8_e4m3_decode
    return np.array([f(int(c)) for c in codes.ravel()], dtype=np.float64).reshape(codes.shape)


def num_threads() -> int:
    return int(lib().aedo_num_threads())
