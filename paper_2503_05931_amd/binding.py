"""ctypes binding of libaed.so (the C ABI declared in include/aed.h).

Argument marshalling only: every step of the decoder runs in the library's
HIP kernels.  PyTorch is used for device memory and streams.  There is no CPU
fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

from . import workloads as _wl

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaed.so")

AED_OK, AED_EINVAL, AED_ECAPACITY, AED_ESTATE, AED_EHIP, AED_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
STATUS_NAMES = {0: "AED_OK", -1: "AED_EINVAL", -2: "AED_ECAPACITY", -3: "AED_ESTATE", -4: "AED_EHIP",
                -5: "AED_EUNSUPPORTED"}
(K_LN_QKV, K_SELF_ATTN, K_SELF_OUT, K_LN_CROSSQ, K_CROSS_ATTN, K_CROSS_OUT, K_LN_FFN1, K_FFN2, K_LN_VOCAB,
 K_SAMPLE, K_EMBED, K_CROSS_KV, K_COUNT) = range(13)
KERNEL_NAMES = ["ln_qkv", "self_attn", "self_out", "ln_crossq", "cross_attn", "cross_out", "ln_ffn1", "ffn2",
                "ln_vocab", "sample", "embed", "cross_kv"]

EXPORTS = ("aed_workspace_bytes", "aed_decoder_create", "aed_decoder_destroy", "aed_cross_kv_precompute",
           "aed_cross_kv_precompute_padded", "aed_decode_step", "aed_decode_step_noalloc", "aed_greedy_decode", "aed_greedy_decode_queue",
           "aed_last_error",
           "aed_layer_matrix_params", "aed_read_cross_kv", "aed_read_self_kv", "aed_read_logits", "aed_time_kernels",
           "aed_kernel_work")


class AedConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "max_positions", "dtype", "norm_type",
        "page_size", "max_batch", "max_total_enc_frames", "max_dec_len", "kv_pages", "eos_id", "pad_id")] + [
        ("ln_eps", C.c_float), ("emb_scale", C.c_float), ("prefill_rows", C.c_int32),
        ("kv_fp8", C.c_int32)]


class AedLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _wl.LAYER_FIELDS]


class AedWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _wl.TOP_FIELDS] + [("layers", C.POINTER(AedLayerWeights))]


class AedError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load():
    """Load libaed.so (built in-tree by paper_2503_05931_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_05931_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    lib.aed_workspace_bytes.argtypes = [C.POINTER(AedConfig), C.POINTER(C.c_size_t)]
    lib.aed_decoder_create.argtypes = [C.POINTER(AedConfig), C.POINTER(AedWeights), vp, C.c_size_t, vp, C.POINTER(vp)]
    lib.aed_decoder_destroy.argtypes = [vp]
    lib.aed_cross_kv_precompute.argtypes = [vp, vp, i32p, C.c_int32]
    lib.aed_cross_kv_precompute_padded.argtypes = [vp, vp, C.c_int32, i32p, C.c_int32]
    lib.aed_decode_step.argtypes = [vp, vp, vp, vp]
    lib.aed_decode_step_noalloc.argtypes = [vp, vp, vp, vp]
    lib.aed_greedy_decode.argtypes = [vp, vp, C.c_int32, C.c_int32, i32p, vp, vp]
    lib.aed_greedy_decode_queue.argtypes = [vp, vp, i32p, C.c_int32, vp, C.c_int32, C.c_int32, i32p, vp, vp, i32p]
    lib.aed_last_error.argtypes = [vp]
    lib.aed_last_error.restype = C.c_char_p
    lib.aed_layer_matrix_params.argtypes = [C.POINTER(AedConfig)]
    lib.aed_layer_matrix_params.restype = C.c_int64
    lib.aed_read_cross_kv.argtypes = [vp, C.c_int32, C.c_int32, f32p, f32p]
    lib.aed_read_self_kv.argtypes = [vp, C.c_int32, C.c_int32, f32p, f32p, i32p]
    lib.aed_read_logits.argtypes = [vp, f32p]
    lib.aed_time_kernels.argtypes = [vp, C.c_int32, C.c_int32, f32p, i32p]
    lib.aed_kernel_work.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    for n in EXPORTS:
        if n not in ("aed_last_error", "aed_layer_matrix_params"):
            getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def make_config(cfg, max_batch: int, max_total_enc_frames: int, max_dec_len: int, kv_pages: int = 0,
                prefill_rows: int = 0) -> AedConfig:
    c = AedConfig()
    c.struct_size = C.sizeof(AedConfig)
    for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "max_positions", "norm_type",
              "page_size", "eos_id", "pad_id"):
        setattr(c, n, int(getattr(cfg, n)))
    c.dtype = 1 if cfg.dtype == "bf16" else 0
    c.max_batch, c.max_total_enc_frames, c.max_dec_len, c.kv_pages = (int(max_batch), int(max_total_enc_frames),
                                                                      int(max_dec_len), int(kv_pages))
    c.ln_eps, c.emb_scale = float(cfg.ln_eps), float(cfg.emb_scale)
    c.prefill_rows = int(prefill_rows)
    c.kv_fp8 = int(getattr(cfg, "kv_fp8", 0))
    return c


# ---- the C entry points under their own names (raw pointers / ctypes objects) ----
def aed_workspace_bytes(c: AedConfig) -> int:
    n = C.c_size_t(0)
    st = load().aed_workspace_bytes(C.byref(c), C.byref(n))
    if st != AED_OK:
        raise AedError(st, load().aed_last_error(None).decode())
    return int(n.value)


def aed_layer_matrix_params(c: AedConfig) -> int:
    return int(load().aed_layer_matrix_params(C.byref(c)))


def _i32_host(a, n=None):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


class Decoder:
    """A decoder handle plus the torch tensors that back it (weights on the
    device, workspace).  Methods carry the C entry points' names."""

    def __init__(self, cfg, weights: Dict, max_batch: int, max_total_enc_frames: int, max_dec_len: int,
                 device: str = "cuda:0", stream=None, kv_pages: int = 0, workspace_fill: Optional[int] = None,
                 prefill_rows: int = 0):
        """workspace_fill: byte value written over the whole workspace before the decoder is
        created (0xFF makes every untouched bf16/fp32 slot read as NaN), for leak checks."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.lib = load()
        self.c_cfg = make_config(cfg, max_batch, max_total_enc_frames, max_dec_len, kv_pages, prefill_rows)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        self._keep = []
        self.handle = C.c_void_p(None)
        nbytes = aed_workspace_bytes(self.c_cfg)
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            if workspace_fill is not None:
                self.workspace.fill_(int(workspace_fill))
            layers = (AedLayerWeights * cfg.n_layers)()
            for i, lw in enumerate(weights["layers"]):
                for n in _wl.LAYER_FIELDS:
                    setattr(layers[i], n, self._dev(lw.get(n)))
            w = AedWeights()
            for n in _wl.TOP_FIELDS:
                setattr(w, n, self._dev(weights.get(n)))
            w.layers = C.cast(layers, C.POINTER(AedLayerWeights))
            torch.cuda.synchronize(self.device)
            st = self.lib.aed_decoder_create(C.byref(self.c_cfg), C.byref(w), C.c_void_p(self.workspace.data_ptr()),
                                             nbytes, C.c_void_p(self.stream.cuda_stream), C.byref(self.handle))
        if st != AED_OK:
            raise AedError(st, self.lib.aed_last_error(None).decode())
        self.batch = 0

    def _dev(self, a):
        if a is None:
            return None
        t = self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(self.tdtype).contiguous()
        self._keep.append(t)
        return t.data_ptr()

    def _check(self, st):
        if st != AED_OK:
            raise AedError(st, self.lib.aed_last_error(self.handle).decode())

    def to_device(self, a):
        """float32 numpy -> device tensor of the decoder's storage type."""
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(self.tdtype).contiguous()

    def close(self):
        if self.handle:
            self.lib.aed_decoder_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _enter(self):
        # inputs were produced on torch's current stream; the library works on self.stream
        self.stream.wait_stream(self.torch.cuda.current_stream(self.device))

    def _exit(self):
        self.torch.cuda.current_stream(self.device).wait_stream(self.stream)

    # ---- entry points ----
    def aed_cross_kv_precompute(self, enc_states, enc_lens: Sequence[int]):
        """enc_states: device tensor [sum(enc_lens), d] of the storage type."""
        lens, p = _i32_host(enc_lens)
        self._enc_keep = enc_states
        self._enter()
        self._check(self.lib.aed_cross_kv_precompute(self.handle, C.c_void_p(enc_states.data_ptr()), p, len(lens)))
        self._exit()
        self.batch = len(lens)

    def aed_cross_kv_precompute_padded(self, enc_padded, enc_lens: Sequence[int]):
        lens, p = _i32_host(enc_lens)
        self._enc_keep = enc_padded
        self._enter()
        self._check(self.lib.aed_cross_kv_precompute_padded(self.handle, C.c_void_p(enc_padded.data_ptr()),
                                                            int(enc_padded.shape[1]), p, len(lens)))
        self._exit()
        self.batch = len(lens)

    def aed_decode_step(self, tokens_in, want_logits: bool = True):
        """tokens_in: device int32 [batch].  Returns (tokens_out, logits or None), device tensors."""
        torch = self.torch
        out = torch.empty(self.batch, dtype=torch.int32, device=self.device)
        logits = torch.empty((self.batch, self.cfg.vocab), dtype=torch.float32, device=self.device) if want_logits else None
        self._enter()
        self._check(self.lib.aed_decode_step(self.handle, C.c_void_p(tokens_in.data_ptr()), C.c_void_p(out.data_ptr()),
                                             C.c_void_p(logits.data_ptr()) if want_logits else None))
        self._exit()
        return out, logits

    def aed_decode_step_noalloc(self, tokens_in, tokens_out, logits_out=None):
        """The step with caller-provided output tensors (device int32 [batch], float32 [batch, vocab] or None);
        nothing is allocated on the way."""
        self._check(self.lib.aed_decode_step_noalloc(
            self.handle, C.c_void_p(tokens_in.data_ptr()), C.c_void_p(tokens_out.data_ptr()),
            C.c_void_p(logits_out.data_ptr()) if logits_out is not None else None))

    def aed_greedy_decode(self, prompt, max_new: int, max_new_per_seq=None, out_tokens=None, out_lens=None):
        """prompt: device int32 [batch, P].  Returns (tokens [batch, max_new], lens [batch]), device tensors."""
        torch = self.torch
        B, P = prompt.shape
        if out_tokens is None:
            out_tokens = torch.empty((B, max_new), dtype=torch.int32, device=self.device)
        if out_lens is None:
            out_lens = torch.empty(B, dtype=torch.int32, device=self.device)
        mn, pmn = _i32_host(max_new_per_seq)
        self._enter()
        self._check(self.lib.aed_greedy_decode(self.handle, C.c_void_p(prompt.data_ptr()), int(P), int(max_new), pmn,
                                               C.c_void_p(out_tokens.data_ptr()), C.c_void_p(out_lens.data_ptr())))
        self._exit()
        return out_tokens, out_lens

    def aed_greedy_decode_queue(self, enc_states, enc_lens, prompts, max_new: int, max_new_per_req=None):
        """All requests at once: enc_states device [sum(enc_lens), d], prompts device int32 [n, P].
        Returns (tokens [n, max_new], lens [n], decoder steps run)."""
        torch = self.torch
        n, P = prompts.shape
        out_tokens = torch.empty((n, max_new), dtype=torch.int32, device=self.device)
        out_lens = torch.empty(n, dtype=torch.int32, device=self.device)
        lens, plens = _i32_host(enc_lens)
        mn, pmn = _i32_host(max_new_per_req)
        steps = C.c_int32(0)
        self._enter()
        self._check(self.lib.aed_greedy_decode_queue(
            self.handle, C.c_void_p(enc_states.data_ptr()), plens, int(n), C.c_void_p(prompts.data_ptr()), int(P),
            int(max_new), pmn, C.c_void_p(out_tokens.data_ptr()), C.c_void_p(out_lens.data_ptr()), C.byref(steps)))
        self._exit()
        return out_tokens, out_lens, int(steps.value)

    def aed_read_cross_kv(self, layer: int, seq: int, enc_len: int):
        d = self.cfg.d_model
        k = np.zeros((enc_len, d), np.float32)
        v = np.zeros((enc_len, d), np.float32)
        fp = C.POINTER(C.c_float)
        self._check(self.lib.aed_read_cross_kv(self.handle, layer, seq, k.ctypes.data_as(fp), v.ctypes.data_as(fp)))
        return k, v

    def aed_read_self_kv(self, layer: int, seq: int):
        d, cap = self.cfg.d_model, int(self.c_cfg.max_dec_len)
        k = np.zeros((cap, d), np.float32)
        v = np.zeros((cap, d), np.float32)
        n = C.c_int32(0)
        fp = C.POINTER(C.c_float)
        self._check(self.lib.aed_read_self_kv(self.handle, layer, seq, k.ctypes.data_as(fp), v.ctypes.data_as(fp),
                                              C.byref(n)))
        return k[:n.value], v[:n.value]

    def aed_read_logits(self):
        """Logits [batch, vocab] of the most recent decoder step (host float32)."""
        out = np.zeros((self.batch, self.cfg.vocab), np.float32)
        self._check(self.lib.aed_read_logits(self.handle, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def aed_time_kernels(self, kernel_class: int, reps: int):
        ms, n = C.c_float(0), C.c_int32(0)
        self._check(self.lib.aed_time_kernels(self.handle, kernel_class, reps, C.byref(ms), C.byref(n)))
        return float(ms.value), int(n.value)

    def aed_kernel_work(self, kernel_class: int):
        b, f = C.c_double(0), C.c_double(0)
        self._check(self.lib.aed_kernel_work(self.handle, kernel_class, C.byref(b), C.byref(f)))
        return float(b.value), float(f.value)
