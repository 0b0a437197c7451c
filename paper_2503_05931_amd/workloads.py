"""Seeded synthetic inputs for the autoregressive AED decoder path.

This module only *draws inputs* (lengths, weights, encoder states, prompts) and
rounds them to the storage type a configuration asks for.  It holds none of
the decoder's arithmetic and is the one module that both the CPU oracle's
tests and the HIP path's tests/benchmarks use, so both sides always see the
same bytes.

Shapes follow the paper's workload: utterances of at most 40 s (its bucket
range, Sec. "Experimental setup"), two ragged axes (encoder frames and
output tokens, Fig. 1), a fixed-length decoder prompt (Fig. 3 caption), and a
24-layer versus 4-layer decoder (Sec. "Transferring model capacity from
decoder to encoder").  The public evaluation sets the paper measured on are
not used; these tensors stand in for them.

Draw order (numpy PCG64, one generator per workload): lengths -> weights in
struct order, layer-major -> encoder states -> prompts.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

LAYER_FIELDS = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_cq", "b_cq", "w_ckv", "b_ckv", "w_co", "b_co",
    "ln3_g", "ln3_b", "w_ff1", "b_ff1", "w_ff2", "b_ff2",
)
TOP_FIELDS = ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "w_out", "b_out")

FRAMES_PER_SECOND = 12.5


# --------------------------------------------------------------------------
# storage rounding (input quantisation; not part of the decoder's arithmetic)
# --------------------------------------------------------------------------
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bfloat16, returned as float32."""
    return bf16_from_bits(bf16_bits(a)).reshape(np.shape(a))


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass
class DecoderConfig:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "fp32" | "bf16": storage of weights, encoder states and KV
    batch: int
    prompt_len: int = 4
    max_new: int = 128
    eos_id: int = -1
    pad_id: int = 0
    ln_eps: float = 1e-5
    emb_scale: float = 1.0
    page_size: int = 16
    norm_type: int = 0
    max_positions: int = 0
    kv_fp8: int = 0  # 1: attention keys and values are stored as 8-bit E4M3 codes (bf16 models only)

    def __post_init__(self):
        if self.max_positions <= 0:
            need = self.prompt_len + self.max_new
            self.max_positions = ((need + 15) // 16) * 16

    @property
    def max_dec_len(self) -> int:
        return self.prompt_len + self.max_new


def config(name: str, **over) -> DecoderConfig:
    """Named configurations: tiny fp32 case, 24-layer and 4-layer decoders,
    the ragged-vs-bucketed stress and the large-batch case."""
    base = dict(d_model=1024, n_heads=8, head_dim=128, d_ffn=4096, vocab=4096,
                dtype="bf16")
    table = {
        "tiny": dict(n_layers=2, d_model=256, n_heads=4, head_dim=64,
                     d_ffn=1024, vocab=512, dtype="fp32", batch=4, max_new=32),
        "canary24_b64": dict(base, n_layers=24, batch=64, max_new=128),
        "flash4_b256": dict(base, n_layers=4, batch=256, max_new=128),
        "ragged24_b128": dict(base, n_layers=24, batch=128, max_new=256,
                              eos_id=2),
        "large24_b1024": dict(base, n_layers=24, batch=1024, max_new=448),
    }
    if name not in table:
        raise KeyError(f"unknown workload {name!r}; have {sorted(table)}")
    kw = dict(table[name])
    kw.update(over)
    return DecoderConfig(name=name, **kw)


# --------------------------------------------------------------------------
# draws
# --------------------------------------------------------------------------
def draw_weights(cfg: DecoderConfig, rng: np.random.Generator,
                 random_ln: bool = False, std: float = 0.02) -> Dict:
    """All decoder weights as float32, N(0, std); LayerNorm gain 1 / shift 0
    unless random_ln.  Values are rounded to bf16 when cfg.dtype == 'bf16'
    (still returned as float32 arrays holding bf16-representable numbers)."""
    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab

    def normal(*shape):
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(std)
        return bf16_round(a) if cfg.dtype == "bf16" else a

    def gain():
        if random_ln:
            a = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32)
            return bf16_round(a) if cfg.dtype == "bf16" else a
        return np.ones(d, dtype=np.float32)

    def shift():
        if random_ln:
            a = (0.1 * rng.standard_normal(d)).astype(np.float32)
            return bf16_round(a) if cfg.dtype == "bf16" else a
        return np.zeros(d, dtype=np.float32)

    w: Dict = {}
    w["tok_emb"] = normal(V, d)
    w["pos_emb"] = normal(cfg.max_positions, d)
    w["lnf_g"] = gain()
    w["lnf_b"] = shift()
    w["w_out"] = normal(V, d)
    w["b_out"] = normal(V)
    layers: List[Dict] = []
    for _ in range(cfg.n_layers):
        l: Dict = {}
        l["ln1_g"], l["ln1_b"] = gain(), shift()
        l["w_qkv"], l["b_qkv"] = normal(3 * d, d), normal(3 * d)
        l["w_o"], l["b_o"] = normal(d, d), normal(d)
        l["ln2_g"], l["ln2_b"] = gain(), shift()
        l["w_cq"], l["b_cq"] = normal(d, d), normal(d)
        l["w_ckv"], l["b_ckv"] = normal(2 * d, d), normal(2 * d)
        l["w_co"], l["b_co"] = normal(d, d), normal(d)
        l["ln3_g"], l["ln3_b"] = gain(), shift()
        l["w_ff1"], l["b_ff1"] = normal(F, d), normal(F)
        l["w_ff2"], l["b_ff2"] = normal(d, F), normal(d)
        layers.append(l)
    w["layers"] = layers
    return w


def draw_durations_lognormal(rng, n, median_s=8.0, sigma=0.7, lo=1.0, hi=40.0):
    dur = np.exp(math.log(median_s) + sigma * rng.standard_normal(n))
    return np.clip(dur, lo, hi)


def frames_from_duration(dur) -> np.ndarray:
    return np.floor(FRAMES_PER_SECOND * np.asarray(dur)).astype(np.int32)


def draw_enc_states(cfg: DecoderConfig, rng, enc_lens) -> np.ndarray:
    """Packed encoder states [sum(enc_lens), d_model], N(0,1), no padding."""
    total = int(np.sum(enc_lens))
    a = rng.standard_normal((total, cfg.d_model), dtype=np.float32)
    return bf16_round(a) if cfg.dtype == "bf16" else a


def draw_prompts(cfg: DecoderConfig, rng, batch=None) -> np.ndarray:
    b = cfg.batch if batch is None else batch
    return rng.integers(3, cfg.vocab, size=(b, cfg.prompt_len)).astype(np.int32)


@dataclass
class Workload:
    cfg: DecoderConfig
    weights: Dict
    enc_lens: np.ndarray          # int32 [B]
    enc: np.ndarray               # float32 [sum(enc_lens), d]
    prompt: np.ndarray            # int32 [B, P]
    max_new_per_seq: Optional[np.ndarray] = None   # int32 [B] or None
    durations_s: Optional[np.ndarray] = None
    extra: Dict = field(default_factory=dict)

    @property
    def enc_offsets(self) -> np.ndarray:
        off = np.zeros(len(self.enc_lens) + 1, dtype=np.int64)
        np.cumsum(self.enc_lens, out=off[1:])
        return off

    def subset(self, idx) -> "Workload":
        """The same workload restricted to sequences idx (sequences are
        independent, so results for a subset equal the rows of the full run)."""
        idx = np.asarray(idx, dtype=np.int64)
        off = self.enc_offsets
        enc = np.concatenate([self.enc[off[i]:off[i + 1]] for i in idx], axis=0)
        mn = None if self.max_new_per_seq is None else self.max_new_per_seq[idx].copy()
        return Workload(self.cfg, self.weights, self.enc_lens[idx].copy(), enc,
                        self.prompt[idx].copy(), mn,
                        None if self.durations_s is None else self.durations_s[idx].copy())


_SEEDS = {"tiny": 0, "canary24_b64": 1, "flash4_b256": 2, "ragged24_b128": 3,
          "large24_b1024": 4}


def make(name: str, seed: Optional[int] = None, random_ln: bool = False,
         with_enc: bool = True, **over) -> Workload:
    """Build the named workload.  with_enc=False skips drawing encoder states
    (the large-batch case holds 2 GB of them) and leaves enc empty."""
    cfg = config(name, **over)
    rng = np.random.default_rng(_SEEDS[name] if seed is None else seed)
    B = cfg.batch
    dur = None
    mnps = None
    extra: Dict = {}
    if name == "tiny":
        enc_lens = rng.integers(20, 101, size=B).astype(np.int32)
    elif name in ("canary24_b64", "flash4_b256"):
        dur = draw_durations_lognormal(rng, B)
        enc_lens = frames_from_duration(dur)
    elif name == "ragged24_b128":
        pool_enc = rng.integers(12, 501, size=2048).astype(np.int32)
        pool_dec = rng.integers(8, 257, size=2048).astype(np.int32)
        perm = rng.permutation(2048)
        extra["pool_enc"], extra["pool_dec"], extra["perm"] = pool_enc, pool_dec, perm
        first = perm[:B]
        enc_lens = pool_enc[first].copy()
        mnps = pool_dec[first].copy()
        dur = enc_lens / FRAMES_PER_SECOND
    elif name == "large24_b1024":
        enc_lens = np.full(B, 500, dtype=np.int32)
        dur = enc_lens / FRAMES_PER_SECOND
    else:  # pragma: no cover
        raise KeyError(name)
    weights = draw_weights(cfg, rng, random_ln=random_ln)
    if with_enc:
        enc = draw_enc_states(cfg, rng, enc_lens)
    else:
        enc = np.zeros((0, cfg.d_model), dtype=np.float32)
    prompt = draw_prompts(cfg, rng)
    return Workload(cfg, weights, enc_lens, enc, prompt, mnps, dur, extra)


def custom(cfg: DecoderConfig, enc_lens, seed: int, random_ln: bool = True,
           max_new_per_seq=None) -> Workload:
    """A free-form workload for unit tests: any dims, explicit lengths."""
    rng = np.random.default_rng(seed)
    enc_lens = np.asarray(enc_lens, dtype=np.int32)
    cfg.batch = len(enc_lens)
    weights = draw_weights(cfg, rng, random_ln=random_ln)
    enc = draw_enc_states(cfg, rng, enc_lens)
    prompt = draw_prompts(cfg, rng)
    mn = None if max_new_per_seq is None else np.asarray(max_new_per_seq, dtype=np.int32)
    return Workload(cfg, weights, enc_lens, enc, prompt, mn)


# --------------------------------------------------------------------------
# batch forming for the ragged-vs-bucketed stress
# --------------------------------------------------------------------------
def random_batches(pool_enc, pool_dec, perm, batch):
    """Case (a): the pool in random order, cut into consecutive batches."""
    n = (len(perm) // batch) * batch
    return [perm[i:i + batch] for i in range(0, n, batch)]


def bucketed_2d_batches(pool_enc, pool_dec, batch, n_enc_bins=8):
    """Case (b): sort by encoder length into equal-count bins, split each bin
    at its output-length median (a small n_enc_bins x 2 version of the paper's
    30 x 2 strict 2D bucketing, Sec. "Experimental setup")."""
    order = np.argsort(pool_enc, kind="stable")
    bins = np.array_split(order, n_enc_bins)
    cells = []
    for b in bins:
        sub = b[np.argsort(pool_dec[b], kind="stable")]
        half = len(sub) // 2
        cells += [sub[:half], sub[half:]]
    out = []
    for c in cells:
        n = (len(c) // batch) * batch
        out += [c[i:i + batch] for i in range(0, n, batch)]
    return out


def padding_fraction(lens_per_batch) -> float:
    """1 - sum(len) / sum_over_batches(B * max len): the share of a padded
    tensor axis that is padding (the quantity of the paper's Fig. 5 text)."""
    real = sum(int(np.sum(l)) for l in lens_per_batch)
    padded = sum(len(l) * int(np.max(l)) for l in lens_per_batch)
    return 1.0 - real / padded
