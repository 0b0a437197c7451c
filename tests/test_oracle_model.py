"""Pins for the oracle's decoder routines (CPU only).

The paper prints no numeric example of the decoder, so these pins are what the
definition fixes: incremental == whole-sequence causal forward, padded+masked
== unpadded (Sec. 1 of the paper: padding masks make padding contribute
nothing), agreement with torch.nn.TransformerDecoder(norm_first=True) on CPU
in float64, closed forms, symmetries, and the paper's parameter count.
"""
import json
import os

import numpy as np
import pytest
import torch

from paper_2503_05931_amd import workloads as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def small_cfg(**over):
    kw = dict(name="unit", n_layers=2, d_model=32, n_heads=4, head_dim=8, d_ffn=48, vocab=50,
              dtype="fp32", batch=3, prompt_len=3, max_new=6, emb_scale=1.0)
    kw.update(over)
    return W.DecoderConfig(**kw)


def small_workload(seed=0, enc_lens=(5, 9, 2), **over):
    cfg = small_cfg(**over)
    wl = W.custom(cfg, enc_lens, seed, random_ln=True)
    # larger weights than N(0, 0.02) so that attention is far from uniform
    rng = np.random.default_rng(seed + 1000)
    for l in wl.weights["layers"]:
        for k in l:
            if k.startswith("w_") or k.startswith("b_"):
                l[k] = (rng.standard_normal(l[k].shape) * 0.3).astype(np.float32)
    for k in ("tok_emb", "pos_emb", "w_out", "b_out"):
        wl.weights[k] = (rng.standard_normal(wl.weights[k].shape) * 0.5).astype(np.float32)
    return wl


def pad_enc(wl, T_max=None, fill=0.0):
    B, d = len(wl.enc_lens), wl.cfg.d_model
    T_max = int(wl.enc_lens.max()) if T_max is None else T_max
    out = np.full((B, T_max, d), fill, dtype=np.float32)
    off = wl.enc_offsets
    for b in range(B):
        out[b, :wl.enc_lens[b]] = wl.enc[off[b]:off[b + 1]]
    return out


def random_tokens(cfg, B, S, seed):
    return np.random.default_rng(seed).integers(0, cfg.vocab, size=(B, S)).astype(np.int32)


# ---- P1: incremental KV-cache decoding == whole-sequence causal forward ----
def test_incremental_equals_full_forward(oracle):
    wl = small_workload(seed=1)
    m = oracle.Model(wl.cfg, wl.weights)
    S = 7
    toks = random_tokens(wl.cfg, 3, S, 11)
    inc = m.decode_forced(wl.enc, wl.enc_lens, toks)
    full = m.forward_full(pad_enc(wl), wl.enc_lens, toks, np.full(3, S, np.int32))
    assert np.abs(inc - full).max() < 1e-10


# ---- P2: padded + masked == unpadded; poisoned padding changes nothing ----
def test_padding_with_masks_contributes_nothing(oracle):
    wl = small_workload(seed=2, enc_lens=(4, 11, 1))
    m = oracle.Model(wl.cfg, wl.weights)
    S_max = 6
    tok_lens = np.array([6, 3, 5], np.int32)
    toks = random_tokens(wl.cfg, 3, S_max, 12)
    ref = m.forward_full(pad_enc(wl), wl.enc_lens, toks, tok_lens)
    # more padding on both axes, filled with NaN / huge values / garbage ids
    toks_p = np.concatenate([toks, np.full((3, 3), 10 ** 6, np.int32)], axis=1)
    for b in range(3):
        toks_p[b, tok_lens[b]:] = -7
    poisoned = m.forward_full(pad_enc(wl, T_max=17, fill=np.nan), wl.enc_lens, toks_p, tok_lens)
    huge = m.forward_full(pad_enc(wl, T_max=13, fill=1e30), wl.enc_lens, toks_p, tok_lens)
    for b in range(3):
        n = tok_lens[b]
        assert np.isfinite(poisoned[b, :n]).all()
        assert np.abs(poisoned[b, :n] - ref[b, :n]).max() < 1e-10
        assert np.abs(huge[b, :n] - ref[b, :n]).max() < 1e-10
        # and equals the unpadded per-sequence incremental result
        one = wl.subset([b])
        inc = m.decode_forced(one.enc, one.enc_lens, toks[b:b + 1, :n])
        assert np.abs(inc[0] - ref[b, :n]).max() < 1e-10


# ---- P5: the same weights in torch.nn.TransformerDecoder (CPU, float64) ----
def _torch_decoder(cfg, w):
    d, H, F = cfg.d_model, cfg.n_heads, cfg.d_ffn
    layer = torch.nn.TransformerDecoderLayer(d, H, dim_feedforward=F, dropout=0.0, activation="relu",
                                             layer_norm_eps=cfg.ln_eps, batch_first=True, norm_first=True)
    dec = torch.nn.TransformerDecoder(layer, cfg.n_layers, norm=torch.nn.LayerNorm(d, eps=cfg.ln_eps)).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        for l, lw in zip(dec.layers, w["layers"]):
            l.self_attn.in_proj_weight.copy_(t(lw["w_qkv"])); l.self_attn.in_proj_bias.copy_(t(lw["b_qkv"]))
            l.self_attn.out_proj.weight.copy_(t(lw["w_o"])); l.self_attn.out_proj.bias.copy_(t(lw["b_o"]))
            l.multihead_attn.in_proj_weight.copy_(t(np.concatenate([lw["w_cq"], lw["w_ckv"]], 0)))
            l.multihead_attn.in_proj_bias.copy_(t(np.concatenate([lw["b_cq"], lw["b_ckv"]], 0)))
            l.multihead_attn.out_proj.weight.copy_(t(lw["w_co"])); l.multihead_attn.out_proj.bias.copy_(t(lw["b_co"]))
            l.linear1.weight.copy_(t(lw["w_ff1"])); l.linear1.bias.copy_(t(lw["b_ff1"]))
            l.linear2.weight.copy_(t(lw["w_ff2"])); l.linear2.bias.copy_(t(lw["b_ff2"]))
            for n_t, n_m in (("norm1", "ln1"), ("norm2", "ln2"), ("norm3", "ln3")):
                getattr(l, n_t).weight.copy_(t(lw[n_m + "_g"])); getattr(l, n_t).bias.copy_(t(lw[n_m + "_b"]))
        dec.norm.weight.copy_(t(w["lnf_g"])); dec.norm.bias.copy_(t(w["lnf_b"]))
    return dec


@pytest.mark.parametrize("emb_scale", [1.0, 2.5])
def test_matches_torch_transformer_decoder(oracle, emb_scale):
    wl = small_workload(seed=3, enc_lens=(6, 3, 10, 1), emb_scale=emb_scale)
    cfg, w = wl.cfg, wl.weights
    m = oracle.Model(cfg, w)
    B, S = 4, 8
    toks = random_tokens(cfg, B, S, 13)
    mine = m.decode_forced(wl.enc, wl.enc_lens, toks)

    dec = _torch_decoder(cfg, w)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x0 = emb_scale * t(w["tok_emb"])[torch.from_numpy(toks).long()] + t(w["pos_emb"])[:S][None]
    mem = t(pad_enc(wl))
    kpm = torch.arange(mem.shape[1])[None, :] >= torch.from_numpy(wl.enc_lens)[:, None]
    causal = torch.triu(torch.ones(S, S, dtype=torch.bool), diagonal=1)
    with torch.no_grad():
        hid = dec(x0, mem, tgt_mask=causal, memory_key_padding_mask=kpm)
        ref = (hid @ t(w["w_out"]).T + t(w["b_out"])).numpy()
    assert np.abs(mine - ref).max() < 1e-9


# ---- P6: structural closed forms ----
def test_zero_output_projections_reduce_to_embedding_path(oracle):
    wl = small_workload(seed=4)
    for l in wl.weights["layers"]:
        for k in ("w_o", "b_o", "w_co", "b_co", "w_ff2", "b_ff2"):
            l[k] = np.zeros_like(l[k])
    cfg, w = wl.cfg, wl.weights
    m = oracle.Model(cfg, w)
    toks = random_tokens(cfg, 3, 5, 14)
    got = m.decode_forced(wl.enc, wl.enc_lens, toks)
    for b in range(3):
        for s in range(5):
            x = cfg.emb_scale * w["tok_emb"][toks[b, s]].astype(np.float64) + w["pos_emb"][s]
            h = torch.nn.functional.layer_norm(torch.from_numpy(x), (cfg.d_model,),
                                               torch.from_numpy(w["lnf_g"]).double(),
                                               torch.from_numpy(w["lnf_b"]).double(), cfg.ln_eps).numpy()
            ref = w["w_out"].astype(np.float64) @ h + w["b_out"]
            assert np.abs(got[b, s] - ref).max() < 1e-11


def test_constant_values_make_attention_length_independent(oracle):
    # V projections with zero weight: every value row equals the bias, so the
    # attention outputs do not depend on scores or on how many keys there are.
    wl = small_workload(seed=5, enc_lens=(3, 3, 3))
    d = wl.cfg.d_model
    for l in wl.weights["layers"]:
        l["w_ckv"][d:] = 0.0
    m = oracle.Model(wl.cfg, wl.weights)
    toks = random_tokens(wl.cfg, 1, 4, 15)
    a = m.decode_forced(wl.enc[:3], [3], toks)
    b = m.decode_forced(wl.enc[:9], [9], toks)          # other frames, other length
    assert np.abs(a - b).max() < 1e-11


# ---- P7: symmetries ----
def test_encoder_frame_permutation_and_batch_independence(oracle):
    wl = small_workload(seed=6, enc_lens=(7, 4, 9))
    m = oracle.Model(wl.cfg, wl.weights)
    toks = random_tokens(wl.cfg, 3, 5, 16)
    base = m.decode_forced(wl.enc, wl.enc_lens, toks)
    # permute the frames inside each sequence: cross-attention has no positional term
    off = wl.enc_offsets
    rng = np.random.default_rng(7)
    enc_p = wl.enc.copy()
    for b in range(3):
        enc_p[off[b]:off[b + 1]] = wl.enc[off[b]:off[b + 1]][rng.permutation(wl.enc_lens[b])]
    assert np.abs(m.decode_forced(enc_p, wl.enc_lens, toks) - base).max() < 1e-10
    # permute the batch
    perm = [2, 0, 1]
    sub = wl.subset(perm)
    assert np.abs(m.decode_forced(sub.enc, sub.enc_lens, toks[perm]) - base[perm]).max() == 0.0
    # a sequence decoded alone equals the same sequence inside the batch
    for b in range(3):
        one = wl.subset([b])
        assert np.abs(m.decode_forced(one.enc, one.enc_lens, toks[b:b + 1])[0] - base[b]).max() == 0.0
    # but the self-attention IS position dependent: permuting tokens changes logits
    assert np.abs(m.decode_forced(wl.enc, wl.enc_lens, toks[:, ::-1].copy())[:, -1] - base[:, -1]).max() > 1e-3


# ---- P8: the paper's parameter count ----
def test_parameter_count_matches_paper(oracle):
    cfg = W.config("canary24_b64")
    removed_layers = GOLD["decoder_layers_before"]["value"] - GOLD["decoder_layers_after"]["value"]
    cfg.n_layers = removed_layers
    m_params = oracle.Model(cfg, {"layers": [{} for _ in range(removed_layers)]}).layer_matrix_params()
    assert m_params == 16 * 1024 * 1024 * 20
    paper_delta = (GOLD["params_before_M"]["value"] - GOLD["params_after_M"]["value"]) * 1e6
    assert abs(m_params - paper_delta) / paper_delta < 0.005   # 335.5M vs the printed 336M


# ---- P9 + greedy semantics ----
def test_greedy_is_argmax_of_forced_logits_and_deterministic(oracle):
    wl = small_workload(seed=8)
    cfg = wl.cfg
    m = oracle.Model(cfg, wl.weights)
    toks, lens, logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new, want_logits=True)
    toks2, lens2 = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new)
    assert (toks == toks2).all() and (lens == lens2).all() and (lens == cfg.max_new).all()
    # feeding prompt + emitted tokens through the teacher-forced routine reproduces the logits
    full = np.concatenate([wl.prompt, toks[:, :-1]], axis=1)
    forced = m.decode_forced(wl.enc, wl.enc_lens, full)
    P = cfg.prompt_len
    assert np.abs(forced[:, P - 1:] - logits).max() == 0.0
    assert (logits.argmax(-1) == toks).all()


def test_greedy_eos_and_forced_eos(oracle):
    wl = small_workload(seed=9)
    cfg = wl.cfg
    free_toks, _ = oracle.Model(cfg, wl.weights).greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new)
    # make the token sequence 0 emits at step 2 the EOS id
    eos = int(free_toks[0, 2])
    cfg2 = small_cfg(eos_id=eos, pad_id=49)
    m = oracle.Model(cfg2, wl.weights)
    toks, lens = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new)
    for b in range(3):
        hits = np.where(free_toks[b] == eos)[0]
        n = (hits[0] + 1) if len(hits) else cfg.max_new
        assert lens[b] == n
        assert (toks[b, :n] == free_toks[b, :n]).all()
        assert (toks[b, n:] == 49).all()
    assert lens[0] <= 3
    # forced EOS at a per-sequence count
    cfg3 = small_cfg(eos_id=48, pad_id=0)
    m3 = oracle.Model(cfg3, wl.weights)
    target = np.array([1, 4, 6], np.int32)
    toks, lens = m3.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new, max_new_per_seq=target)
    for b in range(3):
        if 48 in free_toks[b, :target[b] - 1]:
            continue
        assert lens[b] == target[b]
        assert toks[b, target[b] - 1] == 48
        assert (toks[b, :target[b] - 1] == free_toks[b, :target[b] - 1]).all()
        assert (toks[b, target[b]:] == 0).all()
    with pytest.raises(ValueError):
        oracle.Model(cfg, wl.weights).greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 4, max_new_per_seq=target)


def test_bad_arguments_are_rejected(oracle):
    wl = small_workload(seed=10)
    m = oracle.Model(wl.cfg, wl.weights)
    with pytest.raises(ValueError):
        m.decode_forced(wl.enc, [5, 0, 2], random_tokens(wl.cfg, 3, 2, 1))
    with pytest.raises(ValueError):
        m.decode_forced(wl.enc, wl.enc_lens, np.full((3, 2), wl.cfg.vocab, np.int32))
    with pytest.raises(ValueError):
        m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, wl.cfg.max_positions)


def test_cross_kv_is_the_linear_map(oracle):
    wl = small_workload(seed=11)
    m = oracle.Model(wl.cfg, wl.weights)
    d = wl.cfg.d_model
    enc = wl.enc[:5]
    K, V = m.cross_kv(1, enc)
    lw = wl.weights["layers"][1]
    ref = enc.astype(np.float64) @ lw["w_ckv"].astype(np.float64).T + lw["b_ckv"]
    assert np.abs(K - ref[:, :d]).max() < 1e-12 and np.abs(V - ref[:, d:]).max() < 1e-12


def test_self_kv_of_the_first_layer_is_the_projection_of_the_embedding(oracle):
    wl = small_workload(seed=12)
    cfg, w = wl.cfg, wl.weights
    m = oracle.Model(cfg, w)
    d = cfg.d_model
    toks = np.array([4, 9, 1, 30, 2], np.int32)
    K, V = m.self_kv(0, wl.enc[:wl.enc_lens[0]], toks)
    lw = w["layers"][0]
    for s, t in enumerate(toks):
        x = cfg.emb_scale * w["tok_emb"][t].astype(np.float64) + w["pos_emb"][s]
        mu = x.mean()
        h = (x - mu) / np.sqrt(((x - mu) ** 2).mean() + float(np.float32(cfg.ln_eps))) * lw["ln1_g"] + lw["ln1_b"]
        qkv = lw["w_qkv"].astype(np.float64) @ h + lw["b_qkv"]
        assert np.abs(K[s] - qkv[d:2 * d]).max() < 1e-12 and np.abs(V[s] - qkv[2 * d:]).max() < 1e-12
    # deeper layers: the cache is what attention reads, so feeding one token fewer gives a prefix
    K1, V1 = m.self_kv(1, wl.enc[:wl.enc_lens[0]], toks)
    K1s, V1s = m.self_kv(1, wl.enc[:wl.enc_lens[0]], toks[:3])
    assert np.array_equal(K1[:3], K1s) and np.array_equal(V1[:3], V1s)


# ---- RMSNorm variant (norm_type = 1) ----
def _torch_decoder_rms(cfg, w):
    """torch's pre-norm decoder with every LayerNorm module replaced by torch.nn.RMSNorm (gain only)."""
    dec = _torch_decoder(cfg, w)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))

    def rms(gain):
        mod = torch.nn.RMSNorm(cfg.d_model, eps=cfg.ln_eps).double()
        with torch.no_grad():
            mod.weight.copy_(t(gain))
        return mod

    for l, lw in zip(dec.layers, w["layers"]):
        l.norm1, l.norm2, l.norm3 = rms(lw["ln1_g"]), rms(lw["ln2_g"]), rms(lw["ln3_g"])
    dec.norm = rms(w["lnf_g"])
    return dec.eval()


def _without_norm_shifts(w):
    w = dict(w)
    w["lnf_b"] = None
    w["layers"] = [dict(l, ln1_b=None, ln2_b=None, ln3_b=None) for l in w["layers"]]
    return w


def test_rmsnorm_model_matches_torch_decoder_with_rmsnorm_modules(oracle):
    wl = small_workload(seed=5, enc_lens=(6, 3, 10, 1), norm_type=1)
    cfg = wl.cfg
    w = _without_norm_shifts(wl.weights)
    B, S = 4, 8
    toks = random_tokens(cfg, B, S, 15)
    mine = oracle.Model(cfg, w).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = _torch_decoder_rms(cfg, wl.weights)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x0 = cfg.emb_scale * t(w["tok_emb"])[torch.from_numpy(toks).long()] + t(w["pos_emb"])[:S][None]
    mem = t(pad_enc(wl))
    kpm = torch.arange(mem.shape[1])[None, :] >= torch.from_numpy(wl.enc_lens)[:, None]
    causal = torch.triu(torch.ones(S, S, dtype=torch.bool), diagonal=1)
    with torch.no_grad():
        hid = dec(x0, mem, tgt_mask=causal, memory_key_padding_mask=kpm)
        ref = (hid @ t(w["w_out"]).T + t(w["b_out"])).numpy()
    assert np.abs(mine - ref).max() < 1e-9
    # and it is not the LayerNorm model
    wl_ln = small_workload(seed=5, enc_lens=(6, 3, 10, 1))
    other = oracle.Model(wl_ln.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    assert np.abs(other - mine).max() > 1e-2


def test_rmsnorm_incremental_equals_full_forward_and_padding(oracle):
    wl = small_workload(seed=6, norm_type=1)
    m = oracle.Model(wl.cfg, wl.weights)   # with shift vectors
    S = 7
    toks = random_tokens(wl.cfg, 3, S, 17)
    inc = m.decode_forced(wl.enc, wl.enc_lens, toks)
    full = m.forward_full(pad_enc(wl, fill=np.nan), wl.enc_lens, toks, np.full(3, S, np.int32))
    assert np.abs(inc - full).max() < 1e-10
    # the shift vectors are in use: dropping them changes the logits
    inc0 = oracle.Model(wl.cfg, _without_norm_shifts(wl.weights)).decode_forced(wl.enc, wl.enc_lens, toks)
    assert np.abs(inc0 - inc).max() > 1e-3


def test_rmsnorm_equals_layernorm_while_every_normalised_row_has_zero_mean(oracle):
    """If the embeddings are zero-mean rows and every residual update is (output matrices and biases with zero
    column means), every row that is ever normalised has mean zero, where the two normalisations agree: the
    RMSNorm model then gives the LayerNorm model's logits (which torch's decoder pins)."""
    wl = small_workload(seed=7)
    w = wl.weights
    for k in ("tok_emb", "pos_emb"):
        w[k] = (w[k] - w[k].mean(axis=1, keepdims=True)).astype(np.float32)
    for l in w["layers"]:
        for k in ("w_o", "w_co", "w_ff2"):
            l[k] = (l[k] - l[k].mean(axis=0, keepdims=True)).astype(np.float32)
        for k in ("b_o", "b_co", "b_ff2"):
            l[k] = (l[k] - l[k].mean()).astype(np.float32)
    toks = random_tokens(wl.cfg, 3, 6, 19)
    ln_logits = oracle.Model(wl.cfg, w).decode_forced(wl.enc, wl.enc_lens, toks)
    cfg_rms = small_cfg(norm_type=1)
    rms_logits = oracle.Model(cfg_rms, w).decode_forced(wl.enc, wl.enc_lens, toks)
    assert np.abs(ln_logits - rms_logits).max() < 1e-5   # float32 weights: the means are zero to ~1e-8 only
