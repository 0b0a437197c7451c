"""Pins for the oracle's 8-bit key / value storage option (CPU only).

The format is E4M3 of the OCP 8-bit floating point specification: sign, 4
exponent bits (bias 7), 3 mantissa bits, subnormals, no infinities, one NaN
code per sign, largest magnitude 448.  The codec is pinned against that
closed form written out here, against torch's float8_e4m3fn casts (a library
routine), and by brute force over all codes; its place in the model (keys and
values are replaced by their codes' values when they are cached, nothing
else) is pinned by a numpy forward pass written out for a tiny decoder and by
incremental == whole-sequence agreement."""
import math

import numpy as np
import pytest
import torch

from paper_2503_05931_amd import workloads as W
from tests.test_oracle_model import pad_enc, random_tokens, small_workload


def spec_value(code: int) -> float:
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return math.nan
    v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return -v if s else v


ALL = np.arange(256, dtype=np.uint8)
FINITE = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)


def torch_encode(x32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(x32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_decode_is_the_closed_form_for_all_codes(oracle):
    got = oracle.fp8_e4m3_decode(ALL)
    ref = np.array([spec_value(int(c)) for c in ALL])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got[~np.isnan(ref)], ref[~np.isnan(ref)])
    # landmarks of the format: largest value, smallest normal, smallest subnormal, signed zeros
    assert oracle.fp8_e4m3_decode([0x7E])[0] == 448.0
    assert oracle.fp8_e4m3_decode([0x08])[0] == 2.0 ** -6
    assert oracle.fp8_e4m3_decode([0x01])[0] == 2.0 ** -9
    z = oracle.fp8_e4m3_decode([0x00, 0x80])
    assert z[0] == 0.0 and z[1] == 0.0 and math.copysign(1.0, z[1]) == -1.0
    # and the library's view of the same bytes
    lib = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(got[~np.isnan(ref)], lib[~np.isnan(ref)])


def test_encode_inverts_decode_and_is_monotone(oracle):
    vals = oracle.fp8_e4m3_decode(FINITE).astype(np.float32)
    assert np.array_equal(oracle.fp8_e4m3_encode(vals), FINITE)
    x = np.sort(np.random.default_rng(0).uniform(-460, 460, 20000).astype(np.float32))
    y = oracle.fp8_e4m3_decode(oracle.fp8_e4m3_encode(x))
    assert np.all(np.diff(y) >= 0)


def test_encode_matches_torch_cast(oracle):
    rng = np.random.default_rng(1)
    parts = [rng.standard_normal(200000).astype(np.float32) * s for s in (1e-3, 0.02, 1.0, 30.0)]
    parts.append(rng.uniform(-448, 448, 100000).astype(np.float32))
    # every midpoint between neighbouring codes (the ties) and the floats on either side of it
    pos = np.sort(oracle.fp8_e4m3_decode(FINITE[FINITE < 0x7F]))  # 0 .. 448
    mid = (0.5 * (pos[:-1] + pos[1:])).astype(np.float32)
    for s in (1.0, -1.0):
        parts += [s * mid, s * np.nextafter(mid, np.float32(0)), s * np.nextafter(mid, np.float32(1e9))]
    parts.append(np.array([0.0, -0.0, 1e-30, -1e-30, 2.0 ** -10, 2.0 ** -10 * 1.0001, 448.0, -448.0], np.float32))
    x = np.concatenate(parts)
    x = x[np.abs(x) <= 448.0]
    assert np.array_equal(oracle.fp8_e4m3_encode(x), torch_encode(x))


def test_encode_is_round_to_nearest_even_by_brute_force(oracle):
    table = np.array([spec_value(int(c)) for c in FINITE])
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(3000) * 2.0, rng.uniform(-448, 448, 3000),
                        rng.uniform(-0.05, 0.05, 3000)]).astype(np.float32)
    codes = oracle.fp8_e4m3_encode(x)
    for xi, c in zip(x.astype(np.float64), codes):
        err = np.abs(table - xi)
        best = err.min()
        assert abs(spec_value(int(c)) - xi) == best
        ties = FINITE[err == best]
        ties = [t for t in ties if (t >> 7) == (c >> 7) or best != abs(xi)]  # +0 / -0 stand for the same value
        if len(ties) > 1:
            assert c % 2 == 0, (xi, c, ties)
    # ties written out: halfway between 1.0 (0x38) and 1.125 (0x39) goes to the even code, and so on
    assert list(oracle.fp8_e4m3_encode(np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10], np.float32))) == \
        [0x38, 0x3A, 0x00, 0x02]


def test_encode_saturates_and_keeps_nan(oracle):
    x = np.array([449.0, 464.0, 465.0, 1e30, np.inf, -500.0, -np.inf], np.float32)
    assert list(oracle.fp8_e4m3_encode(x)) == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE]
    assert (oracle.fp8_e4m3_encode(np.array([np.nan], np.float32))[0] & 0x7F) == 0x7F


def q8(a):
    """Independent of the oracle: what a float64 array becomes when stored as E4M3 (torch's casts)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(torch.float32).to(torch.float8_e4m3fn)
    return t.to(torch.float64).numpy()


def test_cross_kv_is_the_quantised_linear_map(oracle):
    wl = small_workload(seed=11, kv_fp8=1)
    m = oracle.Model(wl.cfg, wl.weights)
    d = wl.cfg.d_model
    enc = wl.enc[:5]
    K, V = m.cross_kv(1, enc)
    lw = wl.weights["layers"][1]
    ref = q8(enc.astype(np.float64) @ lw["w_ckv"].astype(np.float64).T + lw["b_ckv"])
    assert np.array_equal(K, ref[:, :d]) and np.array_equal(V, ref[:, d:])
    exact = oracle.Model(small_workload(seed=11).cfg, wl.weights).cross_kv(1, enc)[0]
    assert 0 < np.abs(K - exact).max() <= 2.0 ** -4 * np.abs(exact).max()


def ln(z, g, b, eps):
    mu = z.mean()
    return (z - mu) / math.sqrt(((z - mu) ** 2).mean() + eps) * g + b


def test_self_attention_reads_quantised_keys_and_values(oracle):
    """One layer whose cross-attention and feed-forward outputs are switched off (zero output
    projections), two positions: the whole forward pass written out in numpy with the keys and values
    passed through torch's E4M3 casts where they are cached."""
    wl = small_workload(seed=21, n_layers=1, kv_fp8=1, enc_lens=(4,), batch=1)
    lw = wl.weights["layers"][0]
    for k in ("w_co", "b_co", "w_ff2", "b_ff2"):
        lw[k] = np.zeros_like(lw[k])
    cfg, w = wl.cfg, wl.weights
    d, H, dh = cfg.d_model, cfg.n_heads, cfg.head_dim
    toks = np.array([[7, 3]], np.int32)
    got = oracle.Model(cfg, w).decode_forced(wl.enc, wl.enc_lens, toks)[0]
    f = lambda a: np.asarray(a, dtype=np.float64)
    Ks, Vs = [], []
    for s in range(2):
        x = cfg.emb_scale * f(w["tok_emb"][toks[0, s]]) + f(w["pos_emb"][s])
        qkv = f(lw["w_qkv"]) @ ln(x, f(lw["ln1_g"]), f(lw["ln1_b"]), cfg.ln_eps) + f(lw["b_qkv"])
        Ks.append(q8(qkv[d:2 * d]))
        Vs.append(q8(qkv[2 * d:]))
        att = np.zeros(d)
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            sc = np.array([qkv[sl] @ k[sl] for k in Ks]) / math.sqrt(dh)
            p = np.exp(sc - sc.max())
            p /= p.sum()
            att[sl] = sum(pj * v[sl] for pj, v in zip(p, Vs))
        x = x + f(lw["w_o"]) @ att + f(lw["b_o"])
        logits = f(w["w_out"]) @ ln(x, f(w["lnf_g"]), f(w["lnf_b"]), cfg.ln_eps) + f(w["b_out"])
        assert np.abs(got[s] - logits).max() < 1e-10
    # the cache accessor returns exactly those keys and values
    Kc, Vc = oracle.Model(cfg, w).self_kv(0, wl.enc, toks[0])
    assert np.array_equal(Kc, np.stack(Ks)) and np.array_equal(Vc, np.stack(Vs))
    # the option is not a no-op on this input
    wl0 = small_workload(seed=21, n_layers=1, enc_lens=(4,), batch=1)
    exact = oracle.Model(wl0.cfg, w).decode_forced(wl.enc, wl.enc_lens, toks)[0]
    assert np.abs(got - exact).max() > 1e-6


def test_incremental_equals_full_forward_with_quantised_cache(oracle):
    wl = small_workload(seed=1, kv_fp8=1)
    m = oracle.Model(wl.cfg, wl.weights)
    S = 7
    toks = random_tokens(wl.cfg, 3, S, 11)
    inc = m.decode_forced(wl.enc, wl.enc_lens, toks)
    full = m.forward_full(pad_enc(wl), wl.enc_lens, toks, np.full(3, S, np.int32))
    assert np.abs(inc - full).max() < 1e-10
    exact = oracle.Model(small_workload(seed=1).cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    # storage error of at most 2^-4 relative per element moves the logits a little, not a lot
    assert 1e-6 < np.abs(inc - exact).max() < 0.5 * np.abs(exact).max()
