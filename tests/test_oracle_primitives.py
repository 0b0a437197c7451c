"""Pins for the oracle's primitives: closed forms, brute force written out in
the test, and agreement with library routines (numpy / scipy / torch CPU in
float64).  None of these call the HIP path."""
import math

import numpy as np
import pytest
import torch


def test_layernorm_closed_forms(oracle):
    rng = np.random.default_rng(0)
    n = 37
    z = rng.standard_normal(n) * 3.0 + 5.0
    ones, zeros = np.ones(n, np.float32), np.zeros(n, np.float32)
    eps = 1e-5
    y = oracle.layernorm(z, ones, zeros, eps)
    var = z.var()  # biased
    assert abs(y.mean()) < 1e-12
    assert abs(y.var() - var / (var + eps)) < 1e-12
    # scale invariance up to the eps term
    y2 = oracle.layernorm(7.0 * z, ones, zeros, 0.0)
    y0 = oracle.layernorm(z, ones, zeros, 0.0)
    assert np.allclose(y2, y0, atol=1e-12)
    # a two-point vector: z = [a, b] -> +-1 (eps = 0)
    y = oracle.layernorm(np.array([3.0, 5.0]), np.ones(2, np.float32), np.zeros(2, np.float32), 0.0)
    assert np.allclose(y, [-1.0, 1.0], atol=1e-14)
    # gain and shift apply after normalisation
    g = rng.standard_normal(n).astype(np.float32)
    b = rng.standard_normal(n).astype(np.float32)
    assert np.allclose(oracle.layernorm(z, g, b, eps), g * oracle.layernorm(z, ones, zeros, eps) + b, atol=1e-12)


def test_layernorm_matches_torch(oracle):
    rng = np.random.default_rng(1)
    z = rng.standard_normal(64)
    g = rng.standard_normal(64).astype(np.float32)
    b = rng.standard_normal(64).astype(np.float32)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(z), (64,), torch.from_numpy(g).double(),
                                         torch.from_numpy(b).double(), eps=1e-5).numpy()
    assert np.allclose(oracle.layernorm(z, g, b, 1e-5), ref, atol=1e-12)


def test_linear_is_row_major_out_in(oracle):
    rng = np.random.default_rng(2)
    W = rng.standard_normal((5, 3)).astype(np.float32)  # non-square: a transposed read fails
    b = rng.standard_normal(5).astype(np.float32)
    x = rng.standard_normal(3)
    assert np.allclose(oracle.linear(x, W, b), W.astype(np.float64) @ x + b, atol=1e-13)
    assert np.allclose(oracle.linear(x, W, None), W.astype(np.float64) @ x, atol=1e-13)
    # unit vectors pick out columns
    e1 = np.array([0.0, 1.0, 0.0])
    assert np.allclose(oracle.linear(e1, W, None), W[:, 1], atol=0)


def test_softmax_pins(oracle):
    p = oracle.softmax(np.array([0.0, math.log(2.0)]))
    assert np.allclose(p, [1 / 3, 2 / 3], atol=1e-15)
    rng = np.random.default_rng(3)
    a = rng.standard_normal(100) * 10
    p = oracle.softmax(a)
    assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
    assert np.allclose(oracle.softmax(a + 1000.0), p, atol=1e-12)  # shift invariance, no overflow
    from scipy.special import softmax as sp_softmax
    assert np.allclose(p, sp_softmax(a), atol=1e-14)
    assert np.allclose(oracle.softmax(np.full(7, 3.3)), np.full(7, 1 / 7), atol=1e-15)


def _brute_attention(q, K, V):
    n, dh = len(K), len(q)
    scores = []
    for j in range(n):
        s = 0.0
        for c in range(dh):
            s += q[c] * K[j][c]
        scores.append(s / math.sqrt(dh))
    m = max(scores)
    e = [math.exp(s - m) for s in scores]
    tot = sum(e)
    out = []
    for c in range(dh):
        acc = 0.0
        for j in range(n):
            acc += e[j] / tot * V[j][c]
        out.append(acc)
    return np.array(out), np.array(e) / tot


@pytest.mark.parametrize("n,dh", [(1, 1), (2, 3), (4, 4), (3, 2)])
def test_attend_brute_force(oracle, n, dh):
    rng = np.random.default_rng(10 + n * 7 + dh)
    q, K, V = rng.standard_normal(dh), rng.standard_normal((n, dh)), rng.standard_normal((n, dh))
    out, probs = oracle.attend(q, K, V, want_probs=True)
    ref_out, ref_p = _brute_attention(q.tolist(), K.tolist(), V.tolist())
    assert np.allclose(out, ref_out, atol=1e-14)
    assert np.allclose(probs, ref_p, atol=1e-14)
    assert abs(probs.sum() - 1) < 1e-14


def test_attend_closed_forms(oracle):
    rng = np.random.default_rng(4)
    K, V = rng.standard_normal((6, 8)), rng.standard_normal((6, 8))
    # q = 0 -> uniform weights -> mean of V over the keys given
    assert np.allclose(oracle.attend(np.zeros(8), K, V), V.mean(axis=0), atol=1e-14)
    assert np.allclose(oracle.attend(np.zeros(8), K[:4], V[:4]), V[:4].mean(axis=0), atol=1e-14)
    # one key -> that value row
    q = rng.standard_normal(8)
    assert np.allclose(oracle.attend(q, K[:1], V[:1]), V[0], atol=1e-15)
    # a dominant score -> that value row
    Kd = np.zeros((3, 8))
    Kd[1] = 100.0 * q
    Vd = rng.standard_normal((3, 8))
    assert np.allclose(oracle.attend(q, Kd, Vd), Vd[1], atol=1e-9)
    # the 1/sqrt(dh) scale: two keys, dh = 4, q.k = (4, 0) -> scores (2, 0)
    q4 = np.array([1.0, 1.0, 1.0, 1.0])
    K2 = np.array([[1.0, 1.0, 1.0, 1.0], [0, 0, 0, 0]])
    _, p = oracle.attend(q4, K2, np.eye(2, 4), want_probs=True)
    assert np.allclose(p, [math.e ** 2 / (math.e ** 2 + 1), 1 / (math.e ** 2 + 1)], atol=1e-14)


def test_attend_matches_torch_sdpa(oracle):
    rng = np.random.default_rng(5)
    q, K, V = rng.standard_normal(16), rng.standard_normal((9, 16)), rng.standard_normal((9, 16))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0, 0].numpy()
    assert np.allclose(oracle.attend(q, K, V), ref, atol=1e-12)


def test_argmax_lowest_index_on_ties(oracle):
    assert oracle.argmax(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert oracle.argmax(np.array([5.0, 5.0, 5.0])) == 0
    assert oracle.argmax(np.array([-2.0, -1.0])) == 1


def test_rmsnorm_closed_forms(oracle):
    """Root-mean-square normalisation (Zhang and Sennrich 2019): no mean subtraction."""
    g1, b0 = np.ones(2, np.float32), np.zeros(2, np.float32)
    # [3, 4]: mean square 12.5
    y = oracle.rmsnorm(np.array([3.0, 4.0]), g1, None, 0.0)
    assert np.allclose(y, np.array([3.0, 4.0]) / math.sqrt(12.5), atol=1e-15)
    # eps sits inside the root, next to the mean square
    y = oracle.rmsnorm(np.array([3.0, 4.0]), g1, None, 3.5)
    assert np.allclose(y, np.array([3.0, 4.0]) / 4.0, atol=1e-15)
    # scale invariance at eps = 0, and none under a shift of the input (a LayerNorm would not notice the shift)
    rng = np.random.default_rng(5)
    z = rng.standard_normal(37)
    g = rng.standard_normal(37).astype(np.float32)
    b = rng.standard_normal(37).astype(np.float32)
    assert np.allclose(oracle.rmsnorm(7.5 * z, g, b, 0.0), oracle.rmsnorm(z, g, b, 0.0), atol=1e-13)
    assert np.abs(oracle.rmsnorm(z + 2.0, g, b, 1e-5) - oracle.rmsnorm(z, g, b, 1e-5)).max() > 0.1
    assert np.allclose(oracle.layernorm(z + 2.0, g, b, 1e-5), oracle.layernorm(z, g, b, 1e-5), atol=1e-12)
    # on a zero-mean row it equals LayerNorm (biased variance = mean square)
    z0 = z - z.mean()
    assert np.allclose(oracle.rmsnorm(z0, g, b, 1e-5), oracle.layernorm(z0, g, b, 1e-5), atol=1e-13)
    # gain multiplies, shift adds, a missing shift is zero
    y0 = oracle.rmsnorm(z, np.ones(37, np.float32), None, 1e-5)
    assert np.allclose(oracle.rmsnorm(z, g, b, 1e-5), y0 * g.astype(np.float64) + b.astype(np.float64), atol=1e-14)
    assert np.array_equal(oracle.rmsnorm(z, g, None, 1e-5), oracle.rmsnorm(z, g, np.zeros(37, np.float32), 1e-5))
    # output has mean square n / (n + eps * n / ms) -> 1 for eps -> 0
    assert abs((y0 ** 2).mean() - (z ** 2).mean() / ((z ** 2).mean() + 1e-5)) < 1e-14


def test_rmsnorm_matches_torch(oracle):
    import torch
    rng = np.random.default_rng(6)
    for n in (8, 33, 256):
        z = rng.standard_normal(n) * 3 + 1
        g = rng.standard_normal(n).astype(np.float32)
        ref = torch.nn.functional.rms_norm(torch.from_numpy(z), (n,), torch.from_numpy(g.astype(np.float64)), 1e-5).numpy()
        assert np.abs(oracle.rmsnorm(z, g, None, 1e-5) - ref).max() < 1e-13
