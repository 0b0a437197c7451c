"""GPU parity of the 8-bit key / value cache option (aed_config.kv_fp8): the HIP path against the CPU oracle run
with the same option, i.e. with every cached key and value replaced by the value of its E4M3 code.  Both sides
round from float32 to the nearest code.
Cross-attention keys / values are products of exactly representable bf16 inputs, accumulated in float32 by the
kernels and in float64 by the oracle: the codes are identical except where the exact value lies within a float32
rounding error of the midpoint of two codes (rare; one code step).
Self-attention keys / values are products of activations that already carry the bf16 arithmetic's error, so an
element within that error of a midpoint gets the neighbouring code: a few per cent of the elements differ by one
step (more for elements smaller than the error itself), and the logits tolerance is wider than in bf16 mode
(see gpu_util.TOL)."""
import numpy as np
import pytest

from paper_2503_05931_amd import workloads as W
from tests.test_gpu_parity import random_tokens, unit_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def check_codes(got, ref, what, max_frac=2e-3, noise=0.0):
    """Cache contents read back (decoded codes) against the oracle's: equal but for a fraction max_frac of the
    elements, which are at most one code step (plus `noise`, the error of the value that was encoded) away."""
    assert np.isfinite(got).all(), f"{what}: non-finite cache contents"
    diff = got != ref
    frac = float(diff.mean())
    assert frac < max_frac, f"{what}: {frac:.2e} of the codes differ"
    if diff.any():
        # neighbouring codes are at most 1/8 apart relative to the smaller one (or 2^-9 among subnormals)
        step = np.maximum(np.abs(ref[diff]) * 0.125, 2.0 ** -9)
        assert (np.abs(got[diff] - ref[diff]) <= step * 1.0001 + noise).all(), f"{what}: a code is too far off"
    return frac


@pytest.mark.parametrize("d_model,n_heads,head_dim,enc_lens,steps", [
    (256, 4, 64, [1, 15, 16, 17, 63, 64, 65, 130], 35),   # head_dim 64: 8-byte loads, ragged tails, page boundaries
    (512, 4, 128, [1, 2, 129, 500, 77], 35),               # head_dim 128: 16-byte loads
    (1024, 8, 128, [257, 1, 64], 35),
    (256, 4, 64, [500, 300], 140),                         # keys cut into chunks, last-arriver merge
    (512, 4, 128, [3 + (5 * i) % 40 for i in range(300)], 18),  # more than 1024 workgroups: 4-wavefront kernels
])
def test_fp8_cache_teacher_forced(torch_cuda, oracle, d_model, n_heads, head_dim, enc_lens, steps):
    from tests import gpu_util as G
    wl = unit_workload("bf16", d_model, n_heads, head_dim, enc_lens, seed=len(enc_lens) + d_model + 1,
                       max_new=max(40, steps), kv_fp8=1)
    B = len(enc_lens)
    toks = random_tokens(wl.cfg, B, steps, 5)
    m = oracle.Model(wl.cfg, wl.weights)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16+fp8kv"])
    worst = 0.0
    for b in (0, B - 1):
        Kr, Vr = m.cross_kv(1, wl.subset([b]).enc)
        Kg, Vg = dec.aed_read_cross_kv(1, b, int(enc_lens[b]))
        worst = max(worst, check_codes(Kg, Kr, "cross K"), check_codes(Vg, Vr, "cross V"))
    # the self-attention cache.  First layer: its keys and values depend on nothing cached, so they carry only the
    # bf16 arithmetic's own error and few codes differ from the oracle's.  Second layer: its input has been
    # through the first layer's attention over codes that already differ, so more do.  Every value read back is
    # one a code stands for.
    self_frac = []
    for layer, max_frac, noise in ((0, 0.10, 1e-2), (1, 0.40, 5e-2)):
        Ks, Vs = dec.aed_read_self_kv(layer, B - 1)
        assert Ks.shape == (steps, d_model)
        Kr, Vr = m.self_kv(layer, wl.subset([B - 1]).enc, toks[B - 1])
        self_frac.append(max(check_codes(Ks, Kr, f"self K, layer {layer}", max_frac=max_frac, noise=noise),
                             check_codes(Vs, Vr, f"self V, layer {layer}", max_frac=max_frac, noise=noise)))
        for a in (Ks, Vs):
            assert np.array_equal(oracle.fp8_e4m3_decode(oracle.fp8_e4m3_encode(a)), a.astype(np.float64))
    # what the option changes is visible: the exact-cache oracle is further away than the tolerance check above
    exact_cfg = W.DecoderConfig(**{**wl.cfg.__dict__, "kv_fp8": 0})
    exact = oracle.Model(exact_cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks[:, :4])
    print(f"fp8 caches d={d_model} H={n_heads}x{head_dim}: max |dlogit| = {err:.2e} (oracle with exact caches is "
          f"{np.abs(exact - ref[:, :4]).max():.2e} away), near ties {near}, differing codes: cross {worst:.1e}, "
          f"self {self_frac[0]:.1e} (first layer), {self_frac[1]:.1e} (second)")
    glog2, gids2 = G.forced_logits_gpu(dec, wl, toks)
    assert (glog2 == glog).all() and (gids2 == gids).all()
    dec.close()


@pytest.mark.parametrize("d_model,n_heads,head_dim,enc_lens", [
    (1024, 8, 128, [500, 500, 500, 500, 131]),   # 272 tiles of 128 x 128: the tiled MFMA kernels write the codes
    (1024, 8, 128, [700] * 7 + [411]),           # enough for the persistent 256 x 256 kernel (ragged last row tile)
    (512, 8, 64, [1300] * 7 + [1150]),           # the same kernel, one head per wavefront's 64 columns
])
def test_fp8_cache_large_cross_kv_precompute(torch_cuda, oracle, d_model, n_heads, head_dim, enc_lens):
    from tests import gpu_util as G
    wl = unit_workload("bf16", d_model, n_heads, head_dim, enc_lens, seed=95, n_layers=1, d_ffn=256, vocab=64,
                       max_new=8, kv_fp8=1)
    m = oracle.Model(wl.cfg, wl.weights)
    B = len(enc_lens)
    toks = random_tokens(wl.cfg, B, 4, 8)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    worst = 0.0
    for b in range(B):
        Kr, Vr = m.cross_kv(0, wl.subset([b]).enc)
        Kg, Vg = dec.aed_read_cross_kv(0, b, enc_lens[b])
        worst = max(worst, check_codes(Kg, Kr, "cross K"), check_codes(Vg, Vr, "cross V"))
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16+fp8kv"])
    print(f"fp8 cross K/V precompute, {sum(enc_lens)} frames: differing codes {worst:.1e}, max |dlogit| = {err:.2e}")
    dec.close()


@pytest.mark.parametrize("prefill", [False, True])
def test_fp8_cache_greedy_with_eos(torch_cuda, oracle, prefill):
    """Free-running greedy decoding (launch graph, device-side sampler, optional prompt prefill) with 8-bit
    caches: ids identical to the oracle's up to each sequence's first near-tie step."""
    import torch
    from tests import gpu_util as G
    enc_lens = [33, 7, 120, 64, 250, 18]
    wl = unit_workload("bf16", 512, 4, 128, enc_lens, seed=123, max_new=40, eos_id=2, prompt_len=5, kv_fp8=1)
    cfg = wl.cfg
    B = len(enc_lens)
    limits = np.array([40, 9, 17, 40, 1, 33], np.int32)
    m = oracle.Model(cfg, wl.weights)
    ref_toks, ref_lens, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new,
                                                     max_new_per_seq=limits, want_logits=True)
    dec = G.make_decoder(wl, prefill_rows=(cfg.prompt_len - 1) * 16 if prefill else 0)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new,
                                       max_new_per_seq=limits)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    first = G.first_near_tie(np.nan_to_num(ref_logits, nan=0.0), G.TOL["bf16+fp8kv"])
    for b in range(B):
        n = min(int(first[b]), int(ref_lens[b]))
        assert (toks[b, :n] == ref_toks[b, :n]).all(), f"sequence {b} forks before a near tie"
        if first[b] >= ref_lens[b]:
            assert lens[b] == ref_lens[b] and (toks[b, lens[b]:] == cfg.pad_id).all()
    print("fp8 caches, greedy" + (" with prefill" if prefill else "") + ": identical for", first.tolist(), "steps; lens", lens.tolist())
    assert (lens <= limits).all() and (lens >= 1).all()
    if not prefill:
        # the graph replay and the step-by-step path agree bit for bit: feeding the emitted tokens back through
        # aed_decode_step reproduces them (up to each sequence's end; a forced EOS is not an argmax)
        P = cfg.prompt_len
        fed = np.concatenate([wl.prompt, np.where(toks[:, :-1] == cfg.pad_id, 0, toks[:, :-1])], axis=1)
        _, gids = G.forced_logits_gpu(dec, wl, fed)
        for b in range(B):
            n = int(lens[b]) - 1  # the last emitted token may be a forced EOS
            assert (gids[b, P - 1:P - 1 + n] == toks[b, :n]).all(), f"sequence {b}: graph and step path differ"
    dec.close()


@pytest.mark.parametrize("name,sample,n_new", [
    ("canary24_b64", [17, 63], 40),
    ("flash4_b256", [0, 255], 40),
    ("large24_b1024", [1023], 16),   # about 50 GB of caches; one page boundary
])
def test_fp8_cache_at_the_benchmark_sizes(torch_cuda, oracle, name, sample, n_new):
    """The configurations bench.py --kv-fp8 times: sampled sequences teacher-forced against the oracle, then the
    graph path at full length (every sequence emits max_new tokens; a second run is bit-identical)."""
    import torch
    from tests import gpu_util as G
    from tests.test_gpu_full_size import _forced_check
    wl = W.make(name)
    wl.cfg.kv_fp8 = 1
    dec, err, near = _forced_check(oracle, wl, sample, n_new, G.TOL["bf16+fp8kv"], max_dec_len=wl.cfg.max_dec_len)
    print(f"{name} with fp8 caches, teacher-forced: max |dlogit| = {err:.3e}, near ties {near}")
    if name != "large24_b1024":
        B, P = len(wl.enc_lens), wl.cfg.prompt_len
        dec.close()
        dec = G.make_decoder(wl, prefill_rows=(P - 1) * ((B + 15) // 16 * 16))
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        prompt = torch.from_numpy(wl.prompt).to(dec.device)
        t1, l1 = dec.aed_greedy_decode(prompt, wl.cfg.max_new)
        t1, l1 = t1.cpu().numpy().copy(), l1.cpu().numpy().copy()
        t2, l2 = dec.aed_greedy_decode(prompt, wl.cfg.max_new)
        assert (l1 == wl.cfg.max_new).all() and (t1 == t2.cpu().numpy()).all() and (l1 == l2.cpu().numpy()).all()
    dec.close()


def test_fp8_cache_with_the_request_queue(torch_cuda, oracle):
    """Slot refill writes the new requests' cross K/V through the frame map: with 8-bit caches too, every request's
    tokens equal the oracle's up to its first near tie."""
    import torch
    from tests import gpu_util as G
    rng = np.random.default_rng(5)
    n_req, slots = 14, 4
    enc_lens = rng.integers(3, 90, n_req).tolist()
    wl = unit_workload("bf16", 256, 4, 64, enc_lens, seed=321, max_new=24, eos_id=3, kv_fp8=1)
    cfg = wl.cfg
    limits = rng.integers(1, 24, n_req).astype(np.int32)
    m = oracle.Model(cfg, wl.weights)
    ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new, max_new_per_seq=limits,
                                               want_logits=True)
    dec = G.make_decoder(wl, max_batch=slots, max_total=int(np.sort(wl.enc_lens)[-slots:].sum()) + 64)
    toks, lens, steps = dec.aed_greedy_decode_queue(dec.to_device(wl.enc), wl.enc_lens,
                                                    torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new, limits)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    tol = G.TOL["bf16+fp8kv"]
    whole = 0
    for r in range(n_req):
        n = int(ref_l[r])
        first = int(G.first_near_tie(ref_logits[r:r + 1, :n], tol)[0])
        assert (toks[r, :first] == ref_t[r, :first]).all(), f"request {r} forks before a near tie"
        assert 1 <= lens[r] <= limits[r] and toks[r, lens[r] - 1] == cfg.eos_id and (toks[r, lens[r]:] == cfg.pad_id).all()
        if first >= n:
            whole += 1
            assert lens[r] == n and (toks[r] == ref_t[r]).all()
    print(f"queue with fp8 caches: {n_req} requests through {slots} slots in {steps} steps; {whole} requests fixed to the end")
    dec.close()


def test_fp8_cache_needs_bfloat16(torch_cuda):
    from paper_2503_05931_amd import binding
    from tests import gpu_util as G
    wl = unit_workload("fp32", 256, 4, 64, [5, 6], seed=1, kv_fp8=1)
    with pytest.raises(binding.AedError) as e:
        G.make_decoder(wl)
    assert e.value.status == binding.AED_EUNSUPPORTED
