"""GPU parity at the benchmark's full size and launch configuration: the
24-layer bf16 decoder, batch 64, log-normal lengths, 4-token prompt, 128 greedy
steps through the captured launch graph.  The oracle computes a sample of the
sequences one by one (sequences are independent of their batch)."""
import numpy as np
import pytest

from paper_2503_05931_amd import workloads as W

pytestmark = pytest.mark.gpu

SAMPLE = [0, 17, 40, 63]


def test_canary24_b64_sampled_sequences(oracle):
    import torch
    from tests import gpu_util as G
    wl = W.make("canary24_b64")
    cfg = wl.cfg
    tol = G.TOL["bf16"]
    sub = wl.subset(SAMPLE)
    m = oracle.Model(cfg, wl.weights)
    ref_toks, ref_lens, ref_logits = m.greedy_decode(sub.enc, sub.enc_lens, sub.prompt, cfg.max_new, want_logits=True)

    dec = G.make_decoder(wl, poison=True)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    assert (lens == cfg.max_new).all()
    # free-running: identical ids up to each sequence's first near-tie step
    first = G.first_near_tie(ref_logits, tol)
    for i, b in enumerate(SAMPLE):
        assert (toks[b, :first[i]] == ref_toks[i, :first[i]]).all(), f"sequence {b} forks before a near tie"
    print("free-running ids identical for", first.tolist(), "steps of", cfg.max_new)

    # teacher-forced: the sampled sequences consume the oracle's tokens, the others their own
    forced = np.concatenate([wl.prompt, toks[:, :-1]], axis=1)
    for i, b in enumerate(SAMPLE):
        forced[b, cfg.prompt_len:] = ref_toks[i, :-1]
    glog, gids = G.forced_logits_gpu(dec, wl, forced)
    P = cfg.prompt_len
    err, near = G.check_forced(ref_logits, glog[SAMPLE][:, P - 1:], gids[SAMPLE][:, P - 1:], tol)
    print(f"canary24_b64 teacher-forced: max |dlogit| = {err:.3e}, near-tie steps = {near} of {ref_logits.shape[0] * ref_logits.shape[1]}")
    # the graph replay and the eager step path agree bit for bit on the other sequences' ids
    others = [b for b in range(len(wl.enc_lens)) if b not in SAMPLE]
    assert (gids[others][:, P - 1:] == toks[others]).all()
    dec.close()

    # the configuration bench.py times: the prompt positions before the last prefilled in one pass
    B = len(wl.enc_lens)
    dec = G.make_decoder(wl, poison=True, prefill_rows=(P - 1) * ((B + 15) // 16 * 16))
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks_p, lens_p = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new)
    toks_p, lens_p = toks_p.cpu().numpy(), lens_p.cpu().numpy()
    assert (lens_p == cfg.max_new).all()
    for i, b in enumerate(SAMPLE):
        assert (toks_p[b, :first[i]] == ref_toks[i, :first[i]]).all(), f"with prefill: sequence {b} forks before a near tie"
    same = int((toks_p == toks).all(axis=1).sum())
    print(f"with prompt prefill: {same} of {B} sequences token-identical to the run without it "
          "(the prompt's keys and values come from products of a different shape; forks start at near-ties)")
    dec.close()


def _forced_check(oracle, wl, sample, n_new, tol, max_dec_len=None):
    """Greedy-decode the oracle on the sampled sequences for n_new tokens, then run the whole batch through
    the HIP step path teacher-forced (sampled rows on the oracle's tokens, the rest on token 5) and compare
    every logit of the sampled rows; then the sampled rows' cached self-attention keys and values."""
    import torch
    from tests import gpu_util as G
    cfg = wl.cfg
    sub = wl.subset(sample)
    m = oracle.Model(cfg, wl.weights)
    ref_toks, ref_lens, ref_logits = m.greedy_decode(sub.enc, sub.enc_lens, sub.prompt, n_new, want_logits=True)
    B, P = len(wl.enc_lens), cfg.prompt_len
    forced = np.full((B, P + n_new - 1), 5, np.int32)
    forced[:, :P] = wl.prompt
    for i, b in enumerate(sample):
        forced[b, P:] = ref_toks[i, :-1]
    dec = G.make_decoder(wl, max_dec_len=max_dec_len, poison=True)
    glog, gids = G.forced_logits_gpu(dec, wl, forced, rows=sample)
    err, near = G.check_forced(ref_logits, glog[:, P - 1:], gids[:, P - 1:], tol)
    # the paged cache after the run: every position of the sampled sequences, first and last layer (with 8-bit
    # caches the contents are compared code by code in their own test)
    for i, b in enumerate([] if getattr(cfg, "kv_fp8", 0) else sample[:2]):
        one = wl.subset([b])
        for layer in (0, cfg.n_layers - 1):
            Kr, Vr = m.self_kv(layer, one.enc, forced[b])
            Kg, Vg = dec.aed_read_self_kv(layer, b)
            assert Kg.shape == Kr.shape
            kerr = max(float(np.abs(Kg - Kr).max()), float(np.abs(Vg - Vr).max()))
            assert kerr <= tol, f"self K/V of sequence {b}, layer {layer}: {kerr:.3e} > {tol}"
    return dec, err, near


def test_flash4_b256_sampled_sequences(oracle):
    """4-layer decoder, batch 256 (the shallow-decoder configuration)."""
    from tests import gpu_util as G
    import torch
    wl = W.make("flash4_b256")
    sample = [0, 100, 201, 255]
    # all 128 new tokens: 132 cached positions = 9 pages per sequence, so that each of the attention kernel's four
    # wavefronts goes round its block loop three times (pages looked up in the table, both register buffers refilled)
    dec, err, near = _forced_check(oracle, wl, sample, wl.cfg.max_new, G.TOL["bf16"])
    print(f"flash4_b256 teacher-forced: max |dlogit| = {err:.3e}, near ties {near}")
    # the graph path at full length: every sequence emits exactly max_new tokens, run twice bit-identical
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    prompt = torch.from_numpy(wl.prompt).to(dec.device)
    t1, l1 = dec.aed_greedy_decode(prompt, wl.cfg.max_new)
    t1, l1 = t1.cpu().numpy().copy(), l1.cpu().numpy().copy()
    t2, l2 = dec.aed_greedy_decode(prompt, wl.cfg.max_new)
    assert (l1 == wl.cfg.max_new).all() and (t1 == t2.cpu().numpy()).all() and (l1 == l2.cpu().numpy()).all()
    dec.close()


def test_ragged24_b128_forced_eos(oracle):
    """Ragged stress: 128 sequences with mixed encoder lengths and per-sequence forced EOS."""
    from tests import gpu_util as G
    import torch
    wl = W.make("ragged24_b128")
    cfg = wl.cfg
    target = wl.max_new_per_seq
    order = np.argsort(target)
    sample = [int(order[0]), int(order[3]), int(order[10])]          # short targets keep the oracle cheap
    sub = wl.subset(sample)
    m = oracle.Model(cfg, wl.weights)
    ref_t, ref_l, ref_logits = m.greedy_decode(sub.enc, sub.enc_lens, sub.prompt, cfg.max_new,
                                               max_new_per_seq=target[sample], want_logits=True)
    dec = G.make_decoder(wl, poison=True)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new, max_new_per_seq=target)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    # properties that hold for every sequence
    assert (lens >= 1).all() and (lens <= target).all()
    for b in range(len(target)):
        assert toks[b, lens[b] - 1] == cfg.eos_id                       # ends with EOS (forced or natural)
        assert (toks[b, :lens[b] - 1] != cfg.eos_id).all()
        assert (toks[b, lens[b]:] == cfg.pad_id).all()
    # sampled sequences against the oracle, up to the first near tie
    tol = G.TOL["bf16"]
    for i, b in enumerate(sample):
        n = ref_l[i]
        first = G.first_near_tie(ref_logits[i:i + 1, :n], tol)[0]
        assert (toks[b, :first] == ref_t[i, :first]).all()
        if first >= n:
            assert lens[b] == n and (toks[b] == ref_t[i]).all()
    print("ragged24_b128: lens ok for 128 sequences; sampled targets", target[sample].tolist(), "oracle lens", ref_l.tolist())
    dec.close()


def test_large24_b1024_paged_sampled_sequences(oracle, capsys):
    """Large batch: 1024 sequences of 500 frames, capacity for 452 positions in 16-token pages (about 100 GB of
    workspace).  Teacher-forced on random tokens through all 451 positions (29 pages per sequence): the first and
    the last sequence's logits against the oracle at every step, and the last layer's cached keys and values of
    the first sequence.  The oracle's two passes run side by side (they are independent); a line is printed
    after each phase because the whole test takes a few minutes."""
    import threading
    import time
    from tests import gpu_util as G

    def say(msg):
        with capsys.disabled():
            print(f"\n[large24_b1024] {msg}", flush=True)

    t0 = time.time()
    wl = W.make("large24_b1024")
    cfg = wl.cfg
    tol = G.TOL["bf16"]
    sample = [0, 1023]
    B, S = len(wl.enc_lens), cfg.prompt_len + cfg.max_new - 1
    toks = np.random.default_rng(44).integers(3, cfg.vocab, size=(B, S)).astype(np.int32)
    say(f"inputs drawn ({time.time() - t0:.0f} s); oracle: {len(sample)} sequences x {S} positions x {cfg.n_layers} layers")
    sub = wl.subset(sample)
    m = oracle.Model(cfg, wl.weights)
    res = {}
    first = wl.subset(sample[:1])
    th = threading.Thread(target=lambda: res.update(kv=m.self_kv(cfg.n_layers - 1, first.enc, toks[sample[0]])))
    th.start()
    ref = m.decode_forced(sub.enc, sub.enc_lens, toks[sample])
    say(f"oracle logits done ({time.time() - t0:.0f} s)")
    dec = G.make_decoder(wl, max_dec_len=cfg.max_dec_len, poison=True)
    glog, gids = G.forced_logits_gpu(dec, wl, toks, rows=sample)
    say(f"HIP path done ({time.time() - t0:.0f} s)")
    err, near = G.check_forced(ref, glog, gids, tol)
    th.join()
    Kr, Vr = res["kv"]
    Kg, Vg = dec.aed_read_self_kv(cfg.n_layers - 1, sample[0])
    assert Kg.shape == Kr.shape == (S, cfg.d_model)
    kerr = max(float(np.abs(Kg - Kr).max()), float(np.abs(Vg - Vr).max()))
    assert kerr <= tol, f"self K/V of sequence {sample[0]}, last layer: {kerr:.3e} > {tol}"
    say(f"teacher-forced over {S} positions: max |dlogit| = {err:.3e}, near ties {near}, max |dK,dV| = {kerr:.3e}")
    dec.close()
