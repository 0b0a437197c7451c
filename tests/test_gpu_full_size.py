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
