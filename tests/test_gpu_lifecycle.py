"""GPU tests of the library's state handling: several decoders alive at once on one device (each on its own stream,
their steps interleaved), and handles created and destroyed many times (nothing the library owns may pile up)."""
import numpy as np
import pytest

from paper_2503_05931_amd import workloads as W

pytestmark = pytest.mark.gpu


def _unit(dtype, d_model, n_heads, head_dim, enc_lens, seed, **kw):
    cfg = W.DecoderConfig(name="unit", n_layers=2, d_model=d_model, n_heads=n_heads, head_dim=head_dim, d_ffn=512,
                          vocab=256, dtype=dtype, batch=len(enc_lens), prompt_len=4, max_new=24, **kw)
    return W.custom(cfg, enc_lens, seed, random_ln=True)


def test_two_decoders_interleaved_on_one_device(oracle):
    """A bf16 decoder whose long sequences are cut into merged chunks and an fp32 decoder of another shape take
    turns, step by step, on their own streams; every logit of both is compared with the oracle, as if each had
    run alone."""
    import torch
    from tests import gpu_util as G
    wl_a = _unit("bf16", 256, 4, 64, [300, 7, 150], seed=5)
    wl_b = _unit("fp32", 512, 4, 128, [9, 33, 1, 64, 17], seed=6)
    S = 20
    tok_a = np.random.default_rng(1).integers(0, 256, size=(3, S)).astype(np.int32)
    tok_b = np.random.default_rng(2).integers(0, 256, size=(5, S)).astype(np.int32)
    ref_a = oracle.Model(wl_a.cfg, wl_a.weights).decode_forced(wl_a.enc, wl_a.enc_lens, tok_a)
    ref_b = oracle.Model(wl_b.cfg, wl_b.weights).decode_forced(wl_b.enc, wl_b.enc_lens, tok_b)
    dec_a, dec_b = G.make_decoder(wl_a), G.make_decoder(wl_b)
    dec_a.aed_cross_kv_precompute(dec_a.to_device(wl_a.enc), wl_a.enc_lens)
    dec_b.aed_cross_kv_precompute(dec_b.to_device(wl_b.enc), wl_b.enc_lens)
    dev_a = torch.from_numpy(np.ascontiguousarray(tok_a.T)).to(dec_a.device)
    dev_b = torch.from_numpy(np.ascontiguousarray(tok_b.T)).to(dec_b.device)
    log_a, ids_a, log_b, ids_b = [], [], [], []
    for s in range(S):  # no synchronisation between the two: their launches overlap on the device
        out, lg = dec_a.aed_decode_step(dev_a[s].contiguous())
        log_a.append(lg); ids_a.append(out)
        out, lg = dec_b.aed_decode_step(dev_b[s].contiguous())
        log_b.append(lg); ids_b.append(out)
    torch.cuda.synchronize()
    G.check_forced(ref_a, torch.stack(log_a, 1).cpu().numpy().astype(np.float64), torch.stack(ids_a, 1).cpu().numpy(),
                   G.TOL["bf16"])
    G.check_forced(ref_b, torch.stack(log_b, 1).cpu().numpy().astype(np.float64), torch.stack(ids_b, 1).cpu().numpy(),
                   G.TOL["fp32"])
    # and a greedy decode on one while the other has a step batch open
    dec_b.aed_cross_kv_precompute(dec_b.to_device(wl_b.enc), wl_b.enc_lens)
    ref_t, ref_l, ref_logits = oracle.Model(wl_b.cfg, wl_b.weights).greedy_decode(wl_b.enc, wl_b.enc_lens, wl_b.prompt, 12,
                                                                               want_logits=True)
    toks, lens = dec_b.aed_greedy_decode(torch.from_numpy(wl_b.prompt).to(dec_b.device), 12)
    out, lg = dec_a.aed_decode_step(dev_a[0].contiguous())   # dec_a's batch is still at position S: one more step
    toks = toks.cpu().numpy()
    first = G.first_near_tie(ref_logits, G.TOL["fp32"])
    for b in range(5):
        assert (toks[b, :first[b]] == ref_t[b, :first[b]]).all()
    dec_a.close()
    dec_b.close()


def test_create_destroy_many_times_leaves_nothing_behind():
    """40 handles created, used (one batch, a few greedy tokens: graphs, events and pinned memory come into being) and
    destroyed: the device's free memory afterwards is what it was after the first few (torch's own caches warm up
    during those)."""
    import torch
    from tests import gpu_util as G
    wl = _unit("bf16", 256, 4, 64, [20, 5], seed=9)
    prompt = None
    free_after = []
    for i in range(40):
        dec = G.make_decoder(wl, poison=False)
        if prompt is None:
            prompt = torch.from_numpy(wl.prompt).to(dec.device)
            enc = dec.to_device(wl.enc)
        dec.aed_cross_kv_precompute(enc, wl.enc_lens)
        toks, lens = dec.aed_greedy_decode(prompt, 6)
        assert int(lens.sum().item()) == 12
        dec.close()
        del dec, toks, lens
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        free_after.append(torch.cuda.mem_get_info()[0])
    # allow the allocator's granularity, not a per-handle loss: 35 more handles may not cost 32 MiB
    assert free_after[4] - free_after[-1] < (32 << 20), f"free memory fell from {free_after[4]} to {free_after[-1]}"
