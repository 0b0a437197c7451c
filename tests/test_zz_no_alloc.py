"""aed_decode_step_noalloc (the step with its scratch memory in a static device array, for callers that cannot
allocate) against aed_decode_step, through the C ABI: same tokens, bit-equal logits, on a batch whose long
sequences are cut into chunks (the attention partials and arrival counters live in the array) and then on a
smaller batch that finds the first one's leftovers in the array."""
import ctypes as C

import numpy as np
import pytest

from paper_2503_05931_amd import binding, workloads as W

pytestmark = pytest.mark.gpu


def _workload(enc_lens, seed, max_new):
    cfg = W.DecoderConfig(name="unit", n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=512, vocab=256,
                          dtype="bf16", batch=len(enc_lens), prompt_len=4, max_new=max_new)
    return W.custom(cfg, enc_lens, seed, random_ln=True)


def _run(dec, wl, toks, noalloc):
    """S teacher-forced steps through the raw entry point; returns (logits [S, B, V], ids [S, B]) as numpy."""
    import torch
    lib = dec.lib
    B, S = toks.shape
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    tok_dev = torch.from_numpy(np.ascontiguousarray(toks.T)).to(dec.device)   # [S, B]
    logits = torch.zeros((S, B, wl.cfg.vocab), dtype=torch.float32, device=dec.device)
    ids = torch.zeros((S, B), dtype=torch.int32, device=dec.device)
    torch.cuda.synchronize()
    fn = lib.aed_decode_step_noalloc if noalloc else lib.aed_decode_step
    for s in range(S):
        st = fn(dec.handle, C.c_void_p(tok_dev[s].data_ptr()), C.c_void_p(ids[s].data_ptr()),
                C.c_void_p(logits[s].data_ptr()))
        assert st == binding.AED_OK, lib.aed_last_error(dec.handle).decode()
    dec.stream.synchronize()
    torch.cuda.synchronize()
    return logits.cpu().numpy(), ids.cpu().numpy()


def test_noalloc_step_equals_step_then_a_smaller_batch():
    import torch
    from tests import gpu_util as G
    assert torch.cuda.is_available()
    rng = np.random.default_rng(12)
    # 3 sequences x 4 heads: far fewer than 128 (sequence, head) pairs, so sequences are cut into 64-key chunks:
    # 8 chunks of cross-attention keys, up to 3 of self-attention keys at 140 positions
    big = _workload([500, 300, 77], seed=77, max_new=140)
    small = _workload([33, 5], seed=78, max_new=140)
    cases = [(big, rng.integers(0, 256, size=(3, 140)).astype(np.int32)),
             (small, rng.integers(0, 256, size=(2, 21)).astype(np.int32))]
    for wl, toks in cases:
        # a workspace full of NaN patterns: the static-array path must not depend on the workspace's activations
        dec = G.make_decoder(wl, max_batch=5, max_total=1500, max_dec_len=160, poison=True)
        got_l, got_i = _run(dec, wl, toks, noalloc=True)
        ref_l, ref_i = _run(dec, wl, toks, noalloc=False)
        assert np.isfinite(got_l).all()
        assert (got_i == ref_i).all(), "token ids differ"
        assert (got_l == ref_l).all(), f"logits differ by up to {np.abs(got_l - ref_l).max():.3e}"
        # steps of both kinds mixed in one batch
        mix_l, mix_i = None, None
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        tok_dev = torch.from_numpy(np.ascontiguousarray(toks.T)).to(dec.device)
        lg = torch.zeros((toks.shape[0], wl.cfg.vocab), dtype=torch.float32, device=dec.device)
        out = torch.zeros(toks.shape[0], dtype=torch.int32, device=dec.device)
        torch.cuda.synchronize()
        for s in range(min(20, toks.shape[1])):
            fn = dec.lib.aed_decode_step_noalloc if s % 2 else dec.lib.aed_decode_step
            assert fn(dec.handle, C.c_void_p(tok_dev[s].data_ptr()), C.c_void_p(out.data_ptr()),
                      C.c_void_p(lg.data_ptr())) == binding.AED_OK
            dec.stream.synchronize()
            assert (lg.cpu().numpy() == ref_l[s]).all() and (out.cpu().numpy() == ref_i[s]).all()
        dec.close()


def test_noalloc_step_rejects_a_decoder_that_does_not_fit():
    import torch
    wl = _workload([5] * 4, seed=3, max_new=8)
    cfg = wl.cfg
    # max_batch 2048 of this model needs 28 MiB of step activations: beyond the 8 MiB array
    dec = binding.Decoder(cfg, wl.weights, max_batch=2048, max_total_enc_frames=4096, max_dec_len=16)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    tok = torch.zeros(4, dtype=torch.int32, device=dec.device)
    out = torch.zeros(4, dtype=torch.int32, device=dec.device)
    torch.cuda.synchronize()
    st = dec.lib.aed_decode_step_noalloc(dec.handle, C.c_void_p(tok.data_ptr()), C.c_void_p(out.data_ptr()), None)
    assert st == binding.AED_ECAPACITY
    assert b"static scratch" in dec.lib.aed_last_error(dec.handle)
    # the workspace path still takes the same decoder
    assert dec.lib.aed_decode_step(dec.handle, C.c_void_p(tok.data_ptr()), C.c_void_p(out.data_ptr()), None) == binding.AED_OK
    dec.stream.synchronize()
    dec.close()
